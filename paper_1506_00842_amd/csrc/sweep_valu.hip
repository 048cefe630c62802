// Instantiations of the sweep with the plain vector-ALU network.
#include "net_valu.h"
#include "sweep_kernel.h"

namespace tuner {

// KS = PMAX (inputs padded), NT = padded hidden width / 32; 64 configurations per wave tile
#define TUNER_VALU(PMAX, NT1, NT2, R, NW) \
  {NET_F32_VALU, PMAX, NT1, NT2, R, NW, 64, sweep_kernel<ValuNet<PMAX, NT1 * 32, NT2 * 32>, R, NW>}
static const Variant kValuVariants[] = {
    TUNER_VALU(8, 1, 0, 1, 16),  TUNER_VALU(16, 1, 0, 1, 16),  TUNER_VALU(32, 1, 0, 1, 16),
    TUNER_VALU(8, 2, 0, 1, 16),  TUNER_VALU(16, 2, 0, 1, 16),  TUNER_VALU(32, 2, 0, 1, 16),
    TUNER_VALU(8, 4, 0, 1, 16),  TUNER_VALU(16, 4, 0, 1, 16),  TUNER_VALU(32, 4, 0, 1, 16),
    TUNER_VALU(8, 1, 1, 1, 16),  TUNER_VALU(16, 1, 1, 1, 16),  TUNER_VALU(32, 1, 1, 1, 16),
    TUNER_VALU(8, 2, 2, 1, 16),  TUNER_VALU(16, 2, 2, 1, 16),  TUNER_VALU(32, 2, 2, 1, 16),
    TUNER_VALU(8, 4, 4, 1, 8),   TUNER_VALU(16, 4, 4, 1, 8),   TUNER_VALU(32, 4, 4, 1, 8),
};

const Variant* find_variant_valu(int KS, int NT1, int NT2) {
  for (const Variant& v : kValuVariants)
    if (v.KS == KS && v.NT1 == NT1 && v.NT2 == NT2) return &v;
  return nullptr;
}

}  // namespace tuner
