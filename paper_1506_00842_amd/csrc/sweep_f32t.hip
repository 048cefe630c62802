// Instantiations of the sweep with the fp32 matrix-core network that reads the low
// parameters' layer-1 share from a per-member table and computes the high parameters'
// share once per tile.
#include "net_f32t.h"
#include "sweep_kernel.h"

namespace tuner {

#define TUNER_F32T(NT1, NT2, R, NW) {NET_F32_MFMA, 0, NT1, NT2, R, NW, 32, sweep_kernel<F32TNet<NT1, NT2>, R, NW>}
static const Variant kF32TVariants[] = {
    TUNER_F32T(1, 0, 2, 16), TUNER_F32T(2, 0, 2, 16), TUNER_F32T(4, 0, 2, 8),
    TUNER_F32T(1, 1, 2, 16), TUNER_F32T(2, 2, 2, 16), TUNER_F32T(4, 4, 2, 8),
};

const Variant* find_variant_f32t(int NT1, int NT2) {
  for (const Variant& v : kF32TVariants)
    if (v.NT1 == NT1 && v.NT2 == NT2) return &v;
  return nullptr;
}

}  // namespace tuner
