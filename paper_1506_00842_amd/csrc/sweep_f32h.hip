// Instantiations of the sweep with the fp32 matrix-core network that computes the high
// parameters' layer-1 share once per tile.
#include "net_f32h.h"
#include "sweep_kernel.h"

namespace tuner {

#define TUNER_F32H(KS, NT1, NT2, R, NW) {NET_F32_MFMA, KS, NT1, NT2, R, NW, 32, sweep_kernel<F32HNet<KS, NT1, NT2>, R, NW>}
static const Variant kF32HVariants[] = {
    TUNER_F32H(1, 1, 0, 2, 16), TUNER_F32H(2, 1, 0, 2, 16), TUNER_F32H(3, 1, 0, 2, 16), TUNER_F32H(4, 1, 0, 2, 16),
    TUNER_F32H(1, 2, 0, 2, 16), TUNER_F32H(2, 2, 0, 2, 16), TUNER_F32H(3, 2, 0, 2, 16), TUNER_F32H(4, 2, 0, 2, 16),
    TUNER_F32H(1, 4, 0, 2, 8), TUNER_F32H(2, 4, 0, 2, 8), TUNER_F32H(3, 4, 0, 2, 8), TUNER_F32H(4, 4, 0, 2, 8),
    TUNER_F32H(1, 1, 1, 2, 16), TUNER_F32H(2, 1, 1, 2, 16), TUNER_F32H(3, 1, 1, 2, 16), TUNER_F32H(4, 1, 1, 2, 16),
    TUNER_F32H(1, 2, 2, 2, 16), TUNER_F32H(2, 2, 2, 2, 16), TUNER_F32H(3, 2, 2, 2, 16), TUNER_F32H(4, 2, 2, 2, 16),
    TUNER_F32H(1, 4, 4, 2, 8), TUNER_F32H(2, 4, 4, 2, 8), TUNER_F32H(3, 4, 4, 2, 8), TUNER_F32H(4, 4, 4, 2, 8),
};

const Variant* find_variant_f32h(int KSL, int NT1, int NT2) {
  for (const Variant& v : kF32HVariants)
    if (v.KS == KSL && v.NT1 == NT1 && v.NT2 == NT2) return &v;
  return nullptr;
}

}  // namespace tuner
