// Instantiations of the sweep with the fp32 matrix-core network.
#include "net_f32.h"
#include "sweep_kernel.h"

namespace tuner {

#define TUNER_F32(KS, NT1, NT2, R, NW) {NET_F32_MFMA, KS, NT1, NT2, R, NW, 32, sweep_kernel<F32Net<KS, NT1, NT2>, R, NW>}
static const Variant kF32Variants[] = {
    TUNER_F32(2, 1, 0, 2, 16), TUNER_F32(4, 1, 0, 2, 16), TUNER_F32(6, 1, 0, 2, 16), TUNER_F32(8, 1, 0, 2, 16), TUNER_F32(10, 1, 0, 2, 16), TUNER_F32(12, 1, 0, 2, 16), TUNER_F32(14, 1, 0, 2, 16), TUNER_F32(16, 1, 0, 2, 16),
    TUNER_F32(2, 2, 0, 2, 16), TUNER_F32(4, 2, 0, 2, 16), TUNER_F32(6, 2, 0, 2, 16), TUNER_F32(8, 2, 0, 2, 16), TUNER_F32(10, 2, 0, 2, 16), TUNER_F32(12, 2, 0, 2, 16), TUNER_F32(14, 2, 0, 2, 16), TUNER_F32(16, 2, 0, 2, 16),
    TUNER_F32(2, 4, 0, 2, 8), TUNER_F32(4, 4, 0, 2, 8), TUNER_F32(6, 4, 0, 2, 8), TUNER_F32(8, 4, 0, 2, 8), TUNER_F32(10, 4, 0, 2, 8), TUNER_F32(12, 4, 0, 2, 8), TUNER_F32(14, 4, 0, 2, 8), TUNER_F32(16, 4, 0, 2, 8),
    TUNER_F32(2, 1, 1, 2, 16), TUNER_F32(4, 1, 1, 2, 16), TUNER_F32(6, 1, 1, 2, 16), TUNER_F32(8, 1, 1, 2, 16), TUNER_F32(10, 1, 1, 2, 16), TUNER_F32(12, 1, 1, 2, 16), TUNER_F32(14, 1, 1, 2, 16), TUNER_F32(16, 1, 1, 2, 16),
    TUNER_F32(2, 2, 2, 2, 16), TUNER_F32(4, 2, 2, 2, 16), TUNER_F32(6, 2, 2, 2, 16), TUNER_F32(8, 2, 2, 2, 16), TUNER_F32(10, 2, 2, 2, 16), TUNER_F32(12, 2, 2, 2, 16), TUNER_F32(14, 2, 2, 2, 16), TUNER_F32(16, 2, 2, 2, 16),
    TUNER_F32(2, 4, 4, 2, 8), TUNER_F32(4, 4, 4, 2, 8), TUNER_F32(6, 4, 4, 2, 8), TUNER_F32(8, 4, 4, 2, 8), TUNER_F32(10, 4, 4, 2, 8), TUNER_F32(12, 4, 4, 2, 8), TUNER_F32(14, 4, 4, 2, 8), TUNER_F32(16, 4, 4, 2, 8),
};

const Variant* find_variant_f32(int KS, int NT1, int NT2) {
  for (const Variant& v : kF32Variants)
    if (v.KS == KS && v.NT1 == NT1 && v.NT2 == NT2) return &v;
  return nullptr;
}

}  // namespace tuner
