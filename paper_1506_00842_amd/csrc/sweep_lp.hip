// Instantiations of the sweep with the 16-bit matrix-core networks
// (bf16 single plane; f16 two-plane split).
#include "net_lp.h"
#include "sweep_kernel.h"

namespace tuner {

#define TUNER_BF16(KB, NT1, NT2, R, NW) {NET_BF16, KB, NT1, NT2, R, NW, 32, sweep_kernel<LpNet<__bf16, 1, KB, NT1, NT2>, R, NW>}
// the 128-wide one-plane network: layer 1 tile by tile (LpNet's STREAM), which fits 128
// registers, so 16 waves per workgroup = four per SIMD
#define TUNER_BF16_WIDE(KB) {NET_BF16, KB, 4, 4, 2, 16, 32, sweep_kernel<LpNet<__bf16, 1, KB, 4, 4, true>, 2, 16>}
#define TUNER_F16X2(KB, NT1, NT2, R, NW) {NET_F16X2, KB, NT1, NT2, R, NW, 32, sweep_kernel<LpNet<_Float16, 2, KB, NT1, NT2>, R, NW>}
static const Variant kLpVariants[] = {
    TUNER_BF16(1, 1, 0, 2, 16), TUNER_BF16(2, 1, 0, 2, 16), TUNER_BF16(1, 2, 0, 2, 16), TUNER_BF16(2, 2, 0, 2, 16),
    TUNER_BF16(1, 4, 0, 2, 8), TUNER_BF16(2, 4, 0, 2, 8), TUNER_BF16(1, 1, 1, 2, 16), TUNER_BF16(2, 1, 1, 2, 16),
    TUNER_BF16(1, 2, 2, 2, 16), TUNER_BF16(2, 2, 2, 2, 16), TUNER_BF16_WIDE(1), TUNER_BF16_WIDE(2),
    TUNER_F16X2(1, 1, 0, 2, 16), TUNER_F16X2(2, 1, 0, 2, 16), TUNER_F16X2(1, 2, 0, 2, 16), TUNER_F16X2(2, 2, 0, 2, 16),
    TUNER_F16X2(1, 4, 0, 2, 8), TUNER_F16X2(2, 4, 0, 2, 8), TUNER_F16X2(1, 1, 1, 2, 16), TUNER_F16X2(2, 1, 1, 2, 16),
    TUNER_F16X2(1, 2, 2, 2, 16), TUNER_F16X2(2, 2, 2, 2, 16), TUNER_F16X2(1, 4, 4, 2, 8), TUNER_F16X2(2, 4, 4, 2, 8),
};

const Variant* find_variant_lp(int net, int KS, int NT1, int NT2) {
  for (const Variant& v : kLpVariants)
    if (v.net == net && v.KS == KS && v.NT1 == NT1 && v.NT2 == NT2) return &v;
  return nullptr;
}

}  // namespace tuner
