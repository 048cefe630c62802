// fp32 matrix-core network whose whole layer 1 leaves the per-configuration matrix work:
// the high parameters' share is computed once per tile, the low parameters' share is read
// from a table.  Paper: Section 4.2 (neuron), Section 5.2 (sigmoid hidden layer), Section
// 5.1 (the space is a Cartesian product: consecutive configurations share all but their
// last few parameter values).
//
// A tile is 32 consecutive configurations starting at a multiple of 32.  When the low
// parameters p0 .. P-1 (stride < 32) span exactly 32 configurations (the stride of
// parameter p0-1 is 32), configuration c of EVERY tile has the same low parameter values,
// so their share of the layer-1 pre-activation
//     z_low[u][c] = sum_{p >= p0} W1[u][p] x_p(c)
// is one [units][32] matrix per member: it is tabulated when the weights are packed, in
// the accumulator layout of net_f32.h, and initialises the accumulators.  The share of
// the high parameters and the bias,
//     z_high[u] = b1[u] + sum_{p < p0} W1[u][p] x_p,
// is one vector per (member, tile).  It enters as the A operand of a single matrix step
// whose B operand is all ones: lane (n, h) supplies A[unit n][k = h], so each half of the
// wave sums every other term for its unit and the instruction adds both halves to all 32
// columns.  Layer 1 costs NT1 matrix instructions per member and tile (config of 14
// parameters, 64 units: 2 instead of 16), and no value crosses lanes.
//
// Packed member (fp32 words), hidden-layer weights and biases times -log2(e):
//   ZL  [NT1][4][64 lanes][4]        lane (c, h): z_low[32 t + 8 g + 4 h + j][c]
//   W2A, b2A, woA                    as in net_f32.h
//   WHT [NT1][RQ][64 lanes][4]       lane (n, h), term q = 2 (4 rq + j) + h of unit 32 t + n:
//        W1[unit][q] for q < p0, b1[unit] for q = p0, else 0;  RQ = ceil(ceil((p0 + 1) / 2) / 4)
#pragma once
#include "net_f32.h"

namespace tuner {

__host__ __device__ inline int f32t_term_groups(int p0) { return ((p0 + 2) / 2 + 3) / 4; }

template <int NT1, int NT2>
struct F32TNet {
  static constexpr int kTile = 32;
  static constexpr bool kHoist = true;
  static constexpr int kUnits = NT1 * 32;
  static constexpr int kScratchZ = 0;      // no z scratch: z_high goes straight into the A operand
  struct Feat {};                          // the low parameters' features are in the table

  static __device__ __forceinline__ void load_features(const DevSpace&, uint32_t, int, bool, const NetOffsets&, Feat&) {}
  static __device__ __forceinline__ void zero_features(Feat&) {}

  // Once per tile: the factors of the z_high terms, term q at xs[16 (q % 2) + q / 2]
  // (the feature of parameter q, 1 for the bias term q = p0, 0 beyond), read by every
  // member's forward().  `i` is the lane's own configuration of the tile.
  static __device__ __forceinline__ void load_high(const DevSpace& sp, uint32_t i, int lane, bool pow2,
                                                   const NetOffsets& o, float* xs) {
    if (lane < 32) {
      const uint32_t base = i - (uint32_t)lane;          // lane = the configuration's place in the tile
      const float x = feature_at(sp, lane, base, pow2);
      xs[16 * (lane & 1) + (lane >> 1)] = lane < o.p0 ? x : (lane == o.p0 ? 1.0f : 0.0f);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  static __device__ __forceinline__ float forward(const uint32_t* __restrict__ wm, const Feat&, int lane,
                                                  const NetOffsets& o, const float* xs, float*) {
    const float* w = reinterpret_cast<const float*>(wm);
    const int h = lane >> 5;
    // the table first: its reads are in flight while z_high is summed
    floatx16 a1[NT1];
    const float4* zl = reinterpret_cast<const float4*>(w + o.w1);
#pragma unroll
    for (int t = 0; t < NT1; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 zv = zl[(t * 4 + g) * 64 + lane];
        a1[t][4 * g + 0] = zv.x; a1[t][4 * g + 1] = zv.y; a1[t][4 * g + 2] = zv.z; a1[t][4 * g + 3] = zv.w;
      }
    // this half's terms of z_high for the lane's unit of every tile of units
    float zp[NT1];
#pragma unroll
    for (int t = 0; t < NT1; ++t) zp[t] = 0.0f;
    {
      const float4* wht = reinterpret_cast<const float4*>(w + o.wh);
      const float4* x4 = reinterpret_cast<const float4*>(xs + 16 * h);
      const int RQ = f32t_term_groups(o.p0);
      for (int rq = 0; rq < RQ; ++rq) {
        const float4 x = x4[rq];
#pragma unroll
        for (int t = 0; t < NT1; ++t) {
          const float4 a = wht[(t * RQ + rq) * 64 + lane];
          zp[t] = fmaf(a.x, x.x, zp[t]);
          zp[t] = fmaf(a.y, x.y, zp[t]);
          zp[t] = fmaf(a.z, x.z, zp[t]);
          zp[t] = fmaf(a.w, x.w, zp[t]);
        }
      }
    }
#pragma unroll
    for (int t = 0; t < NT1; ++t) a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(zp[t], 1.0f, a1[t], 0, 0, 0);
    return f32_after_layer1<NT1, NT2>(w, a1, lane, o);
  }
};

// One packed word of a member in this layout (device, used by the prep kernel).
__device__ inline float pack_word_f32t(const Shape& sh, const float* raw, int q, const DevSpace& sp) {
  const int r_w1 = 0, r_b1 = r_w1 + sh.H1 * sh.P;
  float v = 0.0f;
  if (q < sh.o_w2) {                                    // ZL
    const int j = q & 3, lane = (q >> 2) & 63, g = (q >> 8) & 3, t = q >> 10;
    const int c = lane & 31, h = lane >> 5;
    const int unit = 32 * t + 8 * g + 4 * h + j;
    if (unit < sh.H1) {
      const bool pow2 = sp.all_pow2 != 0;
      for (int p = sh.p0; p < sh.P; ++p)
        v = fmaf(raw[r_w1 + unit * sh.P + p] * kNegLog2e, feature_at(sp, p, (uint32_t)c, pow2), v);
    }
  } else if (q < sh.o_wh) {                             // W2A, b2A, woA: the plain layout's
    v = pack_word_f32(sh, raw, q);
  } else {                                              // WHT
    q -= sh.o_wh;
    const int RQ = f32t_term_groups(sh.p0);
    const int j = q & 3, lane = (q >> 2) & 63, rest = q >> 8;
    const int rq = rest % RQ, t = rest / RQ;
    const int n = lane & 31, h = lane >> 5;
    const int unit = 32 * t + n, term = 2 * (4 * rq + j) + h;
    if (unit < sh.H1) {
      if (term < sh.p0) v = raw[r_w1 + unit * sh.P + term] * kNegLog2e;
      else if (term == sh.p0) v = raw[r_b1 + unit] * kNegLog2e;
    }
  }
  return v;
}

}  // namespace tuner
