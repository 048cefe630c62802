// fp32 matrix-core network with the layer-1 contribution of the high parameters
// computed once per tile.  Paper: Section 4.2 (neuron), Section 5.2 (sigmoid hidden
// layer), Section 5.1 (the space is a Cartesian product: consecutive configurations
// share all but their last few parameter values).
//
// A tile is 32 consecutive configurations starting at a multiple of 32, so every
// parameter whose stride is a multiple of 32 (the "high" parameters, indices
// 0 .. p0-1) has one value for the whole tile.  Their part of the layer-1
// pre-activation,
//     z_high[u] = b1[u] + sum_{p < p0} W1[u][p] x_p,
// is the same for all 32 configurations: it is computed once per (member, tile) on
// the vector ALU, one unit per lane, passed through a per-wave LDS scratch into the
// accumulator layout of net_f32.h, and the matrix instructions only contract over the
// "low" parameters p0 .. P-1 (KSL steps of two).  For the 2^27 space this replaces 16
// of the 80 matrix instructions per member and tile by 6.
//
// Packed member (fp32 words), hidden-layer weights and biases times -log2(e):
//   W1A [NT1][ceil(KSL/4)][64 lanes][4]  lane (n, h), step s = 4 sg + j: W1[32 t + n][p0 + 2 s + h]
//   W2A, b2A, woA                        as in net_f32.h
//   WH  [p0 + 1][NT1 * 32]               row p < p0: W1[u][p]; row p0: b1[u]
#pragma once
#include "net_f32.h"

namespace tuner {

template <int KSL, int NT1, int NT2>
struct F32HNet {
  static constexpr int kTile = 32;
  static constexpr bool kHoist = true;
  static constexpr int kUnits = NT1 * 32;
  static constexpr int kScratchZ = kUnits < 64 ? 64 : kUnits;   // floats of the z_high scratch
  struct Feat { float x[KSL]; };   // B operand of layer 1: feature of parameter p0 + 2 s + h

  static __device__ __forceinline__ void load_features(const DevSpace& sp, uint32_t i, int lane, bool pow2,
                                                       const NetOffsets& o, Feat& f) {
    const int p = o.p0 + (lane >> 5);
    if (pow2) {
#pragma unroll
      for (int s = 0; s < KSL; ++s) f.x[s] = feature_at_t<true>(sp, p + 2 * s, i);   // 0 past the last parameter
    } else {
#pragma unroll
      for (int s = 0; s < KSL; ++s) f.x[s] = feature_at_t<false>(sp, p + 2 * s, i);
    }
  }
  static __device__ __forceinline__ void zero_features(Feat& f) {
#pragma unroll
    for (int s = 0; s < KSL; ++s) f.x[s] = 0.0f;
  }

  // Once per tile: xs[p] = feature of high parameter p (0 for p >= p0), p = 0..31, read by
  // every member's forward().  `i` is the lane's own configuration of the tile.
  static __device__ __forceinline__ void load_high(const DevSpace& sp, uint32_t i, int lane, bool pow2,
                                                   const NetOffsets& o, float* xs) {
    if (lane < 32) {
      const uint32_t base = i - (uint32_t)lane;          // lane = the configuration's place in the tile
      const float x = feature_at(sp, lane, base, pow2);
      xs[lane] = lane < o.p0 ? x : 0.0f;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  static __device__ __forceinline__ float forward(const uint32_t* __restrict__ wm, const Feat& f, int lane,
                                                  const NetOffsets& o, const float* xs, float* zs) {
    const float* w = reinterpret_cast<const float*>(wm);
    const int h = lane >> 5;
    // the low parameters' weights first, where the register budget allows (the 128-wide
    // variants run 2 waves per SIMD): their reads are in flight while z_high is summed
    const float4* w1 = reinterpret_cast<const float4*>(w + o.w1);
    constexpr int KG = (KSL + 3) / 4;       // groups of 4 steps in the packed layout
    constexpr bool kEarly = NT1 >= 4;
    float4 wl[KG][NT1];
    if constexpr (kEarly) {
#pragma unroll
      for (int sg = 0; sg < KG; ++sg)
#pragma unroll
        for (int t = 0; t < NT1; ++t) wl[sg][t] = w1[(t * KG + sg) * 64 + lane];
    }
    // z_high, one unit per lane (kUnits / 64 units per lane for the wide nets)
    {
      const float* wh = w + o.wh;
      const int p0 = o.p0;
      constexpr int UPL = kUnits > 64 ? kUnits / 64 : 1;
      float z[UPL];
#pragma unroll
      for (int q = 0; q < UPL; ++q) z[q] = wh[p0 * kUnits + ((lane + 64 * q) % kUnits)];
      int p = 0;
      for (; p + 4 <= p0; p += 4) {
        const float4 x = *reinterpret_cast<const float4*>(xs + p);   // same address in every lane
#pragma unroll
        for (int q = 0; q < UPL; ++q) {
          const int u = (lane + 64 * q) % kUnits;
          z[q] = fmaf(wh[(p + 0) * kUnits + u], x.x, z[q]);
          z[q] = fmaf(wh[(p + 1) * kUnits + u], x.y, z[q]);
          z[q] = fmaf(wh[(p + 2) * kUnits + u], x.z, z[q]);
          z[q] = fmaf(wh[(p + 3) * kUnits + u], x.w, z[q]);
        }
      }
      for (; p < p0; ++p) {
        const float x = xs[p];
#pragma unroll
        for (int q = 0; q < UPL; ++q) z[q] = fmaf(wh[p * kUnits + ((lane + 64 * q) % kUnits)], x, z[q]);
      }
#pragma unroll
      for (int q = 0; q < UPL; ++q) zs[lane + 64 * q] = z[q];
    }
    // a wave's LDS instructions execute in program order: the writes above are in place
    // when the reads below are served; the fence only keeps the compiler from reordering
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    floatx16 a1[NT1];
#pragma unroll
    for (int t = 0; t < NT1; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 zv = *reinterpret_cast<const float4*>(zs + 32 * t + 8 * g + 4 * h);
        a1[t][4 * g + 0] = zv.x; a1[t][4 * g + 1] = zv.y; a1[t][4 * g + 2] = zv.z; a1[t][4 * g + 3] = zv.w;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int sg = 0; sg < KG; ++sg) {
#pragma unroll
      for (int t = 0; t < NT1; ++t) {
        const float4 a = kEarly ? wl[sg][t] : w1[(t * KG + sg) * 64 + lane];
        if (4 * sg + 0 < KSL) a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, f.x[(4 * sg + 0) % KSL], a1[t], 0, 0, 0);
        if (4 * sg + 1 < KSL) a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, f.x[(4 * sg + 1) % KSL], a1[t], 0, 0, 0);
        if (4 * sg + 2 < KSL) a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, f.x[(4 * sg + 2) % KSL], a1[t], 0, 0, 0);
        if (4 * sg + 3 < KSL) a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, f.x[(4 * sg + 3) % KSL], a1[t], 0, 0, 0);
      }
    }
    return f32_after_layer1<NT1, NT2>(w, a1, lane, o);
  }
};

// One packed word of a member in this layout (device, used by the prep kernel).
__device__ inline float pack_word_f32h(const Shape& sh, const float* raw, int q) {
  const int r_w1 = 0, r_b1 = r_w1 + sh.H1 * sh.P;
  float v = 0.0f;
  if (q < sh.o_w2) {                                    // W1A: low parameters only, no bias column
    const int KG = (sh.KS + 3) / 4;
    const int j = q & 3, lane = (q >> 2) & 63, rest = q >> 8;
    const int sg = rest % KG, t = rest / KG;
    const int n = lane & 31, h = lane >> 5, s = 4 * sg + j;
    const int unit = 32 * t + n, p = sh.p0 + 2 * s + h;
    if (unit < sh.H1 && s < sh.KS && p < sh.P) v = raw[r_w1 + unit * sh.P + p] * kNegLog2e;
  } else if (q < sh.o_wh) {                             // W2A, b2A, woA: the plain layout's
    v = pack_word_f32(sh, raw, q);
  } else {                                              // WH
    q -= sh.o_wh;
    const int units = sh.NT1 * 32;
    const int row = q / units, u = q - row * units;
    if (u < sh.H1) {
      if (row < sh.p0) v = raw[r_w1 + u * sh.P + row] * kNegLog2e;
      else if (row == sh.p0) v = raw[r_b1 + u] * kNegLog2e;
    }
  }
  return v;
}

}  // namespace tuner
