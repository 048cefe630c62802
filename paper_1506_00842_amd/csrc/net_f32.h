// Network evaluation on the matrix cores, fp32 in / fp32 accumulate
// (v_mfma_f32_32x32x2_f32).  Paper: Section 4.2 (neuron = weighted sum +
// activation), Section 5.2 (sigmoid hidden layer, linear output).
//
// A wave evaluates a tile of 32 configurations.  The weights are the A operand
// (rows = 32 units of the layer), the activations the B operand (columns = the
// 32 configurations), so a layer's output tile D[unit][config] leaves every lane
// (config c = lane % 32, half h = lane / 32) holding 16 units of its configuration:
//     unit(v, h) = 8 * (v / 4) + 4 * h + (v % 4),  v = 0..15
// which is the ownership the B operand of the next layer needs (lane half h
// supplies one k index per MFMA step), with the k order permuted; the permutation
// is folded into the packed weight layout, so layers chain with no cross-lane
// traffic.  -log2(e) is folded into the hidden layers' weights and biases.
//
// Packed member (fp32 words):
//   W1A [NT1][ceil(KS1/4)][64 lanes][4]   lane (n, h), steps s = 4*sg + j (KS1 is even;
//        the last group of an odd number of step pairs uses j = 0, 1 only):
//        unit = 32 t + n, input f = 2 s + h: W1[unit][f], b1[unit] at f = P, else 0
//   W2A [NT2][NT1][4][64 lanes][4]  lane (n, h): W2[32 u + n][32 t + 8 g + 4 h + j]
//   b2A [NT2][4][2][4]              b2[32 u + 8 g + 4 h + j]
//   woA [NTlast][4][2][4]           w_o[32 u + 8 g + 4 h + j]   (not scaled)
// Padded units have zero incoming and outgoing weights.
#pragma once
#include "sweep_common.h"

namespace tuner {

// Everything after the layer-1 pre-activations (scaled by -log2 e) are in a1: sigmoid,
// second hidden layer if any, output layer.  Returns the lane's share of the output.
// LDS reads are issued one step ahead of their use (the next layer's biases and first
// weights before a sigmoid pass, each group of weights before the matrix steps of the
// previous group), so that a wave is never left waiting for a read it has just issued.
template <int NT1, int NT2>
__device__ __forceinline__ float f32_after_layer1(const float* __restrict__ w, floatx16 (&a1)[NT1], int lane,
                                                  const NetOffsets& o) {
  const int h = lane >> 5;
  float part = 0.0f;
  if constexpr (NT2 > 0) {
    floatx16 a2[NT2];
    const float4* b2 = reinterpret_cast<const float4*>(w + o.b2);
#pragma unroll
    for (int u = 0; u < NT2; ++u)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 b = b2[(u * 4 + g) * 2 + h];
        a2[u][4 * g + 0] = b.x; a2[u][4 * g + 1] = b.y; a2[u][4 * g + 2] = b.z; a2[u][4 * g + 3] = b.w;
      }
    const float4* w2 = reinterpret_cast<const float4*>(w + o.w2);
    float4 a_next = w2[lane];
    // fp32 MFMA and VALU work do not overlap on a SIMD, so nothing is gained by
    // interleaving the sigmoid with the matrix instructions
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < NT1; ++t) sigmoid16(a1[t]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < NT1; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int u = 0; u < NT2; ++u) {
          const float4 a = a_next;
          // the weights of the next group (same nesting order: u fastest, then g, then t)
          const int un = u + 1 < NT2 ? u + 1 : 0;
          const int gn = un ? g : (g + 1 < 4 ? g + 1 : 0);
          const int tn = (un || gn) ? t : t + 1;
          if (tn < NT1) a_next = w2[((un * NT1 + tn) * 4 + gn) * 64 + lane];
          a2[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, a1[t][4 * g + 0], a2[u], 0, 0, 0);
          a2[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, a1[t][4 * g + 1], a2[u], 0, 0, 0);
          a2[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, a1[t][4 * g + 2], a2[u], 0, 0, 0);
          a2[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, a1[t][4 * g + 3], a2[u], 0, 0, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read (the next group's weights)
          __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);   // then this group's four matrix steps
        }
    // (kept behind the matrix steps: layer 1's activations still hold their registers there)
    __builtin_amdgcn_sched_barrier(0);
    const float4* wo = reinterpret_cast<const float4*>(w + o.wo);
    float4 q[NT2 * 4];
#pragma unroll
    for (int x = 0; x < NT2 * 4; ++x) q[x] = wo[x * 2 + h];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < NT2; ++u) sigmoid16(a2[u]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < NT2; ++u)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        part = fmaf(q[u * 4 + g].x, a2[u][4 * g + 0], part);
        part = fmaf(q[u * 4 + g].y, a2[u][4 * g + 1], part);
        part = fmaf(q[u * 4 + g].z, a2[u][4 * g + 2], part);
        part = fmaf(q[u * 4 + g].w, a2[u][4 * g + 3], part);
      }
  } else {
    const float4* wo = reinterpret_cast<const float4*>(w + o.wo);
    float4 q[NT1 * 4];
#pragma unroll
    for (int x = 0; x < NT1 * 4; ++x) q[x] = wo[x * 2 + h];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < NT1; ++t) sigmoid16(a1[t]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < NT1; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        part = fmaf(q[t * 4 + g].x, a1[t][4 * g + 0], part);
        part = fmaf(q[t * 4 + g].y, a1[t][4 * g + 1], part);
        part = fmaf(q[t * 4 + g].z, a1[t][4 * g + 2], part);
        part = fmaf(q[t * 4 + g].w, a1[t][4 * g + 3], part);
      }
  }
  return part;
}

template <int KS1, int NT1, int NT2>
struct F32Net {
  static constexpr int kTile = 32;
  struct Feat { float x[KS1]; };   // B operand of layer 1: feature 2 s + h, 1.0 in the bias slot

  // branch-free: slots past the last parameter decode to feature 0; the slot right
  // after it decodes to the constant 1 that multiplies the bias column (the prep kernel
  // points that slot of the table at the constant)
  static constexpr bool kBiasInput = true;
  static constexpr bool kHoist = false;
  static __device__ __forceinline__ void load_features(const DevSpace& sp, uint32_t i, int lane, bool pow2,
                                                       const NetOffsets&, Feat& f) {
    const int h = lane >> 5;
    if (pow2) {
#pragma unroll
      for (int s = 0; s < KS1; ++s) f.x[s] = feature_at_t<true>(sp, 2 * s + h, i);
    } else {
#pragma unroll
      for (int s = 0; s < KS1; ++s) f.x[s] = feature_at_t<false>(sp, 2 * s + h, i);
    }
  }
  static __device__ __forceinline__ void zero_features(Feat& f) {
#pragma unroll
    for (int s = 0; s < KS1; ++s) f.x[s] = 0.0f;
  }

  static __device__ __forceinline__ float forward(const uint32_t* __restrict__ wm, const Feat& f, int lane,
                                                  const NetOffsets& o) {
    const float* w = reinterpret_cast<const float*>(wm);
    const int h = lane >> 5;
    floatx16 a1[NT1];
#pragma unroll
    for (int t = 0; t < NT1; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) a1[t][v] = 0.0f;
    const float4* w1 = reinterpret_cast<const float4*>(w + o.w1);
    constexpr int KG = (KS1 + 3) / 4;       // groups of 4 steps in the packed layout
#pragma unroll
    for (int sg = 0; sg < KS1 / 4; ++sg) {
#pragma unroll
      for (int t = 0; t < NT1; ++t) {
        const float4 a = w1[(t * KG + sg) * 64 + lane];
        a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, f.x[4 * sg + 0], a1[t], 0, 0, 0);
        a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, f.x[4 * sg + 1], a1[t], 0, 0, 0);
        a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, f.x[4 * sg + 2], a1[t], 0, 0, 0);
        a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, f.x[4 * sg + 3], a1[t], 0, 0, 0);
      }
    }
    if constexpr (KS1 % 4 == 2) {
#pragma unroll
      for (int t = 0; t < NT1; ++t) {
        const float2 a = *reinterpret_cast<const float2*>(&w1[(t * KG + KS1 / 4) * 64 + lane]);
        a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, f.x[KS1 - 2], a1[t], 0, 0, 0);
        a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, f.x[KS1 - 1], a1[t], 0, 0, 0);
      }
    }
    return f32_after_layer1<NT1, NT2>(w, a1, lane, o);
  }
};

// One packed word of a member (device, used by the prep kernel).
__device__ inline float pack_word_f32(const Shape& sh, const float* raw, int q) {
  const int r_w1 = 0, r_b1 = r_w1 + sh.H1 * sh.P;
  const int r_w2 = r_b1 + sh.H1;
  const int r_b2 = r_w2 + sh.H2 * sh.H1;
  const int r_wo = sh.H2 ? r_b2 + sh.H2 : r_w2;
  const int HL = sh.H2 ? sh.H2 : sh.H1;
  float v = 0.0f;
  if (q < sh.o_w2) {                                    // W1A
    const int KG = (sh.KS + 3) / 4;
    const int j = q & 3, lane = (q >> 2) & 63, rest = q >> 8;
    const int sg = rest % KG, t = rest / KG;
    const int n = lane & 31, h = lane >> 5, s = 4 * sg + j;
    const int unit = 32 * t + n, f = 2 * s + h;
    if (unit < sh.H1 && s < sh.KS) {
      if (f < sh.P) v = raw[r_w1 + unit * sh.P + f] * kNegLog2e;
      else if (f == sh.P) v = raw[r_b1 + unit] * kNegLog2e;
    }
  } else if (q < sh.o_b2) {                             // W2A
    q -= sh.o_w2;
    const int j = q & 3, lane = (q >> 2) & 63, rest = q >> 8;
    const int g = rest & 3, t = (rest >> 2) % sh.NT1, u = (rest >> 2) / sh.NT1;
    const int n = lane & 31, h = lane >> 5;
    const int out = 32 * u + n, in = 32 * t + 8 * g + 4 * h + j;
    if (out < sh.H2 && in < sh.H1) v = raw[r_w2 + out * sh.H1 + in] * kNegLog2e;
  } else if (q < sh.o_wo) {                             // b2A
    q -= sh.o_b2;
    const int j = q & 3, h = (q >> 2) & 1, g = (q >> 3) & 3, u = q >> 5;
    const int unit = 32 * u + 8 * g + 4 * h + j;
    if (unit < sh.H2) v = raw[r_b2 + unit] * kNegLog2e;
  } else {                                              // woA
    q -= sh.o_wo;
    const int j = q & 3, h = (q >> 2) & 1, g = (q >> 3) & 3, u = q >> 5;
    const int unit = 32 * u + 8 * g + 4 * h + j;
    if (unit < HL) v = raw[r_wo + unit];
  }
  return v;
}

}  // namespace tuner
