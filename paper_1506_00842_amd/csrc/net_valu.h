// Network evaluation on the plain vector ALU: one configuration per lane, fp32
// v_fma_f32, weights broadcast to all lanes from LDS (every lane reads the same
// address).  Paper: Section 4.2 (neuron), Section 5.2 (sigmoid hidden layer).
// This is the straightforward mapping; it is kept as the reference point against
// which the matrix-core networks are measured (its ceiling is half of theirs:
// one FMA per lane per 4-cycle issue, 78.6 TFLOP/s on the chip).
//
// Packed member (fp32 words), hidden-layer weights and biases times -log2(e):
//   W1v [H1P][PMAX]   rows padded with zeros to PMAX inputs, H1P units
//   W2v [H2P][H1P]    (two hidden layers only)
//   b1v [H1P], b2v [H2P], wov [last hidden width, padded]
#pragma once
#include "sweep_common.h"

namespace tuner {

template <int PMAX, int H1P, int H2P>
struct ValuNet {
  static constexpr int kTile = 64;
  struct Feat { float x[PMAX]; };

  static constexpr bool kBiasInput = false;
  static constexpr bool kHoist = false;
  static __device__ __forceinline__ void load_features(const DevSpace& sp, uint32_t i, int lane, bool pow2,
                                                       const NetOffsets&, Feat& f) {
    if (pow2) {
#pragma unroll
      for (int p = 0; p < PMAX; ++p) f.x[p] = feature_at_t<true>(sp, p, i);   // 0 past the last parameter
    } else {
#pragma unroll
      for (int p = 0; p < PMAX; ++p) f.x[p] = feature_at_t<false>(sp, p, i);
    }
  }
  static __device__ __forceinline__ void zero_features(Feat& f) {
#pragma unroll
    for (int p = 0; p < PMAX; ++p) f.x[p] = 0.0f;
  }

  template <int N>
  static __device__ __forceinline__ float dot_row(const float* __restrict__ row, const float (&v)[N], float acc) {
    const float4* r4 = reinterpret_cast<const float4*>(row);
#pragma unroll
    for (int jj = 0; jj < N / 4; ++jj) {
      const float4 q = r4[jj];
      acc = fmaf(q.x, v[4 * jj + 0], acc);
      acc = fmaf(q.y, v[4 * jj + 1], acc);
      acc = fmaf(q.z, v[4 * jj + 2], acc);
      acc = fmaf(q.w, v[4 * jj + 3], acc);
    }
    return acc;
  }

  // B units of a layer at a time: B independent accumulator chains hide the latency of the
  // dependent multiply-adds and of the broadcast reads (rows past the real width are zero in
  // the packed layout, their output weights too).
  template <int N, int B>
  static __device__ __forceinline__ void dot_rows(const float* __restrict__ rows, const float (&v)[N], float (&z)[B]) {
#pragma unroll
    for (int jj = 0; jj < N / 4; ++jj) {
      float4 q[B];
#pragma unroll
      for (int r = 0; r < B; ++r) q[r] = reinterpret_cast<const float4*>(rows + r * N)[jj];
#pragma unroll
      for (int r = 0; r < B; ++r) z[r] = fmaf(q[r].x, v[4 * jj + 0], z[r]);
#pragma unroll
      for (int r = 0; r < B; ++r) z[r] = fmaf(q[r].y, v[4 * jj + 1], z[r]);
#pragma unroll
      for (int r = 0; r < B; ++r) z[r] = fmaf(q[r].z, v[4 * jj + 2], z[r]);
#pragma unroll
      for (int r = 0; r < B; ++r) z[r] = fmaf(q[r].w, v[4 * jj + 3], z[r]);
    }
  }

  // one block of B units of the last hidden layer: pre-activations, sigmoid, output layer
  template <int N, int B>
  static __device__ __forceinline__ float last_layer_block(const float* __restrict__ rows, const float* __restrict__ bias,
                                                           const float* __restrict__ wo, const float (&v)[N], float y) {
    static_assert(B == 4, "biases and output weights are read four at a time");
    const float4 b4 = *reinterpret_cast<const float4*>(bias);
    const float4 q4 = *reinterpret_cast<const float4*>(wo);
    float z[B] = {b4.x, b4.y, b4.z, b4.w};
    dot_rows<N, B>(rows, v, z);
    y = fmaf(q4.x, sigmoid_prescaled(z[0]), y);
    y = fmaf(q4.y, sigmoid_prescaled(z[1]), y);
    y = fmaf(q4.z, sigmoid_prescaled(z[2]), y);
    y = fmaf(q4.w, sigmoid_prescaled(z[3]), y);
    return y;
  }

  static __device__ __forceinline__ float forward(const uint32_t* __restrict__ wm, const Feat& f, int lane,
                                                  const NetOffsets& o) {
    const float* w = reinterpret_cast<const float*>(wm);
    constexpr int kBlock = 4;
    float y = 0.0f;
    if constexpr (H2P == 0) {
      for (int u = 0; u < o.h1; u += kBlock)
        y = last_layer_block<PMAX, kBlock>(w + o.w1 + u * PMAX, w + o.b1 + u, w + o.wo + u, f.x, y);
    } else {
      float h1[H1P];
#pragma unroll
      for (int u = 0; u < H1P; ++u)
        h1[u] = sigmoid_prescaled(dot_row<PMAX>(w + o.w1 + u * PMAX, f.x, w[o.b1 + u]));
      for (int u = 0; u < o.h2; u += kBlock)
        y = last_layer_block<H1P, kBlock>(w + o.w2 + u * H1P, w + o.b2 + u, w + o.wo + u, h1, y);
    }
    return y;
  }
};

// One packed word of a member (device, used by the prep kernel).  sh.KS = PMAX,
// sh.NT1 * 32 = H1P, sh.NT2 * 32 = H2P.
__device__ inline float pack_word_valu(const Shape& sh, const float* raw, int q) {
  const int r_w1 = 0, r_b1 = r_w1 + sh.H1 * sh.P;
  const int r_w2 = r_b1 + sh.H1;
  const int r_b2 = r_w2 + sh.H2 * sh.H1;
  const int r_wo = sh.H2 ? r_b2 + sh.H2 : r_w2;
  const int HL = sh.H2 ? sh.H2 : sh.H1;
  const int pmax = sh.KS, h1p = sh.NT1 * 32;
  float v = 0.0f;
  if (q < sh.o_w2) {
    const int u = q / pmax, j = q % pmax;
    if (u < sh.H1 && j < sh.P) v = raw[r_w1 + u * sh.P + j] * kNegLog2e;
  } else if (q < sh.o_b1) {
    q -= sh.o_w2;
    const int u = q / h1p, j = q % h1p;
    if (u < sh.H2 && j < sh.H1) v = raw[r_w2 + u * sh.H1 + j] * kNegLog2e;
  } else if (q < sh.o_b2) {
    q -= sh.o_b1;
    if (q < sh.H1) v = raw[r_b1 + q] * kNegLog2e;
  } else if (q < sh.o_wo) {
    q -= sh.o_b2;
    if (q < sh.H2) v = raw[r_b2 + q] * kNegLog2e;
  } else {
    q -= sh.o_wo;
    if (q < HL) v = raw[r_wo + q];
  }
  return v;
}

}  // namespace tuner
