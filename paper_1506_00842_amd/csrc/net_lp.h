// Network evaluation on the 16-bit matrix cores with fp32 accumulation
// (v_mfma_f32_32x32x16_bf16 / _f16).  Paper: Section 4.2, Section 5.2.
//
// Two uses of one code path:
//   NPL = 1, T = bf16: features, weights and hidden activations are rounded to
//       bf16 (nearest even) before each layer's contraction; biases, sigmoid,
//       output dot product and ensemble mean stay in fp32.  Tolerance 1e-2.
//   NPL = 2, T = f16: every operand is split into two f16 planes, x = x_hi + x_lo
//       (x_hi = rn(x), x_lo = rn(x - x_hi): 22 significand bits), and a product is
//       the three terms a_hi b_hi + a_hi b_lo + a_lo b_hi accumulated in fp32, which
//       keeps products to about 2^-21 relative: the fp32 tolerance (1e-5) holds.
//
// Tile mapping as in the fp32 network: weights = A operand (rows = 32 units),
// activations = B operand (columns = 32 configurations); lane (c, h) ends a layer
// holding units 8 (v / 4) + 4 h + (v % 4), v = 0..15, of its configuration.  One
// MFMA contracts a block of 16 inputs: lane half h supplies 8 of them.  Block b
// of a 32-unit tile uses the lane's registers v = 8 b .. 8 b + 7, i.e. units
//     16 b + 8 (j / 4) + 4 h + (j % 4),  j = 0..7
// and the packed weights use the same order, so layers chain without shuffles.
// Layer 1: block kb, lane half h supplies inputs f = 16 kb + 8 h + j.
//
// Packed member (32-bit words; a 16-bit pair per word, element 2 jj in the low half):
//   W1A [NPL][NT1][KB1][64 lanes][4]      lane (n, h): W1[32 t + n][16 kb + 8 h + j]
//   W2A [NPL][NT2][2 NT1][64 lanes][4]    lane (n, h): W2[32 u + n][32 t + 16 b + 8 (j/4) + 4 h + j%4]
//   b1A, b2A, woA  fp32 [NT][4][2][4]     value for unit 32 t + 8 g + 4 h + j
// Hidden-layer weights and biases carry the factor -log2(e).
#pragma once
#include "sweep_common.h"

namespace tuner {

typedef float float2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

struct B4 { uint32_t w[4]; };   // 8 sixteen-bit operands of one lane

template <class T> struct LpTraits;
template <> struct LpTraits<__bf16> {
  typedef bf16x8 V8;
  typedef bf16x2 V2;
  static __device__ __forceinline__ floatx16 mfma(const B4& a, const B4& b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(V8, a), __builtin_bit_cast(V8, b), c, 0, 0, 0);
  }
};
template <> struct LpTraits<_Float16> {
  typedef f16x8 V8;
  typedef f16x2 V2;
  static __device__ __forceinline__ floatx16 mfma(const B4& a, const B4& b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(V8, a), __builtin_bit_cast(V8, b), c, 0, 0, 0);
  }
};

// (a, b) -> one word of two T, round to nearest even; lo word = the remainders
template <class T, int NPL>
__device__ __forceinline__ void pack_pair(float a, float b, uint32_t& hi, uint32_t& lo) {
  typedef typename LpTraits<T>::V2 V2;
  const float2v ab = {a, b};
  const V2 hv = __builtin_convertvector(ab, V2);
  hi = __builtin_bit_cast(uint32_t, hv);
  if constexpr (NPL == 2) {
    // a - hi as a fused multiply-add that reads the 16-bit half directly and rounds its
    // fp32 result into one half of the word (v_fma_mixlo_f16 / v_fma_mixhi_f16): two
    // instructions per pair instead of two conversions, two subtractions and a pack
    // (the factor -1 sits in a register the compiler cannot see through: as a literal it would
    // turn the multiply-add back into a subtraction of a converted value)
    float m1 = -1.0f;
    asm("" : "+v"(m1));
    const V2 lv = {(T)__builtin_fmaf((float)hv[0], m1, a), (T)__builtin_fmaf((float)hv[1], m1, b)};
    lo = __builtin_bit_cast(uint32_t, lv);
  } else {
    lo = 0u;
  }
}

// STREAM (two hidden layers only): layer 1 is evaluated one 32-unit tile at a time, each tile
// going through its sigmoid and into layer 2's accumulators before the next one is computed,
// so that a wave holds one layer-1 tile instead of all of them (128-wide networks then fit
// 128 registers, i.e. four waves per SIMD: the 16-bit matrix instructions of one wave run
// beside the vector work of the others).  Same operations per configuration, in the same
// order, as the plain evaluation: same bits.
template <class T, int NPL, int KB1, int NT1, int NT2, bool STREAM = false>
struct LpNet {
  typedef LpTraits<T> Tr;
  static constexpr int kTile = 32;
  struct Feat { B4 x[NPL][KB1]; };

  static constexpr bool kBiasInput = false;
  template <bool POW2>
  static __device__ __forceinline__ void load_features_t(const DevSpace& sp, uint32_t i, int h, Feat& f) {
#pragma unroll
    for (int kb = 0; kb < KB1; ++kb) {
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = feature_at_t<POW2>(sp, 16 * kb + 8 * h + j, i);   // 0 past the last parameter
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        uint32_t hi, lo;
        pack_pair<T, NPL>(v[2 * jj], v[2 * jj + 1], hi, lo);
        f.x[0][kb].w[jj] = hi;
        if constexpr (NPL == 2) f.x[1][kb].w[jj] = lo;
      }
    }
  }
  static constexpr bool kHoist = false;
  static __device__ __forceinline__ void load_features(const DevSpace& sp, uint32_t i, int lane, bool pow2,
                                                       const NetOffsets&, Feat& f) {
    if (pow2) load_features_t<true>(sp, i, lane >> 5, f);
    else load_features_t<false>(sp, i, lane >> 5, f);
  }
  static __device__ __forceinline__ void zero_features(Feat& f) {
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl)
#pragma unroll
      for (int kb = 0; kb < KB1; ++kb)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) f.x[pl][kb].w[jj] = 0u;
  }

  // The A operand of one block: NPL planes of 8 sixteen-bit weights per lane
  struct A4 { uint4 p[NPL]; };
  static __device__ __forceinline__ A4 load_a(const uint4* __restrict__ wa, int idx0, int plane_stride) {
    A4 a;
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl) a.p[pl] = wa[idx0 + pl * plane_stride];
    return a;
  }
  // acc += A * B with 1 (NPL = 1) or 3 (NPL = 2) matrix instructions
  static __device__ __forceinline__ floatx16 mma(const A4& a, const B4& b_hi, const B4& b_lo, floatx16 acc) {
    const B4 a0 = {{a.p[0].x, a.p[0].y, a.p[0].z, a.p[0].w}};
    acc = Tr::mfma(a0, b_hi, acc);
    if constexpr (NPL == 2) {
      acc = Tr::mfma(a0, b_lo, acc);
      const B4 a1 = {{a.p[NPL - 1].x, a.p[NPL - 1].y, a.p[NPL - 1].z, a.p[NPL - 1].w}};
      acc = Tr::mfma(a1, b_hi, acc);
    }
    return acc;
  }

  static __device__ __forceinline__ void init_bias(const float4* __restrict__ b, int t, int h, floatx16& acc) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 q = b[(t * 4 + g) * 2 + h];
      acc[4 * g + 0] = q.x; acc[4 * g + 1] = q.y; acc[4 * g + 2] = q.z; acc[4 * g + 3] = q.w;
    }
  }

  // LDS reads are issued one step ahead of their use (a block's weights before the matrix
  // steps of the previous block, the next layer's biases and the output weights before a
  // sigmoid pass), and each sigmoid runs as three passes over 16 registers so that no
  // instruction waits on the transcendental before it.
  static __device__ __forceinline__ float forward(const uint32_t* __restrict__ wm, const Feat& f, int lane,
                                                  const NetOffsets& o) {
    if constexpr (STREAM && NT2 > 0) return forward_stream(wm, f, lane, o);
    const int h = lane >> 5;
    floatx16 a1[NT1];
    const float4* b1 = reinterpret_cast<const float4*>(wm + o.b1);
#pragma unroll
    for (int t = 0; t < NT1; ++t) init_bias(b1, t, h, a1[t]);
    const uint4* w1 = reinterpret_cast<const uint4*>(wm + o.w1);
    {
      A4 a_next = load_a(w1, lane, NT1 * KB1 * 64);
#pragma unroll
      for (int kb = 0; kb < KB1; ++kb)
#pragma unroll
        for (int t = 0; t < NT1; ++t) {
          const A4 a = a_next;
          const int tn = t + 1 < NT1 ? t + 1 : 0, kn = tn ? kb : kb + 1;
          if (kn < KB1) a_next = load_a(w1, (tn * KB1 + kn) * 64 + lane, NT1 * KB1 * 64);
          a1[t] = mma(a, f.x[0][kb], f.x[NPL - 1][kb], a1[t]);
        }
    }

    const float4* wo = reinterpret_cast<const float4*>(wm + o.wo);
    float part = 0.0f;
    if constexpr (NT2 == 0) {
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
      return part;
    } else {
      floatx16 a2[NT2];
      const float4* b2 = reinterpret_cast<const float4*>(wm + o.b2);
#pragma unroll
      for (int u = 0; u < NT2; ++u) init_bias(b2, u, h, a2[u]);
      const uint4* w2 = reinterpret_cast<const uint4*>(wm + o.w2);
      A4 a_next = load_a(w2, lane, NT2 * 2 * NT1 * 64);
      // sigmoid of a 32-unit tile of layer 1, repacked as the 16-bit B operands of its two blocks
      B4 hb[NPL][NT1][2];
      auto activate = [&](int t) {
        sigmoid16(a1[t]);
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            uint32_t hi, lo;
            pack_pair<T, NPL>(a1[t][8 * b + 2 * jj], a1[t][8 * b + 2 * jj + 1], hi, lo);
            hb[0][t][b].w[jj] = hi;
            if constexpr (NPL == 2) hb[1][t][b].w[jj] = lo;
          }
      };
      __builtin_amdgcn_sched_barrier(0);
      activate(0);
      __builtin_amdgcn_sched_barrier(0);
      // 16-bit matrix instructions run beside the vector ALU: the matrix steps over tile t
      // are interleaved with the sigmoid of tile t + 1 (one block's steps, then a share of
      // the vector work)
      constexpr int kMper = NPL == 2 ? 3 : 1;                 // matrix instructions per block and output tile
      constexpr int kVper = (NPL == 2 ? 112 : 56) / (2 * NT2);       // vector instructions beside them
#pragma unroll
      for (int t = 0; t < NT1; ++t) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int u = 0; u < NT2; ++u) {
            const A4 a = a_next;
            const int un = u + 1 < NT2 ? u + 1 : 0;
            const int bn = un ? b : (b + 1 < 2 ? b + 1 : 0);
            const int tn = (un || bn) ? t : t + 1;
            if (tn < NT1) a_next = load_a(w2, (un * 2 * NT1 + 2 * tn + bn) * 64 + lane, NT2 * 2 * NT1 * 64);
            a2[u] = mma(a, hb[0][t][b], hb[NPL - 1][t][b], a2[u]);
          }
        if (t + 1 < NT1) {
          activate(t + 1);
#pragma unroll
          for (int i = 0; i < 2 * NT2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, NPL, 0);     // the next block's weights
            __builtin_amdgcn_sched_group_barrier(0x008, kMper, 0);   // this block's matrix steps
            __builtin_amdgcn_sched_group_barrier(0x002, kVper, 0);   // a share of the next tile's sigmoid
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
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
      return part;
    }
  }

  static __device__ __forceinline__ A4 load_w1(const uint4* __restrict__ w1, int t, int kb, int lane) {
    return load_a(w1, (t * KB1 + kb) * 64 + lane, NT1 * KB1 * 64);
  }
  static __device__ __forceinline__ A4 load_w2(const uint4* __restrict__ w2, int t, int b, int u, int lane) {
    return load_a(w2, (u * 2 * NT1 + 2 * t + b) * 64 + lane, NT2 * 2 * NT1 * 64);
  }
  static __device__ __forceinline__ void pack_tile(const floatx16& a1, B4 (&hb)[NPL][2]) {
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        uint32_t hi, lo;
        pack_pair<T, NPL>(a1[8 * b + 2 * jj], a1[8 * b + 2 * jj + 1], hi, lo);
        hb[0][b].w[jj] = hi;
        if constexpr (NPL == 2) hb[1][b].w[jj] = lo;
      }
  }

  // Layer 1 one 32-unit tile at a time: sigmoid and repacking of tile t, then the layer-1
  // steps of tile t + 1 (its accumulator is free once tile t is packed, and its sigmoid then
  // does not wait for the burst of matrix instructions that follows to drain), then the
  // 2 NT2 layer-2 steps that consume tile t.
  static __device__ __forceinline__ float forward_stream(const uint32_t* __restrict__ wm, const Feat& f, int lane,
                                                               const NetOffsets& o) {
    const int h = lane >> 5;
    const float4* b1 = reinterpret_cast<const float4*>(wm + o.b1);
    const float4* b2 = reinterpret_cast<const float4*>(wm + o.b2);
    const uint4* w1 = reinterpret_cast<const uint4*>(wm + o.w1);
    const uint4* w2 = reinterpret_cast<const uint4*>(wm + o.w2);
    const float4* wo = reinterpret_cast<const float4*>(wm + o.wo);
    floatx16 a2[NT2];
#pragma unroll
    for (int u = 0; u < NT2; ++u) init_bias(b2, u, h, a2[u]);
    floatx16 a1;
    B4 hb[NPL][2];
    init_bias(b1, 0, h, a1);
#pragma unroll
    for (int kb = 0; kb < KB1; ++kb) a1 = mma(load_w1(w1, 0, kb, lane), f.x[0][kb], f.x[NPL - 1][kb], a1);
#pragma unroll
    for (int t = 0; t < NT1; ++t) {
      sigmoid16(a1);
      pack_tile(a1, hb);
      if (t + 1 < NT1) {
        init_bias(b1, t + 1, h, a1);
#pragma unroll
        for (int kb = 0; kb < KB1; ++kb) a1 = mma(load_w1(w1, t + 1, kb, lane), f.x[0][kb], f.x[NPL - 1][kb], a1);
      }
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int u = 0; u < NT2; ++u) a2[u] = mma(load_w2(w2, t, b, u, lane), hb[0][b], hb[NPL - 1][b], a2[u]);
    }
    float part = 0.0f;
#pragma unroll
    for (int u = 0; u < NT2; ++u) {
      float4 q[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) q[g] = wo[(u * 4 + g) * 2 + h];
      sigmoid16(a2[u]);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        part = fmaf(q[g].x, a2[u][4 * g + 0], part);
        part = fmaf(q[g].y, a2[u][4 * g + 1], part);
        part = fmaf(q[g].z, a2[u][4 * g + 2], part);
        part = fmaf(q[g].w, a2[u][4 * g + 3], part);
      }
    }
    return part;
  }
};

// One packed word of a member (device, used by the prep kernel).
template <class T>
__device__ inline uint32_t pack_word_lp(const Shape& sh, const float* raw, int q) {
  typedef typename LpTraits<T>::V2 V2;
  const int r_w1 = 0, r_b1 = r_w1 + sh.H1 * sh.P;
  const int r_w2 = r_b1 + sh.H1;
  const int r_b2 = r_w2 + sh.H2 * sh.H1;
  const int r_wo = sh.H2 ? r_b2 + sh.H2 : r_w2;
  const int HL = sh.H2 ? sh.H2 : sh.H1;
  if (q < sh.o_b1) {                 // 16-bit weight planes
    float v[2] = {0.0f, 0.0f};
    int plane;
    if (q < sh.o_w2) {               // W1A [NPL][NT1][KB1][64][4]
      const int jj = q & 3, lane = (q >> 2) & 63, rest = q >> 8;
      const int kb = rest % sh.KS, t = (rest / sh.KS) % sh.NT1;
      plane = rest / (sh.KS * sh.NT1);
      const int n = lane & 31, h = lane >> 5, unit = 32 * t + n;
      for (int e = 0; e < 2; ++e) {
        const int f = 16 * kb + 8 * h + 2 * jj + e;
        if (unit < sh.H1 && f < sh.P) v[e] = raw[r_w1 + unit * sh.P + f] * kNegLog2e;
      }
    } else {                         // W2A [NPL][NT2][2 NT1][64][4]
      q -= sh.o_w2;
      const int jj = q & 3, lane = (q >> 2) & 63, rest = q >> 8;
      const int kbg = rest % (2 * sh.NT1), u = (rest / (2 * sh.NT1)) % sh.NT2;
      plane = rest / (2 * sh.NT1 * sh.NT2);
      const int n = lane & 31, h = lane >> 5, out = 32 * u + n;
      for (int e = 0; e < 2; ++e) {
        const int j = 2 * jj + e;
        const int in = 16 * kbg + 8 * (j >> 2) + 4 * h + (j & 3);
        if (out < sh.H2 && in < sh.H1) v[e] = raw[r_w2 + out * sh.H1 + in] * kNegLog2e;
      }
    }
    const float2v ab = {v[0], v[1]};
    const V2 hv = __builtin_convertvector(ab, V2);
    if (plane == 0) return __builtin_bit_cast(uint32_t, hv);
    const float2v r = {v[0] - (float)hv[0], v[1] - (float)hv[1]};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(r, V2));
  }
  // fp32 tables
  float v = 0.0f;
  if (q < sh.o_b2) {
    q -= sh.o_b1;
    const int j = q & 3, h = (q >> 2) & 1, g = (q >> 3) & 3, t = q >> 5;
    const int unit = 32 * t + 8 * g + 4 * h + j;
    if (unit < sh.H1) v = raw[r_b1 + unit] * kNegLog2e;
  } else if (q < sh.o_wo) {
    q -= sh.o_b2;
    const int j = q & 3, h = (q >> 2) & 1, g = (q >> 3) & 3, u = q >> 5;
    const int unit = 32 * u + 8 * g + 4 * h + j;
    if (unit < sh.H2) v = raw[r_b2 + unit] * kNegLog2e;
  } else {
    q -= sh.o_wo;
    const int j = q & 3, h = (q >> 2) & 1, g = (q >> 3) & 3, u = q >> 5;
    const int unit = 32 * u + 8 * g + 4 * h + j;
    if (unit < HL) v = raw[r_wo + unit];
  }
  return __float_as_uint(v);
}

}  // namespace tuner
