// Device-side description of a tuning space and the index -> digit -> feature /
// validity routines shared by every kernel of the library (and evaluated on
// the host by tuner_space_decode_device_arith for CPU tests).
//
// The space is the Cartesian product of the parameters' value lists (paper
// Section 5.1, Table 2); a configuration index is a mixed-radix number whose
// last parameter is the least significant digit.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define TUNER_HD __host__ __device__ __forceinline__
#else
#define TUNER_HD inline
#endif

namespace tuner {

constexpr int kMaxParams = 32;   // array length (31 usable + one padding slot)
constexpr int kMaxValues = 256;
constexpr int kMaxCons = 8;
constexpr int kMaxEntries = 64;
constexpr int kMaxTermWords = 256;

// Per-parameter decode constants, one 16-byte and one 8-byte LDS read per digit.
// digit_p(i) = (i / stride_p) mod radix_p.  Division by an invariant integer through
// multiply-high and shifts (Granlund & Montgomery 1994):
//   t = mulhi(mul, n);  q = (t + ((n - t) >> sh1)) >> sh2
// *_sh packs sh1 | sh2 << 8 | log2(divisor) << 16 (the last only if the divisor is a
// power of two).  Entries past n_params describe a one-value parameter whose feature is
// 0 (digit always 0, lut_off = kLutZero).
struct ParamA { uint32_t stride_sh, radix, lut_off, stride_mul; };
struct ParamB { uint32_t radix_mul, radix_sh; };

constexpr int kLutZero = kMaxValues - 2;   // lut[kLutZero] = 0.0f
constexpr int kLutOne = kMaxValues - 1;    // lut[kLutOne] = 1.0f

// Passed to kernels by value (about 3.1 KB) and copied to LDS by the sweep.
struct DevSpace {
  int32_t n_params;
  int32_t n_constraints;
  int32_t all_pow2;      // every stride and radix is a power of two
  int32_t pad0;
  ParamA pa[kMaxParams];
  ParamB pb[kMaxParams];
  // validity rule c uses entries [entry_begin[c], entry_begin[c+1]); an entry
  // names a parameter and the start of its term table in terms[].
  uint32_t entry[kMaxEntries];        // param | term_off << 8
  int32_t entry_begin[kMaxCons + 1];
  int32_t bound[kMaxCons];
  int32_t pad1[3];
  float lut[kMaxValues];              // normalised fp32 features (+ the two constants)
  int32_t terms[kMaxTermWords];       // non-zero term tables, back to back
};

TUNER_HD uint32_t mulhi_u32(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __umulhi(a, b);
#else
  return (uint32_t)(((uint64_t)a * (uint64_t)b) >> 32);
#endif
}

TUNER_HD uint32_t fast_div(uint32_t n, uint32_t mul, uint32_t sh) {
  const uint32_t t = mulhi_u32(mul, n);
  return (t + ((n - t) >> (sh & 0xffu))) >> ((sh >> 8) & 0xffu);
}

// S may live in LDS, in kernel-argument memory or on the host.  pow2 = s.all_pow2,
// hoisted by the caller.
template <class S>
TUNER_HD uint32_t digit_of(const S& s, int p, uint32_t index, bool pow2, uint32_t* lut_off = nullptr) {
  const ParamA a = s.pa[p];
  if (lut_off) *lut_off = a.lut_off;
  if (pow2) return (index >> (a.stride_sh >> 16)) & (a.radix - 1u);
  const ParamB b = s.pb[p];
  const uint32_t q = fast_div(index, a.stride_mul, a.stride_sh);
  return q - fast_div(q, b.radix_mul, b.radix_sh) * a.radix;
}

// fp32 network input of parameter p for configuration `index`
template <class S>
TUNER_HD float feature_at(const S& s, int p, uint32_t index, bool pow2) {
  uint32_t off;
  const uint32_t d = digit_of(s, p, index, pow2, &off);
  return s.lut[off + d];
}

// Sum of rule c's terms over the entries e = first, first+step, ... of the rule.
template <class S>
TUNER_HD int32_t rule_partial_sum(const S& s, int c, uint32_t index, int first, int step, bool pow2) {
  int32_t sum = 0;
  for (int e = s.entry_begin[c] + first; e < s.entry_begin[c + 1]; e += step) {
    const uint32_t ent = s.entry[e];
    const int p = (int)(ent & 0xffu);
    sum += s.terms[(ent >> 8) + digit_of(s, p, index, pow2)];
  }
  return sum;
}

template <class S>
TUNER_HD bool is_valid(const S& s, uint32_t index, bool pow2) {
  bool ok = true;
  for (int c = 0; c < s.n_constraints; ++c) ok = ok && (rule_partial_sum(s, c, index, 0, 1, pow2) <= s.bound[c]);
  return ok;
}

}  // namespace tuner
