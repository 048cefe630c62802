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
constexpr int kMaxTermWords = 192;

// Decode constants of one parameter.  digit_p(i) = (i / stride_p) mod radix_p.
//   power-of-two spaces:  digit = (i >> shift) & mask
//   otherwise: division by an invariant integer through multiply-high and shifts
//   (Granlund & Montgomery 1994):  t = mulhi(mul, n);  q = (t + ((n - t) >> sh1)) >> sh2,
//   with *_sh = sh1 | sh2 << 8.
// The A half is all the power-of-two path reads (one 16-byte LDS read per digit).
// Slots past n_params describe a one-value parameter whose feature is 0.
struct ParamA { uint32_t shift, mask, lut_off4, stride_mul; };   // lut_off4: byte offset into lut[]
struct ParamB { uint32_t stride_sh, radix_mul, radix_sh, radix; };
// A validity-rule entry = one parameter with a non-zero term table.
struct RuleEntry { uint32_t param, term_off4; };                // byte offset into terms[]

constexpr int kLutZero = kMaxValues - 2;   // lut[kLutZero] = 0.0f
constexpr int kLutOne = kMaxValues - 1;    // lut[kLutOne] = 1.0f

// Passed to kernels by value (3.4 KB; the kernel-argument limit is 4 KB) and copied to
// LDS by the sweep.
struct DevSpace {
  int32_t n_params;
  int32_t n_constraints;
  int32_t all_pow2;      // every stride and radix is a power of two
  int32_t pad0;
  ParamA pa[kMaxParams];
  ParamB pb[kMaxParams];
  // validity rule c uses entries [entry_begin[c], entry_begin[c+1])
  RuleEntry entry[kMaxEntries];
  int32_t entry_begin[kMaxCons + 1];
  int32_t bound[kMaxCons];
  int32_t pad1[3];
  float lut[kMaxValues];              // normalised fp32 features (+ the two constants)
  int32_t terms[kMaxTermWords];       // non-zero term tables, back to back
};
static_assert(sizeof(DevSpace) <= 3584, "DevSpace must leave room in the 4 KB kernel-argument block");

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

// Any 32-bit index decodes to an in-range digit (the top parameter wraps), so lanes
// past the end of a range may decode safely.
TUNER_HD uint32_t digit_from(const ParamA& a, const ParamB& b, uint32_t index, bool pow2) {
  if (pow2) return (index >> a.shift) & a.mask;
  const uint32_t q = fast_div(index, a.stride_mul, b.stride_sh);
  return q - fast_div(q, b.radix_mul, b.radix_sh) * b.radix;
}

TUNER_HD uint32_t word_at(const void* table, uint32_t byte_off) {
  return *reinterpret_cast<const uint32_t*>(static_cast<const char*>(table) + byte_off);
}

// S may live in LDS, in kernel-argument memory or on the host.  pow2 = s.all_pow2,
// hoisted by the caller.
template <class S>
TUNER_HD uint32_t digit_of(const S& s, int p, uint32_t index, bool pow2) {
  if (pow2) return digit_from(s.pa[p], ParamB{}, index, true);
  return digit_from(s.pa[p], s.pb[p], index, false);
}

// fp32 network input of parameter p for configuration `index`.  POW2 is a template
// argument so that a caller decoding several parameters branches once, not per digit.
template <bool POW2, class S>
TUNER_HD float feature_at_t(const S& s, int p, uint32_t index) {
  const ParamA a = s.pa[p];
  uint32_t d;
  if (POW2) d = digit_from(a, ParamB{}, index, true);
  else d = digit_from(a, s.pb[p], index, false);
  const uint32_t bits = word_at(s.lut, a.lut_off4 + 4u * d);
#if defined(__HIP_DEVICE_COMPILE__)
  return __uint_as_float(bits);
#else
  float f;
  __builtin_memcpy(&f, &bits, 4);
  return f;
#endif
}

template <class S>
TUNER_HD float feature_at(const S& s, int p, uint32_t index, bool pow2) {
  return pow2 ? feature_at_t<true>(s, p, index) : feature_at_t<false>(s, p, index);
}

// Sum of rule c's terms over the entries e = first, first+step, ... of the rule.
template <class S>
TUNER_HD int32_t rule_partial_sum(const S& s, int c, uint32_t index, int first, int step, bool pow2) {
  int32_t sum = 0;
  const int end = s.entry_begin[c + 1];
  for (int e = s.entry_begin[c] + first; e < end; e += step) {
    const RuleEntry ent = s.entry[e];
    sum += (int32_t)word_at(s.terms, ent.term_off4 + 4u * digit_of(s, (int)ent.param, index, pow2));
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
