// CPU ORACLE — TEST INFRASTRUCTURE ONLY.
//
// The tuning space as the oracle sees it: value lists, feature table, mixed-radix
// digits and the static validity rules (paper Section 5.1 / Table 2, Section 5.2
// last paragraph).  Shared by the oracle's translation units only; nothing of
// the HIP library includes it.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

namespace oracle_detail {

struct SpaceView {
  int n_params;
  const int32_t* radices;
  const double* values;          // concatenated value lists
  const int32_t* scales;         // 0 linear, 1 log2
  int n_constraints;
  const int32_t* terms;          // [n_constraints][sum radices]
  const int64_t* bounds;         // [n_constraints]
  std::vector<int64_t> offsets;  // start of each parameter's list
  std::vector<float> lut;        // normalised features, fp32
  int64_t total;                 // sum of radices
};

// Feature table: t(v) = v or log2(v); (t - t_min)/(t_max - t_min) in double,
// rounded once to fp32; a one-value list or a constant list maps to 0.
inline void build_lut(SpaceView& s) {
  s.offsets.assign(s.n_params, 0);
  int64_t off = 0;
  for (int p = 0; p < s.n_params; ++p) { s.offsets[p] = off; off += s.radices[p]; }
  s.total = off;
  s.lut.assign(off, 0.0f);
  for (int p = 0; p < s.n_params; ++p) {
    const int r = s.radices[p];
    std::vector<double> t(r);
    for (int j = 0; j < r; ++j) {
      const double v = s.values[s.offsets[p] + j];
      t[j] = (s.scales[p] == 1) ? std::log2(v) : v;
    }
    double lo = t[0], hi = t[0];
    for (int j = 1; j < r; ++j) { lo = std::min(lo, t[j]); hi = std::max(hi, t[j]); }
    for (int j = 0; j < r; ++j) {
      const double x = (hi > lo) ? (t[j] - lo) / (hi - lo) : 0.0;
      s.lut[s.offsets[p] + j] = static_cast<float>(x);
    }
  }
}

// Mixed-radix digits, last parameter least significant.
inline void digits_of(const SpaceView& s, uint64_t index, int32_t* d) {
  uint64_t q = index;
  for (int p = s.n_params - 1; p >= 0; --p) {
    const uint64_t r = static_cast<uint64_t>(s.radices[p]);
    d[p] = static_cast<int32_t>(q % r);
    q /= r;
  }
}

inline bool is_valid(const SpaceView& s, const int32_t* d) {
  for (int c = 0; c < s.n_constraints; ++c) {
    int64_t sum = 0;
    const int32_t* row = s.terms + static_cast<int64_t>(c) * s.total;
    for (int p = 0; p < s.n_params; ++p) sum += row[s.offsets[p] + d[p]];
    if (sum > s.bounds[c]) return false;
  }
  return true;
}

}  // namespace oracle_detail
