// CPU ORACLE — TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, single-threaded reference for the full-space sweep of the
// ANN performance model of the paper's auto-tuner (Section 5: "predict the
// execution time for all the possible configurations", then take "the M
// configurations with the lowest predicted execution times").  It is the
// definition written out as nested loops in double precision; it is not a
// product code path.  Only tests, the smoke check and the cpu_baseline leg of
// the benchmark may call it.  It shares no code, header, table generator or
// constant with the HIP library.
//
// What is computed, for every configuration index i of the range:
//   digits  d_p(i)   : position of i in the Cartesian product of the value
//                      lists (Section 5.1, Table 2); last parameter fastest.
//   feature x_p      : value v_p[d_p], optionally log2, min-max scaled to
//                      [0,1] over the parameter's list, rounded to fp32.
//                      (The paper does not state the input encoding; this is
//                      the reading documented with the build.)
//   valid(i)         : every static rule  sum_p T_c[p][d_p] <= B_c  holds
//                      (Section 5.2: invalid configurations that "can be
//                      determined statically").
//   y_e              : feed-forward network e (Section 4.2: weighted sum then
//                      activation; Section 5.2: sigmoid hidden units), linear
//                      output, evaluated in double.
//   yhat(i)          : mean over the ensemble (Section 5.2, bagging: "take
//                      the mean of their outputs"), rounded once to fp32;
//                      +infinity if the configuration is invalid.
//   top-k            : the k pairs (yhat, i) that are smallest in
//                      (yhat, then i) order, ascending (Section 5.3).
//
// Pins (tests/test_oracle_*.py): space sizes printed in the paper, closed
// forms for decode/features/zero-weight nets/one-unit nets, analytic valid
// counts, numpy matrix algebra over an itertools.product enumeration (for the
// list evaluation: at scattered indices with digits from plain divmod), and
// brute-force full sorts on spaces of at most 1024 configurations.  A build
// with AddressSanitizer and UndefinedBehaviorSanitizer runs every entry point
// (sanitize_driver.cpp).
// Not pinned: accuracy of a *trained* model (needs the paper's measurements).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <queue>
#include <thread>
#include <utility>
#include <vector>

#include "oracle_api.h"
#include "oracle_space.h"

namespace {

using namespace oracle_detail;

// One network: hidden layers logistic, output layer linear; double throughout.
double network(const float* w, int n_layers, const int32_t* widths,
               const double* x, std::vector<double>& a, std::vector<double>& b) {
  a.assign(x, x + widths[0]);
  for (int l = 0; l < n_layers; ++l) {
    const int fi = widths[l], fo = widths[l + 1];
    const float* W = w;
    const float* bias = w + static_cast<int64_t>(fi) * fo;
    w = bias + fo;
    b.assign(fo, 0.0);
    for (int o = 0; o < fo; ++o) {
      double acc = static_cast<double>(bias[o]);
      for (int j = 0; j < fi; ++j)
        acc += static_cast<double>(W[static_cast<int64_t>(o) * fi + j]) * a[j];
      b[o] = (l + 1 < n_layers) ? 1.0 / (1.0 + std::exp(-acc)) : acc;
    }
    a.swap(b);
  }
  return a[0];
}

int64_t floats_per_member(int n_layers, const int32_t* widths) {
  int64_t n = 0;
  for (int l = 0; l < n_layers; ++l)
    n += static_cast<int64_t>(widths[l]) * widths[l + 1] + widths[l + 1];
  return n;
}

void predict_range(const SpaceView& s, int n_members, int n_layers, const int32_t* widths,
                   const float* weights, uint64_t begin, uint64_t count,
                   float* yhat, uint8_t* valid_out, int32_t* digits_out) {
  std::vector<int32_t> d(s.n_params);
  std::vector<double> x(s.n_params), a, b;
  const int64_t fpm = floats_per_member(n_layers, widths);
  for (uint64_t t = 0; t < count; ++t) {
    const uint64_t i = begin + t;
    digits_of(s, i, d.data());
    if (digits_out) std::memcpy(digits_out + t * s.n_params, d.data(), sizeof(int32_t) * s.n_params);
    const bool ok = is_valid(s, d.data());
    if (valid_out) valid_out[t] = ok ? 1 : 0;
    if (!yhat) continue;
    if (!ok) { yhat[t] = std::numeric_limits<float>::infinity(); continue; }
    for (int p = 0; p < s.n_params; ++p) x[p] = static_cast<double>(s.lut[s.offsets[p] + d[p]]);
    double sum = 0.0;
    for (int e = 0; e < n_members; ++e)
      sum += network(weights + e * fpm, n_layers, widths, x.data(), a, b);
    yhat[t] = static_cast<float>(sum / static_cast<double>(n_members));
  }
}

using Pair = std::pair<float, uint64_t>;  // ordered by value, then index

}  // namespace

extern "C" {

// Fills lut_out[sum radices] with the fp32 feature table.
int oracle_feature_lut(int n_params, const int32_t* radices, const double* values,
                       const int32_t* scales, float* lut_out) {
  SpaceView s{n_params, radices, values, scales, 0, nullptr, nullptr, {}, {}, 0};
  build_lut(s);
  std::copy(s.lut.begin(), s.lut.end(), lut_out);
  return 0;
}

int oracle_digits(int n_params, const int32_t* radices, uint64_t index, int32_t* digits_out) {
  SpaceView s{n_params, radices, nullptr, nullptr, 0, nullptr, nullptr, {}, {}, 0};
  digits_of(s, index, digits_out);
  return 0;
}

// Inverse of oracle_digits (Horner form of the positional system).
int oracle_index(int n_params, const int32_t* radices, const int32_t* digits, uint64_t* index_out) {
  uint64_t i = 0;
  for (int p = 0; p < n_params; ++p) i = i * static_cast<uint64_t>(radices[p]) + static_cast<uint64_t>(digits[p]);
  *index_out = i;
  return 0;
}

// yhat[count] (may be null), valid[count] (may be null), digits[count][P] (may
// be null) for indices begin .. begin+count-1.  n_threads > 1 only partitions
// the index range among threads running the same single-threaded routine.
int oracle_predict_range(int n_params, const int32_t* radices, const double* values,
                         const int32_t* scales, int n_constraints, const int32_t* terms,
                         const int64_t* bounds, int n_members, int n_layers,
                         const int32_t* widths, const float* weights, uint64_t begin,
                         uint64_t count, float* yhat, uint8_t* valid, int32_t* digits,
                         int n_threads) {
  SpaceView s{n_params, radices, values, scales, n_constraints, terms, bounds, {}, {}, 0};
  build_lut(s);
  if (n_threads <= 1) {
    predict_range(s, n_members, n_layers, widths, weights, begin, count, yhat, valid, digits);
    return 0;
  }
  std::vector<std::thread> pool;
  const uint64_t per = (count + n_threads - 1) / n_threads;
  for (int t = 0; t < n_threads; ++t) {
    const uint64_t lo = std::min<uint64_t>(count, per * t), hi = std::min<uint64_t>(count, lo + per);
    if (hi <= lo) continue;
    pool.emplace_back([&, lo, hi] {
      predict_range(s, n_members, n_layers, widths, weights, begin + lo, hi - lo,
                    yhat ? yhat + lo : nullptr, valid ? valid + lo : nullptr,
                    digits ? digits + lo * n_params : nullptr);
    });
  }
  for (auto& th : pool) th.join();
  return 0;
}

// Same as oracle_predict_range for an arbitrary list of indices.
int oracle_predict_indices(int n_params, const int32_t* radices, const double* values,
                           const int32_t* scales, int n_constraints, const int32_t* terms,
                           const int64_t* bounds, int n_members, int n_layers,
                           const int32_t* widths, const float* weights, const uint64_t* indices,
                           uint64_t count, float* yhat, uint8_t* valid, int n_threads) {
  SpaceView s{n_params, radices, values, scales, n_constraints, terms, bounds, {}, {}, 0};
  build_lut(s);
  if (n_threads < 1) n_threads = 1;
  std::vector<std::thread> pool;
  const uint64_t per = (count + n_threads - 1) / n_threads;
  for (int t = 0; t < n_threads; ++t) {
    const uint64_t lo = std::min<uint64_t>(count, per * t), hi = std::min<uint64_t>(count, lo + per);
    if (hi <= lo) continue;
    pool.emplace_back([&, lo, hi] {
      for (uint64_t j = lo; j < hi; ++j)
        predict_range(s, n_members, n_layers, widths, weights, indices[j], 1, yhat + j,
                      valid + j, nullptr);
    });
  }
  for (auto& th : pool) th.join();
  return 0;
}

// Selection from given predictions: the k smallest (value, index) pairs among
// entries with valid[t] != 0, ascending; index reported = index_base + t.
// Bounded max-heap; returns the number found (min(k, #valid)).
int64_t oracle_select_topk(const float* yhat, const uint8_t* valid, uint64_t count,
                           uint64_t index_base, int64_t k, float* values_out,
                           uint64_t* indices_out) {
  std::priority_queue<Pair> heap;  // largest on top
  for (uint64_t t = 0; t < count; ++t) {
    if (valid && !valid[t]) continue;
    Pair p(yhat[t], index_base + t);
    if (static_cast<int64_t>(heap.size()) < k) heap.push(p);
    else if (k > 0 && p < heap.top()) { heap.pop(); heap.push(p); }
  }
  const int64_t n = static_cast<int64_t>(heap.size());
  for (int64_t j = n - 1; j >= 0; --j) {
    values_out[j] = heap.top().first;
    indices_out[j] = heap.top().second;
    heap.pop();
  }
  return n;
}

}  // extern "C"
