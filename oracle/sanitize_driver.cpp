// CPU ORACLE — TEST INFRASTRUCTURE ONLY.
//
// Runs every entry point of the oracle once on the 256-configuration space (4 parameters
// with lists {1,2,4,8}, {1,2,4,8}, {0,1}, {1..8}; one rule so that some configurations are
// invalid) in a build with AddressSanitizer and UndefinedBehaviorSanitizer
// (oracle/build.py --sanitize), without Python in the process.  It checks only what holds
// by construction (round trips, equal results for different thread counts, sorted output);
// the oracle's arithmetic is pinned by the Python tests.  Exit status 0 and the line
// "oracle sanitizer run ok" mean that no sanitizer report was raised.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "oracle_api.h"

#define REQUIRE(cond)                                                        \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "sanitize_driver: %s failed (line %d)\n", #cond, __LINE__); \
      return 1;                                                              \
    }                                                                        \
  } while (0)

int main() {
  const int P = 4;
  const int32_t radices[P] = {4, 4, 2, 8};
  const std::vector<double> values = {1, 2, 4, 8, 1, 2, 4, 8, 0, 1, 1, 2, 3, 4, 5, 6, 7, 8};
  const int32_t scales[P] = {1, 1, 0, 0};
  // rule: digit 0 + digit 1 <= 4
  std::vector<int32_t> terms = {0, 1, 2, 3, 0, 1, 2, 3, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  const int64_t bounds[1] = {4};
  const uint64_t N = 256;

  std::vector<float> lut(values.size());
  REQUIRE(oracle_feature_lut(P, radices, values.data(), scales, lut.data()) == 0);
  REQUIRE(lut[0] == 0.0f && lut[3] == 1.0f && lut[17] == 1.0f);

  for (uint64_t i = 0; i < N; ++i) {
    int32_t d[P];
    uint64_t back = ~0ull;
    REQUIRE(oracle_digits(P, radices, i, d) == 0);
    REQUIRE(oracle_index(P, radices, d, &back) == 0);
    REQUIRE(back == i);
  }

  // one network 4-16-1 and an ensemble of three 4-5-3-1 networks, weights from a small generator
  auto fill = [](std::vector<float>& w, uint32_t seed) {
    for (auto& x : w) { seed = seed * 1664525u + 1013904223u; x = ((seed >> 8) & 0xffff) / 32768.0f - 1.0f; }
  };
  const int32_t widths2[3] = {4, 16, 1};
  std::vector<float> w2(4 * 16 + 16 + 16 + 1);
  fill(w2, 1u);
  const int32_t widths3[4] = {4, 5, 3, 1};
  std::vector<float> w3(3 * (4 * 5 + 5 + 5 * 3 + 3 + 3 + 1));
  fill(w3, 2u);

  std::vector<float> y1(N), y3(N), yl(N);
  std::vector<uint8_t> v1(N), v3(N), vl(N);
  std::vector<int32_t> digs(N * P);
  REQUIRE(oracle_predict_range(P, radices, values.data(), scales, 1, terms.data(), bounds, 1, 2, widths2, w2.data(),
                               0, N, y1.data(), v1.data(), digs.data(), 1) == 0);
  REQUIRE(oracle_predict_range(P, radices, values.data(), scales, 1, terms.data(), bounds, 1, 2, widths2, w2.data(),
                               0, N, y3.data(), v3.data(), nullptr, 3) == 0);
  uint64_t n_valid = 0;
  std::vector<uint64_t> all(N);
  for (uint64_t i = 0; i < N; ++i) {
    REQUIRE(v1[i] == v3[i]);
    REQUIRE(v1[i] ? y1[i] == y3[i] : (std::isinf(y1[i]) && std::isinf(y3[i])));
    n_valid += v1[i];
    all[i] = N - 1 - i;
  }
  REQUIRE(n_valid == 13 * 16);     // 13 of the 16 (digit 0, digit 1) pairs have a sum <= 4
  REQUIRE(oracle_predict_indices(P, radices, values.data(), scales, 1, terms.data(), bounds, 1, 2, widths2,
                                 w2.data(), all.data(), N, yl.data(), vl.data(), 5) == 0);
  for (uint64_t i = 0; i < N; ++i) REQUIRE(vl[i] == v1[N - 1 - i] && (!vl[i] || yl[i] == y1[N - 1 - i]));
  // two hidden layers, a ragged sub-range, no rules, outputs partly omitted
  REQUIRE(oracle_predict_range(P, radices, values.data(), scales, 0, nullptr, nullptr, 3, 3, widths3, w3.data(),
                               7, 201, y3.data(), nullptr, nullptr, 4) == 0);
  REQUIRE(oracle_predict_range(P, radices, values.data(), scales, 1, terms.data(), bounds, 0, 0, widths3, w3.data(),
                               0, N, nullptr, v3.data(), nullptr, 2) == 0);

  std::vector<float> tv(10);
  std::vector<uint64_t> ti(10);
  const int64_t found = oracle_select_topk(y1.data(), v1.data(), N, 0, 10, tv.data(), ti.data());
  REQUIRE(found == 10);
  for (int j = 1; j < 10; ++j) REQUIRE(tv[j] > tv[j - 1] || (tv[j] == tv[j - 1] && ti[j] > ti[j - 1]));
  for (int j = 0; j < 10; ++j) REQUIRE(v1[ti[j]] == 1 && y1[ti[j]] == tv[j]);
  std::vector<float> big(300);
  std::vector<uint64_t> bigi(300);
  REQUIRE(oracle_select_topk(y1.data(), v1.data(), N, 1000, 300, big.data(), bigi.data()) == (int64_t)n_valid);
  REQUIRE(oracle_select_topk(y1.data(), nullptr, N, 0, 0, big.data(), bigi.data()) == 0);

  // sampler -> synthetic times -> training -> metric -> second-stage pick
  std::vector<uint64_t> sample(60);
  const int64_t n_s = oracle_sample_valid(P, radices, 1, terms.data(), bounds, 42u, 60, 4000, sample.data());
  REQUIRE(n_s == 60);
  for (int64_t a = 0; a < n_s; ++a) {
    REQUIRE(sample[a] < N && v1[sample[a]] == 1);
    for (int64_t b = 0; b < a; ++b) REQUIRE(sample[a] != sample[b]);
  }
  std::vector<uint64_t> many(250);                 // more asked for than exist: every valid one comes back
  REQUIRE(oracle_sample_valid(P, radices, 1, terms.data(), bounds, 7u, 250, 100000, many.data()) == (int64_t)n_valid);
  std::vector<float> times(n_s);
  std::vector<int32_t> parts(n_s);
  for (int64_t a = 0; a < n_s; ++a) {
    times[a] = a % 17 == 5 ? -1.0f : std::exp(0.5f * y1[sample[a]]);   // some failed runs
    parts[a] = (int32_t)(a % 3);
  }
  const int E = 3, H = 6;
  std::vector<float> w0(E * (H * P + H + H + 1)), wt(w0.size());
  fill(w0, 3u);
  std::vector<double> loss(E * 6);
  REQUIRE(oracle_train_ensemble(P, radices, values.data(), scales, 1, terms.data(), bounds, E, H, n_s, sample.data(),
                                times.data(), parts.data(), w0.data(), 5, 0.05f, 0.5f, wt.data(), loss.data()) == 0);
  for (double l : loss) REQUIRE(std::isfinite(l) && l >= 0.0);
  REQUIRE(oracle_train_ensemble(P, radices, values.data(), scales, 1, terms.data(), bounds, E, H, n_s, sample.data(),
                                times.data(), parts.data(), w0.data(), 0, 0.05f, 0.5f, wt.data(), nullptr) == 0);
  for (size_t q = 0; q < w0.size(); ++q) REQUIRE(wt[q] == w0[q]);      // no epochs: weights unchanged
  const int32_t widths_t[3] = {P, H, 1};
  std::vector<float> ps(n_s);
  std::vector<uint8_t> pv(n_s);
  REQUIRE(oracle_predict_indices(P, radices, values.data(), scales, 1, terms.data(), bounds, E, 2, widths_t,
                                 wt.data(), sample.data(), n_s, ps.data(), pv.data(), 2) == 0);
  int64_t used = -1;
  const double mre = oracle_mean_relative_error(n_s, ps.data(), times.data(), &used);
  REQUIRE(std::isfinite(mre) && mre >= 0.0 && used > 0 && used < n_s);
  float bt = 0.0f;
  const int64_t pos = oracle_best_of(n_s, times.data(), &bt);
  REQUIRE(pos >= 0 && pos < n_s && times[pos] == bt && bt > 0.0f);
  const float none[3] = {-1.0f, 0.0f, NAN};
  REQUIRE(oracle_best_of(3, none, &bt) == -1 && std::isinf(bt));
  REQUIRE(oracle_mean_relative_error(0, ps.data(), times.data(), &used) == 0.0 && used == 0);

  std::printf("oracle sanitizer run ok\n");
  return 0;
}
