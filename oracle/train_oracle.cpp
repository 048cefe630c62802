// CPU ORACLE — TEST INFRASTRUCTURE ONLY.
//
// Plain, slow, double-precision references for the stages of the paper's tuner
// that surround the full-space sweep: choosing random training configurations,
// training the bagged ensemble, the model-accuracy metric and the second-stage
// pick.  Not a product code path; shares nothing with the HIP library.
//
// oracle_sample_valid      Section 5.2, first paragraph: "randomly chosen parameter
//                          configurations"; invalid ones are ignored (last paragraph).
//                          The draws come from a counter-based generator that both
//                          sides implement (splitmix64 output function); the sample
//                          is the first n distinct valid indices in draw order.
// oracle_train_ensemble    Section 5.2: k networks with one sigmoid hidden layer,
//                          network e trained on all the data except part e, targets
//                          = logarithm of the execution time, loss = mean squared
//                          error.  The paper names no training algorithm: the
//                          reading used is full-batch gradient descent with momentum,
//                          v <- mu v - eta dL/dw, w <- w + v, from given initial weights.
//                          Samples that are statically invalid or whose time is not a
//                          finite number > 0 are ignored.
// oracle_mean_relative_error  Section 6, model accuracy: mean of |exp(prediction) - t| / t
//                          over valid configurations with a usable time.
// oracle_best_of           Section 5.3, third paragraph: the candidate with the lowest
//                          measured time among the M.
//
// Pins (tests/test_oracle_train_pins.py): gradients against central finite
// differences of an independently written loss and against reverse-mode
// automatic differentiation of the same definition (whole trajectories,
// momentum included), the closed-form first step from all-zero weights,
// invariance to the data of the excluded part and of ignored samples,
// brute-force set semantics of the sampler, hand-computed metric values.
// Not pinned: the accuracy the paper reports for its trained models (needs the
// paper's measurements).

#include <cmath>
#include <cstdint>
#include <limits>
#include <unordered_set>
#include <vector>

#include "oracle_api.h"
#include "oracle_space.h"

namespace {

using namespace oracle_detail;

uint64_t splitmix64_at(uint64_t seed, uint64_t counter) {
  uint64_t z = seed + (counter + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

bool usable_time(float t) { return std::isfinite(t) && t > 0.0f; }

}  // namespace

extern "C" {

// indices_out[n_samples]; returns the number written.
int64_t oracle_sample_valid(int n_params, const int32_t* radices, int n_constraints,
                            const int32_t* terms, const int64_t* bounds, uint64_t seed,
                            int64_t n_samples, uint64_t max_draws, uint64_t* indices_out) {
  SpaceView s{n_params, radices, nullptr, nullptr, n_constraints, terms, bounds, {}, {}, 0};
  s.offsets.assign(n_params, 0);
  int64_t off = 0;
  unsigned __int128 n_configs = 1;
  for (int p = 0; p < n_params; ++p) { s.offsets[p] = off; off += radices[p]; n_configs *= (uint64_t)radices[p]; }
  s.total = off;
  std::vector<int32_t> d(n_params);
  std::unordered_set<uint64_t> seen;
  int64_t found = 0;
  for (uint64_t c = 0; c < max_draws && found < n_samples; ++c) {
    const uint64_t z = splitmix64_at(seed, c);
    const uint64_t index = (uint64_t)(((unsigned __int128)z * n_configs) >> 64);
    digits_of(s, index, d.data());
    if (!is_valid(s, d.data())) continue;
    if (!seen.insert(index).second) continue;
    indices_out[found++] = index;
  }
  return found;
}

// Weights per network: W1[H][P], b1[H], w_o[H], b_o (fp32 in, fp32 out; double inside).
// loss_out (may be null): [E][epochs + 1] doubles.
int oracle_train_ensemble(int n_params, const int32_t* radices, const double* values,
                          const int32_t* scales, int n_constraints, const int32_t* terms,
                          const int64_t* bounds, int n_members, int hidden, int64_t n_samples,
                          const uint64_t* sample_indices, const float* sample_times,
                          const int32_t* sample_parts, const float* initial_weights, int epochs,
                          float learning_rate, float momentum, float* weights_out,
                          double* loss_out) {
  SpaceView s{n_params, radices, values, scales, n_constraints, terms, bounds, {}, {}, 0};
  build_lut(s);
  const int P = n_params, H = hidden;
  const int64_t per = (int64_t)H * P + H + H + 1;
  const double eta = (double)learning_rate, mu = (double)momentum;

  // inputs and targets of the usable samples
  std::vector<double> X((size_t)n_samples * P), target(n_samples);
  std::vector<char> usable(n_samples);
  std::vector<int32_t> d(P);
  for (int64_t i = 0; i < n_samples; ++i) {
    digits_of(s, sample_indices[i], d.data());
    usable[i] = is_valid(s, d.data()) && usable_time(sample_times[i]);
    for (int p = 0; p < P; ++p) X[(size_t)i * P + p] = (double)s.lut[s.offsets[p] + d[p]];
    target[i] = usable[i] ? std::log((double)sample_times[i]) : 0.0;
  }

  std::vector<double> w(per), v(per), g(per), h(H);
  for (int e = 0; e < n_members; ++e) {
    for (int64_t q = 0; q < per; ++q) { w[q] = (double)initial_weights[e * per + q]; v[q] = 0.0; }
    double* W1 = w.data();
    double* b1 = W1 + (int64_t)H * P;
    double* wo = b1 + H;
    double* bo = wo + H;
    int64_t n_e = 0;
    for (int64_t i = 0; i < n_samples; ++i) n_e += (usable[i] && sample_parts[i] != e) ? 1 : 0;
    for (int ep = 0; ep <= epochs; ++ep) {
      // loss and gradient at the current weights
      double loss = 0.0;
      for (int64_t q = 0; q < per; ++q) g[q] = 0.0;
      double* gW1 = g.data();
      double* gb1 = gW1 + (int64_t)H * P;
      double* gwo = gb1 + H;
      double* gbo = gwo + H;
      for (int64_t i = 0; i < n_samples; ++i) {
        if (!usable[i] || sample_parts[i] == e) continue;
        const double* x = &X[(size_t)i * P];
        double y = *bo;
        for (int j = 0; j < H; ++j) {
          double z = b1[j];
          for (int p = 0; p < P; ++p) z += W1[(int64_t)j * P + p] * x[p];
          h[j] = 1.0 / (1.0 + std::exp(-z));
          y += wo[j] * h[j];
        }
        const double err = y - target[i];
        loss += err * err;
        const double dy = 2.0 * err / (double)n_e;      // dL/dy for this sample
        *gbo += dy;
        for (int j = 0; j < H; ++j) {
          gwo[j] += dy * h[j];
          const double dz = dy * wo[j] * h[j] * (1.0 - h[j]);
          gb1[j] += dz;
          for (int p = 0; p < P; ++p) gW1[(int64_t)j * P + p] += dz * x[p];
        }
      }
      if (n_e > 0) loss /= (double)n_e;
      if (loss_out) loss_out[(int64_t)e * (epochs + 1) + ep] = loss;
      if (ep == epochs || n_e == 0) continue;
      for (int64_t q = 0; q < per; ++q) {
        v[q] = mu * v[q] - eta * g[q];
        w[q] += v[q];
      }
    }
    for (int64_t q = 0; q < per; ++q) weights_out[e * per + q] = (float)w[q];
  }
  return 0;
}

// Mean of |exp(prediction) - t| / t over entries with a finite prediction and a
// usable time.  Returns the count through *n_used.
double oracle_mean_relative_error(int64_t n, const float* predictions, const float* times,
                                  int64_t* n_used) {
  double sum = 0.0;
  int64_t cnt = 0;
  for (int64_t i = 0; i < n; ++i) {
    if (!std::isfinite(predictions[i]) || !usable_time(times[i])) continue;
    const double t = (double)times[i];
    sum += std::fabs(std::exp((double)predictions[i]) - t) / t;
    ++cnt;
  }
  *n_used = cnt;
  return cnt ? sum / (double)cnt : 0.0;
}

// Position of the lowest usable time (earliest on ties), -1 if none.
int64_t oracle_best_of(int64_t m, const float* times, float* best_time) {
  int64_t best = -1;
  float bt = std::numeric_limits<float>::infinity();
  for (int64_t i = 0; i < m; ++i) {
    if (!usable_time(times[i])) continue;
    if (best < 0 || times[i] < bt) { best = i; bt = times[i]; }
  }
  *best_time = bt;
  return best;
}

}  // extern "C"
