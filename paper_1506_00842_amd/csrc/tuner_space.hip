// Space object: host construction of the decoder tables, host helpers, and the
// decode_range kernel that exposes the device decoder for step-by-step checks.
//
// Paper: the tuning space is the Cartesian product of the per-parameter value
// lists (Section 5.1, Table 2); statically known invalid configurations
// (Section 5.2, last paragraph) are expressed as separable integer rules.
#include <cmath>
#include <cstring>
#include <limits>
#include <map>
#include <mutex>
#include <utility>
#include <new>

#include "tuner_internal.h"

namespace tuner {

static thread_local std::string g_error;

int set_error(int code, const std::string& msg) {
  g_error = msg;
  return code;
}

int hip_error(hipError_t e, const char* what) {
  g_error = std::string("HIP error: ") + hipGetErrorString(e) + " in " + what;
  return TUNER_EHIP;
}

int allow_dynamic_lds(const void* kernel, int bytes) {
  static std::mutex mu;
  static std::map<std::pair<int, const void*>, int> granted;   // (device, kernel) -> limit set so far
  int dev = 0;
  TUNER_HIP_TRY(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(mu);
  int& have = granted[std::make_pair(dev, kernel)];
  if (bytes > have) {
    TUNER_HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    have = bytes;
  }
  return TUNER_OK;
}

static bool is_pow2(uint64_t v) { return v && !(v & (v - 1)); }

static int ceil_log2(uint64_t d) {
  int l = 0;
  while ((1ull << l) < d) ++l;
  return l;
}

// Multiply-shift constants for unsigned 32-bit division by d >= 1.
static void div_constants(uint32_t d, uint32_t* mul, uint32_t* sh) {
  const int l = ceil_log2(d);
  const uint64_t two_l = 1ull << l;  // l <= 32
  const unsigned __int128 num = (unsigned __int128)(two_l - d) << 32;
  *mul = (uint32_t)(num / d) + 1u;
  const uint32_t sh1 = l < 1 ? l : 1, sh2 = l > 1 ? l - 1 : 0;
  *sh = sh1 | (sh2 << 8);
}

// Decode constants of a parameter with the given stride and radix; table_off4 is the
// byte offset of its table (features or rule terms).
static void param_constants(uint64_t stride, uint32_t radix, uint32_t table_off4, ParamA* a, ParamB* b) {
  // a one-value parameter always decodes to digit 0: give it stride 1 so that every
  // stride fits in 32 bits
  if (radix == 1) stride = 1;
  div_constants((uint32_t)stride, &a->stride_mul, &b->stride_sh);
  div_constants(radix, &b->radix_mul, &b->radix_sh);
  b->radix = radix;
  a->shift = is_pow2(stride) ? (uint32_t)ceil_log2(stride) : 0u;
  a->mask = radix - 1u;            // used on the power-of-two path only
  a->lut_off4 = table_off4;
}

}  // namespace tuner

using tuner::set_error;

extern "C" {

const char* tuner_last_error(void) { return tuner::g_error.c_str(); }
const char* tuner_version(void) { return "tuner-hip 0.1 (gfx950)"; }

int tuner_space_create(int32_t n_params, const int32_t* radices, const double* values,
                       const int32_t* scales, int32_t n_constraints,
                       const int32_t* constraint_terms, const int64_t* constraint_bounds,
                       tuner_space** out) {
  if (!radices || !values || !scales || !out) return set_error(TUNER_EINVAL, "null argument");
  if (n_params < 1) return set_error(TUNER_EINVAL, "n_params must be >= 1");
  if (n_params > TUNER_MAX_PARAMS) return set_error(TUNER_ETOOLARGE, "too many parameters");
  if (n_constraints < 0) return set_error(TUNER_EINVAL, "n_constraints < 0");
  if (n_constraints > TUNER_MAX_CONSTRAINTS) return set_error(TUNER_ETOOLARGE, "too many rules");
  if (n_constraints > 0 && (!constraint_terms || !constraint_bounds))
    return set_error(TUNER_EINVAL, "null constraint arrays");

  tuner_space* sp = new (std::nothrow) tuner_space();
  if (!sp) return set_error(TUNER_ENOMEM, "out of host memory");
  struct Guard { tuner_space* p; ~Guard() { delete p; } } guard{sp};

  try {
    sp->n_params = n_params;
    int64_t total = 0;
    unsigned __int128 n = 1;
    for (int p = 0; p < n_params; ++p) {
      if (radices[p] < 1) return set_error(TUNER_EINVAL, "radix < 1");
      sp->offsets.push_back(total);
      total += radices[p];
      n *= (unsigned)radices[p];
      if (n > ((unsigned __int128)1 << 32))
        return set_error(TUNER_ETOOLARGE, "more than 2^32 configurations");
    }
    if (total > TUNER_MAX_VALUES) return set_error(TUNER_ETOOLARGE, "too many values");
    static_assert(TUNER_MAX_VALUES == tuner::kMaxValues - 2, "two table slots hold the constants 0 and 1");
    sp->total_values = total;
    sp->n_configs = (uint64_t)n;
    sp->radices.assign(radices, radices + n_params);
    sp->values.assign(values, values + total);
    sp->scales.assign(scales, scales + n_params);
    sp->strides.assign(n_params, 1);
    for (int p = n_params - 2; p >= 0; --p)
      sp->strides[p] = sp->strides[p + 1] * (uint64_t)radices[p + 1];

    tuner::DevSpace& d = sp->dev;
    std::memset(&d, 0, sizeof(d));
    d.n_params = n_params;
    d.n_constraints = n_constraints;
    d.all_pow2 = 1;
    for (int p = 0; p < n_params; ++p) {
      if (scales[p] != TUNER_SCALE_LINEAR && scales[p] != TUNER_SCALE_LOG2)
        return set_error(TUNER_EINVAL, "bad scale flag");
      if (!tuner::is_pow2((uint64_t)radices[p])) d.all_pow2 = 0;
    }
    d.lut[tuner::kLutZero] = 0.0f;
    d.lut[tuner::kLutOne] = 1.0f;
    for (int p = n_params; p < tuner::kMaxParams; ++p)       // padding: digit 0, feature 0
      tuner::param_constants(1, 1u, 4u * (uint32_t)tuner::kLutZero, &d.pa[p], &d.pb[p]);
    for (int p = 0; p < n_params; ++p) {
      tuner::param_constants(sp->strides[p], (uint32_t)radices[p], 4u * (uint32_t)sp->offsets[p],
                             &d.pa[p], &d.pb[p]);
      // feature table
      const int r = radices[p];
      std::vector<double> t(r);
      for (int j = 0; j < r; ++j) {
        const double v = values[sp->offsets[p] + j];
        if (!std::isfinite(v)) return set_error(TUNER_EINVAL, "non-finite parameter value");
        if (scales[p] == TUNER_SCALE_LOG2) {
          if (!(v > 0.0)) return set_error(TUNER_EINVAL, "log2 scale needs values > 0");
          t[j] = std::log2(v);
        } else {
          t[j] = v;
        }
      }
      double lo = t[0], hi = t[0];
      for (int j = 1; j < r; ++j) { lo = t[j] < lo ? t[j] : lo; hi = t[j] > hi ? t[j] : hi; }
      for (int j = 0; j < r; ++j)
        d.lut[sp->offsets[p] + j] = hi > lo ? (float)((t[j] - lo) / (hi - lo)) : 0.0f;
    }
    // validity rules -> compact (rule, parameter) entries
    if (n_constraints > 0) {
      sp->terms.assign(constraint_terms, constraint_terms + (int64_t)n_constraints * total);
      sp->bounds.assign(constraint_bounds, constraint_bounds + n_constraints);
    }
    sp->n_constraints = n_constraints;
    int n_entries = 0, n_words = 0;
    for (int c = 0; c < n_constraints; ++c) {
      d.entry_begin[c] = n_entries;
      const int32_t* row = constraint_terms + (int64_t)c * total;
      int64_t abs_sum = 0;
      for (int p = 0; p < n_params; ++p) {
        int64_t mx = 0;
        bool any = false;
        for (int j = 0; j < radices[p]; ++j) {
          const int64_t v = row[sp->offsets[p] + j];
          mx = std::max<int64_t>(mx, v < 0 ? -v : v);
          any = any || v != 0;
        }
        abs_sum += mx;
        if (!any) continue;
        if (n_entries >= TUNER_MAX_CONSTRAINT_ENTRIES || n_words + radices[p] > TUNER_MAX_TERM_WORDS)
          return set_error(TUNER_ETOOLARGE, "validity rules need too many table entries");
        d.entry[n_entries].param = (uint32_t)p;
        d.entry[n_entries].term_off4 = 4u * (uint32_t)n_words;
        ++n_entries;
        for (int j = 0; j < radices[p]; ++j) d.terms[n_words++] = row[sp->offsets[p] + j];
      }
      if (abs_sum > std::numeric_limits<int32_t>::max())
        return set_error(TUNER_EINVAL, "rule sum does not fit in 32 bits");
      int64_t b = constraint_bounds[c];
      b = std::min<int64_t>(b, std::numeric_limits<int32_t>::max());
      b = std::max<int64_t>(b, std::numeric_limits<int32_t>::min());
      d.bound[c] = (int32_t)b;
    }
    d.entry_begin[n_constraints] = n_entries;
    for (int c = n_constraints + 1; c <= tuner::kMaxCons; ++c) d.entry_begin[c] = n_entries;
  } catch (const std::bad_alloc&) {
    return set_error(TUNER_ENOMEM, "out of host memory");
  }
  guard.p = nullptr;
  *out = sp;
  return TUNER_OK;
}

void tuner_space_destroy(tuner_space* space) { delete space; }

int tuner_space_size(const tuner_space* space, uint64_t* n_configs) {
  if (!space || !n_configs) return set_error(TUNER_EINVAL, "null argument");
  *n_configs = space->n_configs;
  return TUNER_OK;
}

int tuner_space_decode(const tuner_space* sp, uint64_t index, int32_t* digits, double* values,
                       float* features, int32_t* valid) {
  if (!sp || !digits) return set_error(TUNER_EINVAL, "null argument");
  if (index >= sp->n_configs) return set_error(TUNER_EINVAL, "index outside the space");
  for (int p = 0; p < sp->n_params; ++p) {
    const int32_t dgt = (int32_t)((index / sp->strides[p]) % (uint64_t)sp->radices[p]);
    digits[p] = dgt;
    if (values) values[p] = sp->values[sp->offsets[p] + dgt];
    if (features) features[p] = sp->dev.lut[sp->offsets[p] + dgt];
  }
  if (valid) {
    int ok = 1;
    for (int c = 0; c < sp->n_constraints; ++c) {
      int64_t sum = 0;
      for (int p = 0; p < sp->n_params; ++p)
        sum += sp->terms[(int64_t)c * sp->total_values + sp->offsets[p] + digits[p]];
      if (sum > sp->bounds[c]) ok = 0;
    }
    *valid = ok;
  }
  return TUNER_OK;
}

int tuner_space_encode(const tuner_space* sp, const int32_t* digits, uint64_t* index) {
  if (!sp || !digits || !index) return set_error(TUNER_EINVAL, "null argument");
  uint64_t i = 0;
  for (int p = 0; p < sp->n_params; ++p) {
    if (digits[p] < 0 || digits[p] >= sp->radices[p]) return set_error(TUNER_EINVAL, "digit out of range");
    i += (uint64_t)digits[p] * sp->strides[p];
  }
  *index = i;
  return TUNER_OK;
}

int tuner_space_decode_device_arith(const tuner_space* sp, uint64_t index, int32_t* digits,
                                    float* features, int32_t* valid) {
  if (!sp || !digits) return set_error(TUNER_EINVAL, "null argument");
  if (index >= sp->n_configs) return set_error(TUNER_EINVAL, "index outside the space");
  const uint32_t i = (uint32_t)index;
  const bool pow2 = sp->dev.all_pow2 != 0;
  for (int p = 0; p < sp->n_params; ++p) {
    digits[p] = (int32_t)tuner::digit_of(sp->dev, p, i, pow2);
    if (features) features[p] = tuner::feature_at(sp->dev, p, i, pow2);
  }
  if (valid) *valid = tuner::is_valid(sp->dev, i, pow2) ? 1 : 0;
  return TUNER_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------
// decode_range: one thread per configuration.
// ---------------------------------------------------------------------------
namespace tuner {

__global__ void __launch_bounds__(256)
decode_range_kernel(const DevSpace sp, uint64_t begin, uint64_t count, int32_t* __restrict__ digits,
                    float* __restrict__ features, uint8_t* __restrict__ valid) {
  const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= count) return;
  const uint32_t i = (uint32_t)(begin + t);
  const int P = sp.n_params;
  const bool pow2 = sp.all_pow2 != 0;
  for (int p = 0; p < P; ++p) {
    if (digits) digits[t * P + p] = (int32_t)digit_of(sp, p, i, pow2);
    if (features) features[t * P + p] = feature_at(sp, p, i, pow2);
  }
  if (valid) valid[t] = is_valid(sp, i, pow2) ? 1 : 0;
}

}  // namespace tuner

extern "C" int tuner_decode_range(const tuner_space* sp, uint64_t begin, uint64_t count,
                                  int32_t* digits_dev, float* features_dev, uint8_t* valid_dev,
                                  void* hip_stream) {
  if (!sp) return set_error(TUNER_EINVAL, "null space");
  if (begin > sp->n_configs || count > sp->n_configs - begin)
    return set_error(TUNER_EINVAL, "range outside the space");
  if (count == 0) return TUNER_OK;
  const uint64_t blocks = (count + 255) / 256;
  if (blocks > 0x7fffffffull) return set_error(TUNER_ETOOLARGE, "range too long for one call");
  hipLaunchKernelGGL(tuner::decode_range_kernel, dim3((unsigned)blocks), dim3(256), 0,
                     (hipStream_t)hip_stream, sp->dev, begin, count, digits_dev, features_dev,
                     valid_dev);
  TUNER_HIP_TRY(hipGetLastError());
  return TUNER_OK;
}
