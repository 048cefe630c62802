// Host-side internals shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/tuner.h"
#include "dev_space.h"

struct tuner_space {
  int32_t n_params = 0;
  uint64_t n_configs = 0;
  std::vector<int32_t> radices;
  std::vector<uint64_t> strides;     // true strides (product of the later radices)
  std::vector<int64_t> offsets;      // start of each value list
  std::vector<double> values;
  std::vector<int32_t> scales;
  int32_t n_constraints = 0;
  std::vector<int32_t> terms;        // [C][sum r] as given
  std::vector<int64_t> bounds;
  int64_t total_values = 0;
  tuner::DevSpace dev;               // what the kernels see
};

namespace tuner {

int set_error(int code, const std::string& msg);
int hip_error(hipError_t e, const char* what);

// Raises a kernel's dynamic-LDS limit to at least `bytes` on the current device.  The
// driver call is made only when the limit has to grow: it is a host round trip of several
// microseconds, which a short sweep would pay on every call.
int allow_dynamic_lds(const void* kernel, int bytes);

// Optional timing of the dominant kernels (HIP events on the caller's stream).
enum { PROFILE_SWEEP = 0, PROFILE_TRAIN = 1, PROFILE_KINDS = 2 };
bool profile_on();
void profile_add(int kind, hipEvent_t begin, hipEvent_t end);

#define TUNER_HIP_TRY(expr)                                   \
  do {                                                        \
    hipError_t e_ = (expr);                                   \
    if (e_ != hipSuccess) return tuner::hip_error(e_, #expr); \
  } while (0)

}  // namespace tuner
