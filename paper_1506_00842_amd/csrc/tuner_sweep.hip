// Fused full-space sweep: decode -> features -> validity -> ensemble MLP ->
// mean -> (all predictions | running top-k), for gfx950.
//
// Paper: Section 5.3 (predict every configuration, keep the M lowest),
// Section 5.2 (bagged ensemble of sigmoid networks, mean of the outputs,
// statically invalid configurations), Section 4.2 (neuron = weighted sum +
// activation), Section 5.1 / Table 2 (the space).
//
// Network evaluation on the matrix cores, fp32 in / fp32 accumulate
// (v_mfma_f32_32x32x2_f32).  A wave evaluates a tile of 32 configurations.
// The weights are the A operand (rows = 32 units of the layer), the
// activations are the B operand (columns = the 32 configurations), so a layer's
// output tile D[unit][config] leaves every lane (config c = lane % 32, half
// h = lane / 32) holding 16 units of its configuration:
//     unit(v, h) = 8 * (v / 4) + 4 * h + (v % 4),  v = 0..15
// which is exactly the ownership the B operand of the next layer needs (lane
// half h supplies one k index per MFMA step), with the k order permuted; the
// permutation is folded into the packed weight layout, so layers chain with no
// cross-lane traffic.  The sigmoid runs on the vector ALU between the layers,
// with -log2(e) folded into the packed weights: sigma(z) = 1 / (1 + 2^(z')).
#include <cstdio>
#include <cstring>
#include <mutex>
#include <utility>
#include <vector>

#include "net_f32.h"
#include "net_f32h.h"
#include "net_f32t.h"
#include "net_lp.h"
#include "net_valu.h"
#include "sweep_common.h"
#include "tuner_internal.h"
#include "wave_sort.h"

namespace tuner {

// ---------------------------------------------------------------------------
// prep: packs the weights into the matrix-operand order of the chosen network,
// writes the space tables, resets the queue and the threshold, converts the
// caller's running result into a sorted key list.
// ---------------------------------------------------------------------------
struct PrepParams {
  Shape sh;
  const float* raw;           // caller's weights
  uint32_t* packed;
  DevSpace* space_out;
  WsHeader* hdr;
};

__global__ void __launch_bounds__(256) prep_kernel(const DevSpace sp, const PrepParams pp) {
  const Shape& sh = pp.sh;
  const uint32_t gtid = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t gsize = gridDim.x * blockDim.x;
  const uint32_t total = (uint32_t)sh.E * sh.member_words;
  for (uint32_t x = gtid; x < total; x += gsize) {
    const int e = x / sh.member_words;
    const int q = x - e * sh.member_words;
    const float* raw = pp.raw + (size_t)e * sh.raw_member_floats;
    uint32_t word;
    if (sh.net == NET_BF16) word = pack_word_lp<__bf16>(sh, raw, q);
    else if (sh.net == NET_F16X2) word = pack_word_lp<_Float16>(sh, raw, q);
    else if (sh.net == NET_F32_VALU) word = __float_as_uint(pack_word_valu(sh, raw, q));
    else if (sh.hoist == 2) word = __float_as_uint(pack_word_f32t(sh, raw, q, sp));
    else if (sh.hoist) word = __float_as_uint(pack_word_f32h(sh, raw, q));
    else word = __float_as_uint(pack_word_f32(sh, raw, q));
    pp.packed[x] = word;
  }
  // space tables
  {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(&sp);
    uint32_t* dst = reinterpret_cast<uint32_t*>(pp.space_out);
    for (uint32_t x = gtid; x < sizeof(DevSpace) / 4; x += gsize) dst[x] = src[x];
    // the fp32 matrix network reads its bias column's constant 1 as the feature of the
    // slot after the last parameter (same thread as the plain copy of that word)
    if (sh.net == NET_F32_MFMA && !sh.hoist) {
      const uint32_t word = (uint32_t)((const char*)&sp.pa[sh.P].lut_off4 - (const char*)&sp) / 4u;
      if (gtid == word % gsize) pp.space_out->pa[sh.P].lut_off4 = 4u * (uint32_t)kLutOne;
    }
  }
  // header: the idle state every sweep starts from and its last workgroup restores
  if (gtid == 0) {
    const int r_bo = sh.raw_member_floats - 1;
    float bo = 0.0f;
    for (int e = 0; e < sh.E; ++e) bo += pp.raw[(size_t)e * sh.raw_member_floats + r_bo];
    pp.hdr->bo_sum = bo;
    pp.hdr->work_counter = 0u;
    pp.hdr->n_live = 0u;
    pp.hdr->done = 0u;
    pp.hdr->merge_done = 0u;
    pp.hdr->tau = kKeyMax;
  }
}

// The result of a top-k call over an empty range that merges with nothing: no configuration.
__global__ void __launch_bounds__(256)
empty_result_kernel(int32_t k, float* values, uint32_t* indices, int32_t* n_found) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < k; i += gridDim.x * blockDim.x) {
    values[i] = __builtin_inff();
    indices[i] = 0xffffffffu;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) *n_found = 0;
}

// ---------------------------------------------------------------------------
// Grid merge of sorted lists of kp keys.  The kp smallest of two sorted lists
// are min(A[i], B[kp-1-i]) (a bitonic sequence), which a bitonic merge sorts.
//
// merge_tree_kernel: a workgroup loads 2^levels lists (list indices base + j * stride0)
// into LDS, merges them pairwise level by level there, and writes the result over
// its first list; with `final` set (single workgroup) it also writes the caller's
// outputs.  merge_kernel: one pair per workgroup, in place in global memory, for
// lists too long for LDS.
// ---------------------------------------------------------------------------
constexpr uint32_t kWaveMergeMaxKp = 512;    // lists up to this long are merged one pair per wave (wave_sort.h)

struct MergeParams {
  unsigned long long* pools;
  unsigned long long* extra;   // list index n_pool_lists (the caller's running result)
  uint32_t cap, n_pool_lists, n_lists, kp;
  uint32_t stride0, levels;
  uint32_t fuse_levels;        // > 0: the last workgroup to finish merges the launch's 2^fuse_levels results
  int32_t final, k;
  float* values;
  uint32_t* indices;
  int32_t* n_found;
  WsHeader* hdr;               // final launch: the header goes back to its idle state for the next call
};

__device__ __forceinline__ void reset_header(WsHeader* hdr) {
  hdr->work_counter = 0u;
  hdr->n_live = 0u;
  hdr->done = 0u;
  hdr->merge_done = 0u;
  hdr->tau = kKeyMax;
}

__device__ __forceinline__ void emit_result(const unsigned long long* list, int i, int32_t k, float* values,
                                            uint32_t* indices, int32_t* n_found) {
  const unsigned long long key = list[i];
  const bool real = key != kKeyMax;
  values[i] = real ? unorder_bits((uint32_t)(key >> 32)) : __builtin_inff();
  indices[i] = real ? (uint32_t)key : 0xffffffffu;
  if (i == 0 && !real) *n_found = 0;
  if (real && (i == k - 1 || list[i + 1] == kKeyMax)) *n_found = i + 1;
}

// Loads the lists first + j * stride (j = 0 .. 2^levels - 1; indices >= n_lists read as empty)
// into LDS slots of kp keys: all lists at once, many loads in flight per thread (a loop over
// the lists would pay one memory latency per list): 8 x 16 bytes per thread and round, which
// covers 32 lists of 512 keys in one round.
// COHERENT: the lists were written during this launch by other workgroups (agent-scope
// atomic stores); they are read with agent-scope atomic loads, which are performed at the
// device's coherence point, past the L2 of the XCD this workgroup runs on.
template <bool COHERENT>
__device__ __forceinline__ void merge_load(const MergeParams& mp, unsigned long long* lds, uint32_t first,
                                           uint32_t stride, uint32_t slots, uint32_t n_lists, uint32_t tid) {
  const uint32_t kp = mp.kp;
  auto list_ptr = [&](uint32_t j) -> const unsigned long long* {
    return j < mp.n_pool_lists ? mp.pools + (size_t)j * mp.cap : mp.extra;
  };
  const uint32_t total = slots * kp;
  if constexpr (COHERENT) {
    for (uint32_t t0 = 0; t0 < total; t0 += 8 * kMergeThreads) {
      unsigned long long v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const uint32_t t = t0 + q * kMergeThreads + tid;
        const uint32_t j = t / kp, x = t - j * kp;
        const uint32_t li = first + j * stride;
        v[q] = kKeyMax;
        if (t < total && li < n_lists)
          v[q] = __hip_atomic_load(list_ptr(li) + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const uint32_t t = t0 + q * kMergeThreads + tid;
        if (t < total) lds[t] = v[q];
      }
    }
  } else if ((kp & 1u) == 0u) {
    const uint32_t kp2 = kp >> 1, total2 = total >> 1;
    ulonglong2* lds2 = reinterpret_cast<ulonglong2*>(lds);
    for (uint32_t t0 = 0; t0 < total2; t0 += 8 * kMergeThreads) {
      ulonglong2 v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const uint32_t t = t0 + q * kMergeThreads + tid;
        const uint32_t j = t / kp2, x = t - j * kp2;
        const uint32_t li = first + j * stride;
        v[q] = make_ulonglong2(kKeyMax, kKeyMax);
        if (t < total2 && li < n_lists) v[q] = reinterpret_cast<const ulonglong2*>(list_ptr(li))[x];
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const uint32_t t = t0 + q * kMergeThreads + tid;
        if (t < total2) lds2[t] = v[q];
      }
    }
  } else {                                   // kp = 1
    for (uint32_t t = tid; t < total; t += kMergeThreads) {
      const uint32_t li = first + t * stride;
      lds[t] = li < n_lists ? list_ptr(li)[0] : kKeyMax;
    }
  }
  __syncthreads();
}

// Merges the `slots` sorted lists of kp keys in LDS pairwise, level by level; the kp smallest
// keys of all of them end up sorted in slot 0.
__device__ __forceinline__ void merge_levels(unsigned long long* lds, uint32_t kp, uint32_t slots, uint32_t tid) {
  const uint32_t half = kp >> 1;
  if (kp >= 64 && kp <= kWaveMergeMaxKp) {
    // Lists of 64 .. 512 keys: one wave per pair of lists, the merge network in registers;
    // the workgroup meets once per tree level.
    const uint32_t wave = tid >> 6, lane = tid & 63;
    for (uint32_t s = 1; s < slots; s <<= 1) {
      const uint32_t npairs = slots / (2 * s);
      for (uint32_t m = wave; m < npairs; m += kMergeThreads / 64) {
        unsigned long long* A = lds + (size_t)(2 * m * s) * kp;
        const unsigned long long* B = A + (size_t)s * kp;
        if (kp == 64) wave_pair_merge<1>(A, B, lane);
        else if (kp == 128) wave_pair_merge<2>(A, B, lane);
        else if (kp == 256) wave_pair_merge<4>(A, B, lane);
        else wave_pair_merge<8>(A, B, lane);
      }
      __syncthreads();
    }
  } else if (kp < 64) {
    // Shorter lists: one wave per pair of lists.  A wave's LDS instructions execute in
    // program order, so the steps of its merge network need no workgroup barrier, only a
    // compiler fence; the workgroup meets once per tree level.
    const uint32_t wave = tid >> 6, lane = tid & 63;
    for (uint32_t s = 1; s < slots; s <<= 1) {
      const uint32_t npairs = slots / (2 * s);
      for (uint32_t m = wave; m < npairs; m += kMergeThreads / 64) {
        unsigned long long* A = lds + (size_t)(2 * m * s) * kp;
        const unsigned long long* B = A + (size_t)s * kp;
        for (uint32_t i = lane; i < kp; i += 64) {
          const unsigned long long a = A[i], b = B[kp - 1 - i];
          A[i] = a < b ? a : b;
        }
        for (uint32_t j = half; j > 0; j >>= 1) {
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
          for (uint32_t u = lane; u < half; u += 64) {
            const uint32_t i = ((u & ~(j - 1)) << 1) | (u & (j - 1));
            const uint32_t l = i | j;
            const unsigned long long x = A[i], y = A[l];
            if (x > y) { A[i] = y; A[l] = x; }
          }
        }
      }
      __syncthreads();
    }
  } else {
    for (uint32_t s = 1; s < slots; s <<= 1) {
      const uint32_t npairs = slots / (2 * s);
      // A[i] = min(A[i], B[kp-1-i]) over every pair (A = slot 2 m s, B = slot 2 m s + s)
      for (uint32_t t = tid; t < npairs * kp; t += kMergeThreads) {
        const uint32_t m = t / kp, i = t - m * kp;
        unsigned long long* A = lds + (size_t)(2 * m * s) * kp;
        const unsigned long long a = A[i], b = A[(size_t)s * kp + (kp - 1 - i)];
        A[i] = a < b ? a : b;
      }
      __syncthreads();
      for (uint32_t j = half; j > 0; j >>= 1) {
        for (uint32_t t = tid; t < npairs * half; t += kMergeThreads) {
          const uint32_t m = t / half, u = t - m * half;
          unsigned long long* A = lds + (size_t)(2 * m * s) * kp;
          const uint32_t i = ((u & ~(j - 1)) << 1) | (u & (j - 1));
          const uint32_t l = i | j;
          const unsigned long long x = A[i], y = A[l];
          if (x > y) { A[i] = y; A[l] = x; }
        }
        __syncthreads();
      }
    }
  }
}

__global__ void __launch_bounds__(kMergeThreads) merge_tree_kernel(const MergeParams mp) {
  extern __shared__ __align__(16) unsigned char merge_smem[];
  __shared__ uint32_t s_last;
  unsigned long long* lds = reinterpret_cast<unsigned long long*>(merge_smem);
  const uint32_t tid = threadIdx.x, kp = mp.kp;
  const uint32_t slots = 1u << mp.levels;
  const uint32_t base = blockIdx.x * mp.stride0 * slots;
  merge_load<false>(mp, lds, base, mp.stride0, slots, mp.n_lists, tid);
  merge_levels(lds, kp, slots, tid);
  if (!mp.final) {
    unsigned long long* dst = base < mp.n_pool_lists ? mp.pools + (size_t)base * mp.cap : mp.extra;
    if (!mp.fuse_levels) {
      for (uint32_t x = tid; x < kp; x += kMergeThreads) dst[x] = lds[x];
      return;
    }
    // Second stage in the same launch: the workgroup that finishes last merges the lists the
    // others have written.  The workgroups may sit on different XCDs, each with an L2 of its
    // own, so the lists and the counter travel as agent-scope atomic stores and loads
    // (performed at the device's coherence point), ordered by s_waitcnt vmcnt(0) + the
    // workgroup barrier on the writers' side and by the barrier on the reader's side; no L2
    // write-back or invalidate is issued.
    for (uint32_t x = tid; x < kp; x += kMergeThreads)
      __hip_atomic_store(&dst[x], lds[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wave's stores have been performed
    __syncthreads();
    if (tid == 0)
      s_last = __hip_atomic_fetch_add(&mp.hdr->merge_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1
                   ? 1u : 0u;
    __syncthreads();
    if (!s_last) return;
    const uint32_t stride1 = mp.stride0 * slots;
    merge_load<true>(mp, lds, 0, stride1, 1u << mp.fuse_levels,
                     gridDim.x * stride1 < mp.n_lists ? gridDim.x * stride1 : mp.n_lists, tid);
    merge_levels(lds, kp, 1u << mp.fuse_levels, tid);
  }
  // slot 0 holds kp >= k sorted keys: the caller's outputs
  for (int i = (int)tid; i < mp.k; i += kMergeThreads)
    emit_result(lds, i, mp.k, mp.values, mp.indices, mp.n_found);
  if (tid == 0) reset_header(mp.hdr);
}

__global__ void __launch_bounds__(kMergeThreads)
merge_kernel(unsigned long long* pools, uint32_t cap, unsigned long long* extra, uint32_t n_pool_lists,
             uint32_t kp, uint32_t half) {
  const int tid = threadIdx.x;
  const uint32_t ja = blockIdx.x, jb = blockIdx.x + half;
  unsigned long long* A = ja < n_pool_lists ? pools + (size_t)ja * cap : extra;
  const unsigned long long* B = jb < n_pool_lists ? pools + (size_t)jb * cap : extra;
  for (uint32_t i = tid; i < kp; i += kMergeThreads) {
    const unsigned long long a = A[i], b = B[kp - 1 - i];
    A[i] = a < b ? a : b;
  }
  __syncthreads();
  for (uint32_t j = kp >> 1; j > 0; j >>= 1) {
    for (uint32_t t = tid; t < (kp >> 1); t += kMergeThreads) {
      const uint32_t i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
      const uint32_t l = i | j;
      const unsigned long long x = A[i], y = A[l];
      if (x > y) { A[i] = y; A[l] = x; }
    }
    __syncthreads();
  }
}

__global__ void __launch_bounds__(256)
finalize_kernel(const unsigned long long* list, int32_t k, float* values, uint32_t* indices,
                int32_t* n_found, WsHeader* hdr) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < k; i += gridDim.x * blockDim.x)
    emit_result(list, i, k, values, indices, n_found);
  if (blockIdx.x == 0 && threadIdx.x == 0) reset_header(hdr);
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
static int round_up(int v, int m) { return (v + m - 1) / m * m; }

// allow_hoist: 0 = plain layer 1; 1 = the tile-constant parameters' share once per tile;
// 2 = also the remaining parameters' share from a table, where the space allows it.
static int make_shape(const tuner_space* sp, const tuner_model* m, Shape* sh, int allow_hoist = 0) {
  if (!m->widths || !m->weights_dev) return set_error(TUNER_EINVAL, "null model arrays");
  if (m->n_members < 1) return set_error(TUNER_EINVAL, "n_members < 1");
  if (m->n_layers != 2 && m->n_layers != 3) return set_error(TUNER_EINVAL, "n_layers must be 2 or 3");
  if (m->precision == TUNER_BF16_MFMA) {
    if (m->algo != TUNER_ALGO_AUTO && m->algo != TUNER_ALGO_MFMA)
      return set_error(TUNER_EINVAL, "bf16 precision runs on the matrix cores only");
    sh->net = NET_BF16;
  } else if (m->precision == TUNER_FP32) {
    if (m->algo == TUNER_ALGO_AUTO || m->algo == TUNER_ALGO_MFMA) sh->net = NET_F32_MFMA;
    else if (m->algo == TUNER_ALGO_SPLIT16) sh->net = NET_F16X2;
    else if (m->algo == TUNER_ALGO_VALU) sh->net = NET_F32_VALU;
    else return set_error(TUNER_EINVAL, "unknown algo");
  } else {
    return set_error(TUNER_EINVAL, "unknown precision");
  }
  if (m->widths[0] != sp->n_params) return set_error(TUNER_EINVAL, "model input width != number of parameters");
  if (m->widths[m->n_layers] != 1) return set_error(TUNER_EINVAL, "model output width must be 1");
  sh->P = sp->n_params;
  sh->H1 = m->widths[1];
  sh->H2 = m->n_layers == 3 ? m->widths[2] : 0;
  sh->E = m->n_members;
  if (sh->H1 < 1 || (m->n_layers == 3 && sh->H2 < 1)) return set_error(TUNER_EINVAL, "hidden width < 1");
  if (sh->H1 > TUNER_MAX_WIDTH || sh->H2 > TUNER_MAX_WIDTH) return set_error(TUNER_ETOOLARGE, "hidden layer too wide");
  auto tiles = [](int hgt) { const int t = (hgt + 31) / 32; return t == 3 ? 4 : t; };
  sh->NT1 = tiles(sh->H1);
  sh->NT2 = sh->H2 ? tiles(sh->H2) : 0;
  // hidden layers of different tile counts run on the larger square variant
  if (sh->NT2 && sh->NT1 != sh->NT2) sh->NT1 = sh->NT2 = sh->NT1 > sh->NT2 ? sh->NT1 : sh->NT2;
  const int ntl = sh->NT2 ? sh->NT2 : sh->NT1;
  sh->raw_member_floats = sh->P * sh->H1 + sh->H1 + (sh->H2 ? sh->H1 * sh->H2 + sh->H2 + sh->H2 : sh->H1) + 1;
  // Parameters whose stride is a multiple of the tile size (32) have one value per tile
  // of 32 consecutive configurations that starts at a multiple of 32; they are the leading
  // ones.  The fp32 matrix network can take their layer-1 share out of the matrix
  // instructions (net_f32h.h) when at most 8 parameters remain and at least 2 are taken out.
  sh->hoist = 0;
  if (sh->net == NET_F32_MFMA && allow_hoist) {
    int p0 = 0;
    while (p0 < sh->P && sp->strides[p0] % 32 == 0) ++p0;
    const int n_low = sh->P - p0;
    if (p0 >= 2 && n_low >= 1 && n_low <= 8) {
      sh->hoist = 1;
      sh->p0 = p0;
      // the remaining parameters span exactly one tile: their values repeat from tile to
      // tile, and their layer-1 share is a per-member table (net_f32t.h)
      if (allow_hoist >= 2 && sp->strides[p0 - 1] == 32) sh->hoist = 2;
    }
  }
  if (sh->net == NET_F32_MFMA && sh->hoist == 2) {
    sh->NPL = 1;
    sh->KS = 0;
    sh->o_w1 = 0;                                        // the table
    sh->o_w2 = sh->NT1 * 16 * 64;
    sh->o_b1 = sh->o_w2 + sh->NT2 * sh->NT1 * 16 * 64;
    sh->o_b2 = sh->o_b1;
    sh->o_wo = sh->o_b2 + sh->NT2 * 32;
    sh->o_wh = sh->o_wo + ntl * 32;
    sh->member_words = sh->o_wh + sh->NT1 * f32t_term_groups(sh->p0) * 256;
  } else if (sh->net == NET_F32_MFMA && sh->hoist) {
    sh->NPL = 1;
    sh->KS = (sh->P - sh->p0 + 1) / 2;         // steps of 2 low inputs (no bias column)
    sh->o_w1 = 0;
    sh->o_w2 = sh->NT1 * round_up(sh->KS, 4) * 64;
    sh->o_b1 = sh->o_w2 + sh->NT2 * sh->NT1 * 16 * 64;
    sh->o_b2 = sh->o_b1;
    sh->o_wo = sh->o_b2 + sh->NT2 * 32;
    sh->o_wh = sh->o_wo + ntl * 32;
    sh->member_words = sh->o_wh + round_up((sh->p0 + 1) * sh->NT1 * 32, 4);
  } else if (sh->net == NET_F32_MFMA) {
    sh->NPL = 1;
    sh->KS = round_up(sh->P + 1, 4) / 2;       // steps of 2 inputs (bias column included), even
    sh->o_w1 = 0;
    sh->o_w2 = sh->NT1 * round_up(sh->KS, 4) * 64;   // stored in groups of 4 steps
    sh->o_b1 = sh->o_w2 + sh->NT2 * sh->NT1 * 16 * 64;   // (no separate b1 table: bias rides in W1A)
    sh->o_b2 = sh->o_b1;
    sh->o_wo = sh->o_b2 + sh->NT2 * 32;
    sh->member_words = sh->o_wo + ntl * 32;
  } else if (sh->net == NET_BF16 || sh->net == NET_F16X2) {
    sh->NPL = sh->net == NET_F16X2 ? 2 : 1;
    sh->KS = (sh->P + 15) / 16;                // blocks of 16 inputs
    sh->o_w1 = 0;
    sh->o_w2 = sh->NPL * sh->NT1 * sh->KS * 256;
    sh->o_b1 = sh->o_w2 + sh->NPL * sh->NT2 * 2 * sh->NT1 * 256;
    sh->o_b2 = sh->o_b1 + sh->NT1 * 32;
    sh->o_wo = sh->o_b2 + sh->NT2 * 32;
    sh->member_words = sh->o_wo + ntl * 32;
  } else {                                     // NET_F32_VALU
    sh->NPL = 1;
    sh->KS = sh->P <= 8 ? 8 : (sh->P <= 16 ? 16 : 32);   // inputs padded
    const int h1p = sh->NT1 * 32, h2p = sh->NT2 * 32;
    sh->o_w1 = 0;
    sh->o_w2 = h1p * sh->KS;
    sh->o_b1 = sh->o_w2 + h2p * h1p;
    sh->o_b2 = sh->o_b1 + h1p;
    sh->o_wo = sh->o_b2 + h2p;
    sh->member_words = sh->o_wo + ntl * 32;
  }
  return TUNER_OK;
}

static const Variant* find_variant(const Shape& sh) {
  if (sh.net == NET_F32_MFMA) {
    if (sh.hoist == 2) return find_variant_f32t(sh.NT1, sh.NT2);
    return sh.hoist ? find_variant_f32h(sh.KS, sh.NT1, sh.NT2) : find_variant_f32(sh.KS, sh.NT1, sh.NT2);
  }
  if (sh.net == NET_BF16 || sh.net == NET_F16X2) return find_variant_lp(sh.net, sh.KS, sh.NT1, sh.NT2);
  if (sh.net == NET_F32_VALU) return find_variant_valu(sh.KS, sh.NT1, sh.NT2);
  return nullptr;
}

// ---------------------------------------------------------------------------
// classify: for a long constrained range, the list of chunks the sweep has to visit.
// A chunk whose rule parameters keep their digits over all its configurations (the
// quotient index / stride is the same at both ends, hence throughout) is valid or
// invalid as a whole.  Chunks without any valid configuration are left out of the list
// (predict_all gets their +inf right here); the others carry their state, so that
// wholly valid chunks skip the per-lane rule sums.  The order of the list does not
// matter to any result.
// ---------------------------------------------------------------------------
struct ClassifyParams {
  uint64_t begin, count;
  uint32_t head;              // positions of the range before the caller's first configuration
  uint32_t n_chunks, iter;
  uint32_t per_block;         // chunks classified by one workgroup (<= 256): few when it also fills outputs
  float* pred;                // predict_all: wholly invalid chunks get their +inf (and mask 0) here
  uint8_t* mask;
  uint32_t* live;
  WsHeader* hdr;
};

__global__ void __launch_bounds__(256) classify_kernel(const DevSpace sp, const ClassifyParams cp) {
  __shared__ uint8_t s_state[256];
  const bool pow2 = sp.all_pow2 != 0;
  const uint32_t lane = threadIdx.x & 63;
  for (uint32_t base = blockIdx.x * cp.per_block; base < cp.n_chunks; base += gridDim.x * cp.per_block) {
    const uint32_t c = base + threadIdx.x;
    const bool in = threadIdx.x < cp.per_block && c < cp.n_chunks;
    uint32_t state = CHUNK_ALL_INVALID;
    if (in) {
      const uint64_t t0 = (uint64_t)c * cp.iter;
      const uint64_t left = cp.count - t0 < (uint64_t)cp.iter ? cp.count - t0 : (uint64_t)cp.iter;
      const uint32_t lo = (uint32_t)(cp.begin + t0), hi = (uint32_t)(cp.begin + t0 + left - 1);
      bool uniform = true;
      for (int cc = 0; cc < sp.n_constraints; ++cc)
        for (int e = sp.entry_begin[cc]; e < sp.entry_begin[cc + 1]; ++e) {
          const int p = (int)sp.entry[e].param;
          const uint32_t qa = pow2 ? lo >> sp.pa[p].shift : fast_div(lo, sp.pa[p].stride_mul, sp.pb[p].stride_sh);
          const uint32_t qb = pow2 ? hi >> sp.pa[p].shift : fast_div(hi, sp.pa[p].stride_mul, sp.pb[p].stride_sh);
          uniform = uniform && qa == qb;
        }
      state = uniform ? (is_valid(sp, lo, pow2) ? CHUNK_ALL_VALID : CHUNK_ALL_INVALID) : CHUNK_MIXED;
    }
    const bool keep = in && state != CHUNK_ALL_INVALID;
    const unsigned long long bal = __ballot(keep);
    uint32_t pos = 0;
    if (lane == 0 && bal) pos = atomicAdd(&cp.hdr->n_live, (uint32_t)__popcll(bal));
    pos = __shfl(pos, 0);
    if (keep) cp.live[pos + __popcll(bal & ((1ull << lane) - 1ull))] = c | (state << 30);
    if (cp.pred) {
      // the block fills the outputs of its wholly invalid chunks, coalesced
      __syncthreads();
      s_state[threadIdx.x] = in ? (uint8_t)state : (uint8_t)CHUNK_MIXED;
      __syncthreads();
      for (uint32_t j = 0; j < cp.per_block; ++j) {
        if (s_state[j] != CHUNK_ALL_INVALID) continue;
        const uint64_t t0 = (uint64_t)(base + j) * cp.iter;
        const uint64_t left = cp.count - t0 < (uint64_t)cp.iter ? cp.count - t0 : (uint64_t)cp.iter;
        for (uint64_t x = threadIdx.x; x < left; x += blockDim.x) {
          if (t0 + x < cp.head) continue;
          cp.pred[t0 + x] = __builtin_inff();
          if (cp.mask) cp.mask[t0 + x] = 0;
        }
      }
    }
  }
}

struct Layout {
  size_t o_hdr, o_space, o_packed, o_pools, o_extra, o_live, total;
  uint32_t cap, kp;
};

static uint32_t host_next_pow2(uint32_t v) { uint32_t p = 1; while (p < v) p <<= 1; return p; }


static Layout make_layout(const Shape& sh, int k, uint64_t n_configs, const Variant* var) {
  Layout L{};
  auto al = [](size_t v) { return (v + 255) / 256 * 256; };
  L.o_hdr = 0;
  L.o_space = al(sizeof(WsHeader));
  L.o_packed = L.o_space + kSpaceBytes;
  L.o_pools = L.o_packed + al((size_t)sh.E * sh.member_words * 4);
  L.kp = k > 0 ? host_next_pow2((uint32_t)k) : 0;
  const uint32_t unit_max = (uint32_t)(kMaxIter * kMaxSuper);
  L.cap = k > 0 ? 4u * (L.kp > unit_max ? L.kp : unit_max) : 0;
  L.o_extra = L.o_pools + (size_t)kMaxGroups * L.cap * 8;
  L.o_live = L.o_extra + al((size_t)L.kp * 8);
  // live-chunk list: long ranges only, whose chunks have the variant's full size
  const uint64_t full = (uint64_t)var->waves * var->R * var->tile;
  L.total = L.o_live + al((size_t)((n_configs + full - 1) / full) * 4);
  return L;
}

struct ProfileState {
  bool on = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> events[PROFILE_KINDS];
};
static ProfileState g_profile;
bool profile_on() { return g_profile.on; }
void profile_add(int kind, hipEvent_t begin, hipEvent_t end) { g_profile.events[kind].emplace_back(begin, end); }

struct DeviceInfo { int n_cu = 0; int max_lds = 0; bool ok = false; };

static int device_info(DeviceInfo* out) {
  static thread_local DeviceInfo cache[64];
  int dev = 0;
  TUNER_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return set_error(TUNER_EHIP, "device ordinal out of range");
  if (!cache[dev].ok) {
    TUNER_HIP_TRY(hipDeviceGetAttribute(&cache[dev].n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    TUNER_HIP_TRY(hipDeviceGetAttribute(&cache[dev].max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    cache[dev].ok = true;
  }
  *out = cache[dev];
  return TUNER_OK;
}

// For host-only queries: the current device's attributes when there is a device, else the
// figures of the GPU this library is written for (MI355X: 256 compute units, 160 KB of LDS).
static DeviceInfo device_info_or_default() {
  DeviceInfo di;
  int n = 0;
  if (hipGetDeviceCount(&n) == hipSuccess && n > 0 && device_info(&di) == TUNER_OK) return di;
  (void)hipGetLastError();
  di.n_cu = kMaxGroups;
  di.max_lds = kLdsBytesPerWorkgroup;
  di.ok = true;
  return di;
}

// LDS bytes of the hoisting networks' per-wave scratch: the high features of a wave's
// tiles, and for net_f32h.h one z_high vector.
static int hoist_scratch_bytes(const Shape& sh, const Variant* var) {
  if (!sh.hoist) return 0;
  const int z = sh.hoist == 1 ? std::max(64, sh.NT1 * 32) : 0;
  return var->waves * (var->R * 32 + z) * 4;
}

// How the ensemble goes through LDS: all members resident, or stages of `mps` members.
// Members that do not all fit are streamed through two half-size buffers if a member fits
// one half: the next stage loads while the current one is evaluated.
struct StagePlan { int budget = 0, mps = 0; bool double_buffer = false; };

static StagePlan plan_stages(const Shape& sh, const Variant* var, int max_lds) {
  StagePlan pl;
  pl.budget = max_lds - kSpaceBytes - 64 - hoist_scratch_bytes(sh, var);   // 64 B of static LDS
  const int member_bytes = sh.member_words * 4;
  pl.mps = pl.budget > 0 ? std::min(pl.budget / member_bytes, sh.E) : 0;
  if (pl.mps >= 1 && pl.mps < sh.E && (pl.budget / 2) / member_bytes >= 1) {
    pl.mps = (pl.budget / 2) / member_bytes;
    pl.double_buffer = true;
  }
  return pl;
}

// Shape and kernel variant of a sweep.  Range sweeps (hoist_ok) take the layer-1 shortcuts
// the space allows; the table of the low parameters' share makes a member larger, so it is
// used only while the ensemble stays resident in LDS or keeps its two stage buffers.
static int choose_shape(const tuner_space* sp, const tuner_model* m, bool hoist_ok, int max_lds, Shape* sh,
                        const Variant** var) {
  for (int level = hoist_ok ? 2 : 0; ; --level) {
    const int rc = make_shape(sp, m, sh, level);
    if (rc) return rc;
    *var = find_variant(*sh);
    if (!*var) return set_error(TUNER_ETOOLARGE, "no kernel variant for this model shape");
    if (sh->hoist < 2) return TUNER_OK;
    const StagePlan pl = plan_stages(*sh, *var, max_lds);
    if (pl.mps >= sh->E || pl.double_buffer) return TUNER_OK;
  }
}

// ---------------------------------------------------------------------------
// Scratch of the allocation-free entry point: the workspace of a top-k sweep (header, space
// tables, packed weights, candidate pools, key list of the running result, live-chunk list)
// in a file-scope device array.  Every GPU the library runs on holds its own copy at its own
// address; host code uses the address hipGetSymbolAddress returns for the current device,
// never the array's name.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[TUNER_STATIC_SCRATCH_BYTES];

static int scratch_address(void** out) {
  static std::mutex mu;
  static void* ptr_of_device[64] = {};
  int dev = 0;
  TUNER_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return set_error(TUNER_EHIP, "device ordinal out of range");
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of_device[dev]) {
    void* ptr = nullptr;
    TUNER_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return set_error(TUNER_EHIP, "no device address for the static scratch array");
    ptr_of_device[dev] = ptr;
  }
  *out = ptr_of_device[dev];
  return TUNER_OK;
}

static int launch_prep(const tuner_space* sp, const tuner_model* m, const Shape& sh, WsHeader* hdr,
                       DevSpace* space_dev, uint32_t* packed, hipStream_t stream) {
  PrepParams pp{};
  pp.sh = sh;
  pp.raw = m->weights_dev;
  pp.packed = packed;
  pp.space_out = space_dev;
  pp.hdr = hdr;
  const uint32_t total_packed = (uint32_t)sh.E * sh.member_words;
  const unsigned prep_blocks = std::min<unsigned>(1024, (total_packed + 255) / 256);
  hipLaunchKernelGGL(prep_kernel, dim3(prep_blocks), dim3(256), 0, stream, sp->dev, pp);
  TUNER_HIP_TRY(hipGetLastError());
  return TUNER_OK;
}

// Everything a sweep call decides before it touches the device: the network layout and
// kernel variant, how the range is cut into chunks and queue units, how the ensemble goes
// through LDS, where the candidate pool lives, and the launches of the merge that follows.
// Made from host data and two device attributes only, so that a call can fail before its
// first kernel is enqueued and leave the caller's outputs alone.
struct SweepPlan {
  Shape sh{};
  const Variant* var = nullptr;
  Layout L{};
  uint64_t begin = 0, count = 0;       // the swept range (extended downwards to a tile boundary when hoisting)
  uint32_t head = 0;
  int r_used = 0, iter = 0;
  uint32_t n_chunks = 0, super = 1, n_units = 0, groups = 0;
  bool dynamic = false, use_live = false;
  StagePlan pl{};
  uint32_t stage_words = 0, lds_entries = 0, lds_pool_entries = 0, lds_pool_offset = 0, hoist_offset = 0;
  size_t lds = 0;
  // merge of the workgroups' lists (top-k mode)
  bool merge_in_lds = false;
  uint32_t merge_max_levels = 0;
  size_t merge_lds_max = 0;
  uint32_t n_lists = 0;                // the workgroups' lists, and the running result when the call merges with it
  int merge_launches = 0;
};

// A merge launch of `blocks` workgroups can finish the merge itself (its last workgroup merges
// the blocks' results) when those results fit the LDS of one workgroup: the number of tree
// levels of that second stage, or 0.
static uint32_t merge_fuse_levels(uint32_t blocks, size_t list_bytes, size_t lds_max) {
  if (blocks < 2) return 0;
  uint32_t levels = 1;
  while ((1u << levels) < blocks) ++levels;
  return (list_bytes << levels) <= lds_max ? levels : 0;
}

static int plan_sweep(const tuner_space* sp, const tuner_model* m, uint64_t begin, uint64_t count, int mode,
                      int k, bool merge, bool index_list, const DeviceInfo& di, SweepPlan* out) {
  SweepPlan& P = *out;
  int rc = choose_shape(sp, m, !index_list, di.max_lds, &P.sh, &P.var);
  if (rc) return rc;
  const Shape& sh = P.sh;
  const Variant* var = P.var;
  if (index_list) {
    if (count > (1ull << 32)) return set_error(TUNER_ETOOLARGE, "more than 2^32 list entries");
  } else if (begin > sp->n_configs || count > sp->n_configs - begin) {
    return set_error(TUNER_EINVAL, "range outside the space");
  }
  // The hoisting network needs tiles that start at multiples of 32 in the space: the swept
  // range is extended downwards to one, and the `head` positions before the caller's range
  // are masked (outputs are addressed through pointers shifted by the same amount).  A
  // configuration is then evaluated in the same place of the same tile whatever the range,
  // so results do not depend on how a sweep is cut into calls.
  P.head = 0;
  if (sh.hoist && count > 0) {
    P.head = (uint32_t)(begin % 32);
    begin -= P.head;
    count += P.head;
  }
  P.begin = begin;
  P.count = count;
  P.L = make_layout(sh, k, sp->n_configs, var);

  const int n_cu = di.n_cu > 0 ? di.n_cu : 1;
  const uint32_t max_groups = (uint32_t)std::min(n_cu, kMaxGroups);
  // tiles per wave and chunk: the variant's R, or fewer when the range is so short that
  // smaller chunks finish sooner (rounds of chunks over the workgroups x tiles per chunk)
  int r_used = var->R;
  {
    uint64_t best = ~0ull;
    const uint64_t full = (uint64_t)var->waves * var->R * var->tile;
    const bool is_short = (count + full - 1) / full < 8ull * max_groups;
    for (int r = var->R; r >= (is_short ? 1 : var->R); --r) {
      const uint64_t it = (uint64_t)var->waves * r * var->tile;
      const uint64_t chunks = (count + it - 1) / it;
      const uint64_t cost = (chunks + max_groups - 1) / max_groups * (uint64_t)r;
      if (cost < best) { best = cost; r_used = r; }
    }
  }
  P.r_used = r_used;
  const int iter = var->waves * r_used * var->tile;
  P.iter = iter;
  const uint64_t n_chunks64 = (count + iter - 1) / iter;
  P.n_chunks = (uint32_t)n_chunks64;   // count <= 2^32, iter >= 256
  // queue unit: up to kMaxSuper chunks, while every workgroup still gets >= 8 units
  uint32_t super = 1;
  while (super < (uint32_t)kMaxSuper && 2 * super * (uint32_t)iter <= (uint32_t)(kMaxIter * kMaxSuper) &&
         n_chunks64 / (2 * super) >= 8ull * max_groups)
    super *= 2;
  // a resident ensemble keeps its candidate pool (2 k keys + one queue unit) in LDS too if
  // it fits; a smaller unit is worth that
  if (mode == MODE_TOPK && k > 0) {
    const size_t hoist_b = (size_t)hoist_scratch_bytes(sh, var);
    const size_t free_b = (size_t)di.max_lds - kSpaceBytes - 64 - hoist_b;
    const size_t weights_b = ((size_t)sh.E * sh.member_words * 4 + 15) / 16 * 16;
    if (weights_b < free_b) {
      const uint32_t kp2 = 2u * host_next_pow2((uint32_t)k);
      while (super > 1 && (size_t)host_next_pow2(kp2 + super * (uint32_t)iter) * 8 > free_b - weights_b &&
             (size_t)host_next_pow2(kp2 + (super / 2) * (uint32_t)iter) * 8 <= free_b - weights_b)
        super /= 2;
    }
  }
  P.super = super;
  P.n_units = (uint32_t)((n_chunks64 + super - 1) / super);
  P.groups = std::min<uint32_t>(P.n_units, max_groups);

  if (P.groups > 0) {
    const int hoist_bytes = hoist_scratch_bytes(sh, var);
    P.pl = plan_stages(sh, var, di.max_lds);
    if (P.pl.mps < 1) return set_error(TUNER_ETOOLARGE, "one packed member does not fit in LDS");
    const int budget = P.pl.budget, mps = P.pl.mps, member_bytes = sh.member_words * 4;
    // long ranges take units from the queue counter; constrained ones first get the list
    // of chunks worth visiting (the list is sized for full chunks)
    P.dynamic = P.n_units > 8u * P.groups;
    P.use_live = P.dynamic && !index_list && sp->n_constraints > 0 && r_used == var->R;
    // the region after the space tables holds a stage of weights and doubles as sort
    // scratch for the candidate pool: make it large enough for a pool that is compacted
    // when it reaches 2 k + one queue unit, if the LDS allows
    P.stage_words = (uint32_t)(mps * sh.member_words);
    size_t region = (size_t)mps * member_bytes * (P.pl.double_buffer ? 2 : 1);
    if (mode == MODE_TOPK) {
      const size_t want = 8ull * host_next_pow2(2u * P.L.kp + super * (uint32_t)iter);
      if (want > region && want <= (size_t)budget) region = want;
    }
    P.lds_entries = (uint32_t)(region / 8);
    size_t lds = (size_t)kSpaceBytes + region;
    // resident ensembles that leave room keep the candidate pool in LDS too
    const int n_stages = (sh.E + mps - 1) / mps;
    if (mode == MODE_TOPK && n_stages == 1) {
      const size_t weights_bytes = ((size_t)mps * member_bytes + 15) / 16 * 16;
      const size_t room = (size_t)budget > weights_bytes ? (size_t)budget - weights_bytes : 0;
      // the smallest pool that takes 2 k keys and one queue unit: small pools are sorted
      // more often but much faster, and tighten the threshold sooner
      const uint32_t entries = host_next_pow2(2u * P.L.kp + super * (uint32_t)iter);
      if ((size_t)entries * 8 <= room) {
        P.lds_pool_entries = entries;
        P.lds_pool_offset = (uint32_t)(kSpaceBytes + weights_bytes);
        P.lds_entries = (uint32_t)(weights_bytes / 8);
        lds = (size_t)kSpaceBytes + weights_bytes + (size_t)entries * 8;
      }
    }
    P.hoist_offset = (uint32_t)((lds + 15) / 16 * 16);
    P.lds = (size_t)P.hoist_offset + (size_t)hoist_bytes;
    if (P.lds + 64 > (size_t)di.max_lds) return set_error(TUNER_ETOOLARGE, "the sweep's LDS layout does not fit this device");
  }

  if (mode == MODE_TOPK) {
    // lists: pool 0..groups-1, then the running result when it takes part
    const uint32_t n_lists = P.groups + (merge || P.groups == 0 ? 1u : 0u);
    P.n_lists = n_lists;
    const size_t list_bytes = (size_t)P.L.kp * 8;
    P.merge_lds_max = std::min<size_t>((size_t)di.max_lds, 128u << 10);
    P.merge_in_lds = 2 * list_bytes <= P.merge_lds_max;
    P.merge_launches = 0;
    if (P.merge_in_lds) {
      // in LDS, up to 32 lists per workgroup and launch
      P.merge_max_levels = 0;
      while (P.merge_max_levels < 5 && (list_bytes << (P.merge_max_levels + 1)) <= P.merge_lds_max) ++P.merge_max_levels;
      uint32_t live = n_lists;
      while (live > 1) {
        uint32_t levels = 1;
        while (levels < P.merge_max_levels && (1u << levels) < live) ++levels;
        live = (live + (1u << levels) - 1) >> levels;
        ++P.merge_launches;
        if (live > 1 && merge_fuse_levels(live, list_bytes, P.merge_lds_max)) break;   // second stage in the same launch
      }
      if (n_lists == 1) P.merge_launches = 1;      // finalize only
    } else {
      for (uint32_t n = n_lists; n > 1; n = (n + 1) / 2) ++P.merge_launches;
      ++P.merge_launches;                          // finalize
    }
  }
  return TUNER_OK;
}

// prepared: the workspace already holds the header, the space tables and the packed weights
// of this space and model in the layout of a range sweep (tuner_prepare), so no packing
// kernel is launched.
static int run_sweep(const tuner_space* sp, const tuner_model* m, uint64_t begin, uint64_t count,
                     int mode, int k, int merge, float* values, uint32_t* indices, int32_t* n_found,
                     float* pred, uint8_t* mask, void* ws, size_t ws_bytes, hipStream_t stream,
                     const uint32_t* index_list = nullptr, bool prepared = false, bool timed = true) {
  // ---- everything that can fail comes before the first launch
  // (argument errors are reported even where there is no device to ask: the plan then uses
  // MI355X's figures and the device error comes after them)
  DeviceInfo di;
  const int dev_rc = device_info(&di);
  const std::string dev_msg = dev_rc ? std::string(tuner_last_error()) : std::string();
  if (dev_rc) {
    di.n_cu = kMaxGroups;
    di.max_lds = kLdsBytesPerWorkgroup;
  }
  SweepPlan P;
  int rc = plan_sweep(sp, m, begin, count, mode, k, merge != 0, index_list != nullptr, di, &P);
  if (rc) return rc;
  const Shape& sh = P.sh;
  const Variant* var = P.var;
  const Layout& L = P.L;
  if (!ws || ws_bytes < L.total) return set_error(TUNER_EWORKSPACE, "workspace missing or too small");
  if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0) return set_error(TUNER_EWORKSPACE, "workspace not 256-byte aligned");
  if (dev_rc) return set_error(dev_rc, dev_msg);
  if (P.groups > 0) {
    rc = allow_dynamic_lds(reinterpret_cast<const void*>(var->fn), (int)P.lds);
    if (rc) return rc;
  }
  if (mode == MODE_TOPK && P.merge_in_lds && P.groups > 0) {
    rc = allow_dynamic_lds(reinterpret_cast<const void*>(merge_tree_kernel), (int)P.merge_lds_max);
    if (rc) return rc;
  }
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  if (g_profile.on && timed && P.groups > 0) {
    TUNER_HIP_TRY(hipEventCreate(&ev0));
    const hipError_t e = hipEventCreate(&ev1);
    if (e != hipSuccess) { (void)hipEventDestroy(ev0); return hip_error(e, "hipEventCreate"); }
  }

  // outputs are addressed from the start of the (possibly extended) range
  begin = P.begin;
  count = P.count;
  if (pred) pred -= P.head;
  if (mask) mask -= P.head;
  unsigned char* base = static_cast<unsigned char*>(ws);
  WsHeader* hdr = reinterpret_cast<WsHeader*>(base + L.o_hdr);
  DevSpace* space_dev = reinterpret_cast<DevSpace*>(base + L.o_space);
  uint32_t* packed = reinterpret_cast<uint32_t*>(base + L.o_packed);
  unsigned long long* pools = reinterpret_cast<unsigned long long*>(base + L.o_pools);
  unsigned long long* extra = reinterpret_cast<unsigned long long*>(base + L.o_extra);

  if (!prepared) {
    rc = launch_prep(sp, m, sh, hdr, space_dev, packed, stream);
    if (rc) return rc;
  }

  const uint32_t groups = P.groups;
  if (groups == 0 && mode == MODE_TOPK) {
    // nothing is swept: the running result stays as it is, or there is no result at all
    if (!merge) {
      hipLaunchKernelGGL(empty_result_kernel, dim3((k + 255) / 256), dim3(256), 0, stream, k, values, indices, n_found);
      TUNER_HIP_TRY(hipGetLastError());
    }
    return TUNER_OK;
  }
  if (groups > 0) {
    SweepParams sw{};
    sw.begin = begin;
    sw.count = count;
    sw.head = P.head;
    sw.n_chunks = P.n_chunks;
    sw.n_units = P.n_units;
    sw.super = (int32_t)P.super;
    sw.r_used = P.r_used;
    sw.n_members = sh.E;
    sw.members_per_stage = P.pl.mps;
    sw.n_stages = (sh.E + P.pl.mps - 1) / P.pl.mps;
    sw.member_words = sh.member_words;
    sw.off = NetOffsets{sh.o_w1, sh.o_w2, sh.o_b1, sh.o_b2, sh.o_wo, sh.H1, sh.H2, sh.o_wh, sh.p0};
    sw.mode = mode;
    sw.merge = merge;
    sw.self_reset = (mode == MODE_ALL && (P.dynamic || P.use_live)) ? 1 : 0;
    sw.extra = mode == MODE_TOPK ? extra : nullptr;
    sw.run_values = values;
    sw.run_indices = indices;
    sw.run_found = n_found;
    sw.inv_members = (float)(1.0 / (double)sh.E);
    sw.k = k;
    sw.cap = L.cap;
    sw.kp = L.kp;
    sw.space = space_dev;
    sw.packed = packed;
    sw.index_list = index_list;
    sw.hdr = hdr;
    sw.pools = pools;
    sw.pred = pred;
    sw.mask = mask;
    sw.dynamic = P.dynamic ? 1 : 0;
    sw.live = nullptr;
    if (P.use_live) {
      uint32_t* live = reinterpret_cast<uint32_t*>(base + L.o_live);
      ClassifyParams cp{};
      cp.begin = begin;
      cp.count = count;
      cp.head = P.head;
      cp.n_chunks = P.n_chunks;
      cp.iter = (uint32_t)P.iter;
      cp.pred = mode == MODE_ALL ? pred : nullptr;
      cp.mask = mode == MODE_ALL ? mask : nullptr;
      cp.live = live;
      cp.hdr = hdr;
      // a workgroup that also fills the outputs of its invalid chunks takes few chunks, so
      // that the fill is spread over the chip even when the range has only a few thousand
      cp.per_block = cp.pred ? 16u : 256u;
      hipLaunchKernelGGL(classify_kernel, dim3(std::min<uint32_t>(1u << 16, (P.n_chunks + cp.per_block - 1u) / cp.per_block)),
                         dim3(256), 0, stream, sp->dev, cp);
      TUNER_HIP_TRY(hipGetLastError());
      sw.live = live;
    }
    sw.double_buffer = P.pl.double_buffer ? 1 : 0;
    sw.stage_words = P.stage_words;
    sw.lds_entries = P.lds_entries;
    sw.lds_pool_entries = P.lds_pool_entries;
    sw.lds_pool_offset = P.lds_pool_offset;
    sw.hoist_offset = P.hoist_offset;
    if (ev0) TUNER_HIP_TRY(hipEventRecord(ev0, stream));
    hipLaunchKernelGGL(var->fn, dim3(groups), dim3(var->waves * 64), P.lds, stream, sw);
    TUNER_HIP_TRY(hipGetLastError());
    if (ev0) {
      TUNER_HIP_TRY(hipEventRecord(ev1, stream));
      profile_add(PROFILE_SWEEP, ev0, ev1);
    }
  }

  if (mode == MODE_TOPK) {
    // lists: pool 0..groups-1, then the running result when the call merges with it
    const uint32_t n_lists = P.n_lists;
    const size_t list_bytes = (size_t)L.kp * 8;
    bool finalized = false;
    if (P.merge_in_lds) {
      uint32_t live = n_lists, stride = 1;
      while (live > 1) {
        uint32_t levels = 1;
        while (levels < P.merge_max_levels && (1u << levels) < live) ++levels;
        const uint32_t blocks = (live + (1u << levels) - 1) >> levels;
        const uint32_t fuse = merge_fuse_levels(blocks, list_bytes, P.merge_lds_max);
        MergeParams mp{};
        mp.pools = pools;
        mp.extra = extra;
        mp.cap = L.cap;
        mp.n_pool_lists = groups;
        mp.n_lists = n_lists;
        mp.kp = L.kp;
        mp.stride0 = stride;
        mp.levels = levels;
        mp.fuse_levels = fuse;
        mp.final = blocks == 1 ? 1 : 0;
        mp.k = k;
        mp.values = values;
        mp.indices = indices;
        mp.n_found = n_found;
        mp.hdr = hdr;
        hipLaunchKernelGGL(merge_tree_kernel, dim3(blocks), dim3(kMergeThreads),
                           list_bytes << std::max(levels, fuse), stream, mp);
        TUNER_HIP_TRY(hipGetLastError());
        finalized = blocks == 1 || fuse > 0;
        live = fuse > 0 ? 1 : blocks;
        stride <<= levels;
      }
    } else {
      uint32_t n = n_lists;
      while (n > 1) {
        const uint32_t half = (n + 1) / 2;
        hipLaunchKernelGGL(merge_kernel, dim3(n - half), dim3(kMergeThreads), 0, stream, pools, L.cap, extra,
                           groups, L.kp, half);
        TUNER_HIP_TRY(hipGetLastError());
        n = half;
      }
    }
    if (!finalized) {
      const unsigned long long* list0 = groups > 0 ? pools : extra;
      hipLaunchKernelGGL(finalize_kernel, dim3((k + 255) / 256), dim3(256), 0, stream, list0, k, values,
                         indices, n_found, hdr);
      TUNER_HIP_TRY(hipGetLastError());
    }
  }
  return TUNER_OK;
}

}  // namespace tuner

using tuner::set_error;

extern "C" {

// Bytes of workspace a sweep of this space, model and k may need (any layout of the packed
// weights a call can choose).
static int workspace_need(const tuner_space* space, const tuner_model* model, int32_t k, size_t* need_out) {
  if (!space || !model) return set_error(TUNER_EINVAL, "null argument");
  if (k < 0 || k > TUNER_MAX_K) return set_error(TUNER_ETOOLARGE, "k out of range");
  size_t need = 0;
  for (int level = 0; level <= 2; ++level) {
    tuner::Shape sh{};
    const int rc = tuner::make_shape(space, model, &sh, level);
    if (rc) return rc;
    const tuner::Variant* var = tuner::find_variant(sh);
    if (!var) return set_error(TUNER_ETOOLARGE, "no kernel variant for this model shape");
    need = std::max(need, tuner::make_layout(sh, k, space->n_configs, var).total);
  }
  *need_out = need;
  return TUNER_OK;
}

size_t tuner_workspace_bytes(const tuner_space* space, const tuner_model* model, int32_t k) {
  size_t need = 0;
  return workspace_need(space, model, k, &need) == TUNER_OK ? need : 0;
}

int tuner_hoisted_parameters(const tuner_space* space, const tuner_model* model, int32_t* n_hoisted) {
  if (!space || !model || !n_hoisted) return set_error(TUNER_EINVAL, "null argument");
  tuner::Shape sh{};
  const int rc = tuner::make_shape(space, model, &sh, 1);
  if (rc) return rc;
  *n_hoisted = sh.hoist ? sh.p0 : 0;
  return TUNER_OK;
}

int tuner_tabulated_parameters(const tuner_space* space, const tuner_model* model, int32_t* n_tabulated) {
  if (!space || !model || !n_tabulated) return set_error(TUNER_EINVAL, "null argument");
  tuner::Shape sh{};
  const tuner::Variant* var = nullptr;
  const int rc = tuner::choose_shape(space, model, true, tuner::device_info_or_default().max_lds, &sh, &var);
  if (rc) return rc;
  *n_tabulated = sh.hoist == 2 ? sh.P - sh.p0 : 0;
  return TUNER_OK;
}

int tuner_sweep_plan(const tuner_space* space, const tuner_model* model, uint64_t index_begin,
                     uint64_t index_count, int32_t k, tuner_sweep_plan_info* out) {
  if (!space || !model || !out) return set_error(TUNER_EINVAL, "null argument");
  if (k < 0) return set_error(TUNER_EINVAL, "k must be >= 0");
  if (k > TUNER_MAX_K) return set_error(TUNER_ETOOLARGE, "k > TUNER_MAX_K");
  tuner::SweepPlan P;
  const int rc = tuner::plan_sweep(space, model, index_begin, index_count, k > 0 ? tuner::MODE_TOPK : tuner::MODE_ALL,
                                   k, false, false, tuner::device_info_or_default(), &P);
  if (rc) return rc;
  tuner_sweep_plan_info info{};
  info.network = P.sh.net;
  info.layer1 = P.sh.hoist;
  info.waves = P.var->waves;
  info.tile = P.var->tile;
  info.variant_tiles_per_wave = P.var->R;
  info.tiles_per_wave = P.r_used;
  info.workgroups = (int32_t)P.groups;
  info.n_chunks = P.n_chunks;
  info.chunks_per_unit = (int32_t)P.super;
  info.n_units = P.n_units;
  info.dynamic_queue = P.dynamic ? 1 : 0;
  info.live_chunk_list = P.use_live ? 1 : 0;
  info.members_per_stage = P.groups ? P.pl.mps : 0;
  info.n_stages = P.groups ? (P.sh.E + P.pl.mps - 1) / P.pl.mps : 0;
  info.double_buffer = P.groups && P.pl.double_buffer ? 1 : 0;
  info.pool_in_lds = P.lds_pool_entries > 0 ? 1 : 0;
  info.lds_bytes = (int32_t)P.lds;
  info.merge_launches = P.merge_launches;
  info.workspace_bytes = P.L.total;
  *out = info;
  return TUNER_OK;
}

int tuner_profile_enable(int32_t on) {
  tuner::g_profile.on = on != 0;
  if (!on) {
    // timings nobody read are dropped with their events
    for (auto& kind : tuner::g_profile.events) {
      for (auto& ev : kind) {
        (void)hipEventDestroy(ev.first);
        (void)hipEventDestroy(ev.second);
      }
      kind.clear();
    }
  }
  return TUNER_OK;
}

int64_t tuner_profile_pending(void) {
  int64_t n = 0;
  for (auto& kind : tuner::g_profile.events) n += (int64_t)kind.size();
  return n;
}

static int profile_read(int kind, double* ms_total, int64_t* n_launches) {
  if (!ms_total || !n_launches) return set_error(TUNER_EINVAL, "null argument");
  double total = 0.0;
  int64_t n = 0;
  for (auto& ev : tuner::g_profile.events[kind]) {
    float ms = 0.0f;
    TUNER_HIP_TRY(hipEventSynchronize(ev.second));
    TUNER_HIP_TRY(hipEventElapsedTime(&ms, ev.first, ev.second));
    total += ms;
    ++n;
    (void)hipEventDestroy(ev.first);
    (void)hipEventDestroy(ev.second);
  }
  tuner::g_profile.events[kind].clear();
  *ms_total = total;
  *n_launches = n;
  return TUNER_OK;
}

int tuner_profile_read(double* sweep_ms_total, int64_t* n_sweep_launches) {
  return profile_read(tuner::PROFILE_SWEEP, sweep_ms_total, n_sweep_launches);
}

int tuner_profile_read_train(double* train_ms_total, int64_t* n_train_launches) {
  return profile_read(tuner::PROFILE_TRAIN, train_ms_total, n_train_launches);
}

int tuner_predict_topk(const tuner_space* space, const tuner_model* model, uint64_t index_begin,
                       uint64_t index_count, int32_t k, int32_t merge_with_existing,
                       float* topk_values_dev, uint32_t* topk_indices_dev, int32_t* n_found_dev,
                       void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!space || !model || !topk_values_dev || !topk_indices_dev || !n_found_dev)
    return set_error(TUNER_EINVAL, "null argument");
  if (k < 1) return set_error(TUNER_EINVAL, "k must be >= 1");
  if (k > TUNER_MAX_K) return set_error(TUNER_ETOOLARGE, "k > TUNER_MAX_K");
  return tuner::run_sweep(space, model, index_begin, index_count, tuner::MODE_TOPK, k,
                          merge_with_existing ? 1 : 0, topk_values_dev, topk_indices_dev, n_found_dev,
                          nullptr, nullptr, workspace_dev, workspace_bytes, (hipStream_t)hip_stream);
}

int tuner_prepare(const tuner_space* space, const tuner_model* model, void* workspace_dev,
                  size_t workspace_bytes, void* hip_stream) {
  if (!space || !model) return set_error(TUNER_EINVAL, "null argument");
  tuner::DeviceInfo di;
  const int dev_rc = tuner::device_info(&di);
  const std::string dev_msg = dev_rc ? std::string(tuner_last_error()) : std::string();
  if (dev_rc) di = tuner::device_info_or_default();
  tuner::Shape sh{};
  const tuner::Variant* var = nullptr;
  int rc = tuner::choose_shape(space, model, true, di.max_lds, &sh, &var);
  if (rc) return rc;
  const tuner::Layout L = tuner::make_layout(sh, 0, space->n_configs, var);
  // header, tables and packed weights come first in the workspace, whatever k a later call uses
  if (!workspace_dev || workspace_bytes < L.o_pools)
    return set_error(TUNER_EWORKSPACE, "workspace missing or too small");
  if ((reinterpret_cast<uintptr_t>(workspace_dev) & 255) != 0)
    return set_error(TUNER_EWORKSPACE, "workspace not 256-byte aligned");
  if (dev_rc) return set_error(dev_rc, dev_msg);
  unsigned char* base = static_cast<unsigned char*>(workspace_dev);
  return tuner::launch_prep(space, model, sh, reinterpret_cast<tuner::WsHeader*>(base + L.o_hdr),
                            reinterpret_cast<tuner::DevSpace*>(base + L.o_space),
                            reinterpret_cast<uint32_t*>(base + L.o_packed), (hipStream_t)hip_stream);
}

int tuner_predict_topk_prepared(const tuner_space* space, const tuner_model* model, uint64_t index_begin,
                                uint64_t index_count, int32_t k, int32_t merge_with_existing,
                                float* topk_values_dev, uint32_t* topk_indices_dev, int32_t* n_found_dev,
                                void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!space || !model || !topk_values_dev || !topk_indices_dev || !n_found_dev)
    return set_error(TUNER_EINVAL, "null argument");
  if (k < 1) return set_error(TUNER_EINVAL, "k must be >= 1");
  if (k > TUNER_MAX_K) return set_error(TUNER_ETOOLARGE, "k > TUNER_MAX_K");
  return tuner::run_sweep(space, model, index_begin, index_count, tuner::MODE_TOPK, k,
                          merge_with_existing ? 1 : 0, topk_values_dev, topk_indices_dev, n_found_dev,
                          nullptr, nullptr, workspace_dev, workspace_bytes, (hipStream_t)hip_stream, nullptr, true);
}

int tuner_predict_all_prepared(const tuner_space* space, const tuner_model* model, uint64_t index_begin,
                               uint64_t index_count, float* predictions_dev, uint8_t* valid_mask_dev,
                               void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!space || !model || !predictions_dev) return set_error(TUNER_EINVAL, "null argument");
  return tuner::run_sweep(space, model, index_begin, index_count, tuner::MODE_ALL, 0, 0, nullptr,
                          nullptr, nullptr, predictions_dev, valid_mask_dev, workspace_dev,
                          workspace_bytes, (hipStream_t)hip_stream, nullptr, true);
}

int tuner_predict_topk_static(const tuner_space* space, const tuner_model* model, uint64_t index_begin,
                              uint64_t index_count, int32_t k, int32_t merge_with_existing,
                              float* topk_values_dev, uint32_t* topk_indices_dev, int32_t* n_found_dev,
                              void* hip_stream) {
  if (!space || !model || !topk_values_dev || !topk_indices_dev || !n_found_dev)
    return set_error(TUNER_EINVAL, "null argument");
  if (k < 1) return set_error(TUNER_EINVAL, "k must be >= 1");
  if (k > TUNER_MAX_K) return set_error(TUNER_ETOOLARGE, "k > TUNER_MAX_K");
  size_t need = 0;
  int rc = workspace_need(space, model, k, &need);
  if (rc) return rc;
  if (need > (size_t)TUNER_STATIC_SCRATCH_BYTES)
    return set_error(TUNER_ETOOLARGE,
                     "this space, model and k need " + std::to_string(need) + " bytes of scratch, more than the " +
                         std::to_string((size_t)TUNER_STATIC_SCRATCH_BYTES) +
                         " of the static array: use tuner_predict_topk with a workspace");
  void* ws = nullptr;
  rc = tuner::scratch_address(&ws);
  if (rc) return rc;
  return tuner::run_sweep(space, model, index_begin, index_count, tuner::MODE_TOPK, k,
                          merge_with_existing ? 1 : 0, topk_values_dev, topk_indices_dev, n_found_dev,
                          nullptr, nullptr, ws, (size_t)TUNER_STATIC_SCRATCH_BYTES, (hipStream_t)hip_stream,
                          nullptr, false, /*timed=*/false);   // creates no events either
}

int tuner_predict_all(const tuner_space* space, const tuner_model* model, uint64_t index_begin,
                      uint64_t index_count, float* predictions_dev, uint8_t* valid_mask_dev,
                      void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!space || !model || !predictions_dev) return set_error(TUNER_EINVAL, "null argument");
  return tuner::run_sweep(space, model, index_begin, index_count, tuner::MODE_ALL, 0, 0, nullptr,
                          nullptr, nullptr, predictions_dev, valid_mask_dev, workspace_dev,
                          workspace_bytes, (hipStream_t)hip_stream);
}

int tuner_predict_indices(const tuner_space* space, const tuner_model* model, uint64_t n,
                          const uint32_t* indices_dev, float* predictions_dev, uint8_t* valid_mask_dev,
                          void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!space || !model || !predictions_dev || (n > 0 && !indices_dev))
    return set_error(TUNER_EINVAL, "null argument");
  if (n == 0) return TUNER_OK;
  return tuner::run_sweep(space, model, 0, n, tuner::MODE_ALL, 0, 0, nullptr, nullptr, nullptr,
                          predictions_dev, valid_mask_dev, workspace_dev, workspace_bytes,
                          (hipStream_t)hip_stream, indices_dev);
}

}  // extern "C"
