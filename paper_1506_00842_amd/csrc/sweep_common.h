// Shared device/host definitions of the fused sweep: workspace header, candidate
// keys, model shape, kernel parameters, sorting helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dev_space.h"

namespace tuner {

constexpr int kMergeThreads = 1024;
constexpr int kMaxGroups = 256;           // persistent workgroups (MI355X: 256 CUs)
constexpr int kMaxIter = 1024;            // most configurations per chunk (waves * R * tile) over all variants
constexpr int kMaxSuper = 4;              // most chunks per queue unit
constexpr int kLdsBytesPerWorkgroup = 160 * 1024;   // gfx950; host-only queries plan with it
constexpr unsigned long long kKeyMax = ~0ull;
constexpr int kSpaceBytes = (sizeof(DevSpace) + 255) / 256 * 256;
constexpr float kNegLog2e = -1.44269504088896340736f;

enum { MODE_TOPK = 0, MODE_ALL = 1 };
// validity of the configurations of one chunk, known before the sweep
enum { CHUNK_ALL_INVALID = 0, CHUNK_ALL_VALID = 1, CHUNK_MIXED = 2 };
// how the network is evaluated
enum { NET_F32_MFMA = 0, NET_BF16 = 1, NET_F16X2 = 2, NET_F32_VALU = 3 };

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct WsHeader {
  unsigned long long tau;     // upper bound (as a key) of the final k-th smallest key
  uint32_t work_counter;      // next chunk of the dynamic queue
  float bo_sum;               // sum of the members' output biases
  uint32_t n_live;            // entries of the live-chunk list (long constrained ranges)
  uint32_t done;              // workgroups of the running sweep that have finished (see self_reset)
  uint32_t merge_done;        // workgroups of a two-stage merge launch that have written their list
  uint32_t pad[9];
};

// Model shape and the layout of one packed member, in 32-bit words.
struct Shape {
  int net;                    // NET_*
  int P, H1, H2, E;           // H2 = 0: one hidden layer
  int KS;                     // layer-1 K steps: MFMA steps of 2 inputs (f32) or blocks of 16 (bf16/f16)
  int NT1, NT2;               // 32-unit tiles per hidden layer
  int NPL;                    // operand planes (1, or 2 for the split-precision net)
  int o_w1, o_w2, o_b1, o_b2, o_wo;
  int member_words;           // multiple of 4
  int raw_member_floats;
  // fp32 matrix network with the high parameters' layer-1 share computed once per tile
  int hoist;                  // 0: no; 1: high share once per tile (net_f32h.h); 2: also the low share from a table (net_f32t.h)
  int p0;                     // parameters 0 .. p0-1 are constant over a tile of 32 configurations
  int o_wh;                   // their weights and the bias (layout of the network's header)
};

struct NetOffsets { int w1, w2, b1, b2, wo, h1, h2, wh, p0; };   // word offsets; real hidden widths; hoisting

struct SweepParams {
  uint64_t begin, count;
  uint32_t head;               // positions of the range before the caller's first configuration (masked)
  uint32_t n_chunks, n_units;  // chunks of waves*R*tile configurations; queue units of `super` chunks
  int32_t super;
  int32_t r_used;              // tiles per wave and chunk actually used (1 .. the variant's R)
  int32_t n_members, members_per_stage, n_stages, member_words;
  int32_t mode, k;
  int32_t merge;              // top-k: the caller's outputs hold a running result (values, indices, n_found)
  int32_t self_reset;         // the last workgroup to finish restores the header's idle state (sweeps that
                              // are the last kernel of their call and have used the header's counters)
  float inv_members;          // 1 / n_members, rounded once from double
  uint32_t cap, kp;           // pool capacity per workgroup, k rounded up to a power of two
  uint32_t lds_entries;       // keys that fit the LDS region after the space tables (weights / sort scratch)
  uint32_t lds_pool_entries;  // > 0: the candidate pool lives in LDS (a power of two of keys) ...
  uint32_t lds_pool_offset;   // ... at this byte offset of the dynamic LDS
  uint32_t hoist_offset;      // byte offset in the dynamic LDS of the per-wave scratch of the hoisting network
  int32_t double_buffer;      // two stage buffers in LDS, filled by LDS-direct loads during the evaluation
  uint32_t stage_words;       // words between the two buffers
  int32_t dynamic;            // units beyond a workgroup's first come from the queue counter (else strided)
  const uint32_t* live;       // optional list of chunks to sweep: chunk index | state << 30; its length is
                              // hdr->n_live (chunks with no valid configuration are left out)
  NetOffsets off;
  const DevSpace* space;      // in the workspace
  const uint32_t* packed;
  const uint32_t* index_list;  // optional: configuration t of the "range" is index_list[t]
  WsHeader* hdr;
  unsigned long long* pools;
  unsigned long long* extra;   // top-k: kp keys, the running result as a sorted key list (written by the sweep)
  const float* run_values;     // the caller's top-k outputs, read when merge is set
  const uint32_t* run_indices;
  const int32_t* run_found;
  float* pred;
  uint8_t* mask;
};

typedef void (*SweepFn)(const SweepParams);
struct Variant { int net, KS, NT1, NT2, R, waves, tile; SweepFn fn; };

// Lookups implemented next to the instantiations (one translation unit per family).
const Variant* find_variant_f32(int KS, int NT1, int NT2);
const Variant* find_variant_f32h(int KSL, int NT1, int NT2);
const Variant* find_variant_f32t(int NT1, int NT2);
const Variant* find_variant_lp(int net, int KS, int NT1, int NT2);
const Variant* find_variant_valu(int KS, int NT1, int NT2);

#if defined(__HIPCC__)
__device__ __forceinline__ uint32_t order_bits(float y) {
  const uint32_t u = __float_as_uint(y);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unorder_bits(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}
__device__ __forceinline__ unsigned long long make_key(float y, uint32_t index) {
  return ((unsigned long long)order_bits(y) << 32) | index;
}

// z = -log2(e) * (pre-activation):  1 / (1 + 2^z)
__device__ __forceinline__ float sigmoid_prescaled(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z));
}

// sigma on 16 accumulator registers, in three passes (exp2, +1, rcp) so that no
// instruction waits on the transcendental that precedes it
__device__ __forceinline__ void sigmoid16(floatx16& a) {
#pragma unroll
  for (int v = 0; v < 16; ++v) a[v] = __builtin_amdgcn_exp2f(a[v]);
#pragma unroll
  for (int v = 0; v < 16; ++v) a[v] = 1.0f + a[v];
#pragma unroll
  for (int v = 0; v < 16; ++v) a[v] = __builtin_amdgcn_rcpf(a[v]);
}

// Bitonic sort of a[0..n) ascending, n a power of two, by the whole workgroup.
__device__ inline void bitonic_sort(unsigned long long* a, uint32_t n, int tid, int nthreads) {
  for (uint32_t size = 2; size <= n; size <<= 1) {
    for (uint32_t j = size >> 1; j > 0; j >>= 1) {
      for (uint32_t t = tid; t < (n >> 1); t += nthreads) {
        const uint32_t i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const uint32_t l = i | j;
        const bool asc = (i & size) == 0;
        const unsigned long long x = a[i], y = a[l];
        if ((x > y) == asc) { a[i] = y; a[l] = x; }
      }
      __syncthreads();
    }
  }
}

// Sorts pool[0..n2) (n2 a power of two) ascending: in LDS scratch when it fits
// (lds_entries = capacity of the scratch in keys), else in place in global memory.
__device__ inline void sort_pool(unsigned long long* pool, uint32_t n2, unsigned long long* lds,
                                 uint32_t lds_entries, int tid, int nthreads) {
  if (n2 <= lds_entries) {
    for (uint32_t x = tid; x < n2; x += nthreads) lds[x] = pool[x];
    __syncthreads();
    bitonic_sort(lds, n2, tid, nthreads);
    for (uint32_t x = tid; x < n2; x += nthreads) pool[x] = lds[x];
    __syncthreads();
  } else {
    bitonic_sort(pool, n2, tid, nthreads);
  }
}

__device__ __forceinline__ uint32_t next_pow2(uint32_t v) {
  uint32_t p = 1;
  while (p < v) p <<= 1;
  return p;
}
#endif

}  // namespace tuner
