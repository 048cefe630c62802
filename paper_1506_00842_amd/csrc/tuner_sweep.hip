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
#include <utility>
#include <vector>

#include "tuner_internal.h"

namespace tuner {

constexpr int kThreads = 1024;            // 16 waves per workgroup, one workgroup per CU
constexpr int kWaves = kThreads / 64;
constexpr int kMaxGroups = 256;           // persistent workgroups (MI355X: 256 CUs)
constexpr unsigned long long kKeyMax = ~0ull;
constexpr int kSpaceBytes = (sizeof(DevSpace) + 255) / 256 * 256;
constexpr float kNegLog2e = -1.44269504088896340736f;

enum { MODE_TOPK = 0, MODE_ALL = 1 };

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct WsHeader {
  unsigned long long tau;     // upper bound (as a key) of the final k-th smallest key
  uint32_t work_counter;      // next chunk of the dynamic queue
  float bo_sum;               // sum of the members' output biases
  uint32_t pad[12];
};

// Shape of one packed member (floats), see pack_kernel.
struct Shape {
  int P, H1, H2, E;           // H2 = 0: one hidden layer
  int KS1, NT1, NT2;          // layer-1 MFMA steps (K padded to 2*KS1), 32-unit tiles per hidden layer
  int o_w1, o_w2, o_b2, o_wo; // offsets inside a packed member
  int member_floats;          // multiple of 4
  int raw_member_floats;
};

struct SweepParams {
  uint64_t begin, count;
  uint32_t n_chunks;
  int32_t n_members, members_per_stage, n_stages, member_floats;
  int32_t mode, k;
  float inv_members;          // 1 / n_members, rounded once from double
  uint32_t cap, kp;           // pool capacity per workgroup, k rounded up to a power of two
  const DevSpace* space;      // in the workspace
  const float* packed;
  WsHeader* hdr;
  unsigned long long* pools;
  float* pred;
  uint8_t* mask;
};

// ---------------------------------------------------------------------------
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

__device__ __forceinline__ float sigmoid_prescaled(float z) {
  // z = -log2(e) * (pre-activation)
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z));
}

// ---------------------------------------------------------------------------
// prep: packs the weights into MFMA operand order, writes the space tables,
// resets the queue and the threshold, converts the caller's running result
// into a sorted key list.
//
// Packed member (all fp32, hidden-layer weights and biases times -log2 e):
//   W1A [NT1][KS1/4][64 lanes][4]   lane (n, h), steps s = 4*sg + j:
//        unit = 32 t + n, input f = 2 s + h: W1[unit][f], b1[unit] at f = P, else 0
//   W2A [NT2][NT1][4][64 lanes][4]  lane (n, h): W2[32 u + n][32 t + 8 g + 4 h + j]
//   b2A [NT2][4][2][4]              b2[32 u + 8 g + 4 h + j]
//   woA [NTlast][4][2][4]           w_o[32 u + 8 g + 4 h + j]   (not scaled)
// Padded units have zero incoming and outgoing weights.
// ---------------------------------------------------------------------------
struct PrepParams {
  Shape sh;
  const float* raw;           // caller's weights
  float* packed;
  DevSpace* space_out;
  WsHeader* hdr;
  unsigned long long* extra;  // key list of the running result
  uint32_t kp;
  int32_t k, merge;
  const float* in_values;
  const uint32_t* in_indices;
  const int32_t* in_found;
};

__global__ void __launch_bounds__(256) prep_kernel(const DevSpace sp, const PrepParams pp) {
  const Shape& sh = pp.sh;
  const uint32_t gtid = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t gsize = gridDim.x * blockDim.x;
  // raw member layout
  const int r_w1 = 0, r_b1 = r_w1 + sh.H1 * sh.P;
  const int r_w2 = r_b1 + sh.H1;
  const int r_b2 = r_w2 + sh.H2 * sh.H1;
  const int r_wo = sh.H2 ? r_b2 + sh.H2 : r_w2;
  const int HL = sh.H2 ? sh.H2 : sh.H1;
  const int r_bo = r_wo + HL;
  const uint32_t total = (uint32_t)sh.E * sh.member_floats;
  for (uint32_t x = gtid; x < total; x += gsize) {
    const int e = x / sh.member_floats;
    int q = x - e * sh.member_floats;
    const float* raw = pp.raw + (size_t)e * sh.raw_member_floats;
    float v = 0.0f;
    if (q < sh.o_w2) {                                    // W1A
      const int j = q & 3, lane = (q >> 2) & 63, rest = q >> 8;
      const int sg = rest % (sh.KS1 / 4), t = rest / (sh.KS1 / 4);
      const int n = lane & 31, h = lane >> 5, s = 4 * sg + j;
      const int unit = 32 * t + n, f = 2 * s + h;
      if (unit < sh.H1) {
        if (f < sh.P) v = raw[r_w1 + unit * sh.P + f] * kNegLog2e;
        else if (f == sh.P) v = raw[r_b1 + unit] * kNegLog2e;
      }
    } else if (q < sh.o_b2) {                             // W2A
      q -= sh.o_w2;
      const int j = q & 3, lane = (q >> 2) & 63, rest = q >> 8;
      const int g = rest & 3, t = (rest >> 2) % sh.NT1, u = (rest >> 2) / sh.NT1;
      const int n = lane & 31, h = lane >> 5;
      const int out = 32 * u + n, in = 32 * t + 8 * g + 4 * h + j;
      if (out < sh.H2 && in < sh.H1) v = raw[r_w2 + out * sh.H1 + in] * kNegLog2e;
    } else if (q < sh.o_wo) {                             // b2A
      q -= sh.o_b2;
      const int j = q & 3, h = (q >> 2) & 1, g = (q >> 3) & 3, u = q >> 5;
      const int unit = 32 * u + 8 * g + 4 * h + j;
      if (unit < sh.H2) v = raw[r_b2 + unit] * kNegLog2e;
    } else {                                              // woA
      q -= sh.o_wo;
      const int j = q & 3, h = (q >> 2) & 1, g = (q >> 3) & 3, u = q >> 5;
      const int unit = 32 * u + 8 * g + 4 * h + j;
      if (unit < HL) v = raw[r_wo + unit];
    }
    pp.packed[x] = v;
  }
  // space tables
  {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(&sp);
    uint32_t* dst = reinterpret_cast<uint32_t*>(pp.space_out);
    for (uint32_t x = gtid; x < sizeof(DevSpace) / 4; x += gsize) dst[x] = src[x];
  }
  // running result -> key list
  int found = 0;
  if (pp.merge) {
    found = *pp.in_found;
    found = found < 0 ? 0 : (found > pp.k ? pp.k : found);
  }
  if (pp.extra) {
    for (uint32_t x = gtid; x < pp.kp; x += gsize)
      pp.extra[x] = ((int)x < found) ? make_key(pp.in_values[x], pp.in_indices[x]) : kKeyMax;
  }
  if (gtid == 0) {
    float bo = 0.0f;
    for (int e = 0; e < sh.E; ++e) bo += pp.raw[(size_t)e * sh.raw_member_floats + r_bo];
    pp.hdr->bo_sum = bo;
    pp.hdr->work_counter = 0u;
    pp.hdr->tau = (pp.merge && found == pp.k && pp.k > 0)
                      ? make_key(pp.in_values[pp.k - 1], pp.in_indices[pp.k - 1]) : kKeyMax;
  }
}

// ---------------------------------------------------------------------------
// One member on one tile.  xb[s]: B operand of layer 1 (feature 2 s + h of the
// lane's configuration, 1.0 in the bias slot).  Returns the lane's half of the
// output dot product (sum over the units this lane owns).
// ---------------------------------------------------------------------------
template <int KS1, int NT1, int NT2>
__device__ __forceinline__ float member_forward(const float* __restrict__ w, const float (&xb)[KS1],
                                                int lane, int o_w2, int o_b2, int o_wo) {
  const int h = lane >> 5;
  floatx16 a1[NT1];
#pragma unroll
  for (int t = 0; t < NT1; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) a1[t][v] = 0.0f;
  const float4* w1 = reinterpret_cast<const float4*>(w);
#pragma unroll
  for (int sg = 0; sg < KS1 / 4; ++sg) {
#pragma unroll
    for (int t = 0; t < NT1; ++t) {
      const float4 a = w1[(t * (KS1 / 4) + sg) * 64 + lane];
      a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, xb[4 * sg + 0], a1[t], 0, 0, 0);
      a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, xb[4 * sg + 1], a1[t], 0, 0, 0);
      a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, xb[4 * sg + 2], a1[t], 0, 0, 0);
      a1[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, xb[4 * sg + 3], a1[t], 0, 0, 0);
    }
  }
#pragma unroll
  for (int t = 0; t < NT1; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) a1[t][v] = sigmoid_prescaled(a1[t][v]);

  float part = 0.0f;
  if constexpr (NT2 > 0) {
    floatx16 a2[NT2];
    const float4* b2 = reinterpret_cast<const float4*>(w + o_b2);
#pragma unroll
    for (int u = 0; u < NT2; ++u)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 b = b2[(u * 4 + g) * 2 + h];
        a2[u][4 * g + 0] = b.x; a2[u][4 * g + 1] = b.y; a2[u][4 * g + 2] = b.z; a2[u][4 * g + 3] = b.w;
      }
    const float4* w2 = reinterpret_cast<const float4*>(w + o_w2);
#pragma unroll
    for (int t = 0; t < NT1; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int u = 0; u < NT2; ++u) {
          const float4 a = w2[((u * NT1 + t) * 4 + g) * 64 + lane];
          a2[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, a1[t][4 * g + 0], a2[u], 0, 0, 0);
          a2[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, a1[t][4 * g + 1], a2[u], 0, 0, 0);
          a2[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, a1[t][4 * g + 2], a2[u], 0, 0, 0);
          a2[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, a1[t][4 * g + 3], a2[u], 0, 0, 0);
        }
    const float4* wo = reinterpret_cast<const float4*>(w + o_wo);
#pragma unroll
    for (int u = 0; u < NT2; ++u)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 o = wo[(u * 4 + g) * 2 + h];
        part = fmaf(o.x, sigmoid_prescaled(a2[u][4 * g + 0]), part);
        part = fmaf(o.y, sigmoid_prescaled(a2[u][4 * g + 1]), part);
        part = fmaf(o.z, sigmoid_prescaled(a2[u][4 * g + 2]), part);
        part = fmaf(o.w, sigmoid_prescaled(a2[u][4 * g + 3]), part);
      }
  } else {
    const float4* wo = reinterpret_cast<const float4*>(w + o_wo);
#pragma unroll
    for (int t = 0; t < NT1; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 o = wo[(t * 4 + g) * 2 + h];
        part = fmaf(o.x, a1[t][4 * g + 0], part);
        part = fmaf(o.y, a1[t][4 * g + 1], part);
        part = fmaf(o.z, a1[t][4 * g + 2], part);
        part = fmaf(o.w, a1[t][4 * g + 3], part);
      }
  }
  return part;
}

// Bitonic sort of a[0..n) ascending, n a power of two, by the whole workgroup.
__device__ void bitonic_sort(unsigned long long* a, uint32_t n, int tid) {
  for (uint32_t size = 2; size <= n; size <<= 1) {
    for (uint32_t j = size >> 1; j > 0; j >>= 1) {
      for (uint32_t t = tid; t < (n >> 1); t += kThreads) {
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
__device__ void sort_pool(unsigned long long* pool, uint32_t n2, unsigned long long* lds,
                          uint32_t lds_entries, int tid) {
  if (n2 <= lds_entries) {
    for (uint32_t x = tid; x < n2; x += kThreads) lds[x] = pool[x];
    __syncthreads();
    bitonic_sort(lds, n2, tid);
    for (uint32_t x = tid; x < n2; x += kThreads) pool[x] = lds[x];
    __syncthreads();
  } else {
    bitonic_sort(pool, n2, tid);
  }
}

__device__ __forceinline__ uint32_t next_pow2(uint32_t v) {
  uint32_t p = 1;
  while (p < v) p <<= 1;
  return p;
}

// ---------------------------------------------------------------------------
// The sweep.  Persistent workgroups pull chunks of kWaves * R tiles from a
// global queue.  LDS: [space tables][one stage of packed members].
// ---------------------------------------------------------------------------
template <int KS1, int NT1, int NT2, int R>
__global__ void __launch_bounds__(kThreads)
sweep_kernel(const SweepParams prm, const int o_w2, const int o_b2, const int o_wo) {
  extern __shared__ __align__(16) unsigned char smem[];
  DevSpace& sp = *reinterpret_cast<DevSpace*>(smem);
  float* wts = reinterpret_cast<float*>(smem + kSpaceBytes);
  __shared__ uint32_t s_chunk, s_cnt, s_compact;
  __shared__ unsigned long long s_tau, s_tau_local;

  constexpr int kIter = kWaves * R * 32;   // configurations per chunk
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, h = lane >> 5;
  unsigned long long* pool = prm.pools + (size_t)blockIdx.x * prm.cap;

  {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(prm.space);
    uint32_t* dst = reinterpret_cast<uint32_t*>(smem);
    for (int x = tid; x < (int)(sizeof(DevSpace) / 4); x += kThreads) dst[x] = src[x];
  }
  if (tid == 0) { s_cnt = 0; s_tau_local = kKeyMax; s_compact = 0; }
  auto load_stage = [&](int st) {
    const int first = st * prm.members_per_stage;
    int nm = prm.n_members - first;
    nm = nm < prm.members_per_stage ? nm : prm.members_per_stage;
    const float4* src = reinterpret_cast<const float4*>(prm.packed + (size_t)first * prm.member_floats);
    float4* dst = reinterpret_cast<float4*>(wts);
    const int n4 = nm * prm.member_floats / 4;
    for (int x = tid; x < n4; x += kThreads) dst[x] = src[x];
  };
  if (prm.n_stages == 1) load_stage(0);
  const float bo_sum = prm.hdr->bo_sum;
  // the weight stage doubles as sort scratch during pool compaction
  unsigned long long* lds_keys = reinterpret_cast<unsigned long long*>(wts);
  const uint32_t lds_entries = (uint32_t)prm.members_per_stage * (uint32_t)prm.member_floats / 2u;
  // thread 0 keeps one chunk index in flight so the queue's latency is hidden
  uint32_t next_chunk = 0;
  if (tid == 0) next_chunk = atomicAdd(&prm.hdr->work_counter, 1u);

  for (;;) {
    __syncthreads();
    if (tid == 0) {
      s_chunk = next_chunk;
      if (prm.mode == MODE_TOPK) {
        const unsigned long long g =
            __hip_atomic_load(&prm.hdr->tau, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_tau = g < s_tau_local ? g : s_tau_local;
        s_compact = (s_cnt + kIter > prm.cap) ? 1u : 0u;
      }
    }
    __syncthreads();
    const uint32_t chunk = s_chunk;
    if (chunk >= prm.n_chunks) break;
    if (tid == 0) next_chunk = atomicAdd(&prm.hdr->work_counter, 1u);

    if (prm.mode == MODE_TOPK && s_compact) {
      const uint32_t n = s_cnt;
      const uint32_t n2 = next_pow2(n);
      for (uint32_t x = n + tid; x < n2; x += kThreads) pool[x] = kKeyMax;
      __syncthreads();
      sort_pool(pool, n2, lds_keys, lds_entries, tid);
      if (prm.n_stages == 1 && n2 <= lds_entries) load_stage(0);   // scratch held the weights
      if (tid == 0) {
        if (n >= (uint32_t)prm.k) {
          const unsigned long long t = pool[prm.k - 1];
          s_tau_local = t;
          atomicMin(&prm.hdr->tau, t);
          if (t < s_tau) s_tau = t;
          s_cnt = prm.k;
        }
      }
      __syncthreads();
    }
    const unsigned long long tau = s_tau;

    // ---- decode, features, validity for this wave's R tiles
    float xb[R][KS1];
    float ysum[R];
    bool ok[R], any[R];
    uint32_t idx[R];
    uint64_t pos[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const uint64_t p0 = (uint64_t)chunk * kIter + (uint32_t)((wave * R + r) * 32 + c);
      const bool in_range = p0 < prm.count;
      pos[r] = p0;
      const uint32_t i = (uint32_t)(prm.begin + (in_range ? p0 : prm.count - 1));
      idx[r] = i;
      bool v = in_range;
      for (int cc = 0; cc < sp.n_constraints; ++cc) {
        int ps = rule_partial_sum(sp, cc, i, h, 2);
        ps += __shfl_xor(ps, 32);
        v = v && (ps <= sp.bound[cc]);
      }
      ok[r] = v;
      any[r] = __ballot(v) != 0ull;
      ysum[r] = 0.0f;
      if (any[r]) {
#pragma unroll
        for (int s = 0; s < KS1; ++s) {
          const int p = 2 * s + h;
          float f = 0.0f;
          if (p < sp.n_params) f = feature_of(sp, p, digit_of(sp, p, i));
          else if (p == sp.n_params) f = 1.0f;
          xb[r][s] = f;
        }
      } else {
#pragma unroll
        for (int s = 0; s < KS1; ++s) xb[r][s] = 0.0f;
      }
    }

    // ---- ensemble
    for (int st = 0; st < prm.n_stages; ++st) {
      if (prm.n_stages > 1) {
        __syncthreads();
        load_stage(st);
        __syncthreads();
      }
      const int first = st * prm.members_per_stage;
      int nm = prm.n_members - first;
      nm = nm < prm.members_per_stage ? nm : prm.members_per_stage;
      for (int m = 0; m < nm; ++m) {
        const float* w = wts + (size_t)m * prm.member_floats;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          if (any[r]) ysum[r] += member_forward<KS1, NT1, NT2>(w, xb[r], lane, o_w2, o_b2, o_wo);
        }
      }
    }

    // ---- mean, mask, output
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float y = ysum[r] + __shfl_xor(ysum[r], 32);
      y = (y + bo_sum) * prm.inv_members + 0.0f;
      if (prm.mode == MODE_ALL) {
        if (h == 0 && pos[r] < prm.count) {
          prm.pred[pos[r]] = ok[r] ? y : __builtin_inff();
          if (prm.mask) prm.mask[pos[r]] = ok[r] ? 1 : 0;
        }
      } else {
        const unsigned long long key = make_key(y, idx[r]);
        const bool pass = ok[r] && h == 0 && key < tau;
        const unsigned long long bal = __ballot(pass);
        if (bal) {
          uint32_t base = 0;
          if (lane == 0) base = atomicAdd(&s_cnt, (uint32_t)__popcll(bal));
          base = __shfl(base, 0);
          if (pass) pool[base + __popcll(bal & ((1ull << lane) - 1ull))] = key;
        }
      }
    }
  }

  if (prm.mode == MODE_TOPK) {
    // final: sorted list of at least kp entries (padded with the sentinel)
    __syncthreads();
    const uint32_t n = s_cnt;
    uint32_t n2 = next_pow2(n);
    n2 = n2 < prm.kp ? prm.kp : n2;
    for (uint32_t x = n + tid; x < n2; x += kThreads) pool[x] = kKeyMax;
    __syncthreads();
    sort_pool(pool, n2, lds_keys, lds_entries, tid);
  }
}

// ---------------------------------------------------------------------------
// Grid merge: lists of kp sorted keys, pairwise: the kp smallest of two sorted
// lists are min(A[i], B[kp-1-i]) (a bitonic sequence), then a bitonic merge.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads)
merge_kernel(unsigned long long* pools, uint32_t cap, unsigned long long* extra, uint32_t n_pool_lists,
             uint32_t kp, uint32_t half) {
  const int tid = threadIdx.x;
  const uint32_t ja = blockIdx.x, jb = blockIdx.x + half;
  unsigned long long* A = ja < n_pool_lists ? pools + (size_t)ja * cap : extra;
  const unsigned long long* B = jb < n_pool_lists ? pools + (size_t)jb * cap : extra;
  for (uint32_t i = tid; i < kp; i += kThreads) {
    const unsigned long long a = A[i], b = B[kp - 1 - i];
    A[i] = a < b ? a : b;
  }
  __syncthreads();
  for (uint32_t j = kp >> 1; j > 0; j >>= 1) {
    for (uint32_t t = tid; t < (kp >> 1); t += kThreads) {
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
                int32_t* n_found) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < k; i += gridDim.x * blockDim.x) {
    const unsigned long long key = list[i];
    const bool real = key != kKeyMax;
    values[i] = real ? unorder_bits((uint32_t)(key >> 32)) : __builtin_inff();
    indices[i] = real ? (uint32_t)key : 0xffffffffu;
    if (i == 0 && !real) *n_found = 0;
    if (real && (i == k - 1 || list[i + 1] == kKeyMax)) *n_found = i + 1;
  }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
static int round_up(int v, int m) { return (v + m - 1) / m * m; }

static int make_shape(const tuner_space* sp, const tuner_model* m, Shape* sh) {
  if (!m->widths || !m->weights_dev) return set_error(TUNER_EINVAL, "null model arrays");
  if (m->n_members < 1) return set_error(TUNER_EINVAL, "n_members < 1");
  if (m->n_layers != 2 && m->n_layers != 3) return set_error(TUNER_EINVAL, "n_layers must be 2 or 3");
  if (m->precision != TUNER_FP32) return set_error(TUNER_EINVAL, "precision not supported by this build");
  if (m->algo != TUNER_ALGO_AUTO && m->algo != TUNER_ALGO_MFMA)
    return set_error(TUNER_EINVAL, "algo not supported by this build");
  if (m->widths[0] != sp->n_params) return set_error(TUNER_EINVAL, "model input width != number of parameters");
  if (m->widths[m->n_layers] != 1) return set_error(TUNER_EINVAL, "model output width must be 1");
  sh->P = sp->n_params;
  sh->H1 = m->widths[1];
  sh->H2 = m->n_layers == 3 ? m->widths[2] : 0;
  sh->E = m->n_members;
  if (sh->H1 < 1 || (m->n_layers == 3 && sh->H2 < 1)) return set_error(TUNER_EINVAL, "hidden width < 1");
  if (sh->H1 > TUNER_MAX_WIDTH || sh->H2 > TUNER_MAX_WIDTH) return set_error(TUNER_ETOOLARGE, "hidden layer too wide");
  sh->KS1 = round_up(sh->P + 1, 8) / 2;       // steps of 2 inputs, multiple of 4
  auto tiles = [](int hgt) { const int t = (hgt + 31) / 32; return t == 3 ? 4 : t; };
  sh->NT1 = tiles(sh->H1);
  sh->NT2 = sh->H2 ? tiles(sh->H2) : 0;
  sh->o_w1 = 0;
  sh->o_w2 = sh->NT1 * sh->KS1 * 64;
  sh->o_b2 = sh->o_w2 + sh->NT2 * sh->NT1 * 16 * 64;
  sh->o_wo = sh->o_b2 + sh->NT2 * 32;
  sh->member_floats = sh->o_wo + (sh->NT2 ? sh->NT2 : sh->NT1) * 32;
  sh->raw_member_floats = sh->P * sh->H1 + sh->H1 + (sh->H2 ? sh->H1 * sh->H2 + sh->H2 + sh->H2 : sh->H1) + 1;
  return TUNER_OK;
}

struct Layout {
  size_t o_hdr, o_space, o_packed, o_pools, o_extra, total;
  uint32_t cap, kp;
};

static uint32_t host_next_pow2(uint32_t v) { uint32_t p = 1; while (p < v) p <<= 1; return p; }

constexpr int kMaxIter = kWaves * 2 * 32;   // largest chunk over the instantiated R

static Layout make_layout(const Shape& sh, int k) {
  Layout L{};
  auto al = [](size_t v) { return (v + 255) / 256 * 256; };
  L.o_hdr = 0;
  L.o_space = al(sizeof(WsHeader));
  L.o_packed = L.o_space + kSpaceBytes;
  L.o_pools = L.o_packed + al((size_t)sh.E * sh.member_floats * 4);
  L.kp = k > 0 ? host_next_pow2((uint32_t)k) : 0;
  L.cap = k > 0 ? 4u * (L.kp > (uint32_t)kMaxIter ? L.kp : (uint32_t)kMaxIter) : 0;
  L.o_extra = L.o_pools + (size_t)kMaxGroups * L.cap * 8;
  L.total = L.o_extra + al((size_t)L.kp * 8);
  return L;
}

typedef void (*SweepFn)(const SweepParams, const int, const int, const int);
struct Variant { int KS1, NT1, NT2, R; SweepFn fn; };

#define TUNER_VARIANT(KS1, NT1, NT2, R) {KS1, NT1, NT2, R, sweep_kernel<KS1, NT1, NT2, R>}
static const Variant kVariants[] = {
    TUNER_VARIANT(4, 1, 0, 2),  TUNER_VARIANT(8, 1, 0, 2),  TUNER_VARIANT(12, 1, 0, 2), TUNER_VARIANT(16, 1, 0, 2),
    TUNER_VARIANT(4, 2, 0, 2),  TUNER_VARIANT(8, 2, 0, 2),  TUNER_VARIANT(12, 2, 0, 2), TUNER_VARIANT(16, 2, 0, 2),
    TUNER_VARIANT(4, 4, 0, 2),  TUNER_VARIANT(8, 4, 0, 2),  TUNER_VARIANT(12, 4, 0, 2), TUNER_VARIANT(16, 4, 0, 2),
    TUNER_VARIANT(4, 1, 1, 2),  TUNER_VARIANT(8, 1, 1, 2),  TUNER_VARIANT(12, 1, 1, 2), TUNER_VARIANT(16, 1, 1, 2),
    TUNER_VARIANT(4, 2, 2, 2),  TUNER_VARIANT(8, 2, 2, 2),  TUNER_VARIANT(12, 2, 2, 2), TUNER_VARIANT(16, 2, 2, 2),
    TUNER_VARIANT(4, 4, 4, 1),  TUNER_VARIANT(8, 4, 4, 1),  TUNER_VARIANT(12, 4, 4, 1), TUNER_VARIANT(16, 4, 4, 1),
};

static const Variant* find_variant(Shape* sh) {
  // hidden layers of different tile counts run on the larger square variant
  if (sh->NT2 && sh->NT1 != sh->NT2) {
    const int nt = sh->NT1 > sh->NT2 ? sh->NT1 : sh->NT2;
    sh->NT1 = sh->NT2 = nt;
    sh->o_w2 = sh->NT1 * sh->KS1 * 64;
    sh->o_b2 = sh->o_w2 + sh->NT2 * sh->NT1 * 16 * 64;
    sh->o_wo = sh->o_b2 + sh->NT2 * 32;
    sh->member_floats = sh->o_wo + sh->NT2 * 32;
  }
  for (const Variant& v : kVariants)
    if (v.KS1 == sh->KS1 && v.NT1 == sh->NT1 && v.NT2 == sh->NT2) return &v;
  return nullptr;
}

// Optional timing of the sweep kernel alone (HIP events on the caller's stream).
struct ProfileState {
  bool on = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> events;
};
static ProfileState g_profile;

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

static int run_sweep(const tuner_space* sp, const tuner_model* m, uint64_t begin, uint64_t count,
                     int mode, int k, int merge, float* values, uint32_t* indices, int32_t* n_found,
                     float* pred, uint8_t* mask, void* ws, size_t ws_bytes, hipStream_t stream) {
  Shape sh{};
  int rc = make_shape(sp, m, &sh);
  if (rc) return rc;
  const Variant* var = find_variant(&sh);
  if (!var) return set_error(TUNER_ETOOLARGE, "no kernel variant for this model shape");
  if (begin > sp->n_configs || count > sp->n_configs - begin)
    return set_error(TUNER_EINVAL, "range outside the space");
  const Layout L = make_layout(sh, k);
  if (!ws || ws_bytes < L.total) return set_error(TUNER_EWORKSPACE, "workspace missing or too small");
  if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0) return set_error(TUNER_EWORKSPACE, "workspace not 256-byte aligned");
  DeviceInfo di;
  rc = device_info(&di);
  if (rc) return rc;

  unsigned char* base = static_cast<unsigned char*>(ws);
  WsHeader* hdr = reinterpret_cast<WsHeader*>(base + L.o_hdr);
  DevSpace* space_dev = reinterpret_cast<DevSpace*>(base + L.o_space);
  float* packed = reinterpret_cast<float*>(base + L.o_packed);
  unsigned long long* pools = reinterpret_cast<unsigned long long*>(base + L.o_pools);
  unsigned long long* extra = reinterpret_cast<unsigned long long*>(base + L.o_extra);

  PrepParams pp{};
  pp.sh = sh;
  pp.raw = m->weights_dev;
  pp.packed = packed;
  pp.space_out = space_dev;
  pp.hdr = hdr;
  pp.extra = mode == MODE_TOPK ? extra : nullptr;
  pp.kp = L.kp;
  pp.k = k;
  pp.merge = merge;
  pp.in_values = values;
  pp.in_indices = indices;
  pp.in_found = n_found;
  const uint32_t total_packed = (uint32_t)sh.E * sh.member_floats;
  const unsigned prep_blocks = std::min<unsigned>(1024, (total_packed + 255) / 256);
  hipLaunchKernelGGL(prep_kernel, dim3(prep_blocks), dim3(256), 0, stream, sp->dev, pp);
  TUNER_HIP_TRY(hipGetLastError());

  const int iter = kWaves * var->R * 32;
  const uint64_t n_chunks64 = (count + iter - 1) / iter;
  const uint32_t n_chunks = (uint32_t)n_chunks64;   // count <= 2^32, iter >= 512
  const int n_cu = di.n_cu > 0 ? di.n_cu : 1;
  uint32_t groups = (uint32_t)std::min<uint64_t>(n_chunks64, (uint64_t)std::min(n_cu, kMaxGroups));

  if (groups > 0) {
    const int budget = di.max_lds - kSpaceBytes - 64;   // 64 B of static LDS
    const int member_bytes = sh.member_floats * 4;
    int mps = budget / member_bytes;
    if (mps < 1) return set_error(TUNER_ETOOLARGE, "one packed member does not fit in LDS");
    mps = std::min(mps, sh.E);
    SweepParams sw{};
    sw.begin = begin;
    sw.count = count;
    sw.n_chunks = n_chunks;
    sw.n_members = sh.E;
    sw.members_per_stage = mps;
    sw.n_stages = (sh.E + mps - 1) / mps;
    sw.member_floats = sh.member_floats;
    sw.mode = mode;
    sw.inv_members = (float)(1.0 / (double)sh.E);
    sw.k = k;
    sw.cap = L.cap;
    sw.kp = L.kp;
    sw.space = space_dev;
    sw.packed = packed;
    sw.hdr = hdr;
    sw.pools = pools;
    sw.pred = pred;
    sw.mask = mask;
    const size_t lds = (size_t)kSpaceBytes + (size_t)mps * member_bytes;
    TUNER_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(var->fn),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (g_profile.on) {
      TUNER_HIP_TRY(hipEventCreate(&ev0));
      TUNER_HIP_TRY(hipEventCreate(&ev1));
      TUNER_HIP_TRY(hipEventRecord(ev0, stream));
    }
    hipLaunchKernelGGL(var->fn, dim3(groups), dim3(kThreads), lds, stream, sw, sh.o_w2, sh.o_b2, sh.o_wo);
    TUNER_HIP_TRY(hipGetLastError());
    if (g_profile.on) {
      TUNER_HIP_TRY(hipEventRecord(ev1, stream));
      g_profile.events.emplace_back(ev0, ev1);
    }
  }

  if (mode == MODE_TOPK) {
    // lists: pool 0..groups-1, then the running result
    uint32_t n = groups + 1;
    while (n > 1) {
      const uint32_t half = (n + 1) / 2;
      hipLaunchKernelGGL(merge_kernel, dim3(n - half), dim3(kThreads), 0, stream, pools, L.cap, extra,
                         groups, L.kp, half);
      TUNER_HIP_TRY(hipGetLastError());
      n = half;
    }
    const unsigned long long* list0 = groups > 0 ? pools : extra;
    hipLaunchKernelGGL(finalize_kernel, dim3((k + 255) / 256), dim3(256), 0, stream, list0, k, values,
                       indices, n_found);
    TUNER_HIP_TRY(hipGetLastError());
  }
  return TUNER_OK;
}

}  // namespace tuner

using tuner::set_error;

extern "C" {

size_t tuner_workspace_bytes(const tuner_space* space, const tuner_model* model, int32_t k) {
  if (!space || !model) { set_error(TUNER_EINVAL, "null argument"); return 0; }
  if (k < 0 || k > TUNER_MAX_K) { set_error(TUNER_ETOOLARGE, "k out of range"); return 0; }
  tuner::Shape sh{};
  if (tuner::make_shape(space, model, &sh)) return 0;
  if (!tuner::find_variant(&sh)) { set_error(TUNER_ETOOLARGE, "no kernel variant for this model shape"); return 0; }
  return tuner::make_layout(sh, k).total;
}

int tuner_profile_enable(int32_t on) {
  tuner::g_profile.on = on != 0;
  return TUNER_OK;
}

int tuner_profile_read(double* sweep_ms_total, int64_t* n_sweep_launches) {
  if (!sweep_ms_total || !n_sweep_launches) return set_error(TUNER_EINVAL, "null argument");
  double total = 0.0;
  int64_t n = 0;
  for (auto& ev : tuner::g_profile.events) {
    float ms = 0.0f;
    TUNER_HIP_TRY(hipEventSynchronize(ev.second));
    TUNER_HIP_TRY(hipEventElapsedTime(&ms, ev.first, ev.second));
    total += ms;
    ++n;
    hipEventDestroy(ev.first);
    hipEventDestroy(ev.second);
  }
  tuner::g_profile.events.clear();
  *sweep_ms_total = total;
  *n_sweep_launches = n;
  return TUNER_OK;
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

int tuner_predict_all(const tuner_space* space, const tuner_model* model, uint64_t index_begin,
                      uint64_t index_count, float* predictions_dev, uint8_t* valid_mask_dev,
                      void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!space || !model || !predictions_dev) return set_error(TUNER_EINVAL, "null argument");
  return tuner::run_sweep(space, model, index_begin, index_count, tuner::MODE_ALL, 0, 0, nullptr,
                          nullptr, nullptr, predictions_dev, valid_mask_dev, workspace_dev,
                          workspace_bytes, (hipStream_t)hip_stream);
}

}  // extern "C"
