// The stages of the tuner around the sweep, for gfx950: random choice of valid
// training configurations, training of the bagged ensemble, the accuracy
// metric and the second-stage pick.
//
// Paper: Section 5.2 (random training configurations, one sigmoid hidden layer,
// bagging with k networks each trained on all parts but one, logarithm of the
// execution time as target, mean squared error, invalid configurations
// ignored), Section 4.2 (training starts from random weights and adjusts them),
// Section 5.3 third paragraph (best of the M measured candidates), Section 6
// (mean relative error on configurations not used for training).
#include <cstdio>
#include <cstring>

#include <algorithm>

#include "lane_ops.h"
#include "tuner_internal.h"

namespace tuner {

// ---------------------------------------------------------------------------
// Sampler
// ---------------------------------------------------------------------------
constexpr unsigned long long kEmptySlot = ~0ull;

__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t counter) {
  uint64_t z = seed + (counter + 1ull) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// draw c -> configuration index floor(z_c * N / 2^64); N <= 2^32
__device__ __forceinline__ uint32_t draw_index(uint64_t seed, uint64_t c, uint64_t n_configs) {
  return (uint32_t)__umul64hi(splitmix64_at(seed, c), n_configs);
}

__device__ __forceinline__ uint32_t slot_of(uint32_t index, uint32_t log_slots) {
  return (index * 2654435761u) >> (32u - log_slots);
}

__global__ void __launch_bounds__(256) sample_clear_kernel(unsigned long long* table, uint32_t n_slots) {
  for (uint32_t x = blockIdx.x * blockDim.x + threadIdx.x; x < n_slots; x += gridDim.x * blockDim.x)
    table[x] = kEmptySlot;
}

// Open-addressing table keyed by configuration index; a slot holds
// (index << 32 | lowest draw number that produced it).  Only valid draws enter.
__global__ void __launch_bounds__(256)
sample_insert_kernel(const DevSpace sp, uint64_t seed, uint64_t n_configs, uint32_t max_draws,
                     unsigned long long* table, uint32_t log_slots) {
  const bool pow2 = sp.all_pow2 != 0;
  const uint32_t mask = (1u << log_slots) - 1u;
  for (uint32_t c = blockIdx.x * blockDim.x + threadIdx.x; c < max_draws; c += gridDim.x * blockDim.x) {
    const uint32_t index = draw_index(seed, c, n_configs);
    if (!is_valid(sp, index, pow2)) continue;
    const unsigned long long key = ((unsigned long long)index << 32) | c;
    uint32_t slot = slot_of(index, log_slots);
    for (uint32_t probe = 0; probe <= mask; ++probe) {        // the table has 2x more slots than draws
      unsigned long long cur = __hip_atomic_load(&table[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (cur == kEmptySlot) {
        cur = atomicCAS(&table[slot], kEmptySlot, key);
        if (cur == kEmptySlot) break;                         // claimed
      }
      if ((uint32_t)(cur >> 32) == index) {                   // the slot belongs to this index
        atomicMin(&table[slot], key);
        break;
      }
      slot = (slot + 1u) & mask;
    }
  }
}

// One workgroup: draw c is kept iff it is the first draw of its (valid) index; kept
// draws are written in draw order until n_samples are out.
__global__ void __launch_bounds__(1024)
sample_compact_kernel(uint64_t seed, uint64_t n_configs, uint32_t max_draws, const unsigned long long* table,
                      uint32_t log_slots, uint32_t n_samples, uint32_t* __restrict__ out,
                      int32_t* __restrict__ n_found) {
  __shared__ uint32_t s_count[1024];
  const uint32_t tid = threadIdx.x;
  const uint32_t mask = (1u << log_slots) - 1u;
  const uint32_t per = (max_draws + 1023u) / 1024u;
  const uint32_t c0 = tid * per, c1 = min(max_draws, c0 + per);
  auto kept = [&](uint32_t c) -> bool {
    const uint32_t index = draw_index(seed, c, n_configs);
    uint32_t slot = slot_of(index, log_slots);
    for (uint32_t probe = 0; probe <= mask; ++probe) {
      const unsigned long long cur = table[slot];
      if (cur == kEmptySlot) return false;                    // an invalid draw: never inserted
      if ((uint32_t)(cur >> 32) == index) return (uint32_t)cur == c;
      slot = (slot + 1u) & mask;
    }
    return false;
  };
  uint32_t mine = 0;
  for (uint32_t c = c0; c < c1; ++c) mine += kept(c) ? 1u : 0u;
  s_count[tid] = mine;
  __syncthreads();
  // inclusive scan of the 1024 counts
  for (uint32_t d = 1; d < 1024; d <<= 1) {
    const uint32_t v = tid >= d ? s_count[tid - d] : 0u;
    __syncthreads();
    s_count[tid] += v;
    __syncthreads();
  }
  const uint32_t total = s_count[1023];
  uint32_t pos = s_count[tid] - mine;
  for (uint32_t c = c0; c < c1 && pos < n_samples; ++c)
    if (kept(c)) out[pos++] = draw_index(seed, c, n_configs);
  const uint32_t found = total < n_samples ? total : n_samples;
  for (uint32_t x = found + tid; x < n_samples; x += 1024) out[x] = 0xffffffffu;
  if (tid == 0) *n_found = (int32_t)found;
}

// ---------------------------------------------------------------------------
// Training
// ---------------------------------------------------------------------------
constexpr int kPartSkip = -0x7fffffff;       // record's part id for a sample nobody trains on
constexpr float kNegLog2eT = -1.44269504088896340736f;
constexpr int kMaxTrainGroups = 256;         // workgroups of one launch that exchange partial sums
constexpr int kMaxSplit = 16;                // workgroups per network
constexpr uint32_t kSpinLimit = 1u << 22;    // polls of the per-epoch barrier before a run gives up

__device__ __forceinline__ bool usable_time(float t) { return t > 0.0f && t < __builtin_inff(); }

// Workspace header: one arrival flag per workgroup (the number of epochs it has
// finished, in a 64-byte line of its own) for the per-epoch barrier among a network's
// workgroups, and the give-up flag.  Cleared by train_prep_kernel before every run.
struct TrainHeader {
  uint32_t arrived[kMaxTrainGroups][16];
  uint32_t abort;
  uint32_t pad[63];
};

// records[s] = { x_0 .. x_{P-1}, 0.., ln t, part }: RS floats (RS = round_up(P, 4) + 4,
// target at RS - 2, part id (int bits) at RS - 1)
__global__ void __launch_bounds__(256)
train_prep_kernel(const DevSpace sp, uint32_t n, const uint32_t* __restrict__ indices,
                  const float* __restrict__ times, const int32_t* __restrict__ parts, int rs,
                  float* __restrict__ records, TrainHeader* __restrict__ hdr) {
  if (blockIdx.x == 0) {
    for (int x = threadIdx.x; x < kMaxTrainGroups; x += blockDim.x) hdr->arrived[x][0] = 0u;
    if (threadIdx.x == 0) hdr->abort = 0u;
  }
  const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= n) return;
  const bool pow2 = sp.all_pow2 != 0;
  const uint32_t i = indices[s];
  float* r = records + (size_t)s * rs;
  for (int p = 0; p < rs - 2; ++p) r[p] = p < sp.n_params ? feature_at(sp, p, i, pow2) : 0.0f;
  const float t = times[s];
  const bool ok = usable_time(t) && is_valid(sp, i, pow2);
  r[rs - 2] = ok ? logf(t) : 0.0f;
  r[rs - 1] = __int_as_float(ok ? parts[s] : kPartSkip);
}

struct TrainParams {
  int32_t P, H, E;
  int32_t rs;                   // floats per record
  uint32_t n;                   // samples
  int32_t epochs;
  float eta, mu;
  int32_t split;                // workgroups per network (each takes a contiguous slice of the samples)
  uint32_t slice;               // samples per slice
  int32_t rec_in_lds;           // the slice's records are staged in LDS once
  const float* records;
  const float* w_in;
  float* w_out;
  float* loss;                  // optional [E][epochs + 1]
  TrainHeader* hdr;
  float* partials;              // [2][E * split][NQ]
  uint32_t poll_limit;
};

// split workgroups per network; workgroup (e, g) works on the samples of slice g.  A
// lane stands for one hidden unit (lane % GROUP) of one of the 64 / GROUP samples a
// wave works on at a time; the slice's samples are dealt to the waves round robin.
// Per sample the only cross-lane step is the sum of the units' contributions to the
// output; every gradient entry is accumulated over the samples in the registers of
// the lane that owns the unit.  Per epoch the partial sums of the waves are added
// through LDS, those of the network's workgroups through global memory (one barrier
// among them per epoch), always in the same order, and every workgroup applies the
// same update to its own copy of the weights: a run is reproducible bit for bit.
// The barrier is a bounded spin: if the workgroups of a network are not all running
// within the poll limit the run gives up and returns NaN weights and losses.
template <int PMAX, int GROUP, int THREADS>
__global__ void __launch_bounds__(THREADS) train_kernel(const TrainParams tp) {
  constexpr int kWaves = THREADS / 64;
  constexpr int G = 64 / GROUP;             // samples per wave and step
  constexpr int NA = PMAX + 3;              // accumulator slots per unit: W1 row, b1, w_o, (b_o | loss)
  constexpr int NQ = GROUP * NA;            // gradient entries (padded units and inputs included)
  constexpr int KQ = (NQ + THREADS - 1) / THREADS;   // entries owned by a thread
  constexpr int NV = PMAX / 4 + 1;          // 16-byte words of a record
  extern __shared__ __align__(16) float smem[];
  float* s_w = smem;                        // current weights, [GROUP][NA] (slot PMAX+2 of unit 0 = b_o)
  float* s_red = smem + NQ;                 // [kWaves / 2][NQ] partial sums
  const float4* s_rec = reinterpret_cast<const float4*>(smem + NQ + (kWaves / 2) * NQ);
  __shared__ uint32_t s_ne[kWaves];
  __shared__ uint32_t s_abort;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane % GROUP, g = lane / GROUP;
  const int split = tp.split;
  const int e = blockIdx.x / split, part_g = blockIdx.x % split;
  const int P = tp.P, H = tp.H, rs = tp.rs;
  const int per = H * P + 2 * H + 1;
  const float* w_raw = tp.w_in + (size_t)e * per;
  const uint32_t s_begin = min(tp.n, (uint32_t)part_g * tp.slice);
  const uint32_t s_count = min(tp.n - s_begin, tp.slice);
  const bool rec_in_lds = tp.rec_in_lds != 0;
  if (tid == 0) s_abort = 0u;

  if (rec_in_lds) {
    float4* dst = reinterpret_cast<float4*>(smem + NQ + (kWaves / 2) * NQ);
    const float4* src = reinterpret_cast<const float4*>(tp.records + (size_t)s_begin * rs);
    const uint32_t n4 = s_count * (uint32_t)(rs / 4);
    for (uint32_t x = tid; x < n4; x += THREADS) dst[x] = src[x];
  }

  // thread owns the gradient entries q = tid + k * THREADS (unit q / NA, slot q % NA) and,
  // where an entry is a real weight, that weight and its momentum
  int raw[KQ];                              // position in the caller's layout, -1: none, -2: the loss slot
  float w_own[KQ], v_own[KQ];
#pragma unroll
  for (int k = 0; k < KQ; ++k) {
    const int q = tid + k * THREADS;
    const int uq = q / NA, aq = q % NA;
    raw[k] = -1;
    if (q < NQ) {
      if (uq < H) {
        if (aq < P) raw[k] = uq * P + aq;
        else if (aq == PMAX) raw[k] = H * P + uq;
        else if (aq == PMAX + 1) raw[k] = H * P + H + uq;
        else if (aq == PMAX + 2 && uq == 0) raw[k] = H * P + 2 * H;
      }
      if (uq == 1 && aq == PMAX + 2) raw[k] = -2;
    }
    w_own[k] = raw[k] >= 0 ? w_raw[raw[k]] : 0.0f;
    v_own[k] = 0.0f;
    if (q < NQ) s_w[q] = w_own[k];
  }

  // number of training samples of this network (over all slices)
  uint32_t cnt = 0;
  for (uint32_t s = tid; s < tp.n; s += THREADS) {
    const int part = __float_as_int(tp.records[(size_t)s * rs + rs - 1]);
    cnt += (part != kPartSkip && part != e) ? 1u : 0u;
  }
  for (int d = 32; d > 0; d >>= 1) cnt += __shfl_xor(cnt, d);
  if (lane == 0) s_ne[wave] = cnt;
  __syncthreads();
  uint32_t n_e = 0;
  for (int x = 0; x < kWaves; ++x) n_e += s_ne[x];
  const float inv_ne = n_e ? 1.0f / (float)n_e : 0.0f;

  const uint32_t n_steps = (s_count + G - 1) / G;
  bool aborted = false;
  for (int ep = 0; ep <= tp.epochs; ++ep) {
    __syncthreads();
    // this lane's unit: W1 row (pre-scaled for the exp2-based sigmoid), b1, w_o; b_o
    float w1s[PMAX], acc[PMAX];
#pragma unroll
    for (int p = 0; p < PMAX; ++p) { w1s[p] = s_w[j * NA + p] * kNegLog2eT; acc[p] = 0.0f; }
    const float b1s = s_w[j * NA + PMAX] * kNegLog2eT;
    const float wo = s_w[j * NA + PMAX + 1];
    const float bo = s_w[PMAX + 2];
    float g_b1 = 0.0f, g_wo = 0.0f, g_bo = 0.0f, sq = 0.0f;

    auto load_record = [&](uint32_t step, float4* dst) {
      const uint32_t s = step * G + g;        // within the slice
      if (step < n_steps && s < s_count) {
        if (rec_in_lds) {
          const float4* src = s_rec + (size_t)s * NV;
#pragma unroll
          for (int x = 0; x < NV; ++x) dst[x] = src[x];
        } else {
          const float4* src = reinterpret_cast<const float4*>(tp.records + (size_t)(s_begin + s) * rs);
#pragma unroll
          for (int x = 0; x < NV; ++x) dst[x] = src[x];
        }
      } else {
#pragma unroll
        for (int x = 0; x < NV - 1; ++x) dst[x] = make_float4(0.f, 0.f, 0.f, 0.f);
        dst[NV - 1] = make_float4(0.f, 0.f, 0.f, __int_as_float(kPartSkip));
      }
    };
    auto one_sample = [&](const float4* rec) {
      float x[PMAX];
#pragma unroll
      for (int v = 0; v < PMAX / 4; ++v) {
        x[4 * v + 0] = rec[v].x; x[4 * v + 1] = rec[v].y; x[4 * v + 2] = rec[v].z; x[4 * v + 3] = rec[v].w;
      }
      const float target = rec[NV - 1].z;
      const int part = __float_as_int(rec[NV - 1].w);
      const bool active = part != kPartSkip && part != e;
      // forward
      float z = b1s;
#pragma unroll
      for (int p = 0; p < PMAX; ++p) z = fmaf(w1s[p], x[p], z);
      const float h = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z));
      const float y = bo + group_sum<GROUP>(wo * h);
      // backward
      const float err = active ? y - target : 0.0f;
      sq = fmaf(err, err, sq);
      g_bo += err;
      g_wo = fmaf(err, h, g_wo);
      const float dz = (err * wo) * (h - h * h);
      g_b1 += dz;
#pragma unroll
      for (int p = 0; p < PMAX; ++p) acc[p] = fmaf(dz, x[p], acc[p]);
    };
    // two records in flight per wave, alternating registers
    float4 rec_a[NV], rec_b[NV];
    load_record(wave, rec_a);
    for (uint32_t step = wave; step < n_steps; step += 2 * kWaves) {
      load_record(step + kWaves, rec_b);
      one_sample(rec_a);
      load_record(step + 2 * kWaves, rec_a);
      one_sample(rec_b);                      // past the end: an inactive all-zero record
    }

    // the wave's G groups first (lane pairs 32 apart), then the waves through LDS
    if constexpr (G == 2) {
#pragma unroll
      for (int p = 0; p < PMAX; ++p) acc[p] = pair_sum(acc[p]);
      g_b1 = pair_sum(g_b1); g_wo = pair_sum(g_wo); g_bo = pair_sum(g_bo); sq = pair_sum(sq);
    }
    float tail = j == 0 ? g_bo : (j == 1 ? sq : 0.0f);
    auto put = [&](float* dst) {
#pragma unroll
      for (int p = 0; p < PMAX; ++p) dst[j * NA + p] = acc[p];
      dst[j * NA + PMAX] = g_b1; dst[j * NA + PMAX + 1] = g_wo; dst[j * NA + PMAX + 2] = tail;
    };
    if (wave >= kWaves / 2 && g == 0) put(s_red + (wave - kWaves / 2) * NQ);
    __syncthreads();
    if (wave < kWaves / 2 && g == 0) {
      const float* src = s_red + wave * NQ;
#pragma unroll
      for (int p = 0; p < PMAX; ++p) acc[p] += src[j * NA + p];
      g_b1 += src[j * NA + PMAX]; g_wo += src[j * NA + PMAX + 1]; tail += src[j * NA + PMAX + 2];
    }
    __syncthreads();
    if (wave < kWaves / 2 && g == 0) put(s_red + wave * NQ);
    __syncthreads();

    // sums of this workgroup, by owner
    float sum[KQ];
#pragma unroll
    for (int k = 0; k < KQ; ++k) {
      const int q = tid + k * THREADS;
      sum[k] = 0.0f;
      if (q >= NQ || raw[k] == -1) continue;
#pragma unroll
      for (int x = 0; x < kWaves / 2; ++x) sum[k] += s_red[x * NQ + q];
    }
    if (split > 1) {
      // exchange among the network's workgroups: write, arrive, wait for all, read all
      float* mine = tp.partials + ((size_t)(ep & 1) * tp.E * split + blockIdx.x) * NQ;
#pragma unroll
      for (int k = 0; k < KQ; ++k) {
        const int q = tid + k * THREADS;
        if (q < NQ && raw[k] != -1) __hip_atomic_store(&mine[q], sum[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      // The partial sums and the flags travel as agent-scope atomic stores and loads
      // (performed at the device's coherence point, past the per-XCD L2), so no cache
      // write-back or invalidate is needed: L2-wide fences cost ~0.35 us per workgroup and
      // epoch here and serialise.  Ordering: a wave's stores are complete (vmcnt = 0, which
      // the barrier waits for) before lane 0 raises the flag, and the partial sums are
      // loaded only after the barrier that follows the poll.
      __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wave's stores have been performed
      __syncthreads();
      if (wave == 0) {
        // arrive: this workgroup's flag <- epochs finished (a plain store of its own line:
        // no read-modify-write on a shared word); wait: lane x polls the flag of the
        // network's workgroup x
        if (lane == 0)
          __hip_atomic_store(&tp.hdr->arrived[blockIdx.x][0], (uint32_t)(ep + 1), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t* flag = &tp.hdr->arrived[e * split + (lane < split ? lane : 0)][0];
        uint32_t polls = 0;
        bool ok = true;
        for (;;) {
          const bool here = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= (uint32_t)(ep + 1);
          if (__all(here)) break;
          if (++polls > tp.poll_limit ||
              __hip_atomic_load(&tp.hdr->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
            ok = false;
            break;
          }
          __builtin_amdgcn_s_sleep(2);
        }
        if (!ok && lane == 0) {
          __hip_atomic_store(&tp.hdr->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          s_abort = 1u;
        }
      }
      __syncthreads();
      if (s_abort) { aborted = true; break; }
      const float* all = tp.partials + (size_t)(ep & 1) * tp.E * split * NQ + (size_t)e * split * NQ;
#pragma unroll
      for (int k = 0; k < KQ; ++k) {
        const int q = tid + k * THREADS;
        if (q >= NQ || raw[k] == -1) continue;
        // all loads first (one memory latency, not `split` of them), then the adds in order
        float v[kMaxSplit];
#pragma unroll
        for (int x = 0; x < kMaxSplit; ++x)
          v[x] = x < split ? __hip_atomic_load(&all[(size_t)x * NQ + q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0f;
        float total = v[0];
#pragma unroll
        for (int x = 1; x < kMaxSplit; ++x) total += v[x];
        sum[k] = total;
      }
    }
#pragma unroll
    for (int k = 0; k < KQ; ++k) {
      const int q = tid + k * THREADS;
      if (q >= NQ || raw[k] == -1) continue;
      if (raw[k] == -2) {                                   // sum of squared errors
        if (tp.loss && part_g == 0) tp.loss[(size_t)e * (tp.epochs + 1) + ep] = sum[k] * inv_ne;
      } else if (ep < tp.epochs && n_e > 0) {
        const float grad = 2.0f * inv_ne * sum[k];
        v_own[k] = tp.mu * v_own[k] - tp.eta * grad;
        w_own[k] += v_own[k];
        s_w[q] = w_own[k];
      }
    }
  }
  if (part_g != 0) return;
  const float nan = __builtin_nanf("");
#pragma unroll
  for (int k = 0; k < KQ; ++k)
    if (raw[k] >= 0) tp.w_out[(size_t)e * per + raw[k]] = aborted ? nan : w_own[k];
  if (aborted && tp.loss)
    for (int x = tid; x <= tp.epochs; x += THREADS) tp.loss[(size_t)e * (tp.epochs + 1) + x] = nan;
}

typedef void (*TrainFn)(const TrainParams);
struct TrainVariant { int pmax, group, threads; TrainFn fn; };
// wide inputs need more registers per lane: half the waves
#define TUNER_TRAIN(PMAX, T) {PMAX, 32, T, train_kernel<PMAX, 32, T>}, {PMAX, 64, T, train_kernel<PMAX, 64, T>}
static const TrainVariant kTrainVariants[] = {
    TUNER_TRAIN(4, 1024), TUNER_TRAIN(8, 1024), TUNER_TRAIN(12, 1024), TUNER_TRAIN(16, 1024),
    TUNER_TRAIN(20, 512), TUNER_TRAIN(24, 512), TUNER_TRAIN(28, 512), TUNER_TRAIN(32, 512),
};

// ---------------------------------------------------------------------------
// Metrics
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
mean_relative_error_kernel(uint64_t n, const float* __restrict__ pred, const float* __restrict__ times,
                           float* __restrict__ mean_out, int32_t* __restrict__ n_used) {
  __shared__ float s_sum[1024];
  __shared__ uint32_t s_cnt[1024];
  const uint32_t tid = threadIdx.x;
  float sum = 0.0f;
  uint32_t cnt = 0;
  for (uint64_t i = tid; i < n; i += 1024) {
    const float y = pred[i], t = times[i];
    if (usable_time(t) && fabsf(y) < __builtin_inff()) {
      sum += fabsf(expf(y) - t) / t;
      ++cnt;
    }
  }
  s_sum[tid] = sum;
  s_cnt[tid] = cnt;
  __syncthreads();
  for (uint32_t d = 512; d > 0; d >>= 1) {
    if (tid < d) { s_sum[tid] += s_sum[tid + d]; s_cnt[tid] += s_cnt[tid + d]; }
    __syncthreads();
  }
  if (tid == 0) {
    *mean_out = s_cnt[0] ? s_sum[0] / (float)s_cnt[0] : 0.0f;
    *n_used = (int32_t)s_cnt[0];
  }
}

__global__ void __launch_bounds__(1024)
best_of_kernel(uint64_t m, const float* __restrict__ times, int32_t* __restrict__ best_pos,
               float* __restrict__ best_time) {
  __shared__ unsigned long long s_key[1024];
  const uint32_t tid = threadIdx.x;
  unsigned long long best = ~0ull;                 // (time bits << 32 | position); positive floats order as integers
  for (uint64_t i = tid; i < m; i += 1024) {
    const float t = times[i];
    if (usable_time(t)) {
      const unsigned long long key = ((unsigned long long)__float_as_uint(t) << 32) | (uint32_t)i;
      best = key < best ? key : best;
    }
  }
  s_key[tid] = best;
  __syncthreads();
  for (uint32_t d = 512; d > 0; d >>= 1) {
    if (tid < d) s_key[tid] = s_key[tid] < s_key[tid + d] ? s_key[tid] : s_key[tid + d];
    __syncthreads();
  }
  if (tid == 0) {
    const unsigned long long k = s_key[0];
    *best_pos = k == ~0ull ? -1 : (int32_t)(uint32_t)k;
    *best_time = k == ~0ull ? __builtin_inff() : __uint_as_float((uint32_t)(k >> 32));
  }
}

static uint32_t log2_ceil_u64(uint64_t v) { uint32_t l = 0; while ((1ull << l) < v) ++l; return l; }

}  // namespace tuner

using tuner::set_error;

extern "C" {

size_t tuner_sample_workspace_bytes(uint64_t max_draws) {
  if (max_draws < 1 || max_draws > (1ull << 24)) { set_error(TUNER_ETOOLARGE, "max_draws out of range"); return 0; }
  const uint32_t log_slots = tuner::log2_ceil_u64(2 * max_draws) < 4 ? 4 : tuner::log2_ceil_u64(2 * max_draws);
  return ((size_t)8 << log_slots);
}

int tuner_sample_valid(const tuner_space* space, uint64_t seed, uint32_t n_samples, uint64_t max_draws,
                       uint32_t* indices_dev, int32_t* n_found_dev, void* workspace_dev,
                       size_t workspace_bytes, void* hip_stream) {
  if (!space || !indices_dev || !n_found_dev) return set_error(TUNER_EINVAL, "null argument");
  if (n_samples < 1) return set_error(TUNER_EINVAL, "n_samples must be >= 1");
  if (max_draws < n_samples) return set_error(TUNER_EINVAL, "max_draws < n_samples");
  if (max_draws > (1ull << 24)) return set_error(TUNER_ETOOLARGE, "max_draws > 2^24");
  const size_t need = tuner_sample_workspace_bytes(max_draws);
  if (!workspace_dev || workspace_bytes < need) return set_error(TUNER_EWORKSPACE, "workspace missing or too small");
  if ((reinterpret_cast<uintptr_t>(workspace_dev) & 255) != 0) return set_error(TUNER_EWORKSPACE, "workspace not 256-byte aligned");
  hipStream_t stream = (hipStream_t)hip_stream;
  const uint32_t log_slots = tuner::log2_ceil_u64(need / 8);
  const uint32_t n_slots = 1u << log_slots;
  unsigned long long* table = static_cast<unsigned long long*>(workspace_dev);
  const uint32_t md = (uint32_t)max_draws;
  hipLaunchKernelGGL(tuner::sample_clear_kernel, dim3(std::min<uint32_t>(1024, (n_slots + 255) / 256)), dim3(256), 0,
                     stream, table, n_slots);
  TUNER_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(tuner::sample_insert_kernel, dim3(std::min<uint32_t>(1024, (md + 255) / 256)), dim3(256), 0,
                     stream, space->dev, seed, space->n_configs, md, table, log_slots);
  TUNER_HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(tuner::sample_compact_kernel, dim3(1), dim3(1024), 0, stream, seed, space->n_configs, md,
                     table, log_slots, n_samples, indices_dev, n_found_dev);
  TUNER_HIP_TRY(hipGetLastError());
  return TUNER_OK;
}

static int train_record_floats(const tuner_space* space) { return (space->n_params + 3) / 4 * 4 + 4; }

// Workspace: [records n x RS floats][TrainHeader][partial sums 2 x kMaxTrainGroups x NQ floats]
struct TrainLayout { size_t o_hdr, o_partials, total; int nq_max; };
static TrainLayout train_layout(const tuner_space* space, uint64_t n_samples) {
  TrainLayout L{};
  const int rs = train_record_floats(space);
  const size_t rec = ((size_t)n_samples * rs * 4 + 255) / 256 * 256;
  L.nq_max = 64 * (rs - 4 + 3);
  L.o_hdr = rec;
  L.o_partials = L.o_hdr + sizeof(tuner::TrainHeader);
  L.total = L.o_partials + (size_t)2 * tuner::kMaxTrainGroups * L.nq_max * 4;
  return L;
}

size_t tuner_train_workspace_bytes(const tuner_space* space, uint64_t n_samples) {
  if (!space) { set_error(TUNER_EINVAL, "null space"); return 0; }
  if (n_samples > (1ull << 24)) { set_error(TUNER_ETOOLARGE, "n_samples > 2^24"); return 0; }
  return train_layout(space, n_samples).total;
}

int tuner_train_ensemble(const tuner_space* space, int32_t n_members, int32_t hidden, uint64_t n_samples,
                         const uint32_t* sample_indices_dev, const float* sample_times_dev,
                         const int32_t* sample_parts_dev, const float* initial_weights_dev,
                         const tuner_train_options* options, float* weights_out_dev,
                         float* loss_history_dev, void* workspace_dev, size_t workspace_bytes,
                         void* hip_stream) {
  if (!space || !initial_weights_dev || !options || !weights_out_dev)
    return set_error(TUNER_EINVAL, "null argument");
  if (n_samples > 0 && (!sample_indices_dev || !sample_times_dev || !sample_parts_dev))
    return set_error(TUNER_EINVAL, "null sample arrays");
  if (n_members < 1) return set_error(TUNER_EINVAL, "n_members < 1");
  if (n_members > 65535) return set_error(TUNER_ETOOLARGE, "n_members > 65535");
  if (hidden < 1) return set_error(TUNER_EINVAL, "hidden < 1");
  if (hidden > 64) return set_error(TUNER_ETOOLARGE, "hidden > 64");
  if (options->epochs < 0) return set_error(TUNER_EINVAL, "epochs < 0");
  if (options->workgroups_per_network < 0 || options->workgroups_per_network > tuner::kMaxSplit)
    return set_error(TUNER_EINVAL, "workgroups_per_network outside 0..16");
  if (options->barrier_poll_limit < 0) return set_error(TUNER_EINVAL, "barrier_poll_limit < 0");
  if (!(options->learning_rate == options->learning_rate) || !(options->momentum == options->momentum))
    return set_error(TUNER_EINVAL, "learning rate or momentum is not a number");
  if (n_samples > (1ull << 24)) return set_error(TUNER_ETOOLARGE, "n_samples > 2^24");
  const TrainLayout L = train_layout(space, n_samples);
  if (!workspace_dev || workspace_bytes < L.total) return set_error(TUNER_EWORKSPACE, "workspace missing or too small");
  if ((reinterpret_cast<uintptr_t>(workspace_dev) & 255) != 0) return set_error(TUNER_EWORKSPACE, "workspace not 256-byte aligned");
  hipStream_t stream = (hipStream_t)hip_stream;
  const int rs = train_record_floats(space);
  char* ws = static_cast<char*>(workspace_dev);
  float* records = reinterpret_cast<float*>(ws);
  tuner::TrainHeader* hdr = reinterpret_cast<tuner::TrainHeader*>(ws + L.o_hdr);
  const uint32_t n = (uint32_t)n_samples;

  const int pmax = rs - 4, group = hidden <= 32 ? 32 : 64;
  const tuner::TrainVariant* var = nullptr;
  for (const auto& v : tuner::kTrainVariants)
    if (v.pmax == pmax && v.group == group) var = &v;
  if (!var) return set_error(TUNER_ETOOLARGE, "no training kernel for this many parameters");

  int dev = 0, n_cu = 0, max_lds = 0;
  TUNER_HIP_TRY(hipGetDevice(&dev));
  TUNER_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  TUNER_HIP_TRY(hipDeviceGetAttribute(&max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
  // Workgroups per network: all workgroups of the launch must run at the same time (they
  // meet at a barrier every epoch), so the launch stays within 3/4 of the compute units;
  // a slice has at least 4 steps of work for every wave.
  const int waves = var->threads / 64, per_step = 64 / group;
  int split = std::min(tuner::kMaxSplit, std::max(1, (n_cu * 3 / 4) / n_members));
  split = std::min<int>(split, std::max<uint32_t>(1u, n / (uint32_t)(4 * waves * per_step)));
  if (options->workgroups_per_network > 0) split = options->workgroups_per_network;
  if ((long long)n_members * split > tuner::kMaxTrainGroups) split = 1;
  uint32_t slice = (n + split - 1) / split;
  slice = (slice + per_step - 1) / per_step * per_step;
  if (slice == 0) slice = per_step;

  hipLaunchKernelGGL(tuner::train_prep_kernel, dim3(std::max(1u, (n + 255) / 256)), dim3(256), 0, stream,
                     space->dev, n, sample_indices_dev, sample_times_dev, sample_parts_dev, rs, records, hdr);
  TUNER_HIP_TRY(hipGetLastError());

  const int nq = group * (pmax + 3);
  const size_t lds_fixed = (size_t)(1 + var->threads / 128) * nq * 4;
  const size_t lds_rec = (size_t)slice * rs * 4;
  const size_t lds_budget = std::min<size_t>((size_t)max_lds, 96u << 10) - 64;   // the kernel's static LDS
  const bool rec_in_lds = lds_fixed + lds_rec <= lds_budget;
  const size_t lds = lds_fixed + (rec_in_lds ? lds_rec : 0);

  tuner::TrainParams tp{};
  tp.P = space->n_params;
  tp.H = hidden;
  tp.E = n_members;
  tp.rs = rs;
  tp.n = n;
  tp.epochs = options->epochs;
  tp.eta = options->learning_rate;
  tp.mu = options->momentum;
  tp.split = split;
  tp.slice = slice;
  tp.rec_in_lds = rec_in_lds ? 1 : 0;
  tp.records = records;
  tp.w_in = initial_weights_dev;
  tp.w_out = weights_out_dev;
  tp.loss = loss_history_dev;
  tp.hdr = hdr;
  tp.partials = reinterpret_cast<float*>(ws + L.o_partials);
  tp.poll_limit = options->barrier_poll_limit > 0 ? (uint32_t)options->barrier_poll_limit : tuner::kSpinLimit;
  {
    const int rc = tuner::allow_dynamic_lds(reinterpret_cast<const void*>(var->fn), (int)lds);
    if (rc) return rc;
  }
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  if (tuner::profile_on()) {
    TUNER_HIP_TRY(hipEventCreate(&ev0));
    TUNER_HIP_TRY(hipEventCreate(&ev1));
    TUNER_HIP_TRY(hipEventRecord(ev0, stream));
  }
  hipLaunchKernelGGL(var->fn, dim3(n_members * split), dim3(var->threads), lds, stream, tp);
  TUNER_HIP_TRY(hipGetLastError());
  if (tuner::profile_on()) {
    TUNER_HIP_TRY(hipEventRecord(ev1, stream));
    tuner::profile_add(tuner::PROFILE_TRAIN, ev0, ev1);
  }
  return TUNER_OK;
}

int tuner_mean_relative_error(uint64_t n, const float* predictions_dev, const float* times_dev,
                              float* mean_error_dev, int32_t* n_used_dev, void* hip_stream) {
  if (!mean_error_dev || !n_used_dev || (n > 0 && (!predictions_dev || !times_dev)))
    return set_error(TUNER_EINVAL, "null argument");
  if (n > (1ull << 31)) return set_error(TUNER_ETOOLARGE, "n > 2^31");
  hipLaunchKernelGGL(tuner::mean_relative_error_kernel, dim3(1), dim3(1024), 0, (hipStream_t)hip_stream, n,
                     predictions_dev, times_dev, mean_error_dev, n_used_dev);
  TUNER_HIP_TRY(hipGetLastError());
  return TUNER_OK;
}

int tuner_best_of(uint64_t m, const float* times_dev, int32_t* best_pos_dev, float* best_time_dev,
                  void* hip_stream) {
  if (!best_pos_dev || !best_time_dev || (m > 0 && !times_dev)) return set_error(TUNER_EINVAL, "null argument");
  if (m > (1ull << 31)) return set_error(TUNER_ETOOLARGE, "m > 2^31");
  hipLaunchKernelGGL(tuner::best_of_kernel, dim3(1), dim3(1024), 0, (hipStream_t)hip_stream, m, times_dev,
                     best_pos_dev, best_time_dev);
  TUNER_HIP_TRY(hipGetLastError());
  return TUNER_OK;
}

}  // extern "C"
