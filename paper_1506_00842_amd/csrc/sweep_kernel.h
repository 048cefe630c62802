// The fused sweep kernel, parameterised by how the network is evaluated.
//
// Paper: Section 5.3 (predict every configuration, keep the M lowest), Section
// 5.2 (ensemble mean, statically invalid configurations), Section 5.1 (space).
//
// Persistent workgroups (NW waves) pull chunks of NW * R tiles (32 consecutive
// configurations each) from a global queue.  LDS: [space tables][one stage of
// packed members].  A Net policy supplies
//   static constexpr int kTile                    configurations per wave and tile: 32 (each
//                                                 configuration is shared by the lane pair
//                                                 (lane, lane ^ 32)) or 64 (one per lane)
//   struct Feat                                   per-tile network input registers
//   static void load_features(sp, index, lane, pow2, offsets, Feat&)
//   static void zero_features(Feat&)
//   static float forward(const uint32_t* member_lds, const Feat&, int lane, const NetOffsets&)
//        -> the lane's share of the member's output (both halves of a lane pair
//           (lane, lane ^ 32) are summed by the caller)
#pragma once
#include "lane_ops.h"
#include "sweep_common.h"
#include "wave_sort.h"

namespace tuner {

template <class Net, int R, int NW>
__global__ void __launch_bounds__(NW * 64) sweep_kernel(const SweepParams prm) {
  constexpr int kThreads = NW * 64;
  constexpr int kWaves = NW;
  extern __shared__ __align__(16) unsigned char smem[];
  DevSpace& sp = *reinterpret_cast<DevSpace*>(smem);
  uint32_t* wts = reinterpret_cast<uint32_t*>(smem + kSpaceBytes);
  __shared__ uint32_t s_chunk, s_cnt, s_compact;
  __shared__ unsigned long long s_tau, s_tau_local;

  constexpr int kTile = Net::kTile;
  // configurations per chunk: every wave takes r_used (<= R) tiles of it; small spaces
  // use fewer tiles per wave so that their chunks still cover every compute unit
  const int r_used = prm.r_used;
  const uint32_t kIter = (uint32_t)(kWaves * kTile) * (uint32_t)r_used;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave_u = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, known uniform
  const int c = kTile == 32 ? (lane & 31) : lane, h = kTile == 32 ? (lane >> 5) : 0;
  // candidate pool: in LDS behind the weights when there is room for 2 k + one queue
  // unit of keys (then no candidate ever travels to HBM and back, and a compaction
  // leaves the weights alone); otherwise in the workgroup's slice of the workspace
  // (two pointers and explicit branches: one pointer that may be either would make every
  // access a flat one)
  unsigned long long* gpool = prm.pools + (size_t)blockIdx.x * prm.cap;
  unsigned long long* lpool = reinterpret_cast<unsigned long long*>(smem + prm.lds_pool_offset);
  const bool pool_in_lds = prm.lds_pool_entries > 0;

  {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(prm.space);
    uint32_t* dst = reinterpret_cast<uint32_t*>(smem);
    for (int x = tid; x < (int)(sizeof(DevSpace) / 4); x += kThreads) dst[x] = src[x];
  }
  if (tid == 0) { s_cnt = 0; s_tau_local = kKeyMax; s_compact = 0; }
  if (prm.mode == MODE_TOPK) {
    // The running result of earlier calls becomes one more sorted key list for the merge
    // that follows this kernel (every workgroup converts a slice), and its k-th key, if it
    // has k entries, is an upper bound of the final k-th key from the start.
    int found = 0;
    if (prm.merge) {
      found = *prm.run_found;
      found = found < 0 ? 0 : (found > prm.k ? prm.k : found);
    }
    for (uint32_t x = blockIdx.x * kThreads + tid; x < prm.kp; x += gridDim.x * kThreads)
      prm.extra[x] = ((int)x < found) ? make_key(prm.run_values[x], prm.run_indices[x]) : kKeyMax;
    if (tid == 0 && found == prm.k && found > 0)
      s_tau_local = make_key(prm.run_values[prm.k - 1], prm.run_indices[prm.k - 1]);
  }
  auto load_stage = [&](int st) {
    const int first = st * prm.members_per_stage;
    int nm = prm.n_members - first;
    nm = nm < prm.members_per_stage ? nm : prm.members_per_stage;
    const uint4* src = reinterpret_cast<const uint4*>(prm.packed + (size_t)first * prm.member_words);
    uint4* dst = reinterpret_cast<uint4*>(wts);
    const int n4 = nm * prm.member_words / 4;
    for (int x = tid; x < n4; x += kThreads) dst[x] = src[x];
  };
  // The same copy without registers and without waiting: LDS-direct loads (every wave
  // moves 64 x 16 bytes per instruction; lane l's bytes land at the wave's base + 16 l).
  // Completion is the wave's vmcnt; the stage is visible to the workgroup after
  // s_waitcnt vmcnt(0) and a barrier.
  auto issue_stage = [&](int st, int buf) {
    const int first = st * prm.members_per_stage;
    int nm = prm.n_members - first;
    nm = nm < prm.members_per_stage ? nm : prm.members_per_stage;
    const uint4* src = reinterpret_cast<const uint4*>(prm.packed + (size_t)first * prm.member_words);
    uint4* dst = reinterpret_cast<uint4*>(wts + (size_t)buf * prm.stage_words);
    const int n4 = nm * prm.member_words / 4;
    for (int x = wave_u * 64; x < n4; x += kThreads) {
      if (x + lane < n4)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + x + lane),
                                         (__attribute__((address_space(3))) void*)(dst + x), 16, 0, 0);
    }
  };
  const bool double_buffer = prm.double_buffer != 0;
  // per-wave scratch of the hoisting network: the tiles' high features, then one z_high vector
  float* hoist_xs = nullptr;
  float* hoist_zs = nullptr;
  if constexpr (Net::kHoist) {
    hoist_xs = reinterpret_cast<float*>(smem + prm.hoist_offset) + (size_t)wave_u * (R * 32 + Net::kScratchZ);
    hoist_zs = hoist_xs + R * 32;
  }
  if (prm.n_stages == 1) load_stage(0);
  const float bo_sum = prm.hdr->bo_sum;
  const bool pow2 = prm.space->all_pow2 != 0;
  const int n_constraints = prm.space->n_constraints;
  // the weight stage doubles as sort scratch during pool compaction
  unsigned long long* lds_keys = reinterpret_cast<unsigned long long*>(wts);
  const uint32_t lds_entries = prm.lds_entries;
  // Queue unit = prm.super consecutive chunks.  Thread 0 keeps two unit indices in
  // flight so that the queue's latency is hidden even across runs of invalid units.
  const uint32_t super_iter = (uint32_t)prm.super * kIter;
  // pools are compacted while they still fit the LDS sort scratch, if that leaves room
  uint32_t eff_cap = prm.cap;
  if (pool_in_lds) {
    eff_cap = prm.lds_pool_entries;
  } else {
    uint32_t lds_pow2 = 1;
    while (lds_pow2 * 2 <= lds_entries) lds_pow2 *= 2;
    if (lds_pow2 < eff_cap && lds_pow2 >= 2u * prm.kp + super_iter) eff_cap = lds_pow2;
  }
  // The first unit of a workgroup is its own index.  Long ranges take further units
  // from the queue counter (units differ in cost); short ranges stride through the units
  // instead and touch no atomic at all (a thousand read-modify-writes of one word would
  // take longer than such a sweep).  Long constrained ranges come with a list of the
  // chunks to sweep, made by classify_kernel: runs of chunks without any valid
  // configuration would otherwise turn the queue counter into the bottleneck (every
  // workgroup claims such units as fast as the atomic unit serves them).
  // Leaves the smallest keys of the pool's n candidates sorted at its front: at least
  // max(kp, what the pool held) of them when everything was sorted, else the kp smallest,
  // followed by padding keys up to kp.  Lists of up to 512 keys (k <= 512) go through the
  // register-level selection (a barrier per merge level); longer ones through the
  // workgroup-wide sorting network.  A pool in the workspace is sorted in the LDS region of
  // the weights when it fits there (the resident ensemble is then loaded again).
  auto sort_candidates = [&](uint32_t n, bool sweep_goes_on) {
    uint32_t n2 = next_pow2(n);
    n2 = n2 < prm.kp ? prm.kp : n2;
    const uint32_t keep = prm.kp < 64u ? 64u : prm.kp;
    const bool select = prm.kp <= kSelectMaxKeep;
    const uint32_t m2 = (select && n2 < 64u) ? 64u : n2;       // the selection works on runs of 64 keys
    if (pool_in_lds) {
      for (uint32_t x = n + tid; x < m2; x += kThreads) lpool[x] = kKeyMax;
      __syncthreads();
      if (select && m2 <= prm.lds_pool_entries) select_sorted(lpool, m2, keep, tid, kThreads);
      else bitonic_sort(lpool, n2, tid, kThreads);
    } else if (select && m2 <= lds_entries) {
      for (uint32_t x = tid; x < m2; x += kThreads) lds_keys[x] = x < n ? gpool[x] : kKeyMax;
      __syncthreads();
      select_sorted(lds_keys, m2, keep, tid, kThreads);
      for (uint32_t x = tid; x < prm.kp; x += kThreads) gpool[x] = lds_keys[x];
      __syncthreads();
      if (sweep_goes_on && prm.n_stages == 1) load_stage(0);    // the scratch held the weights
    } else {
      for (uint32_t x = n + tid; x < n2; x += kThreads) gpool[x] = kKeyMax;
      __syncthreads();
      sort_pool(gpool, n2, lds_keys, lds_entries, tid, kThreads);
      if (sweep_goes_on && prm.n_stages == 1 && n2 <= lds_entries) load_stage(0);   // scratch held the weights
    }
  };
  const bool dynamic = prm.dynamic != 0;
  const uint32_t n_chunks = prm.live ? prm.hdr->n_live : prm.n_chunks;
  const uint32_t n_units = prm.live ? (n_chunks + (uint32_t)prm.super - 1u) / (uint32_t)prm.super : prm.n_units;
  uint32_t next0 = 0, next1 = 0;
  if (tid == 0) {
    next0 = blockIdx.x;
    next1 = dynamic ? gridDim.x + atomicAdd(&prm.hdr->work_counter, 1u) : blockIdx.x + gridDim.x;
  }

  for (;;) {
    __syncthreads();
    if (tid == 0) {
      s_chunk = next0;
      if (prm.mode == MODE_TOPK) {
        const unsigned long long g =
            __hip_atomic_load(&prm.hdr->tau, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_tau = g < s_tau_local ? g : s_tau_local;
        s_compact = (s_cnt + super_iter > eff_cap) ? 1u : 0u;
      }
    }
    __syncthreads();
    const uint32_t unit = __builtin_amdgcn_readfirstlane(s_chunk);
    if (unit >= n_units) break;
    if (tid == 0) {
      next0 = next1;
      next1 = dynamic ? gridDim.x + atomicAdd(&prm.hdr->work_counter, 1u) : next1 + gridDim.x;
    }

    if (prm.mode == MODE_TOPK && s_compact) {
      // pool nearly full: keep its k smallest keys, lower the thresholds
      const uint32_t n = s_cnt;
      sort_candidates(n, true);
      if (tid == 0) {
        if (n >= (uint32_t)prm.k) {
          const unsigned long long t = pool_in_lds ? lpool[prm.k - 1] : gpool[prm.k - 1];
          if (t < s_tau_local) s_tau_local = t;
          // (the returned value is used, so the atomic has completed before this workgroup
          // reports itself done at the end of the kernel)
          const unsigned long long before = atomicMin(&prm.hdr->tau, t);
          if (t < s_tau) s_tau = t;
          if (before < s_tau) s_tau = before;
          s_cnt = prm.k;
        }
      }
      __syncthreads();
    }
    const unsigned long long tau = s_tau;

    // chunks of this unit; with two stage buffers the first stage's weights start
    // their way into LDS now and every later stage while its predecessor is evaluated
    const uint32_t n_sub = min((uint32_t)prm.super, n_chunks - unit * (uint32_t)prm.super);
    uint32_t stage_seq = 0;
    if (double_buffer) issue_stage(0, 0);
    for (uint32_t sub = 0; sub < n_sub; ++sub) {
    const uint32_t slot = unit * (uint32_t)prm.super + sub;
    const uint32_t entry = prm.live ? prm.live[slot] : (slot | ((uint32_t)CHUNK_MIXED << 30));
    const uint32_t chunk = entry & 0x3fffffffu;
    const uint32_t state = __builtin_amdgcn_readfirstlane(entry >> 30);

    // ---- validity, then digits -> features, for this wave's R tiles
    typename Net::Feat feat[R];
    float ysum[R];
    bool ok[R], any[R];
    uint32_t idx[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      // uniform: tile start inside the range, and how many of its configurations exist
      const uint64_t t0 = (uint64_t)chunk * kIter + (uint32_t)((wave_u * r_used + r) * kTile);
      const uint32_t left =
          (r < r_used && t0 < prm.count) ? (uint32_t)min((uint64_t)kTile, prm.count - t0) : 0u;
      uint32_t i = (uint32_t)(prm.begin + t0) + (uint32_t)c;   // any 32-bit index decodes safely
      if (prm.index_list) i = (uint32_t)c < left ? prm.index_list[t0 + (uint32_t)c] : 0u;
      idx[r] = i;
      bool v = (uint32_t)c < left && t0 + (uint32_t)c >= prm.head;
      if (state == CHUNK_MIXED) {
        for (int cc = 0; cc < n_constraints; ++cc) {
          int ps;
          if constexpr (kTile == 32) {
            ps = pair_sum(rule_partial_sum(sp, cc, i, h, 2, pow2));   // the lane pair splits the entries
          } else {
            ps = rule_partial_sum(sp, cc, i, 0, 1, pow2);
          }
          v = v && (ps <= sp.bound[cc]);
        }
      } else {
        v = v && state == CHUNK_ALL_VALID;
      }
      ok[r] = v;
      any[r] = __ballot(v) != 0ull;
      ysum[r] = 0.0f;
      if (any[r]) {
        Net::load_features(sp, i, lane, pow2, prm.off, feat[r]);
        if constexpr (Net::kHoist) Net::load_high(sp, i, lane, pow2, prm.off, hoist_xs + r * 32);
      } else {
        Net::zero_features(feat[r]);
      }
    }

    // ---- ensemble
    for (int st = 0; st < prm.n_stages; ++st) {
      const uint32_t* stage = wts;
      if (double_buffer) {
        // stage st has landed in its buffer, and every wave has left the other buffer
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        const int buf = (int)(stage_seq & 1u);
        ++stage_seq;
        if (st + 1 < prm.n_stages) issue_stage(st + 1, buf ^ 1);
        else if (sub + 1 < n_sub) issue_stage(0, buf ^ 1);
        stage = wts + (size_t)buf * prm.stage_words;
      } else if (prm.n_stages > 1) {
        __syncthreads();
        load_stage(st);
        __syncthreads();
      }
      const int first = st * prm.members_per_stage;
      int nm = prm.n_members - first;
      nm = nm < prm.members_per_stage ? nm : prm.members_per_stage;
      for (int m = 0; m < nm; ++m) {
        const uint32_t* w = stage + (size_t)m * prm.member_words;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          if (any[r]) {
            if constexpr (Net::kHoist) ysum[r] += Net::forward(w, feat[r], lane, prm.off, hoist_xs + r * 32, hoist_zs);
            else ysum[r] += Net::forward(w, feat[r], lane, prm.off);
          }
        }
      }
    }

    // ---- mean, mask, output
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float y = ysum[r];
      if constexpr (kTile == 32) y = pair_sum(y);
      y = (y + bo_sum) * prm.inv_members + 0.0f;
      if (prm.mode == MODE_ALL) {
        const uint64_t t0 = (uint64_t)chunk * kIter + (uint32_t)((wave_u * r_used + r) * kTile);
        const uint32_t left =
            (r < r_used && t0 < prm.count) ? (uint32_t)min((uint64_t)kTile, prm.count - t0) : 0u;
        if (h == 0 && (uint32_t)c < left && t0 + (uint32_t)c >= prm.head) {
          prm.pred[t0 + (uint32_t)c] = ok[r] ? y : __builtin_inff();
          if (prm.mask) prm.mask[t0 + (uint32_t)c] = ok[r] ? 1 : 0;
        }
      } else {
        const unsigned long long key = make_key(y, idx[r]);
        const bool pass = ok[r] && h == 0 && key < tau;
        const unsigned long long bal = __ballot(pass);
        if (bal) {
          uint32_t base = 0;
          if (lane == 0) base = atomicAdd(&s_cnt, (uint32_t)__popcll(bal));
          base = __shfl(base, 0);
          if (pass) {
            const uint32_t at = base + __popcll(bal & ((1ull << lane) - 1ull));
            if (pool_in_lds) lpool[at] = key;
            else gpool[at] = key;
          }
        }
      }
    }
    }  // sub
  }

  if (prm.mode == MODE_TOPK) {
    // final: sorted list of at least kp entries (padded with the sentinel)
    __syncthreads();
    const uint32_t n = s_cnt;
    sort_candidates(n, false);
    if (pool_in_lds)
      for (uint32_t x = tid; x < prm.kp; x += kThreads) gpool[x] = lpool[x];
  }
  // A call on a prepared workspace has no kernel that resets the header before it.  Top-k
  // calls leave that to their last merge launch; a sweep that is the last kernel of its call
  // does it here: the last workgroup to finish restores the idle state (every other
  // workgroup's accesses to these words have completed: their results were consumed before
  // the increment below).
  if (prm.self_reset && tid == 0) {
    const uint32_t finished = atomicAdd(&prm.hdr->done, 1u);
    if (finished == gridDim.x - 1) {
      prm.hdr->work_counter = 0u;
      prm.hdr->n_live = 0u;
      prm.hdr->tau = kKeyMax;
      prm.hdr->done = 0u;
    }
  }
}

}  // namespace tuner
