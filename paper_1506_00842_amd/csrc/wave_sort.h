// Sorting and merging of 64-bit candidate keys in the registers of one wave (64 lanes), for
// the top-k selection of the sweep (paper, Section 5.3: the M configurations with the lowest
// predictions).  A wave holds 64 * E keys, element i = lane + 64 r in register r of its lane.
// Compare-exchange steps whose partners sit in different registers stay inside the lane; those
// between lanes (distance 1 .. 32) fetch the partner's key with data-parallel-primitive moves
// inside a row of 16 lanes and with the row/half swaps across rows: no LDS round trip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lane_ops.h"

namespace tuner {

// x[lane ^ J] for J = 1, 2, 4, 8, 16, 32.
template <int J>
__device__ __forceinline__ uint32_t xor_lane(uint32_t x, uint32_t lane) {
  static_assert(J == 1 || J == 2 || J == 4 || J == 8 || J == 16 || J == 32, "power of two below 64");
  const int v = (int)x;
  if constexpr (J == 1) {                      // quad_perm [1, 0, 3, 2]
    return (uint32_t)__builtin_amdgcn_update_dpp(v, v, 0xB1, 0xf, 0xf, false);
  } else if constexpr (J == 2) {               // quad_perm [2, 3, 0, 1]
    return (uint32_t)__builtin_amdgcn_update_dpp(v, v, 0x4E, 0xf, 0xf, false);
  } else if constexpr (J == 4) {
    // lanes 0-3 and 8-11 of a row read four lanes up (row_shl:4), the others four lanes down
    // (row_shr:4); the bank mask selects which groups of four lanes an instruction writes
    const int up = __builtin_amdgcn_update_dpp(v, v, 0x104, 0xf, 0x5, false);
    return (uint32_t)__builtin_amdgcn_update_dpp(up, v, 0x114, 0xf, 0xa, false);
  } else if constexpr (J == 8) {               // row_ror:8 (half a row: lane ^ 8)
    return (uint32_t)__builtin_amdgcn_update_dpp(v, v, 0x128, 0xf, 0xf, false);
  } else if constexpr (J == 16) {
    // swaps the odd rows of the first operand with the even rows of the second: afterwards the
    // first holds the even rows twice, the second the odd rows twice
    const auto r = __builtin_amdgcn_permlane16_swap(x, opaque_copy(x), false, false);
    return (lane & 16u) ? r[0] : r[1];
  } else {
    // swaps the upper half of the first operand with the lower half of the second
    const auto r = __builtin_amdgcn_permlane32_swap(x, opaque_copy(x), false, false);
    return (lane & 32u) ? r[0] : r[1];
  }
}

template <int J>
__device__ __forceinline__ unsigned long long xor_lane64(unsigned long long x, uint32_t lane) {
  const uint32_t lo = xor_lane<J>((uint32_t)x, lane), hi = xor_lane<J>((uint32_t)(x >> 32), lane);
  return ((unsigned long long)hi << 32) | lo;
}

// One compare-exchange step between lanes at distance J on every register: the lane with
// bit J clear keeps the smaller key when `ascending`, the larger one otherwise.  (Keys are
// distinct except for the padding key, so "not smaller" stands for "larger".)
template <int J, int E>
__device__ __forceinline__ void exchange_lanes(unsigned long long (&v)[E], uint32_t lane, bool ascending) {
  const bool keep_large = ((lane & (uint32_t)J) == 0u) != ascending;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const unsigned long long o = xor_lane64<J>(v[r], lane);
    const bool take = (o < v[r]) != keep_large;
    v[r] = take ? o : v[r];
  }
}

// The same step, ascending in every lane, for J = 16 or 32 on a pair of registers: one row
// (half) swap puts the two partners of every exchange into the same lane of the two
// registers, a second one puts the smaller and the larger key back where they belong.
template <int J>
__device__ __forceinline__ void swap_pair(uint32_t& a, uint32_t& b) {
  static_assert(J == 16 || J == 32, "row swap or half swap");
  if constexpr (J == 16) {
    const auto r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
    a = r[0]; b = r[1];
  } else {
    const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    a = r[0]; b = r[1];
  }
}
template <int J>
__device__ __forceinline__ void exchange_rows_pair(unsigned long long& x, unsigned long long& y) {
  uint32_t xl = (uint32_t)x, xh = (uint32_t)(x >> 32), yl = (uint32_t)y, yh = (uint32_t)(y >> 32);
  swap_pair<J>(xl, yl);
  swap_pair<J>(xh, yh);
  const unsigned long long p = ((unsigned long long)xh << 32) | xl, q = ((unsigned long long)yh << 32) | yl;
  const bool lt = p < q;
  const unsigned long long lo = lt ? p : q, hi = lt ? q : p;
  xl = (uint32_t)lo; xh = (uint32_t)(lo >> 32); yl = (uint32_t)hi; yh = (uint32_t)(hi >> 32);
  swap_pair<J>(xl, yl);
  swap_pair<J>(xh, yh);
  x = ((unsigned long long)xh << 32) | xl;
  y = ((unsigned long long)yh << 32) | yl;
}
template <int J, int E>
__device__ __forceinline__ void exchange_rows(unsigned long long (&v)[E], uint32_t lane) {
  if constexpr (E >= 2) {
#pragma unroll
    for (int r = 0; r < E; r += 2) exchange_rows_pair<J>(v[r], v[r + 1]);
  } else {
    exchange_lanes<J, E>(v, lane, true);
  }
}

// v holds a bitonic sequence of 64 * E keys -> sorted ascending.
template <int E>
__device__ __forceinline__ void bitonic_merge_regs(unsigned long long (&v)[E], uint32_t lane) {
#pragma unroll
  for (int jr = E / 2; jr > 0; jr >>= 1)
#pragma unroll
    for (int r = 0; r < E; ++r)
      if ((r & jr) == 0) {
        const unsigned long long x = v[r], y = v[r | jr];
        v[r] = x < y ? x : y;
        v[r | jr] = x < y ? y : x;
      }
  exchange_rows<32, E>(v, lane);
  exchange_rows<16, E>(v, lane);
  exchange_lanes<8, E>(v, lane, true);
  exchange_lanes<4, E>(v, lane, true);
  exchange_lanes<2, E>(v, lane, true);
  exchange_lanes<1, E>(v, lane, true);
}

// One wave merges two sorted lists of 64 * E keys in LDS (A, B) into the 64 * E smallest,
// sorted, in A: min(A[i], B[n - 1 - i]) is a bitonic sequence holding the n smallest of both.
template <int E>
__device__ __forceinline__ void wave_pair_merge(unsigned long long* A, const unsigned long long* B, uint32_t lane) {
  constexpr uint32_t n = 64u * E;
  unsigned long long v[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const uint32_t i = lane + 64u * r;
    const unsigned long long a = A[i], b = B[n - 1 - i];
    v[r] = a < b ? a : b;
  }
  bitonic_merge_regs<E>(v, lane);
#pragma unroll
  for (int r = 0; r < E; ++r) A[lane + 64u * r] = v[r];
}

// One wave merges two sorted lists of 32 * E keys each (A, then B) into one sorted list of
// 64 * E keys, written to `out` (which may be A when B follows A directly): A followed by B
// reversed is a bitonic sequence.
template <int E>
__device__ __forceinline__ void wave_full_merge(const unsigned long long* A, const unsigned long long* B,
                                                unsigned long long* out, uint32_t lane) {
  constexpr uint32_t half = 32u * E;
  unsigned long long v[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const uint32_t i = lane + 64u * r;
    v[r] = i < half ? A[i] : B[2u * half - 1u - i];
  }
  bitonic_merge_regs<E>(v, lane);
#pragma unroll
  for (int r = 0; r < E; ++r) out[lane + 64u * r] = v[r];
}

// One wave sorts 64 keys (one per lane) ascending.
__device__ __forceinline__ unsigned long long wave_sort64(unsigned long long key, uint32_t lane) {
  unsigned long long v[1] = {key};
  // blocks of 2, 4, ..., 32 alternate in direction so that the next size finds bitonic runs
  exchange_lanes<1, 1>(v, lane, (lane & 2u) == 0u);
  exchange_lanes<2, 1>(v, lane, (lane & 4u) == 0u);
  exchange_lanes<1, 1>(v, lane, (lane & 4u) == 0u);
  exchange_lanes<4, 1>(v, lane, (lane & 8u) == 0u);
  exchange_lanes<2, 1>(v, lane, (lane & 8u) == 0u);
  exchange_lanes<1, 1>(v, lane, (lane & 8u) == 0u);
  exchange_lanes<8, 1>(v, lane, (lane & 16u) == 0u);
  exchange_lanes<4, 1>(v, lane, (lane & 16u) == 0u);
  exchange_lanes<2, 1>(v, lane, (lane & 16u) == 0u);
  exchange_lanes<1, 1>(v, lane, (lane & 16u) == 0u);
  exchange_lanes<16, 1>(v, lane, (lane & 32u) == 0u);
  exchange_lanes<8, 1>(v, lane, (lane & 32u) == 0u);
  exchange_lanes<4, 1>(v, lane, (lane & 32u) == 0u);
  exchange_lanes<2, 1>(v, lane, (lane & 32u) == 0u);
  exchange_lanes<1, 1>(v, lane, (lane & 32u) == 0u);
  bitonic_merge_regs<1>(v, lane);
  return v[0];
}

// The whole workgroup leaves the `keep` smallest keys of a[0 .. n2) sorted at the front of a
// (LDS; n2 a power of two >= 64, unused entries hold the largest key; keep = 64, 128, 256 or
// 512, at most n2).  Every wave sorts runs of 64 keys in registers; then levels of pairwise
// merges, one wave per pair: two runs become one of twice the length until the runs are `keep`
// long, after that a pair leaves its `keep` smallest keys in its first run.  One workgroup
// barrier per level instead of one per step of a workgroup-wide sorting network.
constexpr uint32_t kSelectMaxKeep = 512;

__device__ inline void select_sorted(unsigned long long* a, uint32_t n2, uint32_t keep, int tid, int nthreads) {
  const uint32_t wave = (uint32_t)tid >> 6, lane = (uint32_t)tid & 63u, nwaves = (uint32_t)nthreads >> 6;
  uint32_t runs = n2 >> 6;
  for (uint32_t r = wave; r < runs; r += nwaves) a[r * 64 + lane] = wave_sort64(a[r * 64 + lane], lane);
  __syncthreads();
  uint32_t len = 64, stride = 64;                 // run length; distance between the starts of two runs
  while (runs > 1) {
    const uint32_t pairs = runs >> 1;
    const bool grow = 2 * len <= keep;
    for (uint32_t p = wave; p < pairs; p += nwaves) {
      unsigned long long* A = a + (size_t)(2 * p) * stride;
      unsigned long long* B = A + stride;
      if (grow) {                                 // stride == len here: B follows A directly
        if (len == 64) wave_full_merge<2>(A, B, A, lane);
        else if (len == 128) wave_full_merge<4>(A, B, A, lane);
        else wave_full_merge<8>(A, B, A, lane);
      } else {
        if (len == 64) wave_pair_merge<1>(A, B, lane);
        else if (len == 128) wave_pair_merge<2>(A, B, lane);
        else if (len == 256) wave_pair_merge<4>(A, B, lane);
        else wave_pair_merge<8>(A, B, lane);
      }
    }
    __syncthreads();
    if (grow) len <<= 1;
    stride <<= 1;
    runs = pairs;
  }
}

}  // namespace tuner
