// Exact selection of nearest points on one wave: 64-bit keys (fp32 squared distance bits, index) compared
// as integers, a bitonic sort network on DPP lane patterns and the gfx950 row / half swaps, and a running
// top-64.  Distances are evaluated without fused multiply-add: every translation unit that includes this
// header is compiled with -ffp-contract=off.
#pragma once

#include "device_util.h"

namespace affmae {

typedef unsigned long long key_t;
constexpr key_t kKeyMax = ~0ull;

// fp32 squared distance, each operation rounded separately.
__device__ __forceinline__ float dist2(float ax, float ay, float bx, float by) {
#pragma clang fp contract(off)
  float dx = ax - bx;
  float dy = ay - by;
  float xx = dx * dx;
  float yy = dy * dy;
  return xx + yy;
}

__device__ __forceinline__ key_t make_key(float d2, int idx) {
  return ((key_t)__float_as_uint(d2) << 32) | (key_t)(uint32_t)idx;
}

__device__ __forceinline__ key_t shfl_key(key_t k, int src) {
  uint32_t lo = (uint32_t)k, hi = (uint32_t)(k >> 32);
  lo = __shfl(lo, src);
  hi = __shfl(hi, src);
  return ((key_t)hi << 32) | lo;
}

// The key held by lane (lane ^ J), J a power of two, moved on the VALU: DPP lane
// patterns inside a row of 16 lanes, the gfx950 row / half swaps across rows.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t x) {
  // every pattern used here reads an existing lane, so no value is needed for lanes without a source: leaving it
  // undefined saves the instruction that would otherwise set it before every move
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, CTRL, 0xf, 0xf, true);
}
template <int J>
__device__ __forceinline__ uint32_t lane_xor_u32(uint32_t x, int lane) {
  typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
  if constexpr (J == 1) {
    return dpp_mov<0xB1>(x);  // quad_perm [1,0,3,2]
  } else if constexpr (J == 2) {
    return dpp_mov<0x4E>(x);  // quad_perm [2,3,0,1]
  } else if constexpr (J == 4) {
    return dpp_mov<0x1B>(dpp_mov<0x141>(x));  // reverse 8 lanes, then reverse each quad: i -> i ^ 7 ^ 3
  } else if constexpr (J == 8) {
    return dpp_mov<0x128>(x);  // rotate the row by 8
  } else if constexpr (J == 16) {
    const u32x2 t = __builtin_amdgcn_permlane16_swap(x, x, false, false);  // [0]: even rows doubled, [1]: odd rows
    return (lane & 16) ? t[0] : t[1];
  } else {
    const u32x2 t = __builtin_amdgcn_permlane32_swap(x, x, false, false);  // [0]: low half doubled, [1]: high half
    return (lane & 32) ? t[0] : t[1];
  }
}
template <int J>
__device__ __forceinline__ key_t lane_xor_key(key_t k, int lane) {
  const uint32_t lo = lane_xor_u32<J>((uint32_t)k, lane);
  const uint32_t hi = lane_xor_u32<J>((uint32_t)(k >> 32), lane);
  return ((key_t)hi << 32) | lo;
}

// One compare-exchange step of a bitonic network: partner lane ^ J; the lane keeps
// the smaller key when keep_min.
template <int J>
__device__ __forceinline__ key_t exchange(key_t key, int lane, bool keep_min) {
  const key_t other = lane_xor_key<J>(key, lane);
  return ((key < other) == keep_min) ? key : other;
}
template <int K2, int J>
__device__ __forceinline__ key_t sort_stage(key_t key, int lane) {
  // blocks of K2 lanes alternate ascending / descending; within a block the lower lane of a pair keeps the minimum
  key = exchange<J>(key, lane, ((lane & K2) == 0) == ((lane & J) == 0));
  if constexpr (J > 1) key = sort_stage<K2, J / 2>(key, lane);
  return key;
}

// Sort one key per lane ascending across the 64 lanes of the wave.
__device__ __forceinline__ key_t wave_sort(key_t key, int lane) {
  key = sort_stage<2, 1>(key, lane);
  key = sort_stage<4, 2>(key, lane);
  key = sort_stage<8, 4>(key, lane);
  key = sort_stage<16, 8>(key, lane);
  key = sort_stage<32, 16>(key, lane);
  key = sort_stage<64, 32>(key, lane);  // lane & 64 == 0 everywhere: ascending
  return key;
}

// Input: bitonic across lanes.  Output: ascending across lanes.
__device__ __forceinline__ key_t wave_bitonic_merge(key_t key, int lane) {
  return sort_stage<64, 32>(key, lane);
}

// Keeps the 64 smallest keys seen so far, ascending across lanes.  `row` holds 64
// new keys in any order; `kth` is the lane whose key bounds what can still enter
// the first `kth+1` places.
__device__ __forceinline__ key_t topk_push(key_t best, key_t row, int lane, int kth) {
  key_t bound = shfl_key(best, kth);
  if (__ballot(row < bound) == 0ull) return best;  // wave-uniform: nothing can enter
  row = wave_sort(row, lane);
  key_t rev = shfl_key(row, kWave - 1 - lane);
  best = best < rev ? best : rev;  // the 64 smallest of both, bitonic
  return wave_bitonic_merge(best, lane);
}

// The K nearest of up to 64 * ROWS candidates held one per lane and row: d2[row] = bit pattern of the lane's
// squared distance (ordered like the value, since d2 >= +0; all ones where the lane has no candidate), id[row] =
// its index (all ones likewise).  Returns the keys ascending across the lanes (the first K are the answer).
//
// The wave looks for a distance threshold T with K <= #{d2 <= T} <= 64 by counting with ballots: it starts from
// `guess` (the threshold that worked for the previous, nearby query; 0 = none), scales it by wanted / found (the
// count grows like the area, i.e. like d2), then bisects on the bit pattern.  Everything at or below T is nearer
// than everything above it, so the K nearest are among the counted candidates: they are compacted into one row
// (through `pend`, 128 keys of LDS owned by the wave) and sorted once.  When no such T exists (more than
// 64 - K + 1 candidates at one distance) the first row is sorted and later candidates that beat the current K-th
// key are queued and merged 64 at a time.  Either way the result is exact.
template <int ROWS>
__device__ __forceinline__ key_t select_nearest(const uint32_t (&d2)[ROWS], const uint32_t (&id)[ROWS], int K,
                                                uint32_t& guess, key_t* pend, int lane) {
  const uint32_t kInfBits = 0x7f800000u;
  auto count_le = [&](uint32_t t) -> int {
    int n = 0;
#pragma unroll
    for (int row = 0; row < ROWS; ++row) n += __popcll(__ballot(d2[row] <= t));
    return n;
  };
  // invariant: count(lo) < K (lo = -1: nothing known), count(hi) > 64 or hi = +inf bits
  long long lo = -1, hi = (long long)kInfBits;
  uint32_t t = guess;
  if (t == 0u) {  // first token of the wave: the farthest of the first 64 candidates, so the count is not 0
    t = min(d2[0], kInfBits);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) t = max(t, (uint32_t)__shfl_xor((int)t, o));
    t = __builtin_amdgcn_readfirstlane(t);
  }
  bool found = false;
  for (int it = 0; it < 48; ++it) {
    const int n = count_le(t);
    if (n >= K && n <= kWave) { found = true; break; }
    if (n < K) lo = t; else hi = t;
    if (hi - lo <= 1) break;  // neighbouring bit patterns straddle the window
    long long next = -1;
    if (it < 4 && n > 0) {
      const float scaled = __uint_as_float(t) * ((float)(K + kWave) * 0.5f / (float)n);
      next = (long long)__float_as_uint(scaled);
    }
    if (next <= lo || next >= hi) next = lo + (hi - lo) / 2;
    t = (uint32_t)next;
  }
  key_t best;
  if (found) {
    guess = t;
    int fill = 0;
#pragma unroll
    for (int row = 0; row < ROWS; ++row) {
      const bool in = d2[row] <= t;
      const unsigned long long mask = __ballot(in);
      const int rank =
          __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
      if (in) pend[fill + rank] = ((key_t)d2[row] << 32) | id[row];
      fill += __popcll(mask);
    }
    wave_lds_sync();
    best = wave_sort((lane < fill) ? pend[lane] : kKeyMax, lane);
    wave_lds_sync();
  } else {
    best = wave_sort(((key_t)d2[0] << 32) | id[0], lane);
    key_t bound = shfl_key(best, K - 1);
    int fill = 0;
#pragma unroll
    for (int row = 1; row < ROWS; ++row) {
      const key_t key = ((key_t)d2[row] << 32) | id[row];
      const bool in = key < bound;
      const unsigned long long mask = __ballot(in);
      if (mask != 0ull) {
        const int rank =
            __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        if (in) pend[fill + rank] = key;
        fill += __popcll(mask);
        if (fill >= kWave) {
          wave_lds_sync();
          const key_t full = pend[lane];
          const key_t rest = pend[kWave + lane];
          wave_lds_sync();
          fill -= kWave;
          if (lane < fill) pend[lane] = rest;
          best = topk_push(best, full, lane, K - 1);
          bound = shfl_key(best, K - 1);
        }
      }
    }
    if (fill > 0) {
      wave_lds_sync();
      best = topk_push(best, (lane < fill) ? pend[lane] : kKeyMax, lane, K - 1);
    }
    wave_lds_sync();
  }
  return best;
}

}  // namespace affmae
