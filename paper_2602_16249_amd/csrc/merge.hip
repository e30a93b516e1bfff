// Neighbourhood merging (paper, Sec. "AutoFocusFormer", the paragraph on downsampling: an importance score per
// token, the top-ranked tokens kept as anchors, the remaining tokens merged into nearby anchors through a
// differentiable, location-aware aggregation; the paper leaves the operator itself to the AFF paper).  What this
// file computes:
//   select  : the n_keep tokens of every image with the largest score, equal scores going to the lower index,
//             listed in ascending token index.  One workgroup per image finds, on the order-preserving bit pattern
//             of the scores, the score of the last kept token and how many tokens of exactly that score are kept
//             (up to 32768 tokens per image: keys in registers, the pattern built bit by bit from counts; larger
//             images: a radix select, four 8-bit digits, histograms in LDS); then, in index order, the larger
//             scores and the first so many of the equal ones are kept, their places given by block-wide prefix counts.
//   forward : one wave per anchor.  Lane j holds neighbour j of the anchor's row of the stage's neighbour table:
//             distance to the anchor, z_j = score_j - p dist_j, w = softmax_j(z) by wave reductions.  The weighted
//             sum of the feature rows moves 16 bytes per lane: a row takes PP lanes, 64 / PP rows are in flight per
//             trip, and the row groups are added up with lane shuffles at the end.
//   backward: the same wave forms g_j = <dout_anchor, feat_j> (partial dot per lane, reduced inside a row's
//             lanes), dz_j = w_j (d_j - sum_i w_i d_i) with d_i = g_i - g_ref relative to the neighbour of largest
//             weight (differences first: the form does not cancel when one weight saturates), its part of dp
//             (distances relative to the nearest neighbour's, for the same reason), and keeps w, dz and the token of every (anchor, neighbour) pair.  dfeat and dscore are then
//             gathered, not scattered: the pairs are filed per token (the list builder of the virtual-token
//             backward) and every token adds up w * dout, respectively dz, over its own list.
#include <algorithm>

#include "device_util.h"
#include "launch.h"
#include "timing.h"

namespace affmae {
namespace {

inline unsigned round_up8(long long blocks) { return (unsigned)((blocks + 7) / 8 * 8); }
__device__ __forceinline__ long long xcd_contiguous_block() {
  // workgroups are dealt round-robin to the 8 XCDs (one L2 each): consecutive anchors share rows, so every XCD
  // gets a contiguous range; the grid is a multiple of 8
  const unsigned per_xcd = gridDim.x >> 3;
  return (long long)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
}

// Order-preserving 32-bit pattern of a finite score: a larger score has a larger pattern; -0 and +0 share one.
__device__ __forceinline__ uint32_t score_key(float s) {
  const uint32_t u = (s == 0.f) ? 0u : __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;

// Number of earlier threads of the workgroup whose flag is set, and the total (two barriers).
__device__ __forceinline__ int block_rank(bool flag, int* wave_total, int& total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const unsigned long long mask = __ballot(flag);
  const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
  __syncthreads();  // the previous use of wave_total has been read
  if (lane == 0) wave_total[wave] = __popcll(mask);
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = wave_total[w];
    before += w < wave ? t : 0;
    all += t;
  }
  total = all;
  return before + rank;
}

__global__ __launch_bounds__(kSelThreads) void merge_select_kernel(const float* __restrict__ score,
                                                                  const float* __restrict__ coords, int N, int n_keep,
                                                                  int32_t* __restrict__ anchor_idx,
                                                                  float* __restrict__ anchor_xy) {
  __shared__ int hist[kSelWaves][256];  // one histogram per wave: fewer lanes meet in one counter
  __shared__ int wave_total[kSelWaves];
  __shared__ uint32_t s_prefix;
  __shared__ int s_remaining;
  const int tid = threadIdx.x, wave = tid / kWave;
  const int b = blockIdx.x;
  const float* sc = score + (size_t)b * N;
  // the key of the last kept token, digit by digit from the top: among the keys that agree with the digits found
  // so far, `remaining` are still to be kept
  uint32_t prefix = 0u, mask = 0u;
  int remaining = n_keep;
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = tid; i < kSelWaves * 256; i += kSelThreads) (&hist[0][0])[i] = 0;
    __syncthreads();
    for (int i = tid; i < N; i += kSelThreads) {
      const uint32_t key = score_key(sc[i]);
      if ((key & mask) == prefix) atomicAdd(&hist[wave][(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (tid < 256) {
      int t = 0;
#pragma unroll
      for (int w = 0; w < kSelWaves; ++w) t += hist[w][tid];
      hist[0][tid] = t;  // (each thread reads and writes its own column only)
    }
    __syncthreads();
    if (tid < 256) {
      // the largest digit whose keys, with all larger ones, reach `remaining`: thread d adds up the digits above d
      // (independent loads; one thread walking down the 256 counters is a chain of 256 dependent LDS reads)
      int above = 0;
      for (int d = tid + 1; d < 256; ++d) above += hist[0][d];
      if (above < remaining && above + hist[0][tid] >= remaining) {  // true for exactly one digit
        s_prefix = prefix | ((uint32_t)tid << shift);
        s_remaining = remaining - above;
      }
    }
    __syncthreads();
    prefix = s_prefix;
    remaining = s_remaining;
    mask |= 0xffu << shift;
    __syncthreads();
  }
  // sweep in index order: every larger key is kept, and the first `remaining` tokens whose key equals `prefix`
  int equal_before = 0, kept_before = 0;
  for (int base = 0; base < N; base += kSelThreads) {
    const int i = base + tid;
    const bool in = i < N;
    const uint32_t key = in ? score_key(sc[i]) : 0u;
    const bool equal = in && key == prefix;
    int equal_total, kept_total;
    const int equal_rank = block_rank(equal, wave_total, equal_total);
    const bool keep = in && (key > prefix || (equal && equal_before + equal_rank < remaining));
    const int place = kept_before + block_rank(keep, wave_total, kept_total);
    if (keep && place < n_keep) {
      anchor_idx[(size_t)b * n_keep + place] = i;
      if (anchor_xy) {
        anchor_xy[2 * ((size_t)b * n_keep + place)] = coords[2 * ((size_t)b * N + i)];
        anchor_xy[2 * ((size_t)b * n_keep + place) + 1] = coords[2 * ((size_t)b * N + i) + 1];
      }
    }
    equal_before += equal_total;
    kept_before += kept_total;
  }
}

// Sum of v over the earlier threads of the workgroup, and over all of them (two barriers).
__device__ __forceinline__ int block_exclusive_sum(int v, int* wave_total, int& total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  int incl = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(incl, o);
    incl += lane >= o ? up : 0;
  }
  __syncthreads();  // the previous use of wave_total has been read
  if (lane == kWave - 1) wave_total[wave] = incl;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = wave_total[w];
    before += w < wave ? t : 0;
    all += t;
  }
  total = all;
  return before + incl - v;
}

// The same selection for images of at most KPT * 1024 tokens, with the keys held in registers: thread t keeps the
// keys of tokens t KPT .. t KPT + KPT - 1.  The key of the last kept token is built bit by bit from the top: a bit
// stays set when at least n_keep keys are >= the candidate (a compare and a wave-wide count per key, one barrier per
// bit).  The radix form above re-reads the scores for each digit and adds into LDS counters, where the lanes of a
// wave meet in the few counters that the leading bits of real scores fall into; this form has no contended address.
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void merge_select_bits_kernel(const float* __restrict__ score,
                                                                       const float* __restrict__ coords, int N,
                                                                       int n_keep, int32_t* __restrict__ anchor_idx,
                                                                       float* __restrict__ anchor_xy) {
  __shared__ int wave_count[2][kSelWaves];
  __shared__ int wave_total[kSelWaves];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int b = blockIdx.x;
  const float* sc = score + (size_t)b * N;
  const int first = tid * KPT;
  uint32_t key[KPT];  // 0 past the end: below the key of every finite score
  if (KPT % 4 == 0 && N % 4 == 0 && reinterpret_cast<uintptr_t>(sc) % 16 == 0) {
#pragma unroll
    for (int e = 0; e < KPT; e += 4) {
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      const bool in = first + e < N;  // N % 4 == 0: a piece is inside or outside as a whole
      if (in) v = *reinterpret_cast<const float4*>(sc + first + e);
      key[e] = in ? score_key(v.x) : 0u;
      key[e + 1] = in ? score_key(v.y) : 0u;
      key[e + 2] = in ? score_key(v.z) : 0u;
      key[e + 3] = in ? score_key(v.w) : 0u;
    }
  } else {
#pragma unroll
    for (int e = 0; e < KPT; ++e) key[e] = first + e < N ? score_key(sc[first + e]) : 0u;
  }
  // number of keys of the workgroup that are >= cand (cand > 0); `turn` alternates the LDS row so that one barrier
  // per count is enough: a row is rewritten only after every thread has passed the barrier of the next count
  auto count_at_least = [&](uint32_t cand, int turn) {
    int c = 0;
#pragma unroll
    for (int e = 0; e < KPT; ++e) c += __popcll(__ballot(key[e] >= cand));  // wave-uniform
    if (lane == 0) wave_count[turn][wave] = c;
    __syncthreads();
    int all = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) all += wave_count[turn][w];
    return all;
  };
  uint32_t prefix = 0u;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = prefix | (1u << bit);
    if (count_at_least(cand, bit & 1) >= n_keep) prefix = cand;
  }
  // prefix = key of the last kept token; `remaining` of the tokens with exactly that key are kept, lowest index first
  // (row 1 was last used for bit 1; the barrier of bit 0 lies between)
  const int larger = prefix == 0xffffffffu ? 0 : count_at_least(prefix + 1u, 1);
  const int remaining = n_keep - larger;
  int equal = 0;
#pragma unroll
  for (int e = 0; e < KPT; ++e) equal += key[e] == prefix ? 1 : 0;
  int total;
  int equal_before = block_exclusive_sum(equal, wave_total, total);
  int kept = 0;
#pragma unroll
  for (int e = 0; e < KPT; ++e) {
    const bool eq = key[e] == prefix;
    kept += (key[e] > prefix || (eq && equal_before < remaining)) ? 1 : 0;
    equal_before += eq ? 1 : 0;
  }
  equal_before -= equal;
  int place = block_exclusive_sum(kept, wave_total, total);
  int32_t* idx_out = anchor_idx + (size_t)b * n_keep;
#pragma unroll
  for (int e = 0; e < KPT; ++e) {
    const bool eq = key[e] == prefix;
    const bool keep = key[e] > prefix || (eq && equal_before < remaining);
    equal_before += eq ? 1 : 0;
    if (keep && first + e < N && place < n_keep) idx_out[place] = first + e;
    place += keep ? 1 : 0;
  }
  if (!anchor_xy) return;
  // the anchors' coordinates: the list just written is read back in order (its writes are visible to the workgroup
  // after the fence and the barrier), so the gathers of a thread are independent loads and the stores are coalesced
  __threadfence_block();
  __syncthreads();
  const float2* xy_in = reinterpret_cast<const float2*>(coords) + (size_t)b * N;
  float2* xy_out = reinterpret_cast<float2*>(anchor_xy) + (size_t)b * n_keep;
  for (int a = tid; a < n_keep; a += kSelThreads) xy_out[a] = xy_in[min(max(idx_out[a], 0), N - 1)];
}

// 16 bytes of channels
template <typename T>
struct Piece16;
template <>
struct Piece16<float> {
  static constexpr int kCh = 4;
  static __device__ __forceinline__ void load(const float* p, float (&v)[8]) {
    const float4 x = *reinterpret_cast<const float4*>(p);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    v[4] = v[5] = v[6] = v[7] = 0.f;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <>
struct Piece16<bf16_t> {
  static constexpr int kCh = 8;
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const uint4 x = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[2 * e] = __uint_as_float(w[e] << 16);
      v[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    uint4 x;
    x.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
    x.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
    x.z = (uint32_t)f32_to_bf16(v[4]) | ((uint32_t)f32_to_bf16(v[5]) << 16);
    x.w = (uint32_t)f32_to_bf16(v[6]) | ((uint32_t)f32_to_bf16(v[7]) << 16);
    *reinterpret_cast<uint4*>(p) = x;
  }
};

// <a, b> over 16 bytes: bf16 by four two-element dot instructions on the packed values, fp32 by multiply-adds
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ float dot16(const bf16_t* pa, const uint4& b) {
  const uint4 a = *reinterpret_cast<const uint4*>(pa);
  float acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), 0.f, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), acc, false);
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), acc, false);
}
__device__ __forceinline__ float dot16(const float* pa, const uint4& b) {
  const float4 a = *reinterpret_cast<const float4*>(pa);
  return fmaf(a.w, __uint_as_float(b.w), fmaf(a.z, __uint_as_float(b.z), fmaf(a.y, __uint_as_float(b.y), a.x * __uint_as_float(b.x))));
}

// The anchor of this wave and the neighbour of this lane: index, distance, weight.  Every lane runs this.
struct Nbr {
  int anchor_slot;  // b * n_keep + a
  int b, tok;       // image, the anchor's token
  int idx;          // neighbour token of this lane (lanes >= K: the anchor's own token, weight 0)
  float dist, w;
};
__device__ __forceinline__ Nbr load_neighbour(const float* __restrict__ coords, const float* __restrict__ score,
                                              const int32_t* __restrict__ nbr, const int32_t* __restrict__ anchor,
                                              long long slot, int N, int K, int n_keep, float p, int lane) {
  Nbr r;
  r.anchor_slot = (int)slot;
  r.b = (int)(slot / n_keep);
  r.tok = min(max(anchor[slot], 0), N - 1);
  const bool on = lane < K;
  const int32_t* row = nbr + ((size_t)r.b * N + r.tok) * K;
  r.idx = on ? min(max(row[lane], 0), N - 1) : r.tok;
  const float2 xa = *reinterpret_cast<const float2*>(coords + 2 * ((size_t)r.b * N + r.tok));
  const float2 xn = *reinterpret_cast<const float2*>(coords + 2 * ((size_t)r.b * N + r.idx));
  const float dx = xn.x - xa.x, dy = xn.y - xa.y;
  r.dist = sqrtf(dx * dx + dy * dy);  // correctly rounded: an error of the distance is multiplied by p in the exponent
  const float z = on ? score[(size_t)r.b * N + r.idx] - p * r.dist : -INFINITY;
  const float zmax = wave_max(z);
  const float e = on ? __expf(z - zmax) : 0.f;
  r.w = e / wave_sum(e);  // the sum is in [1, K]
  // broadcast from their lanes later: pinned here, where every lane is active
  asm volatile("" : "+v"(r.w), "+v"(r.idx));
  return r;
}

// PIECES: rows are whole 16-byte pieces and 16-byte aligned; a row takes PP lanes (the next power of two of its
// piece count, at most 64), RW = 64 / PP rows are in flight per trip.  Otherwise lanes are channels.
template <typename T, bool PIECES>
__global__ __launch_bounds__(256) void merge_fwd_kernel(const T* __restrict__ feat, const float* __restrict__ coords,
                                                       const float* __restrict__ score,
                                                       const int32_t* __restrict__ nbr,
                                                       const int32_t* __restrict__ anchor, int B, int N, int C, int K,
                                                       int n_keep, float p, int PP, T* __restrict__ out) {
  const int lane = threadIdx.x & (kWave - 1);
  const long long slot = xcd_contiguous_block() * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (slot >= (long long)B * n_keep) return;  // wave-uniform
  const Nbr nb = load_neighbour(coords, score, nbr, anchor, slot, N, K, n_keep, p, lane);
  const T* rows = feat + (size_t)nb.b * N * C;
  T* orow = out + (size_t)slot * C;
  if (PIECES) {
    constexpr int CH = Piece16<T>::kCh;
    const int pieces = C / CH;
    const int RW = kWave / PP;
    const int pc = lane & (PP - 1), rs = lane / PP;  // piece and row of this lane inside a trip
    for (int pc0 = 0; pc0 < pieces; pc0 += PP) {      // one trip unless a row has more than 64 pieces
      const bool pon = pc0 + pc < pieces;
      const int c0 = min(pc0 + pc, pieces - 1) * CH;  // lanes past the row's end repeat its last piece (unused)
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int j0 = 0; j0 < K; j0 += RW) {
        const int j = j0 + rs;
        const int jj = min(j, K - 1);
        const float wraw = __shfl(nb.w, jj);  // (every lane takes part in the shuffles; rows past K get weight 0)
        const int ij = __shfl(nb.idx, jj);
        const float wj = j < K ? wraw : 0.f;
        float f[8];
        Piece16<T>::load(rows + (uint32_t)(ij * C + c0), f);  // (row offsets inside an image fit 32 bits on this path)
#pragma unroll
        for (int e = 0; e < CH; ++e) acc[e] = fmaf(wj, f[e], acc[e]);
      }
      for (int o = PP; o < kWave; o <<= 1) {  // add up the row groups
#pragma unroll
        for (int e = 0; e < CH; ++e) acc[e] += __shfl_xor(acc[e], o);
      }
      if (rs == 0 && pon) Piece16<T>::store(orow + c0, acc);
    }
  } else {
    for (int base = 0; base < C; base += kWave) {  // wave-uniform trips; only the memory accesses are predicated
      const int c = base + lane;
      const bool on = c < C;
      float a = 0.f;
      for (int j = 0; j < K; ++j) {
        const float wj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(nb.w), j));
        const int ij = __builtin_amdgcn_readlane(nb.idx, j);
        if (on) a = fmaf(wj, Elem<T>::load(rows + (size_t)ij * C + c), a);
      }
      if (on) Elem<T>::store(orow + c, a);
    }
  }
}

template <typename T, bool PIECES>
__global__ __launch_bounds__(256) void merge_bwd_kernel(const T* __restrict__ feat, const float* __restrict__ coords,
                                                       const float* __restrict__ score,
                                                       const int32_t* __restrict__ nbr,
                                                       const int32_t* __restrict__ anchor, const T* __restrict__ dout,
                                                       int B, int N, int C, int K, int n_keep, float p, int PP,
                                                       float* __restrict__ wpair, float* __restrict__ dzpair,
                                                       int32_t* __restrict__ pair_token, int2* __restrict__ pair_bounds,
                                                       float* __restrict__ dp_part) {
  __shared__ float g_all[4][kWave];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const long long slot = xcd_contiguous_block() * 4 + wave;
  if (slot >= (long long)B * n_keep) return;  // wave-uniform; no workgroup barrier below
  float* g = g_all[wave];
  const Nbr nb = load_neighbour(coords, score, nbr, anchor, slot, N, K, n_keep, p, lane);
  const T* rows = feat + (size_t)nb.b * N * C;
  const T* grow = dout + (size_t)slot * C;
  g[lane] = 0.f;
  wave_lds_sync();
  if (PIECES) {
    constexpr int CH = Piece16<T>::kCh;
    const int pieces = C / CH;
    const int RW = kWave / PP;
    const int pc = lane & (PP - 1), rs = lane / PP;
    for (int pc0 = 0; pc0 < pieces; pc0 += PP) {
      const bool pon = pc0 + pc < pieces;
      const int c0 = min(pc0 + pc, pieces - 1) * CH;
      const uint4 go = *reinterpret_cast<const uint4*>(grow + c0);
      for (int j0 = 0; j0 < K; j0 += RW) {
        const int j = j0 + rs;
        const int ij = __shfl(nb.idx, min(j, K - 1));
        // (row offsets inside an image fit 32 bits on this path)
        float part = dot16(rows + (uint32_t)(ij * C + c0), go);
        part = pon ? part : 0.f;
        for (int o = 1; o < PP; o <<= 1) part += __shfl_xor(part, o);  // over the lanes of the row
        if (pc == 0 && j < K) g[j] += part;                            // (one lane per j: no two lanes add to one cell)
      }
    }
  } else {
    for (int j = 0; j < K; ++j) {
      const int ij = __builtin_amdgcn_readlane(nb.idx, j);
      float part = 0.f;
      for (int c = lane; c < C; c += kWave) part = fmaf(Elem<T>::load(grow + c), Elem<T>::load(rows + (size_t)ij * C + c), part);
      part = wave_sum(part);
      if (lane == 0) g[j] = part;
    }
  }
  wave_lds_sync();
  float g_mine = lane < K ? g[lane] : 0.f;
  asm volatile("" : "+v"(g_mine));
  // dz_j = w_j (g_j - sum_i w_i g_i).  Taken relative to the neighbour with the largest weight (the first of
  // them), d_i = g_i - g_ref: dz_j = w_j (d_j - sum_i w_i d_i), since the weights add up to 1.  The differences are
  // formed first, the reference's own term is exactly 0 and every other term carries a small weight when one
  // weight saturates - the form does not cancel then, like sum_i w_i (g_j - g_i), at two wave reductions instead of
  // K broadcasts per lane.
  const float wmax = wave_max(nb.w);  // lanes >= K hold weight 0
  const unsigned long long at_max = __ballot(lane < K && nb.w == wmax);  // not empty: K >= 1 and wmax is some lane's
  const int ref = __builtin_amdgcn_readfirstlane((int)__builtin_ctzll(at_max));
  const float gref = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(g_mine), ref));
  const float delta = g_mine - gref;
  const float spread = delta - wave_sum(nb.w * delta);
  const float dz = nb.w * spread;  // lanes >= K hold weight 0
  // sum_j dz_j (-dist_j) with sum_j dz_j = 0: distances relative to the nearest neighbour's
  const float dnear = -wave_max(lane < K ? -nb.dist : -INFINITY);
  const float dpv = wave_sum(lane < K ? dz * (dnear - nb.dist) : 0.f);
  if (lane < K) {
    const size_t pair = (size_t)slot * K + lane;
    wpair[pair] = nb.w;
    dzpair[pair] = dz;
    pair_token[pair] = nb.b * N + nb.idx;
  }
  if (lane == 0 && dp_part) dp_part[slot] = dpv;
  // the lowest and highest token of the anchor's pairs, for the list builder (lanes >= K hold the anchor's token)
  int tmin = nb.b * N + nb.idx, tmax = tmin;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    tmin = min(tmin, __shfl_xor(tmin, o));
    tmax = max(tmax, __shfl_xor(tmax, o));
  }
  if (lane == 0) pair_bounds[slot] = make_int2(tmin, tmax);
}


size_t merge_align(size_t n) { return (n + 255) / 256 * 256; }
struct MergeBwdLayout {
  size_t w_off, dz_off, pair_off, bounds_off, offset_off, list_off, dp_off, dp2_off, total;
};
MergeBwdLayout merge_bwd_layout(int B, int N, int K, int n_keep) {
  MergeBwdLayout L;
  const size_t pairs = (size_t)B * n_keep * K, tokens = (size_t)B * N, anchors = (size_t)B * n_keep;
  size_t off = 0;
  L.w_off = off;      off += merge_align(pairs * sizeof(float));
  L.dz_off = off;     off += merge_align(pairs * sizeof(float));
  L.pair_off = off;   off += merge_align(pairs * sizeof(int32_t));
  L.bounds_off = off; off += merge_align(anchors * 2 * sizeof(int32_t));
  L.offset_off = off; off += merge_align((tokens + 1) * sizeof(int32_t));
  L.list_off = off;   off += merge_align(pairs * sizeof(int32_t));
  L.dp_off = off;     off += merge_align(anchors * sizeof(float));
  L.dp2_off = off;    off += merge_align(sum_parts_scratch_floats(anchors) * sizeof(float));
  L.total = off;
  return L;
}

// rows of whole 16-byte pieces, 16-byte aligned, row offsets inside an image within 32 bits
bool merge_pieces(const MergeArgs& a, const void* t0, const void* t1) {
  const size_t row = (size_t)a.C * (a.dtype == 1 ? 2 : 4);
  auto al = [](const void* p) { return p == nullptr || reinterpret_cast<uintptr_t>(p) % 16 == 0; };
  return row % 16 == 0 && al(t0) && al(t1) && reinterpret_cast<uintptr_t>(a.coords) % 8 == 0 &&
         (long long)a.N * a.C < (1ll << 31);
}
int lanes_per_row(const MergeArgs& a) {
  const int pieces = a.C / (a.dtype == 1 ? 8 : 4);
  int pp = 1;
  while (pp < pieces && pp < kWave) pp <<= 1;
  return pp;
}

}  // namespace

hipError_t launch_merge_select(const float* score, const float* coords, int B, int N, int n_keep, int32_t* anchor_idx,
                               float* anchor_xy, hipStream_t stream) {
#define AFFMAE_SELECT(KERNEL) \
  AFFMAE_LAUNCH("merge_select_kernel", stream, KERNEL, dim3(B), dim3(kSelThreads), 0, stream, score, coords, N, \
                n_keep, anchor_idx, anchor_xy)
  if (N <= 4 * kSelThreads) AFFMAE_SELECT(merge_select_bits_kernel<4>);
  else if (N <= 16 * kSelThreads) AFFMAE_SELECT(merge_select_bits_kernel<16>);
  else if (N <= 32 * kSelThreads) AFFMAE_SELECT(merge_select_bits_kernel<32>);
  else AFFMAE_SELECT(merge_select_kernel);  // larger images: the keys do not fit a workgroup's registers
#undef AFFMAE_SELECT
  return hipGetLastError();
}

hipError_t launch_merge_fwd(const MergeArgs& a, hipStream_t stream) {
  const dim3 grid(round_up8(((long long)a.B * a.n_keep + 3) / 4));
  const bool pieces = merge_pieces(a, a.feat, a.out);
  const int pp = lanes_per_row(a);
#define AFFMAE_MERGE_FWD(T, P)                                                                                     \
  AFFMAE_LAUNCH("merge_fwd_kernel", stream, (merge_fwd_kernel<T, P>), grid, dim3(256), 0, stream, (const T*)a.feat, \
                a.coords, a.score, a.nbr_idx, a.anchor_idx, a.B, a.N, a.C, a.K, a.n_keep, a.p, pp, (T*)a.out)
  if (a.dtype == 1 && pieces) AFFMAE_MERGE_FWD(bf16_t, true);
  else if (a.dtype == 1) AFFMAE_MERGE_FWD(bf16_t, false);
  else if (pieces) AFFMAE_MERGE_FWD(float, true);
  else AFFMAE_MERGE_FWD(float, false);
#undef AFFMAE_MERGE_FWD
  return hipGetLastError();
}

size_t merge_bwd_workspace_bytes(int B, int N, int K, int n_keep) { return merge_bwd_layout(B, N, K, n_keep).total; }

hipError_t launch_merge_bwd(const MergeArgs& a, hipStream_t stream) {
  const MergeBwdLayout L = merge_bwd_layout(a.B, a.N, a.K, a.n_keep);
  char* ws = static_cast<char*>(a.workspace);
  float* wpair = reinterpret_cast<float*>(ws + L.w_off);
  float* dzpair = reinterpret_cast<float*>(ws + L.dz_off);
  int32_t* pair_token = reinterpret_cast<int32_t*>(ws + L.pair_off);
  int2* pair_bounds = reinterpret_cast<int2*>(ws + L.bounds_off);
  int32_t* offset = reinterpret_cast<int32_t*>(ws + L.offset_off);
  int32_t* list = reinterpret_cast<int32_t*>(ws + L.list_off);
  float* dp_part = a.dp ? reinterpret_cast<float*>(ws + L.dp_off) : nullptr;
  float* dp_part2 = reinterpret_cast<float*>(ws + L.dp2_off);
  const size_t tokens = (size_t)a.B * a.N, anchors = (size_t)a.B * a.n_keep;
  const dim3 grid(round_up8(((long long)anchors + 3) / 4));
  const bool pieces = merge_pieces(a, a.feat, a.dout);
  const int pp = lanes_per_row(a);
#define AFFMAE_MERGE_BWD(T, P)                                                                                     \
  AFFMAE_LAUNCH("merge_bwd_kernel", stream, (merge_bwd_kernel<T, P>), grid, dim3(256), 0, stream, (const T*)a.feat, \
                a.coords, a.score, a.nbr_idx, a.anchor_idx, (const T*)a.dout, a.B, a.N, a.C, a.K, a.n_keep, a.p, pp, \
                wpair, dzpair, pair_token, pair_bounds, dp_part)
  if (a.dtype == 1 && pieces) AFFMAE_MERGE_BWD(bf16_t, true);
  else if (a.dtype == 1) AFFMAE_MERGE_BWD(bf16_t, false);
  else if (pieces) AFFMAE_MERGE_BWD(float, true);
  else AFFMAE_MERGE_BWD(float, false);
#undef AFFMAE_MERGE_BWD
  if (a.dp) {
    const hipError_t e = launch_sum_parts(dp_part, anchors, dp_part2, a.dp, stream);
    if (e != hipSuccess) return e;
  }
  hipError_t e = launch_pair_lists(pair_token, a.B, a.N, a.n_keep * a.K, offset, list, stream,
                                   reinterpret_cast<const int32_t*>(pair_bounds), a.K);
  if (e != hipSuccess) return e;
  // one walk over every token's list serves both sums: dfeat = sum of w * dout, dscore = sum of dz
  const bool gpieces = merge_pieces(a, a.dout, a.dfeat) && (long long)a.n_keep * a.C < (1ll << 31);
  return launch_pair_gather(a.dout, wpair, offset, list, tokens, a.C, a.K, a.dtype, a.dfeat, gpieces, stream, dzpair,
                            a.dscore);
}

}  // namespace affmae
