// Virtual sampled tokens of the point decoder (paper, Sec. "AFFMAE": a decoder query gathers the nearest
// visible tokens and aggregates their features with the exponential distance kernel softmax_i(-p d_i),
// d_i = |q - x_i| + eps; Sec. "Flash-style Cluster Attention and Fast Decoder KNN" and supplement
// "Point-based decoder": the nearest visible tokens come from a table cached over the dense patch grid,
// the query is rounded to its nearest grid point, and lookup, distances, weights and the weighted sum
// are one kernel).
//
//   table   : one wave per grid point; the image's visible tokens stream past 64 at a time; the first 64
//             are sorted, later ones are queued only when they beat the current Kt-th key and merged 64
//             at a time.  Keys = (fp32 squared distance bits, token index): exact and unique.
//   forward : a group of 4 lanes (Kt <= 4; 16 lanes up to Kt = 16, else a whole wave) per query; lane l of the
//             group holds candidate l (index, distance, weight), then the lanes split the channels of the
//             gathered feature rows, 16 bytes at a time, for the weighted sum.
//   backward: the same groups: g_i = <dout, feat_i> by group reductions, dz_i = w_i (g_i - sum w g), dquery
//             and a part of dp per wave (added up in a fixed order afterwards) from the lanes that hold
//             candidates; the weights and the token of every (query, candidate) pair are kept.  dfeat is then
//             gathered, not scattered: the pairs are filed per token (counted, prefix-summed and placed in LDS,
//             one workgroup per range of tokens of an image: no atomics on global memory), and a group of
//             lanes per visible token adds up w * dout over its pairs (no floating-point atomics; the order
//             inside a token's list, hence the last bits of dfeat, follows the filing order of the run).
// This file is compiled with -ffp-contract=off (grid points and table distances are defined unfused).
#include <algorithm>

#include "cluster_common.h"
#include "device_util.h"
#include "launch.h"
#include "select_util.h"
#include "timing.h"

namespace affmae {
namespace {

// Workgroups are dealt round-robin to the 8 XCDs (one L2 each).  Consecutive queries and tokens belong to one
// image and share its feature rows, so every XCD gets a contiguous range.  The grid is a multiple of 8.
__device__ __forceinline__ long long xcd_contiguous_block() {
  const unsigned per_xcd = gridDim.x >> 3;
  return (long long)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
}
inline unsigned round_up8(long long blocks) { return (unsigned)((blocks + 7) / 8 * 8); }

struct Grid {
  int Hg, Wg;
  float x0, y0, cell;
};

__global__ __launch_bounds__(256) void vts_table_kernel(const float* __restrict__ vis_xy, int B, int Nv, Grid gr, int Kt,
                                                       int32_t* __restrict__ table) {
  __shared__ key_t pend_all[4][2 * kWave];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const long long cells = (long long)B * gr.Hg * gr.Wg;
  const long long gcell = (long long)blockIdx.x * 4 + wave;
  if (gcell >= cells) return;  // wave-uniform; no workgroup barrier below
  key_t* pend = pend_all[wave];
  const int per_image = gr.Hg * gr.Wg;
  const int b = (int)(gcell / per_image);
  const int c = (int)(gcell - (long long)b * per_image);
  const int iy = c / gr.Wg, ix = c - iy * gr.Wg;
  // patch centre, each operation rounded separately
  const float hx = (float)ix + 0.5f, hy = (float)iy + 0.5f;
  const float sx = hx * gr.cell, sy = hy * gr.cell;
  const float gx = gr.x0 + sx, gy = gr.y0 + sy;
  const float* xy = vis_xy + (size_t)b * Nv * 2;
  auto key_of = [&](int i) -> key_t {
    if (i >= Nv) return kKeyMax;
    return make_key(dist2(gx, gy, xy[2 * (size_t)i], xy[2 * (size_t)i + 1]), i);
  };
  key_t best = wave_sort(key_of(lane), lane);
  key_t bound = shfl_key(best, Kt - 1);
  int fill = 0;  // queued keys, wave-uniform, always < 64 between rows
  for (int base = kWave; base < Nv; base += kWave) {
    const key_t key = key_of(base + lane);
    const bool in = key < bound;
    const unsigned long long mask = __ballot(in);
    if (mask == 0ull) continue;  // wave-uniform
    const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
    if (in) pend[fill + rank] = key;
    fill += __popcll(mask);
    if (fill >= kWave) {
      wave_lds_sync();
      const key_t row = pend[lane];
      const key_t rest = pend[kWave + lane];
      wave_lds_sync();
      fill -= kWave;
      if (lane < fill) pend[lane] = rest;
      best = topk_push(best, row, lane, Kt - 1);
      bound = shfl_key(best, Kt - 1);
    }
  }
  if (fill > 0) {
    wave_lds_sync();
    best = topk_push(best, (lane < fill) ? pend[lane] : kKeyMax, lane, Kt - 1);
  }
  if (lane < Kt) table[(size_t)gcell * Kt + lane] = (int32_t)(uint32_t)best;
}

// At most 1024 visible tokens per image: every lane keeps its 16 tokens in registers and the wave serves a run
// of consecutive grid points of one image, each by a counted distance threshold and a single sort (the
// threshold of one grid point is the first guess for the next).
constexpr int kTableRows = 16;
constexpr int kTableRun = 16;  // grid points per wave
__global__ __launch_bounds__(256) void vts_table_fast_kernel(const float* __restrict__ vis_xy, int B, int Nv, Grid gr,
                                                            int Kt, int32_t* __restrict__ table) {
  __shared__ key_t pend_all[4][2 * kWave];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int per_image = gr.Hg * gr.Wg;
  const int runs_per_image = (per_image + kTableRun - 1) / kTableRun;
  const long long grun = (long long)blockIdx.x * 4 + wave;
  if (grun >= (long long)B * runs_per_image) return;  // wave-uniform; no workgroup barrier below
  key_t* pend = pend_all[wave];
  const int b = (int)(grun / runs_per_image);
  const int first = (int)(grun - (long long)b * runs_per_image) * kTableRun;
  const float* xy = vis_xy + (size_t)b * Nv * 2;
  float cx[kTableRows], cy[kTableRows];
  uint32_t cid[kTableRows];
#pragma unroll
  for (int row = 0; row < kTableRows; ++row) {
    const int i = row * kWave + lane;
    const bool ok = i < Nv;
    cx[row] = ok ? xy[2 * (size_t)i] : 0.f;
    cy[row] = ok ? xy[2 * (size_t)i + 1] : 0.f;
    cid[row] = ok ? (uint32_t)i : 0xffffffffu;
  }
  uint32_t guess = 0u;
  for (int c = first; c < min(first + kTableRun, per_image); ++c) {
    const int iy = c / gr.Wg, ix = c - iy * gr.Wg;
    // patch centre, each operation rounded separately
    const float hx = (float)ix + 0.5f, hy = (float)iy + 0.5f;
    const float sx = hx * gr.cell, sy = hy * gr.cell;
    const float gx = gr.x0 + sx, gy = gr.y0 + sy;
    uint32_t d2[kTableRows];
#pragma unroll
    for (int row = 0; row < kTableRows; ++row)
      d2[row] = cid[row] != 0xffffffffu ? __float_as_uint(dist2(gx, gy, cx[row], cy[row])) : 0xffffffffu;
    const key_t best = select_nearest<kTableRows>(d2, cid, Kt, guess, pend, lane);
    if (lane < Kt) table[((size_t)b * per_image + c) * Kt + lane] = (int32_t)(uint32_t)best;
  }
}

// Grid cell of a query coordinate: floor((q - x0) / cell), clamped to 0..n-1 (NaN goes to 0).
__device__ __forceinline__ int cell_of(float q, float x0, float cell, int n) {
  const float t = q - x0;
  const float u = t / cell;
  const float f = floorf(u);
  if (!(f >= 0.f)) return 0;
  if (f > (float)(n - 1)) return n - 1;
  return (int)f;
}

// Table by a search over the grid itself, for small Kt.  A workgroup bins the image's visible tokens by grid
// cell in LDS (count, prefix sum, fill: tokens of a cell, and of consecutive cells of a grid row, end up
// adjacent), then every thread serves one grid point: it scans the tokens of a square window of cells around the
// point, keeping the best Kt keys in registers, and widens the window until the Kt-th key is closer than
// anything outside the window can be.  A token binned outside a window of radius r cells is at least
// (r + 1/2) cell widths away along one axis (tokens outside the grid are binned to border cells and are farther
// still); the test leaves a margin of 2^-10 for the rounding of the bin and of the distances.  Same keys, hence
// the same table, as the exhaustive kernels above.
constexpr int kGridThreads = 1024;
constexpr int kGridLdsBytes = 64 * 1024;
template <int CAP>
__global__ __launch_bounds__(kGridThreads) void vts_table_grid_kernel(const float* __restrict__ vis_xy, int B, int Nv,
                                                                     Grid gr, int Kt, int r0, int slabs,
                                                                     int32_t* __restrict__ table) {
  extern __shared__ __align__(16) unsigned char grid_lds[];
  const int cells = gr.Hg * gr.Wg;
  int32_t* cend = reinterpret_cast<int32_t*>(grid_lds);                      // [cells] counts, then starts, then ends
  float2* sxy = reinterpret_cast<float2*>(grid_lds + (size_t)((cells + 1) & ~1) * 4);  // [Nv] tokens in cell order
  int32_t* sidx = reinterpret_cast<int32_t*>(sxy + Nv);                     // [Nv]
  __shared__ int32_t wave_total[kGridThreads / kWave];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int b = blockIdx.x / slabs, slab = blockIdx.x - b * slabs;
  const float2* xy = reinterpret_cast<const float2*>(vis_xy) + (size_t)b * Nv;
  auto bin_of = [&](const float2& t) { return cell_of(t.y, gr.y0, gr.cell, gr.Hg) * gr.Wg + cell_of(t.x, gr.x0, gr.cell, gr.Wg); };
  // the first kHeld tokens of a thread stay in registers between the counting and the filing
  constexpr int kHeld = 4;
  float2 held[kHeld];
  int held_bin[kHeld];
#pragma unroll
  for (int i = 0; i < kHeld; ++i) {
    const int t = tid + i * kGridThreads;
    held[i] = xy[min(t, Nv - 1)];
  }
  for (int c = tid; c < cells; c += kGridThreads) cend[c] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kHeld; ++i) {
    held_bin[i] = bin_of(held[i]);
    if (tid + i * kGridThreads < Nv) atomicAdd(&cend[held_bin[i]], 1);
  }
  for (int t = tid + kHeld * kGridThreads; t < Nv; t += kGridThreads) atomicAdd(&cend[bin_of(xy[t])], 1);
  __syncthreads();
  // exclusive prefix sum in place: thread tid owns a run of consecutive cells
  const int per = (cells + kGridThreads - 1) / kGridThreads;
  const int c_lo = min(tid * per, cells), c_hi = min(c_lo + per, cells);
  int mine = 0;
  for (int c = c_lo; c < c_hi; ++c) mine += cend[c];
  int incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  if (lane == kWave - 1) wave_total[wave] = incl;
  __syncthreads();
  int run = incl - mine;
  for (int w = 0; w < wave; ++w) run += wave_total[w];
  for (int c = c_lo; c < c_hi; ++c) {
    const int n = cend[c];
    cend[c] = run;
    run += n;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kHeld; ++i) {
    const int t = tid + i * kGridThreads;
    if (t < Nv) {
      const int pos = atomicAdd(&cend[held_bin[i]], 1);  // leaves the end of every cell behind
      sxy[pos] = held[i];
      sidx[pos] = t;
    }
  }
  for (int t = tid + kHeld * kGridThreads; t < Nv; t += kGridThreads) {
    const float2 v = xy[t];
    const int pos = atomicAdd(&cend[bin_of(v)], 1);
    sxy[pos] = v;
    sidx[pos] = t;
  }
  __syncthreads();

  const int c = slab * kGridThreads + tid;
  if (c >= cells) return;  // no barrier below
  const int iy = c / gr.Wg, ix = c - iy * gr.Wg;
  // patch centre, each operation rounded separately
  const float hx = (float)ix + 0.5f, hy = (float)iy + 0.5f;
  const float sx = hx * gr.cell, sy = hy * gr.cell;
  const float gx = gr.x0 + sx, gy = gr.y0 + sy;
  key_t best[CAP];
  for (int r = r0;; r += max(1, r >> 1)) {
#pragma unroll
    for (int i = 0; i < CAP; ++i) best[i] = kKeyMax;
    const int x_lo = max(ix - r, 0), x_hi = min(ix + r, gr.Wg - 1);
    const int y_lo = max(iy - r, 0), y_hi = min(iy + r, gr.Hg - 1);
    for (int y = y_lo; y <= y_hi; ++y) {
      const int first = y * gr.Wg + x_lo, last = y * gr.Wg + x_hi;
      const int t_lo = first > 0 ? cend[first - 1] : 0, t_hi = cend[last];
      for (int t = t_lo; t < t_hi; ++t) {
        const float2 v = sxy[t];
        const key_t key = make_key(dist2(gx, gy, v.x, v.y), sidx[t]);
        if (key < best[CAP - 1]) {
          best[CAP - 1] = key;
#pragma unroll
          for (int i = CAP - 1; i > 0; --i) {
            const key_t a = best[i - 1], bb = best[i];
            best[i - 1] = a < bb ? a : bb;
            best[i] = a < bb ? bb : a;
          }
        }
      }
    }
    if (x_lo == 0 && y_lo == 0 && x_hi == gr.Wg - 1 && y_hi == gr.Hg - 1) break;  // every token has been seen
    key_t kth = kKeyMax;
#pragma unroll
    for (int i = 0; i < CAP; ++i) kth = (i == Kt - 1) ? best[i] : kth;
    const float reach = ((float)r + 0.5f) * gr.cell;
    const float safe = reach * reach * (1.f - 0x1p-10f);
    if (kth != kKeyMax && __uint_as_float((uint32_t)(kth >> 32)) < safe) break;
  }
#pragma unroll
  for (int i = 0; i < CAP; ++i)
    if (i < Kt) table[((size_t)b * cells + c) * Kt + i] = (int32_t)(uint32_t)best[i];
}

// Two consecutive channels (even channel index, 4-byte aligned rows): one 32-bit access for bf16.
__device__ __forceinline__ void load2(const float* p, float& a, float& b) {
  a = p[0];
  b = p[1];
}
__device__ __forceinline__ void load2(const bf16_t* p, float& a, float& b) {
  const uint32_t w = *reinterpret_cast<const uint32_t*>(p);
  a = __uint_as_float(w << 16);
  b = __uint_as_float(w & 0xffff0000u);
}
__device__ __forceinline__ void store2(float* p, float a, float b) {
  p[0] = a;
  p[1] = b;
}
__device__ __forceinline__ void store2(bf16_t* p, float a, float b) {
  *reinterpret_cast<uint32_t*>(p) = (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

struct Cand {
  int idx;       // visible token of this lane (lanes >= Kt: token 0, weight 0)
  float dx, dy;  // q - x_i
  float dist;    // |q - x_i|
  float w;       // softmax_i(-p (dist + eps))
};

__device__ __forceinline__ Cand load_candidate(const float* __restrict__ query_xy, const float* __restrict__ vis_xy,
                                               const int32_t* __restrict__ table, int b, long long gq, int Nv,
                                               const Grid& gr, int Kt, float p, float eps, int lane) {
  const float qx = query_xy[2 * (size_t)gq], qy = query_xy[2 * (size_t)gq + 1];
  const int ix = cell_of(qx, gr.x0, gr.cell, gr.Wg), iy = cell_of(qy, gr.y0, gr.cell, gr.Hg);
  const int32_t* row = table + (((size_t)b * gr.Hg + iy) * gr.Wg + ix) * Kt;
  Cand c;
  const bool on = lane < Kt;
  c.idx = on ? min(max(row[lane], 0), Nv - 1) : 0;
  const float* x = vis_xy + ((size_t)b * Nv + c.idx) * 2;
  c.dx = qx - x[0];
  c.dy = qy - x[1];
  c.dist = sqrtf(c.dx * c.dx + c.dy * c.dy);
  const float z = on ? -p * (c.dist + eps) : -INFINITY;
  const float zmax = wave_max(z);
  const float e = on ? __expf(z - zmax) : 0.f;
  c.w = e / wave_sum(e);
  // the weights and indices are broadcast from their lanes later: pin their values here, where every lane is
  // active, so that no part of their computation moves under a lane predicate
  asm volatile("" : "+v"(c.w), "+v"(c.idx));
  return c;
}

template <typename T>
__global__ __launch_bounds__(256) void vts_fwd_kernel(const float* __restrict__ query_xy, const float* __restrict__ vis_xy,
                                                     const T* __restrict__ feat, const int32_t* __restrict__ table,
                                                     int B, int Mq, int Nv, int C, Grid gr, int Kt, float p, float eps,
                                                     T* __restrict__ out) {
  const int lane = threadIdx.x & (kWave - 1);
  const long long gq = xcd_contiguous_block() * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (gq >= (long long)B * Mq) return;  // wave-uniform
  const int b = (int)(gq / Mq);
  const Cand cd = load_candidate(query_xy, vis_xy, table, b, gq, Nv, gr, Kt, p, eps, lane);
  // C is even: two channels per lane and trip.  The trip loop is wave-uniform and only the memory accesses
  // are predicated, so that the lane broadcasts below always run with every lane active.
  for (int base = 0; base < C; base += 2 * kWave) {
    const int c0 = base + 2 * lane;
    const bool on = c0 < C;
    float a0 = 0.f, a1 = 0.f;
    for (int i = 0; i < Kt; ++i) {
      const float w = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(cd.w), i));
      const int idx = __builtin_amdgcn_readlane(cd.idx, i);
      const T* f = feat + ((size_t)b * Nv + idx) * C + c0;
      if (on) {
        float f0, f1;
        load2(f, f0, f1);
        a0 = fmaf(w, f0, a0);
        a1 = fmaf(w, f1, a1);
      }
    }
    if (on) store2(out + (size_t)gq * C + c0, a0, a1);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void vts_bwd_kernel(const float* __restrict__ query_xy, const float* __restrict__ vis_xy,
                                                     const T* __restrict__ feat, const int32_t* __restrict__ table,
                                                     const T* __restrict__ dout, int B, int Mq, int Nv, int C, Grid gr,
                                                     int Kt, float p, float eps, float* __restrict__ weights,
                                                     int32_t* __restrict__ pair_token, float* __restrict__ dquery,
                                                     float* __restrict__ dp_part) {
  const int lane = threadIdx.x & (kWave - 1);
  const long long gq = xcd_contiguous_block() * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (gq >= (long long)B * Mq) return;  // wave-uniform
  const int b = (int)(gq / Mq);
  const Cand cd = load_candidate(query_xy, vis_xy, table, b, gq, Nv, gr, Kt, p, eps, lane);
  // g_i = <dout, feat_i>: lanes <-> channels, then one wave reduction per candidate; lane i keeps g_i
  float g_mine = 0.f;
  for (int i = 0; i < Kt; ++i) {
    const int idx = __builtin_amdgcn_readlane(cd.idx, i);
    const T* f = feat + ((size_t)b * Nv + idx) * C;
    float part = 0.f;
    for (int c0 = 2 * lane; c0 < C; c0 += 2 * kWave) {
      float g0, g1, f0, f1;
      load2(dout + (size_t)gq * C + c0, g0, g1);
      load2(f + c0, f0, f1);
      part = fmaf(g0, f0, part);
      part = fmaf(g1, f1, part);
    }
    const float gi = wave_sum(part);
    if (lane == i) g_mine = gi;
  }
  // dz_i = w_i (g_i - sum_j w_j g_j) = w_i sum_j w_j (g_i - g_j): the differences are taken first.  When one weight
  // is close to 1 the first form subtracts two nearly equal numbers and leaves rounding noise of the size of
  // eps |g| where the true value is of the size of (1 - w_i) |g_i - g_j|.
  float spread = 0.f;
  for (int j = 0; j < Kt; ++j) {
    const float wj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(cd.w), j));
    const float gj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(g_mine), j));
    spread = fmaf(wj, g_mine - gj, spread);
  }
  const float dz = cd.w * spread;  // lanes >= Kt hold weight 0
  const float inv = cd.dist > 0.f ? 1.f / cd.dist : 0.f;
  const float qx = wave_sum(dz * (-p) * cd.dx * inv);
  const float qy = wave_sum(dz * (-p) * cd.dy * inv);
  // sum_i dz_i (-(d_i + eps)) with sum_i dz_i = 0: the distances are taken relative to the nearest candidate's, so
  // that the sum does not cancel terms of the size of |dz| d against a result of the size of |dz| (d_i - d_j)
  const float dnear = -wave_max(lane < Kt ? -cd.dist : -INFINITY);
  const float dpv = wave_sum(lane < Kt ? dz * (dnear - cd.dist) : 0.f);
  if (lane < Kt) {
    weights[(size_t)gq * Kt + lane] = cd.w;
    pair_token[(size_t)gq * Kt + lane] = b * Nv + cd.idx;
  }
  if (lane == 0) {
    dquery[2 * (size_t)gq] = qx;
    dquery[2 * (size_t)gq + 1] = qy;
    if (dp_part) dp_part[gq] = dpv;
  }
}

// ---- several queries per wave --------------------------------------------------------------------------------
// A row of C channels is moved 16 bytes per lane; when Kt <= 16 a group of 16 lanes (of 4 when Kt <= 4) serves
// one query (lane l of the group holds candidate l), so a wave carries 4 (16) independent chains of dependent
// loads (query -> table row -> token coordinates -> feature rows) instead of one, and the per-query arithmetic
// (cell, distances, weights) is spread over the lanes instead of repeated by all of them.  Needs rows that are
// whole 16-byte pieces.
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  const f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}
template <typename T>
struct Piece;  // 16 bytes of channels
template <>
struct Piece<float> {
  static constexpr int kCh = 4;
  static __device__ __forceinline__ void load(const float* p, float (&v)[8]) {
    const float4 x = *reinterpret_cast<const float4*>(p);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <>
struct Piece<bf16_t> {
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
    uint4 x;  // round to nearest even, two values per conversion instruction
    x.x = pack2_bf16(v[0], v[1]);
    x.y = pack2_bf16(v[2], v[3]);
    x.z = pack2_bf16(v[4], v[5]);
    x.w = pack2_bf16(v[6], v[7]);
    *reinterpret_cast<uint4*>(p) = x;
  }
};

// A group of G lanes (4 or 16) serves one query: lane l of the group holds candidate l and moves every G-th
// 16-byte piece of a row, so the lanes of a group read G x 16 contiguous bytes per load.  Reductions and
// broadcasts inside a group run on the VALU (DPP), not through LDS.
template <int CTRL>
__device__ __forceinline__ float dpp_movf(float x) {
  return __uint_as_float(dpp_mov<CTRL>(__float_as_uint(x)));
}
template <int G>
struct Group;
template <>
struct Group<16> {  // a DPP row: rotating it by 8, 4, 2 and 1 lanes leaves every lane with the reduction of all 16
  static __device__ __forceinline__ float max(float x) {
    x = fmaxf(x, dpp_movf<0x128>(x));  // row_ror:8
    x = fmaxf(x, dpp_movf<0x124>(x));  // row_ror:4
    x = fmaxf(x, dpp_movf<0x122>(x));  // row_ror:2
    x = fmaxf(x, dpp_movf<0x121>(x));  // row_ror:1
    return x;
  }
  static __device__ __forceinline__ float sum(float x) {
    x += dpp_movf<0x128>(x);
    x += dpp_movf<0x124>(x);
    x += dpp_movf<0x122>(x);
    x += dpp_movf<0x121>(x);
    return x;
  }
  template <int I0>
  static __device__ __forceinline__ void bcast4_at(uint32_t x, uint32_t (&out)[4]) {
    out[0] = dpp_mov<0x150 + I0 + 0>(x);  // row_newbcast: one lane of the row to all of them
    out[1] = dpp_mov<0x150 + I0 + 1>(x);
    out[2] = dpp_mov<0x150 + I0 + 2>(x);
    out[3] = dpp_mov<0x150 + I0 + 3>(x);
  }
  // out[u] = the value that lane i0 + u of the group holds, u = 0..3, i0 in {0, 4, 8, 12} (wave-uniform)
  static __device__ __forceinline__ void bcast4(uint32_t x, int i0, uint32_t (&out)[4]) {
    if (i0 == 0) bcast4_at<0>(x, out);
    else if (i0 == 4) bcast4_at<4>(x, out);
    else if (i0 == 8) bcast4_at<8>(x, out);
    else bcast4_at<12>(x, out);
  }
};
template <>
struct Group<4> {  // a DPP quad
  static __device__ __forceinline__ float max(float x) {
    x = fmaxf(x, dpp_movf<0xB1>(x));  // quad_perm [1,0,3,2]
    x = fmaxf(x, dpp_movf<0x4E>(x));  // quad_perm [2,3,0,1]
    return x;
  }
  static __device__ __forceinline__ float sum(float x) {
    x += dpp_movf<0xB1>(x);
    x += dpp_movf<0x4E>(x);
    return x;
  }
  static __device__ __forceinline__ void bcast4(uint32_t x, int, uint32_t (&out)[4]) {  // i0 is always 0
    out[0] = dpp_mov<0x00>(x);
    out[1] = dpp_mov<0x55>(x);
    out[2] = dpp_mov<0xAA>(x);
    out[3] = dpp_mov<0xFF>(x);
  }
};

// Candidate of lane (lane % G) for the group's query; every lane of the wave runs this (queries past the end
// repeat the last one and are not stored).
template <int G>
__device__ __forceinline__ Cand load_candidate_g(const float* __restrict__ query_xy, const float* __restrict__ vis_xy,
                                                 const int32_t* __restrict__ table, int b, int gq, int Nv,
                                                 const Grid& gr, int Kt, float p, float eps, int sub) {
  const float2 qxy = *reinterpret_cast<const float2*>(query_xy + 2 * (size_t)gq);
  const float qx = qxy.x, qy = qxy.y;
  const int ix = cell_of(qx, gr.x0, gr.cell, gr.Wg), iy = cell_of(qy, gr.y0, gr.cell, gr.Hg);
  const int cell = (b * gr.Hg + iy) * gr.Wg + ix;  // < 2^31 cells
  const int32_t* row = table + (size_t)cell * Kt;
  Cand c;
  const bool on = sub < Kt;
  c.idx = on ? min(max(row[sub], 0), Nv - 1) : 0;
  const float2 x = *reinterpret_cast<const float2*>(vis_xy + 2 * (size_t)(b * Nv + c.idx));
  c.dx = qx - x.x;
  c.dy = qy - x.y;
  c.dist = sqrtf(c.dx * c.dx + c.dy * c.dy);  // correctly rounded: an error of d is multiplied by p in the exponent
  const float z = on ? -p * (c.dist + eps) : -INFINITY;
  const float zmax = Group<G>::max(z);
  const float e = on ? __expf(z - zmax) : 0.f;
  c.w = e * __builtin_amdgcn_rcpf(Group<G>::sum(e));  // the sum is in [1, Kt]
  return c;
}

// The query of this lane's group (clamped to the last one) and its image.  The wave's first query is divided by
// Mq on the scalar unit; a wave spans at most 16 queries, so with Mq >= 16 the image index moves on at most once.
struct QueryOfLane {
  int gq, b;
  bool live;
};
template <int G>
__device__ __forceinline__ QueryOfLane query_of_lane(int B, int Mq, int lane) {
  constexpr int QW = kWave / G;  // queries per wave
  const int total = B * Mq;      // < 2^31
  const long long wave_id = xcd_contiguous_block() * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const long long wave_first = wave_id * QW;
  QueryOfLane q;
  q.live = wave_first + lane / G < total;
  q.gq = q.live ? (int)wave_first + lane / G : total - 1;
  if (Mq >= QW) {
    const int first = (int)min(wave_first, (long long)total - 1);
    const int b0 = first / Mq;  // wave-uniform
    q.b = b0 + (q.gq - b0 * Mq >= Mq ? 1 : 0);
  } else {
    q.b = q.gq / Mq;
  }
  return q;
}

template <typename T, int G>
__global__ __launch_bounds__(256) void vts_fwdg_kernel(const float* __restrict__ query_xy,
                                                      const float* __restrict__ vis_xy, const T* __restrict__ feat,
                                                      const int32_t* __restrict__ table, int B, int Mq, int Nv, int C,
                                                      Grid gr, int Kt, float p, float eps, T* __restrict__ out) {
  constexpr int CH = Piece<T>::kCh;
  const int lane = threadIdx.x & (kWave - 1), sub = lane & (G - 1);
  const QueryOfLane ql = query_of_lane<G>(B, Mq, lane);
  const Cand cd = load_candidate_g<G>(query_xy, vis_xy, table, ql.b, ql.gq, Nv, gr, Kt, p, eps, sub);
  const int pieces = C / CH;  // rows are whole 16-byte pieces
  const T* rows = feat + (size_t)ql.b * Nv * C;
  T* orow = out + (size_t)ql.gq * C;
  for (int p0 = 0; p0 < pieces; p0 += G) {  // wave-uniform trips
    const bool on = ql.live && p0 + sub < pieces;
    const int c0 = min(p0 + sub, pieces - 1) * CH;  // lanes past the row's end repeat its last piece: all loads are valid
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // four candidates per trip, their rows in flight together (past Kt: the trip's first one again, at weight 0)
    for (int i0 = 0; i0 < Kt; i0 += 4) {
      uint32_t wb[4], ib[4];
      Group<G>::bcast4(__float_as_uint(cd.w), i0, wb);
      Group<G>::bcast4((uint32_t)cd.idx, i0, ib);
      float f[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t idx = i0 + u < Kt ? ib[u] : ib[0];
        Piece<T>::load(rows + (size_t)(idx * (uint32_t)C) + c0, f[u]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float w = i0 + u < Kt ? __uint_as_float(wb[u]) : 0.f;
#pragma unroll
        for (int e = 0; e < CH; ++e) acc[e] = fmaf(w, f[u][e], acc[e]);
      }
    }
    if (on) Piece<T>::store(orow + c0, acc);
  }
}

template <typename T, int G>
__global__ __launch_bounds__(256) void vts_bwdg_kernel(const float* __restrict__ query_xy,
                                                      const float* __restrict__ vis_xy, const T* __restrict__ feat,
                                                      const int32_t* __restrict__ table, const T* __restrict__ dout,
                                                      int B, int Mq, int Nv, int C, Grid gr, int Kt, float p, float eps,
                                                      float* __restrict__ weights, int32_t* __restrict__ pair_token,
                                                      float* __restrict__ dquery, float* __restrict__ dp_part) {
  constexpr int CH = Piece<T>::kCh;
  const int lane = threadIdx.x & (kWave - 1), sub = lane & (G - 1);
  const QueryOfLane ql = query_of_lane<G>(B, Mq, lane);
  const int gq = ql.gq, b = ql.b;
  const Cand cd = load_candidate_g<G>(query_xy, vis_xy, table, b, gq, Nv, gr, Kt, p, eps, sub);
  const int pieces = C / CH;  // rows are whole 16-byte pieces
  const T* rows = feat + (size_t)b * Nv * C;
  const T* grow = dout + (size_t)gq * C;
  float g_mine = 0.f;
  // four candidates per trip, their rows in flight together (past Kt: the trip's first one again, result unused)
  for (int i0 = 0; i0 < Kt; i0 += 4) {
    uint32_t ib[4];
    Group<G>::bcast4((uint32_t)cd.idx, i0, ib);
    float part[4] = {0.f, 0.f, 0.f, 0.f};
    for (int p0 = 0; p0 < pieces; p0 += G) {
      const bool on = p0 + sub < pieces;
      const int c0 = min(p0 + sub, pieces - 1) * CH;  // lanes past the row's end repeat its last piece, unused
      float g[8], f[4][8];
      Piece<T>::load(grow + c0, g);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t idx = i0 + u < Kt ? ib[u] : ib[0];
        Piece<T>::load(rows + (size_t)(idx * (uint32_t)C) + c0, f[u]);
      }
      if (on) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int e = 0; e < CH; ++e) part[u] = fmaf(g[e], f[u][e], part[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float gi = Group<G>::sum(part[u]);
      if (sub == i0 + u && sub < Kt) g_mine = gi;
    }
  }
  // dz_i = w_i (g_i - sum_j w_j g_j) = w_i sum_j w_j (g_i - g_j), the differences taken first: when one weight is
  // close to 1, g_i minus the weighted mean cancels to rounding noise of the size of eps |g|, while the true value is
  // of the size of (1 - w_i) |g_i - g_j|.  Lanes past Kt hold weight 0 and add nothing.
  float spread = 0.f;
  for (int i0 = 0; i0 < Kt; i0 += 4) {
    uint32_t wb[4], gb[4];
    Group<G>::bcast4(__float_as_uint(cd.w), i0, wb);
    Group<G>::bcast4(__float_as_uint(g_mine), i0, gb);
#pragma unroll
    for (int u = 0; u < 4; ++u) spread = fmaf(__uint_as_float(wb[u]), g_mine - __uint_as_float(gb[u]), spread);
  }
  const float dz = cd.w * spread;
  const float inv = cd.dist > 0.f ? __builtin_amdgcn_rcpf(cd.dist) : 0.f;
  const float qx = Group<G>::sum(dz * (-p) * cd.dx * inv);
  const float qy = Group<G>::sum(dz * (-p) * cd.dy * inv);
  // sum_i dz_i (-(d_i + eps)) with sum_i dz_i = 0: distances relative to the nearest candidate's, so that the sum
  // does not cancel terms of the size of |dz| d against a result of the size of |dz| (d_i - d_j)
  const float dnear = -Group<G>::max(sub < Kt ? -cd.dist : -INFINITY);
  const float dpv = Group<G>::sum(sub < Kt ? dz * (dnear - cd.dist) : 0.f);
  if (ql.live && sub < Kt) {
    weights[(size_t)gq * Kt + sub] = cd.w;
    pair_token[(size_t)gq * Kt + sub] = b * Nv + cd.idx;
  }
  if (ql.live && sub == 0) *reinterpret_cast<float2*>(dquery + 2 * (size_t)gq) = make_float2(qx, qy);
  if (dp_part) {  // one part per wave (0 from a wave past the end)
    const float wave_part = wave_sum(ql.live && sub == 0 ? dpv : 0.f);
    const long long wave_id = xcd_contiguous_block() * 4 + threadIdx.x / kWave;
    if (lane == 0) dp_part[wave_id] = wave_part;
  }
}

// dp = sum of the per-query parts in a fixed order, in two steps: workgroup j adds up parts [j per, (j + 1) per)
// into out[j]; a second launch with one workgroup adds up those sums.
constexpr int kDpPer = 16384;
__global__ __launch_bounds__(1024) void vts_dp_kernel(const float* __restrict__ part, size_t n, size_t per,
                                                      float* __restrict__ out) {
  __shared__ float acc[16];
  const size_t lo = (size_t)blockIdx.x * per, hi = min(n, lo + per);  // per is a multiple of 4 or the only block's n
  float s = 0.f;
  const size_t n4 = (hi - lo) / 4;  // the workspace slots are 256-byte aligned: whole 16-byte pieces first
  for (size_t i = threadIdx.x; i < n4; i += blockDim.x) {
    const float4 v = reinterpret_cast<const float4*>(part + lo)[i];
    s += (v.x + v.y) + (v.z + v.w);
  }
  for (size_t i = lo + n4 * 4 + threadIdx.x; i < hi; i += blockDim.x) s += part[i];
  s = wave_sum(s);
  if ((threadIdx.x & (kWave - 1)) == 0) acc[threadIdx.x / kWave] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int w = 0; w < 16; ++w) t += acc[w];
    out[blockIdx.x] = t;
  }
}

// Files every (query, candidate) pair in the list of its token, with no atomic on global memory.  A
// workgroup owns a range of at most kListRange tokens of one image; it walks all pairs of that image twice
// (they sit in L2): first it counts the pairs of each of its tokens in LDS (and the pairs of the image's earlier
// tokens), a prefix sum turns the counts into list starts (every image holds exactly pairs_per_image pairs,
// so the image's first list starts at a known place), then every pair takes the next free place of its list.
constexpr int kListThreads = 1024;
constexpr int kListRange = 4 * kListThreads;
// NP > 0: a thread keeps its NP 16-byte pieces of the pair array in registers between the two walks (the image's
// pairs must fit: NP * kListThreads pieces); NP == 0: it reads them again.
template <int NP>
__global__ __launch_bounds__(kListThreads) void vts_lists_kernel(const int32_t* __restrict__ pair_token, int B, int Nv,
                                                                 int pairs_per_image, int range, int ranges,
                                                                 int32_t* __restrict__ offset,
                                                                 int32_t* __restrict__ list) {
  __shared__ int32_t cnt[kListRange];
  __shared__ int32_t wave_total[kListThreads / kWave], wave_below[kListThreads / kWave];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int b = blockIdx.x / ranges, rg = blockIdx.x - b * ranges;
  const int t0 = rg * range;
  const int span = min(range, Nv - t0);  // >= 1: ranges = ceil(Nv / range)
  // the image's pairs [lo, hi), read 16 bytes at a time from the aligned place at or before lo (the slot of the
  // pair array is padded to 256 bytes, so the last piece may reach past hi but not past the slot)
  const int lo = b * pairs_per_image, hi = lo + pairs_per_image;
  const int a0 = lo & ~3;
  const int pieces = (hi - a0 + 3) >> 2;
  const int first = b * Nv + t0;
  int4 held[NP > 0 ? NP : 1];
  if constexpr (NP > 0) {
#pragma unroll
    for (int i = 0; i < NP; ++i)  // threads past the end repeat the last piece and skip it below
      held[i] = *reinterpret_cast<const int4*>(pair_token + a0 + 4 * min(tid + i * kListThreads, pieces - 1));
  }
  // fn(token, pair) for every pair of the image that this thread looks at
  auto each_pair = [&](auto&& fn) {
    auto piece = [&](const int4& v, int g4, bool in) {
      const int tok[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (in && g4 + j >= lo && g4 + j < hi) fn(tok[j], g4 + j);
    };
    if constexpr (NP > 0) {
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        const int k = tid + i * kListThreads;
        piece(held[i], a0 + 4 * k, k < pieces);
      }
    } else {
#pragma unroll 2
      for (int k = tid; k < pieces; k += kListThreads)
        piece(*reinterpret_cast<const int4*>(pair_token + a0 + 4 * k), a0 + 4 * k, true);
    }
  };
#pragma unroll
  for (int i = 0; i < 4; ++i) cnt[4 * tid + i] = 0;
  __syncthreads();
  int below = 0;
  each_pair([&](int tok, int) {
    const int rel = tok - first;
    below += rel < 0 ? 1 : 0;
    if ((unsigned)rel < (unsigned)span) atomicAdd(&cnt[rel], 1);
  });
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) below += __shfl_xor(below, o);
  __syncthreads();
  int c[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) c[i] = cnt[4 * tid + i];  // zero past the span
  const int mine = c[0] + c[1] + c[2] + c[3];
  int incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  if (lane == kWave - 1) wave_total[wave] = incl;
  if (lane == 0) wave_below[wave] = below;
  __syncthreads();
  int run = lo + incl - mine;
  for (int w = 0; w < kListThreads / kWave; ++w) run += wave_below[w] + (w < wave ? wave_total[w] : 0);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (4 * tid + i < span) offset[(size_t)first + 4 * tid + i] = run;
    cnt[4 * tid + i] = run;  // from here on: the next free place of the token's list
    run += c[i];
  }
  if (blockIdx.x == gridDim.x - 1 && tid == 0) offset[(size_t)B * Nv] = B * pairs_per_image;
  __syncthreads();
  each_pair([&](int tok, int pair) {
    const int rel = tok - first;
    if ((unsigned)rel < (unsigned)span) list[atomicAdd(&cnt[rel], 1)] = pair;
  });
}

// The same filing when the pairs come in groups of `gs` consecutive pairs (one group per anchor or per query) whose
// lowest and highest token are known (bounds[group] = (min, max), global token ids): a workgroup lists the groups
// that can hold a token of its range, kGroupCap groups of the image at a time, and walks only their pairs.  Groups
// that end before the range count as a whole for the range's first list start; those that begin before it and
// reach into it are among the listed ones.  With tokens stored along a space-filling curve a group spans a small
// part of the image, so a range walks a fraction of the image's pairs instead of all of them.
constexpr int kGroupCap = 8192;  // groups of one image that a workgroup lists at a time
__global__ __launch_bounds__(kListThreads) void pair_lists_grouped_kernel(
    const int32_t* __restrict__ pair_token, const int2* __restrict__ bounds, int B, int Nv, int groups, int gs,
    uint32_t gs_magic, int range, int ranges, int32_t* __restrict__ offset, int32_t* __restrict__ list) {
  __shared__ int32_t cnt[kListRange];
  __shared__ int32_t glist[kGroupCap];
  __shared__ int32_t wave_total[kListThreads / kWave], wave_below[kListThreads / kWave];
  __shared__ int32_t s_listed, s_whole;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int b = blockIdx.x / ranges, rg = blockIdx.x - b * ranges;
  const int t0 = rg * range;
  const int span = min(range, Nv - t0);  // >= 1: ranges = ceil(Nv / range)
  const int first = b * Nv + t0, end = first + span;
  const int lo = b * groups * gs;  // the image's first pair
  if (tid == 0) s_whole = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) cnt[4 * tid + i] = 0;
  // fn(token, pair) for every pair of the groups [g0, g0 + kGroupCap) that reach into the range; `whole` counts the
  // groups that end before it
  int whole = 0;
  auto each_pair = [&](int g0, bool count_whole, auto&& fn) {
    __syncthreads();  // the previous list has been walked (and, the first time, cnt / s_whole are set)
    if (tid == 0) s_listed = 0;
    __syncthreads();
    const int g1 = min(g0 + kGroupCap, groups);
    for (int g = g0 + tid; g < g1; g += kListThreads) {
      const int2 bd = bounds[(size_t)b * groups + g];
      if (bd.y < first) whole += count_whole ? 1 : 0;
      else if (bd.x < end) glist[atomicAdd(&s_listed, 1)] = g;
    }
    __syncthreads();
    const int items = s_listed * gs;
    for (int i = tid; i < items; i += kListThreads) {
      const int gi = exact_div(i, gs, gs_magic);
      const int pair = lo + glist[gi] * gs + (i - gi * gs);
      fn(pair_token[pair], pair);
    }
  };
  int below = 0;
  for (int g0 = 0; g0 < groups; g0 += kGroupCap)
    each_pair(g0, true, [&](int tok, int) {
      const int rel = tok - first;
      below += rel < 0 ? 1 : 0;
      if ((unsigned)rel < (unsigned)span) atomicAdd(&cnt[rel], 1);
    });
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    below += __shfl_xor(below, o);
    whole += __shfl_xor(whole, o);
  }
  if (lane == 0 && whole) atomicAdd(&s_whole, whole);
  __syncthreads();
  int c[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) c[i] = cnt[4 * tid + i];  // zero past the span
  const int mine = c[0] + c[1] + c[2] + c[3];
  int incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  if (lane == kWave - 1) wave_total[wave] = incl;
  if (lane == 0) wave_below[wave] = below;
  __syncthreads();
  int run = lo + s_whole * gs + incl - mine;
  for (int w = 0; w < kListThreads / kWave; ++w) run += wave_below[w] + (w < wave ? wave_total[w] : 0);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (4 * tid + i < span) offset[(size_t)first + 4 * tid + i] = run;
    cnt[4 * tid + i] = run;  // from here on: the next free place of the token's list
    run += c[i];
  }
  if (blockIdx.x == gridDim.x - 1 && tid == 0) offset[(size_t)B * Nv] = B * groups * gs;
  for (int g0 = 0; g0 < groups; g0 += kGroupCap)
    each_pair(g0, false, [&](int tok, int pair) {
      const int rel = tok - first;
      if ((unsigned)rel < (unsigned)span) list[atomicAdd(&cnt[rel], 1)] = pair;
    });
}

// Four visible tokens per wave (16 lanes each) when the rows are whole 16-byte pieces: dfeat = sum over the
// token's pairs of w * dout[query]; with `extra`, also extra_sum[token] = sum over the same pairs of extra[pair].
template <typename T>
__global__ __launch_bounds__(256) void vts_dfeat16_kernel(const T* __restrict__ dout, const float* __restrict__ weights,
                                                         const int32_t* __restrict__ offset,
                                                         const int32_t* __restrict__ list, int tokens, int C, int Kt,
                                                         T* __restrict__ dfeat, const float* __restrict__ extra,
                                                         float* __restrict__ extra_sum) {
  constexpr int CH = Piece<T>::kCh;
  const int lane = threadIdx.x & (kWave - 1), sub = lane & 15;
  const long long want = (xcd_contiguous_block() * 4 + threadIdx.x / kWave) * 4 + (lane >> 4);
  const bool live = want < tokens;
  const long long tok = live ? want : tokens - 1;
  const int lo = offset[tok], n = live ? offset[tok + 1] - lo : 0;
  // the longest list of the wave's four tokens sets the (wave-uniform) trip count of the pair loop
  int nmax = n;
  nmax = max(nmax, __shfl_xor(nmax, 16));
  nmax = max(nmax, __shfl_xor(nmax, 32));
  float xsum = 0.f;
  for (int base = 0; base < C; base += 16 * CH) {
    const int c0 = base + sub * CH;
    const bool on = live && c0 < C;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int chunk = 0; chunk < nmax; chunk += 16) {
      const bool have = chunk + sub < n;
      // places past the end of a list repeat its last pair at weight 0 (an empty list: pair 0)
      const int mine = n > 0 ? list[lo + min(chunk + sub, n - 1)] : 0;
      const float wmine = have ? weights[mine] : 0.f;
      if (extra && base == 0 && have) xsum += extra[mine];
      const int qmine = mine / Kt;
      const int m = min(16, nmax - chunk);
      // four pairs per trip, their rows in flight together
      for (int i0 = 0; i0 < m; i0 += 4) {
        float w[4];
        int q[4];
        {
          uint32_t wb[4], qb[4];
          Group<16>::bcast4(__float_as_uint(wmine), i0, wb);
          Group<16>::bcast4((uint32_t)qmine, i0, qb);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            w[u] = __uint_as_float(wb[u]);
            q[u] = (int)qb[u];
          }
        }
        if (on) {
          float g[4][8];
#pragma unroll
          for (int u = 0; u < 4; ++u) Piece<T>::load(dout + (size_t)q[u] * C + c0, g[u]);
#pragma unroll
          for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < CH; ++e) acc[e] = fmaf(w[u], g[u][e], acc[e]);
        }
      }
    }
    if (on) Piece<T>::store(dfeat + (size_t)tok * C + c0, acc);
  }
  if (extra) {  // wave-uniform
    xsum = Group<16>::sum(xsum);
    if (live && sub == 0) extra_sum[tok] = xsum;
  }
}

// One wave per visible token: dfeat = sum over the token's pairs of w * dout[query] (and extra_sum, as above).
template <typename T>
__global__ __launch_bounds__(256) void vts_dfeat_kernel(const T* __restrict__ dout, const float* __restrict__ weights,
                                                       const int32_t* __restrict__ offset,
                                                       const int32_t* __restrict__ list, int tokens, int C, int Kt,
                                                       T* __restrict__ dfeat, const float* __restrict__ extra,
                                                       float* __restrict__ extra_sum) {
  const int lane = threadIdx.x & (kWave - 1);
  const long long tok = xcd_contiguous_block() * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (tok >= tokens) return;  // wave-uniform
  const int lo = offset[tok], n = offset[tok + 1] - lo;
  float xsum = 0.f;
  for (int base = 0; base < C; base += 2 * kWave) {  // wave-uniform trips; only the memory accesses are predicated
    const int c0 = base + 2 * lane;
    const bool on = c0 < C;
    float a0 = 0.f, a1 = 0.f;
    for (int chunk = 0; chunk < n; chunk += kWave) {
      const int m = min(kWave, n - chunk);
      const int mine = lane < m ? list[lo + chunk + lane] : 0;
      float wmine = lane < m ? weights[mine] : 0.f;
      if (extra && base == 0 && lane < m) xsum += extra[mine];
      int qmine = mine / Kt;
      asm volatile("" : "+v"(wmine), "+v"(qmine));  // broadcast below: computed here with every lane active
      for (int i = 0; i < m; ++i) {
        const float w = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(wmine), i));
        const int q = __builtin_amdgcn_readlane(qmine, i);
        if (on) {
          float g0, g1;
          load2(dout + (size_t)q * C + c0, g0, g1);
          a0 = fmaf(w, g0, a0);
          a1 = fmaf(w, g1, a1);
        }
      }
    }
    if (on) store2(dfeat + (size_t)tok * C + c0, a0, a1);
  }
  if (extra) {  // wave-uniform
    xsum = wave_sum(xsum);
    if (lane == 0) extra_sum[tok] = xsum;
  }
}

}  // namespace

hipError_t launch_vts_table(const VtsArgs& a, hipStream_t stream) {
  const Grid gr = {a.Hg, a.Wg, a.x0, a.y0, a.cell};
  const long long cells = (long long)a.B * a.Hg * a.Wg;
  const size_t grid_lds = (size_t)((a.Hg * a.Wg + 1) & ~1) * 4 + (size_t)a.Nv * 12;
  if (a.Kt <= 8 && (long long)a.Hg * a.Wg <= 16384 && grid_lds <= (size_t)kGridLdsBytes &&
      reinterpret_cast<uintptr_t>(a.vis_xy) % 8 == 0) {
    // first window: about twice Kt tokens expected inside at the image's mean density
    const int per_image = a.Hg * a.Wg;
    int r0 = 1;
    while ((2ll * r0 + 1) * (2 * r0 + 1) * a.Nv < 2ll * a.Kt * per_image && r0 < 64) ++r0;
    const int slabs = (per_image + kGridThreads - 1) / kGridThreads;
    const dim3 grid((unsigned)(a.B * slabs));
    if (a.Kt <= 4)
      AFFMAE_LAUNCH("vts_table_kernel", stream, vts_table_grid_kernel<4>, grid, dim3(kGridThreads), grid_lds, stream,
                    a.vis_xy, a.B, a.Nv, gr, a.Kt, r0, slabs, a.table_out);
    else
      AFFMAE_LAUNCH("vts_table_kernel", stream, vts_table_grid_kernel<8>, grid, dim3(kGridThreads), grid_lds, stream,
                    a.vis_xy, a.B, a.Nv, gr, a.Kt, r0, slabs, a.table_out);
    return hipGetLastError();
  }
  if (a.Nv <= kTableRows * kWave) {
    const long long runs = (long long)a.B * ((a.Hg * a.Wg + kTableRun - 1) / kTableRun);
    AFFMAE_LAUNCH("vts_table_kernel", stream, vts_table_fast_kernel, dim3((unsigned)((runs + 3) / 4)), dim3(256), 0,
                  stream, a.vis_xy, a.B, a.Nv, gr, a.Kt, a.table_out);
    return hipGetLastError();
  }
  AFFMAE_LAUNCH("vts_table_kernel", stream, vts_table_kernel, dim3((unsigned)((cells + 3) / 4)), dim3(256), 0, stream,
                a.vis_xy, a.B, a.Nv, gr, a.Kt, a.table_out);
  return hipGetLastError();
}

// Four queries per wave when a group of 16 lanes can hold the candidates and the rows are whole 16-byte pieces.
static bool vts_grouped(const VtsArgs& a, const void* t0, const void* t1, const void* t2) {
  const size_t row = (size_t)a.C * (a.dtype == 1 ? 2 : 4);
  auto al = [](const void* p) { return p == nullptr || reinterpret_cast<uintptr_t>(p) % 16 == 0; };
  auto al8 = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 8 == 0; };  // (x, y) pairs are moved whole
  if ((long long)a.Nv * a.C >= (1ll << 31)) return false;                             // 32-bit offsets inside an image
  return a.Kt <= 16 && row % 16 == 0 && al(t0) && al(t1) && al8(t2) && al8(a.query_xy) && al8(a.vis_xy);
}

hipError_t launch_vts_fwd(const VtsArgs& a, hipStream_t stream) {
  const Grid gr = {a.Hg, a.Wg, a.x0, a.y0, a.cell};
  if (vts_grouped(a, a.feat, a.out, nullptr)) {
    // groups of 4 lanes (16 queries per wave) when they can hold the candidates, else groups of 16
    const long long total = (long long)a.B * a.Mq;
    const bool quad = a.Kt <= 4;
    const int per_block = quad ? 64 : 16;
    const dim3 gridg(round_up8((total + per_block - 1) / per_block));
#define AFFMAE_VTS_FWDG(T, G)                                                                                     \
  AFFMAE_LAUNCH("vts_fwd_kernel", stream, (vts_fwdg_kernel<T, G>), gridg, dim3(256), 0, stream, a.query_xy,       \
                a.vis_xy, (const T*)a.feat, a.table, a.B, a.Mq, a.Nv, a.C, gr, a.Kt, a.p, a.eps, (T*)a.out)
    if (a.dtype == 1 && quad) AFFMAE_VTS_FWDG(bf16_t, 4);
    else if (a.dtype == 1) AFFMAE_VTS_FWDG(bf16_t, 16);
    else if (quad) AFFMAE_VTS_FWDG(float, 4);
    else AFFMAE_VTS_FWDG(float, 16);
#undef AFFMAE_VTS_FWDG
    return hipGetLastError();
  }
  const dim3 grid(round_up8(((long long)a.B * a.Mq + 3) / 4));
  if (a.dtype == 1)
    AFFMAE_LAUNCH("vts_fwd_kernel", stream, vts_fwd_kernel<bf16_t>, grid, dim3(256), 0, stream, a.query_xy, a.vis_xy,
                  (const bf16_t*)a.feat, a.table, a.B, a.Mq, a.Nv, a.C, gr, a.Kt, a.p, a.eps, (bf16_t*)a.out);
  else
    AFFMAE_LAUNCH("vts_fwd_kernel", stream, vts_fwd_kernel<float>, grid, dim3(256), 0, stream, a.query_xy, a.vis_xy,
                  (const float*)a.feat, a.table, a.B, a.Mq, a.Nv, a.C, gr, a.Kt, a.p, a.eps, (float*)a.out);
  return hipGetLastError();
}

namespace {
struct VtsBwdLayout {
  size_t weights_off, pair_off, offset_off, list_off, dp_off, dp2_off, total;
};
size_t vts_align(size_t n) { return (n + 255) / 256 * 256; }
size_t vts_dp_blocks(int B, int Mq) { return ((size_t)B * Mq + kDpPer - 1) / kDpPer; }
VtsBwdLayout vts_bwd_layout(int B, int Mq, int Nv, int Kt) {
  VtsBwdLayout L;
  const size_t pairs = (size_t)B * Mq * Kt, tokens = (size_t)B * Nv;
  size_t off = 0;
  L.weights_off = off; off += vts_align(pairs * sizeof(float));
  L.pair_off = off;    off += vts_align(pairs * sizeof(int32_t));
  L.offset_off = off;  off += vts_align((tokens + 1) * sizeof(int32_t));
  L.list_off = off;    off += vts_align(pairs * sizeof(int32_t));
  L.dp_off = off;      off += vts_align(((size_t)B * Mq + 64) * sizeof(float));  // per query, or per wave (+ grid padding)
  L.dp2_off = off;     off += vts_align(vts_dp_blocks(B, Mq) * sizeof(float));
  L.total = off;
  return L;
}
}  // namespace

size_t vts_bwd_workspace_bytes(int B, int Mq, int Nv, int Kt) { return vts_bwd_layout(B, Mq, Nv, Kt).total; }

hipError_t launch_vts_bwd(const VtsArgs& a, hipStream_t stream) {
  const Grid gr = {a.Hg, a.Wg, a.x0, a.y0, a.cell};
  const dim3 grid(round_up8(((long long)a.B * a.Mq + 3) / 4));
  const VtsBwdLayout L = vts_bwd_layout(a.B, a.Mq, a.Nv, a.Kt);
  char* ws = static_cast<char*>(a.workspace);
  float* weights = reinterpret_cast<float*>(ws + L.weights_off);
  int32_t* pair_token = reinterpret_cast<int32_t*>(ws + L.pair_off);
  int32_t* offset = reinterpret_cast<int32_t*>(ws + L.offset_off);
  int32_t* list = reinterpret_cast<int32_t*>(ws + L.list_off);
  float* dp_part = a.dp ? reinterpret_cast<float*>(ws + L.dp_off) : nullptr;
  float* dp_part2 = reinterpret_cast<float*>(ws + L.dp2_off);
  const size_t tokens = (size_t)a.B * a.Nv;
  const bool grouped = vts_grouped(a, a.feat, a.dout, a.dquery);
  const bool quad = a.Kt <= 4;
  const int per_block = quad ? 64 : 16;
  const dim3 gridg(round_up8(((long long)a.B * a.Mq + per_block - 1) / per_block));
#define AFFMAE_VTS_BWDG(T, G)                                                                                      \
  AFFMAE_LAUNCH("vts_bwd_kernel", stream, (vts_bwdg_kernel<T, G>), gridg, dim3(256), 0, stream, a.query_xy,        \
                a.vis_xy, (const T*)a.feat, a.table, (const T*)a.dout, a.B, a.Mq, a.Nv, a.C, gr, a.Kt, a.p, a.eps, \
                weights, pair_token, a.dquery, dp_part)
  if (grouped && a.dtype == 1 && quad) AFFMAE_VTS_BWDG(bf16_t, 4);
  else if (grouped && a.dtype == 1) AFFMAE_VTS_BWDG(bf16_t, 16);
  else if (grouped && quad) AFFMAE_VTS_BWDG(float, 4);
  else if (grouped) AFFMAE_VTS_BWDG(float, 16);
#undef AFFMAE_VTS_BWDG
  else if (a.dtype == 1)
    AFFMAE_LAUNCH("vts_bwd_kernel", stream, vts_bwd_kernel<bf16_t>, grid, dim3(256), 0, stream, a.query_xy, a.vis_xy,
                  (const bf16_t*)a.feat, a.table, (const bf16_t*)a.dout, a.B, a.Mq, a.Nv, a.C, gr, a.Kt, a.p, a.eps,
                  weights, pair_token, a.dquery, dp_part);
  else
    AFFMAE_LAUNCH("vts_bwd_kernel", stream, vts_bwd_kernel<float>, grid, dim3(256), 0, stream, a.query_xy, a.vis_xy,
                  (const float*)a.feat, a.table, (const float*)a.dout, a.B, a.Mq, a.Nv, a.C, gr, a.Kt, a.p, a.eps,
                  weights, pair_token, a.dquery, dp_part);
  if (a.dp) {
    // parts: one per wave of the grouped kernels, one per query otherwise
    const size_t n = grouped ? (size_t)gridg.x * 4 : (size_t)a.B * a.Mq;
    const hipError_t e = launch_sum_parts(dp_part, n, dp_part2, a.dp, stream);
    if (e != hipSuccess) return e;
  }
  const hipError_t e = launch_pair_lists(pair_token, a.B, a.Nv, a.Mq * a.Kt, offset, list, stream);
  if (e != hipSuccess) return e;
  const bool pieces = vts_grouped(a, a.dout, a.dfeat, nullptr);  // (Kt <= 16 is not needed here, only the row shape)
  return launch_pair_gather(a.dout, weights, offset, list, tokens, a.C, a.Kt, a.dtype, a.dfeat, pieces, stream);
}

// out = sum of part[0..n) in a fixed order (part2: room for ceil(n / 16384) floats).
size_t sum_parts_scratch_floats(size_t n) { return (n + kDpPer - 1) / kDpPer; }
hipError_t launch_sum_parts(const float* part, size_t n, float* part2, float* out, hipStream_t stream) {
  const size_t blocks = (n + kDpPer - 1) / kDpPer;
  if (blocks <= 8) {  // up to 128 values per thread: one workgroup is quicker than a second launch
    AFFMAE_LAUNCH("vts_dp_kernel", stream, vts_dp_kernel, dim3(1), dim3(1024), 0, stream, part, n, n, out);
  } else {
    AFFMAE_LAUNCH("vts_dp_kernel", stream, vts_dp_kernel, dim3((unsigned)blocks), dim3(1024), 0, stream, part, n,
                  (size_t)kDpPer, part2);
    AFFMAE_LAUNCH("vts_dp_kernel", stream, vts_dp_kernel, dim3(1), dim3(1024), 0, stream, part2, blocks, blocks, out);
  }
  return hipGetLastError();
}

// Files pairs per token: pair_token[b * pairs_per_image + i] = the (global, b * Nv + t) token of pair i of image b
// -> offset [B * Nv + 1] (start of every token's list) and list [B * pairs_per_image] (pair ids grouped by token).
// group_bounds (optional): [B * pairs_per_image / group_size][2], the lowest and highest token of every run of
// group_size consecutive pairs.
hipError_t launch_pair_lists(const int32_t* pair_token, int B, int Nv, int pairs_per_image, int32_t* offset,
                             int32_t* list, hipStream_t stream, const int32_t* group_bounds, int group_size) {
  if (group_bounds && group_size >= 1 && pairs_per_image % group_size == 0) {
    // a range walks only the groups that reach into it: many small ranges cost little
    const int groups = pairs_per_image / group_size;
    const int want = (512 + B - 1) / B;
    int range = std::max(64, (Nv + want - 1) / want);
    range = std::min(range, kListRange);
    const int ranges = (Nv + range - 1) / range;
    AFFMAE_LAUNCH("vts_lists_kernel", stream, pair_lists_grouped_kernel, dim3((unsigned)(B * ranges)),
                  dim3(kListThreads), 0, stream, pair_token, reinterpret_cast<const int2*>(group_bounds), B, Nv, groups,
                  group_size, div_magic(group_size), range, ranges, offset, list);
    return hipGetLastError();
  }
  // token ranges per image: enough workgroups to fill the chip, never more tokens than the LDS counters hold
  const int want = (192 + B - 1) / B;
  int range = std::max(64, (Nv + want - 1) / want);
  range = std::min(range, kListRange);
  const int ranges = (Nv + range - 1) / range;
  const dim3 lgrid((unsigned)(B * ranges));
  const int ppi = pairs_per_image, pieces_max = (ppi + 3) / 4 + 1;  // + 1: an image may start inside a piece
#define AFFMAE_VTS_LISTS(NP)                                                                                         \
  AFFMAE_LAUNCH("vts_lists_kernel", stream, vts_lists_kernel<NP>, lgrid, dim3(kListThreads), 0, stream, pair_token, \
                B, Nv, ppi, range, ranges, offset, list)
  if (pieces_max <= 4 * kListThreads) AFFMAE_VTS_LISTS(4);
  else if (pieces_max <= 9 * kListThreads) AFFMAE_VTS_LISTS(9);
  else AFFMAE_VTS_LISTS(0);
#undef AFFMAE_VTS_LISTS
  return hipGetLastError();
}

// dfeat[token] = sum over the token's pairs of weights[pair] * dout[pair / Kt]  (rows of C channels of `dtype`;
// `pieces`: rows are whole 16-byte pieces, 16-byte aligned, and every row offset fits 32 bits).  With `extra`
// (one value per pair), also extra_sum[token] = sum over the token's pairs of extra[pair].
hipError_t launch_pair_gather(const void* dout, const float* weights, const int32_t* offset, const int32_t* list,
                              size_t tokens, int C, int Kt, int dtype, void* dfeat, bool pieces, hipStream_t stream,
                              const float* extra, float* extra_sum) {
  if (pieces) {
    const dim3 per4(round_up8(((long long)tokens + 15) / 16));
    if (dtype == 1)
      AFFMAE_LAUNCH("vts_dfeat_kernel", stream, vts_dfeat16_kernel<bf16_t>, per4, dim3(256), 0, stream,
                    (const bf16_t*)dout, weights, offset, list, (int)tokens, C, Kt, (bf16_t*)dfeat, extra, extra_sum);
    else
      AFFMAE_LAUNCH("vts_dfeat_kernel", stream, vts_dfeat16_kernel<float>, per4, dim3(256), 0, stream,
                    (const float*)dout, weights, offset, list, (int)tokens, C, Kt, (float*)dfeat, extra, extra_sum);
    return hipGetLastError();
  }
  const dim3 per_token(round_up8(((long long)tokens + 3) / 4));
  if (dtype == 1)
    AFFMAE_LAUNCH("vts_dfeat_kernel", stream, vts_dfeat_kernel<bf16_t>, per_token, dim3(256), 0, stream,
                  (const bf16_t*)dout, weights, offset, list, (int)tokens, C, Kt, (bf16_t*)dfeat, extra, extra_sum);
  else
    AFFMAE_LAUNCH("vts_dfeat_kernel", stream, vts_dfeat_kernel<float>, per_token, dim3(256), 0, stream,
                  (const float*)dout, weights, offset, list, (int)tokens, C, Kt, (float*)dfeat, extra, extra_sum);
  return hipGetLastError();
}

}  // namespace affmae
