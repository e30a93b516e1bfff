// Batched clustered neighbour search (paper, Sec. "AutoFocusFormer": equal-size
// clusters, fixed-size neighbourhoods by nearest-neighbour search over 2-D token
// coordinates).  Four kernels:
//   members  (only with an explicit cluster_id): token lists per cluster
//   centroid : double-precision mean of each cluster's coordinates -> fp32
//   near     : per cluster the M clusters with nearest centroids
//   knn      : per token the K nearest among the members of those M clusters
//              (up to 512 candidates: kept in registers, selected by a counted
//              distance threshold and one sort; more: staged in LDS and merged)
// Selection is exact and unique: 64-bit keys (fp32 distance bits, index) compared
// as integers; distances are evaluated without fused multiply-add.  This file is
// compiled with -ffp-contract=off.
#include "device_util.h"
#include "launch.h"
#include "select_util.h"
#include "timing.h"

namespace affmae {
namespace {

// Clusters hold S tokens, except that the last one (cluster G - 1, G = ceil(N / S)) holds what is left.
__device__ __forceinline__ int cluster_size(int c, int N, int S, int G) { return c == G - 1 ? N - (G - 1) * S : S; }

// members[b, c*S + r] = r-th token (ascending) whose cluster id is c.  One
// workgroup per image; a thread owns a cluster and scans the id array, which is
// staged through LDS in chunks.  Slots that an invalid assignment leaves unset
// keep the in-range default c*S + r.
constexpr int kMemChunk = 2048;
__global__ __launch_bounds__(256) void members_kernel(const int32_t* __restrict__ cluster_id, int N, int S, int G,
                                                     int32_t* __restrict__ members) {
  __shared__ int32_t ids[kMemChunk];
  const int b = blockIdx.x;
  const int32_t* cid = cluster_id + (size_t)b * N;
  int32_t* mem = members + (size_t)b * N;
  for (int i = threadIdx.x; i < N; i += blockDim.x) mem[i] = i;
  __syncthreads();
  for (int c0 = 0; c0 < G; c0 += blockDim.x) {
    const int c = c0 + threadIdx.x;
    int count = 0;
    for (int base = 0; base < N; base += kMemChunk) {
      const int n = min(kMemChunk, N - base);
      __syncthreads();
      for (int t = threadIdx.x; t < n; t += blockDim.x) ids[t] = cid[base + t];
      __syncthreads();
      if (c < G) {
        for (int t = 0; t < n; ++t) {
          if (ids[t] == c && count < cluster_size(c, N, S, G)) {
            mem[(size_t)c * S + count] = base + t;
            ++count;
          }
        }
      }
    }
  }
}

// One wave per cluster: the lanes fetch the members' coordinates 64 at a time (coalesced), then every
// lane forms the same sequential double-precision sum in member order from lane broadcasts.
__global__ __launch_bounds__(256) void centroid_kernel(const float* __restrict__ coords,
                                                      const int32_t* __restrict__ members, int B, int N, int S,
                                                      int G, float* __restrict__ centroid) {
  const int lane = threadIdx.x & (kWave - 1);
  const int gc = blockIdx.x * (blockDim.x / kWave) + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (gc >= B * G) return;  // wave-uniform
  const int b = gc / G, c = gc % G;
  const float* xy = coords + (size_t)b * N * 2;
  double sx = 0.0, sy = 0.0;
  const int size = cluster_size(c, N, S, G);
  for (int base = 0; base < size; base += kWave) {
    const int n = min(kWave, size - base);
    float x = 0.f, y = 0.f;
    if (lane < n) {
      int tok = c * S + base + lane;
      if (members) tok = min(max(members[(size_t)b * N + tok], 0), N - 1);
      x = xy[2 * (size_t)tok];
      y = xy[2 * (size_t)tok + 1];
    }
    for (int r = 0; r < n; ++r) {
      sx += (double)__uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), r));
      sy += (double)__uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(y), r));
    }
  }
  if (lane == 0) {
    centroid[2 * (size_t)gc + 0] = (float)(sx / (double)size);
    centroid[2 * (size_t)gc + 1] = (float)(sy / (double)size);
  }
}

// One wave per cluster: the M nearest centroids of the image, ascending.
__global__ __launch_bounds__(256) void near_kernel(const float* __restrict__ centroid, int B, int G, int M,
                                                  int32_t* __restrict__ near) {
  const int lane = threadIdx.x & (kWave - 1);
  const int gc = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
  if (gc >= B * G) return;  // wave-uniform
  const int b = gc / G;
  const float* cen = centroid + (size_t)b * G * 2;
  const float cx = centroid[2 * (size_t)gc], cy = centroid[2 * (size_t)gc + 1];
  key_t best = kKeyMax;
  for (int base = 0; base < G; base += kWave) {
    const int e = base + lane;
    key_t key = kKeyMax;
    if (e < G) key = make_key(dist2(cx, cy, cen[2 * e], cen[2 * e + 1]), e);
    best = topk_push(best, key, lane, M - 1);
  }
  if (lane < M) near[(size_t)gc * M + lane] = (int32_t)(uint32_t)best;
}

// One workgroup per cluster.  The coordinates and token ids of the M*S candidate
// tokens are staged in LDS once; each wave then serves the cluster's tokens in
// turn.  The first 64 candidates (the nearest cluster's) are sorted to give a
// first bound on the K-th key; later candidates are compared against the
// current bound, 64 at a time, and only those below it are queued (compacted in
// a per-wave LDS buffer).  Whenever 64 are queued they are merged into the
// running top-64, which tightens the bound for what follows.  A candidate is
// dropped only when K smaller keys are already known, so the result is exact.
constexpr int kKnnWaves = 4;
__global__ __launch_bounds__(kKnnWaves* kWave) void knn_kernel(const float* __restrict__ coords,
                                                              const int32_t* __restrict__ members,
                                                              const int32_t* __restrict__ near, int N, int S, int M,
                                                              int K, int G, int32_t* __restrict__ nbr_idx) {
  extern __shared__ float4 cand[];  // x, y, token id (bits), unused
  __shared__ key_t pend_all[kKnnWaves][2 * kWave];
  const int b = blockIdx.x / G, c = blockIdx.x % G;
  const int Cn = M * S;
  const float* xy = coords + (size_t)b * N * 2;
  const int32_t* mem = members ? members + (size_t)b * N : nullptr;
  for (int p = threadIdx.x; p < Cn; p += blockDim.x) {
    const int m = p / S, r = p - m * S;
    int e = near[((size_t)b * G + c) * M + m];
    e = min(max(e, 0), G - 1);
    const bool real = r < cluster_size(e, N, S, G);  // a short last cluster fills only part of its places
    int tok = min(e * S + r, N - 1);
    if (mem) tok = min(max(mem[tok], 0), N - 1);
    cand[p] = make_float4(xy[2 * (size_t)tok], xy[2 * (size_t)tok + 1], __int_as_float(real ? tok : -1), 0.f);
  }
  __syncthreads();
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  key_t* pend = pend_all[wave];
  auto cand_key = [&](int p, float qx, float qy) -> key_t {
    if (p >= Cn) return kKeyMax;
    const float4 cp = cand[p];
    if (__float_as_int(cp.z) < 0) return kKeyMax;  // an empty place of a short cluster
    return make_key(dist2(qx, qy, cp.x, cp.y), __float_as_int(cp.z));
  };
  const int my_size = cluster_size(c, N, S, G);
  for (int r = wave; r < my_size; r += kKnnWaves) {
    int qtok = c * S + r;
    if (mem) qtok = min(max(mem[qtok], 0), N - 1);
    const float qx = xy[2 * (size_t)qtok], qy = xy[2 * (size_t)qtok + 1];
    key_t best = wave_sort(cand_key(lane, qx, qy), lane);
    key_t bound = shfl_key(best, K - 1);
    int fill = 0;  // queued keys, wave-uniform, always < 64 between rows
    for (int base = kWave; base < Cn; base += kWave) {
      const key_t key = cand_key(base + lane, qx, qy);
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
        best = topk_push(best, row, lane, K - 1);
        bound = shfl_key(best, K - 1);
      }
    }
    if (fill > 0) {
      wave_lds_sync();
      const key_t row = (lane < fill) ? pend[lane] : kKeyMax;
      best = topk_push(best, row, lane, K - 1);
    }
    wave_lds_sync();  // the next token's queue starts after this one's reads
    if (lane < K) nbr_idx[((size_t)b * N + qtok) * K + lane] = (int32_t)(uint32_t)best;
  }
}

// At most 512 candidates: each lane keeps its 8 candidates in registers for all of the
// cluster's tokens.  Per token the wave looks for a distance threshold T with
// K <= #{candidates with d2 <= T} <= 64 by counting (ballots), starting from the previous
// token's threshold and scaling it by the ratio of the wanted to the found count (the count grows
// like the area, i.e. like d2), then by bisection on the bit pattern.  Everything at or below T is
// closer than everything above it, so the K nearest are among the counted candidates: they are
// compacted into one row and sorted once by (d2, index).  When no such T exists (more than
// 64 - K + 1 candidates at one distance) the token takes the queue-and-merge route of the
// general kernel.  Either way the result is the exact, unique answer.
constexpr int kFastRows = 8;
__global__ __launch_bounds__(kKnnWaves* kWave) void knn_fast_kernel(const float* __restrict__ coords,
                                                                   const int32_t* __restrict__ members,
                                                                   const int32_t* __restrict__ near, int N, int S,
                                                                   int M, int K, int G,
                                                                   int32_t* __restrict__ nbr_idx) {
  __shared__ key_t pend_all[kKnnWaves][2 * kWave];
  const int b = blockIdx.x / G, c = blockIdx.x % G;
  const int Cn = M * S;
  const float* xy = coords + (size_t)b * N * 2;
  const int32_t* mem = members ? members + (size_t)b * N : nullptr;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  key_t* pend = pend_all[wave];
  float cx[kFastRows], cy[kFastRows];
  uint32_t cid[kFastRows];
  bool cok[kFastRows];
#pragma unroll
  for (int row = 0; row < kFastRows; ++row) {
    const int p = row * kWave + lane;
    const int pp = p < Cn ? p : 0;
    const int m = pp / S, r = pp - m * S;
    int e = near[((size_t)b * G + c) * M + m];
    e = min(max(e, 0), G - 1);
    cok[row] = p < Cn && r < cluster_size(e, N, S, G);  // a short last cluster fills only part of its places
    int tok = min(e * S + r, N - 1);
    if (mem) tok = min(max(mem[tok], 0), N - 1);
    cx[row] = xy[2 * (size_t)tok];
    cy[row] = xy[2 * (size_t)tok + 1];
    cid[row] = cok[row] ? (uint32_t)tok : 0xffffffffu;
  }
  uint32_t guess = 0u;  // threshold that worked for the previous token (0: none yet)
  const int my_size = cluster_size(c, N, S, G);
  for (int r = wave; r < my_size; r += kKnnWaves) {
    int qtok = c * S + r;
    if (mem) qtok = min(max(mem[qtok], 0), N - 1);
    const float qx = xy[2 * (size_t)qtok], qy = xy[2 * (size_t)qtok + 1];
    uint32_t d2[kFastRows];  // bit pattern of the squared distance: ordered like the value (d2 >= +0)
#pragma unroll
    for (int row = 0; row < kFastRows; ++row)
      d2[row] = cok[row] ? __float_as_uint(dist2(qx, qy, cx[row], cy[row])) : 0xffffffffu;
    const key_t best = select_nearest<kFastRows>(d2, cid, K, guess, pend, lane);
    if (lane < K) nbr_idx[((size_t)b * N + qtok) * K + lane] = (int32_t)(uint32_t)best;
  }
}

}  // namespace

hipError_t launch_knn(const KnnArgs& a, hipStream_t stream) {
  const int32_t* members = nullptr;
  if (a.cluster_id) {
    AFFMAE_LAUNCH("members_kernel", stream, members_kernel, dim3(a.B), dim3(256), 0, stream, a.cluster_id, a.N, a.S, a.G, a.members);
    members = a.members;
  }
  const int BG = a.B * a.G;
  AFFMAE_LAUNCH("centroid_kernel", stream, centroid_kernel, dim3((BG + 3) / 4), dim3(256), 0, stream, a.coords, members, a.B, a.N,
                     a.S, a.G, a.centroid);
  AFFMAE_LAUNCH("near_kernel", stream, near_kernel, dim3((BG + 3) / 4), dim3(256), 0, stream, a.centroid, a.B, a.G, a.M,
                     a.near_clusters);
  if (a.M * a.S <= kFastRows * kWave) {
    AFFMAE_LAUNCH("knn_kernel", stream, knn_fast_kernel, dim3(BG), dim3(kKnnWaves * kWave), 0, stream, a.coords, members,
                  a.near_clusters, a.N, a.S, a.M, a.K, a.G, a.nbr_idx);
  } else {
    const size_t lds = (size_t)a.M * a.S * sizeof(float4);
    AFFMAE_LAUNCH("knn_kernel", stream, knn_kernel, dim3(BG), dim3(kKnnWaves * kWave), lds, stream, a.coords, members,
                  a.near_clusters, a.N, a.S, a.M, a.K, a.G, a.nbr_idx);
  }
  return hipGetLastError();
}

}  // namespace affmae
