// Batched clustered neighbour search (paper, Sec. "AutoFocusFormer": equal-size
// clusters, fixed-size neighbourhoods by nearest-neighbour search over 2-D token
// coordinates).  Four kernels:
//   members  (only with an explicit cluster_id): token lists per cluster
//   centroid : double-precision mean of each cluster's coordinates -> fp32
//   near     : per cluster the M clusters with nearest centroids
//   knn      : per token the K nearest among the members of those M clusters
// Selection is exact and unique: 64-bit keys (fp32 distance bits, index) compared
// as integers; distances are evaluated without fused multiply-add.  This file is
// compiled with -ffp-contract=off.
#include "device_util.h"
#include "launch.h"
#include "timing.h"

namespace affmae {
namespace {

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

__device__ __forceinline__ key_t shfl_key_xor(key_t k, int mask) {
  uint32_t lo = (uint32_t)k, hi = (uint32_t)(k >> 32);
  lo = __shfl_xor(lo, mask);
  hi = __shfl_xor(hi, mask);
  return ((key_t)hi << 32) | lo;
}
__device__ __forceinline__ key_t shfl_key(key_t k, int src) {
  uint32_t lo = (uint32_t)k, hi = (uint32_t)(k >> 32);
  lo = __shfl(lo, src);
  hi = __shfl(hi, src);
  return ((key_t)hi << 32) | lo;
}

// Sort one key per lane ascending across the 64 lanes of the wave.
__device__ __forceinline__ key_t wave_sort(key_t key, int lane) {
#pragma unroll
  for (int k = 2; k <= kWave; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      key_t other = shfl_key_xor(key, j);
      bool up = (lane & k) == 0;
      bool lower = (lane & j) == 0;
      key_t lo = key < other ? key : other;
      key_t hi = key < other ? other : key;
      key = (lower == up) ? lo : hi;
    }
  }
  return key;
}

// Input: bitonic across lanes.  Output: ascending across lanes.
__device__ __forceinline__ key_t wave_bitonic_merge(key_t key, int lane) {
#pragma unroll
  for (int j = kWave / 2; j > 0; j >>= 1) {
    key_t other = shfl_key_xor(key, j);
    key_t lo = key < other ? key : other;
    key_t hi = key < other ? other : key;
    key = ((lane & j) == 0) ? lo : hi;
  }
  return key;
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
          if (ids[t] == c && count < S) {
            mem[(size_t)c * S + count] = base + t;
            ++count;
          }
        }
      }
    }
  }
}

// One thread per cluster: sequential double-precision sum in member order.
__global__ __launch_bounds__(256) void centroid_kernel(const float* __restrict__ coords,
                                                      const int32_t* __restrict__ members, int B, int N, int S,
                                                      int G, float* __restrict__ centroid) {
  const int gc = blockIdx.x * blockDim.x + threadIdx.x;
  if (gc >= B * G) return;
  const int b = gc / G, c = gc % G;
  const float* xy = coords + (size_t)b * N * 2;
  double sx = 0.0, sy = 0.0;
  for (int r = 0; r < S; ++r) {
    int tok = c * S + r;
    if (members) tok = min(max(members[(size_t)b * N + tok], 0), N - 1);
    sx += (double)xy[2 * (size_t)tok + 0];
    sy += (double)xy[2 * (size_t)tok + 1];
  }
  centroid[2 * (size_t)gc + 0] = (float)(sx / (double)S);
  centroid[2 * (size_t)gc + 1] = (float)(sy / (double)S);
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
// turn: 64 candidates at a time, one per lane, pushed into a running top-64.
__global__ __launch_bounds__(256) void knn_kernel(const float* __restrict__ coords,
                                                 const int32_t* __restrict__ members,
                                                 const int32_t* __restrict__ near, int N, int S, int M, int K,
                                                 int G, int32_t* __restrict__ nbr_idx) {
  extern __shared__ float4 cand[];  // x, y, token id (bits), unused
  const int b = blockIdx.x / G, c = blockIdx.x % G;
  const int Cn = M * S;
  const float* xy = coords + (size_t)b * N * 2;
  const int32_t* mem = members ? members + (size_t)b * N : nullptr;
  for (int p = threadIdx.x; p < Cn; p += blockDim.x) {
    const int m = p / S, r = p - m * S;
    int e = near[((size_t)b * G + c) * M + m];
    e = min(max(e, 0), G - 1);
    int tok = e * S + r;
    if (mem) tok = min(max(mem[tok], 0), N - 1);
    cand[p] = make_float4(xy[2 * (size_t)tok], xy[2 * (size_t)tok + 1], __int_as_float(tok), 0.f);
  }
  __syncthreads();
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave, nwaves = blockDim.x / kWave;
  for (int r = wave; r < S; r += nwaves) {
    int qtok = c * S + r;
    if (mem) qtok = min(max(mem[qtok], 0), N - 1);
    const float qx = xy[2 * (size_t)qtok], qy = xy[2 * (size_t)qtok + 1];
    key_t best = kKeyMax;
    for (int base = 0; base < Cn; base += kWave) {
      const int p = base + lane;
      key_t key = kKeyMax;
      if (p < Cn) {
        const float4 cp = cand[p];
        key = make_key(dist2(qx, qy, cp.x, cp.y), __float_as_int(cp.z));
      }
      best = topk_push(best, key, lane, K - 1);
    }
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
  AFFMAE_LAUNCH("centroid_kernel", stream, centroid_kernel, dim3((BG + 255) / 256), dim3(256), 0, stream, a.coords, members, a.B, a.N,
                     a.S, a.G, a.centroid);
  AFFMAE_LAUNCH("near_kernel", stream, near_kernel, dim3((BG + 3) / 4), dim3(256), 0, stream, a.centroid, a.B, a.G, a.M,
                     a.near_clusters);
  const size_t lds = (size_t)a.M * a.S * sizeof(float4);
  AFFMAE_LAUNCH("knn_kernel", stream, knn_kernel, dim3(BG), dim3(256), lds, stream, a.coords, members, a.near_clusters, a.N, a.S,
                     a.M, a.K, a.G, a.nbr_idx);
  return hipGetLastError();
}

}  // namespace affmae
