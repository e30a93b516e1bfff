// Relative-position bias (paper, Sec. "AutoFocusFormer": within a neighbourhood, attention uses relative
// position derived from the 2-D token coordinates; it enters the FlashNbhdAttn equation as B_n).  The paper
// gives no function; the reading taken here is a learned table per head over quantised offsets:
//   bias[b,i,h,j] = table[h][by][bx],  bx = clamp(rint((x_n - x_i) * rate), -R, R) + R  (fp32, ties to even),
//   by alike, n = nbr_idx[b,i,j].
// This file holds the two stand-alone kernels: the bias written out as a tensor (for the gather kernels, which
// take any neighbour table), and the gradient of the table from the bias gradients.  The tiled kernels compute
// the same bias themselves from the coordinates of the token tiles they stage (pla_cluster_*.hip).
#include <algorithm>

#include "device_util.h"
#include "launch.h"
#include "timing.h"

namespace affmae {
namespace {

// the same arithmetic everywhere: fp32 offset, fp32 product, round to nearest even, clamp
__device__ __forceinline__ int relpos_bin(float nbr, float query, float rate, int R) {
#pragma clang fp contract(off)
  const float d = nbr - query;
  const float t = d * rate;
  const float r = __builtin_rintf(t);
  if (!(r >= (float)(-R))) return 0;  // also NaN
  if (r > (float)R) return 2 * R;
  return (int)r + R;
}

// one thread per (token, neighbour): the bin once, then one value per head
template <typename T>
__global__ __launch_bounds__(256) void relpos_bias_kernel(const float* __restrict__ coords,
                                                          const int32_t* __restrict__ nbr_idx,
                                                          const T* __restrict__ table, int B, int N, int H, int K,
                                                          int R, float rate, T* __restrict__ bias) {
  const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (long long)B * N * K) return;
  const long long tok = e / K;  // b * N + i
  const int j = (int)(e - tok * K);
  const int b = (int)(tok / N);
  const int n = min(max(nbr_idx[e], 0), N - 1);
  const float2 ci = reinterpret_cast<const float2*>(coords)[tok];
  const float2 cn = reinterpret_cast<const float2*>(coords)[(long long)b * N + n];
  const int W = 2 * R + 1;
  const int cell = relpos_bin(cn.y, ci.y, rate, R) * W + relpos_bin(cn.x, ci.x, rate, R);
  for (int h = 0; h < H; ++h) bias[(tok * H + h) * K + j] = table[(size_t)h * W * W + cell];
}

// Gradient of the table.  A workgroup adds the bias gradients of a slab of tokens into a table in LDS (the
// neighbours of one token have different offsets, so the lanes of a wave seldom meet in a bin), then stores
// its table; a second launch adds up the workgroups' tables in a fixed order.
constexpr int kDtableThreads = 256;
template <typename T>
__global__ __launch_bounds__(kDtableThreads) void relpos_dtable_part_kernel(const float* __restrict__ coords,
                                                                           const int32_t* __restrict__ nbr_idx,
                                                                           const T* __restrict__ dbias, int B, int N,
                                                                           int H, int K, int R, float rate,
                                                                           long long per_block,
                                                                           float* __restrict__ part) {
  extern __shared__ float acc[];  // [H][W*W]
  const int W = 2 * R + 1, cells = W * W;
  for (int i = threadIdx.x; i < H * cells; i += kDtableThreads) acc[i] = 0.f;
  __syncthreads();
  const long long total = (long long)B * N * K;
  const long long lo = (long long)blockIdx.x * per_block, hi = min(total, lo + per_block);
  for (long long e = lo + threadIdx.x; e < hi; e += kDtableThreads) {
    const long long tok = e / K;
    const int j = (int)(e - tok * K);
    const int b = (int)(tok / N);
    const int n = min(max(nbr_idx[e], 0), N - 1);
    const float2 ci = reinterpret_cast<const float2*>(coords)[tok];
    const float2 cn = reinterpret_cast<const float2*>(coords)[(long long)b * N + n];
    const int cell = relpos_bin(cn.y, ci.y, rate, R) * W + relpos_bin(cn.x, ci.x, rate, R);
    for (int h = 0; h < H; ++h) atomicAdd(&acc[h * cells + cell], Elem<T>::load(dbias + (tok * H + h) * K + j));
  }
  __syncthreads();
  for (int i = threadIdx.x; i < H * cells; i += kDtableThreads) part[(size_t)blockIdx.x * H * cells + i] = acc[i];
}

__global__ __launch_bounds__(256) void relpos_dtable_sum_kernel(const float* __restrict__ part, int blocks, int cells,
                                                                float* __restrict__ dtable) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= cells) return;
  float s = 0.f;
  for (int b = 0; b < blocks; ++b) s += part[(size_t)b * cells + i];
  dtable[i] = s;
}

}  // namespace

hipError_t launch_relpos_bias(const RelposArgs& r, int B, int N, int H, int K, int dtype, void* bias,
                              hipStream_t stream) {
  const long long total = (long long)B * N * K;
  const dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == 1)
    AFFMAE_LAUNCH("relpos_bias_kernel", stream, relpos_bias_kernel<bf16_t>, grid, dim3(256), 0, stream, r.coords,
                  r.nbr_idx, (const bf16_t*)r.table, B, N, H, K, r.R, r.rate, (bf16_t*)bias);
  else
    AFFMAE_LAUNCH("relpos_bias_kernel", stream, relpos_bias_kernel<float>, grid, dim3(256), 0, stream, r.coords,
                  r.nbr_idx, (const float*)r.table, B, N, H, K, r.R, r.rate, (float*)bias);
  return hipGetLastError();
}

int relpos_dtable_blocks(int B, int N, int K) {
  const long long total = (long long)B * N * K;
  return (int)std::min<long long>(1024, (total + 4095) / 4096);
}
size_t relpos_dtable_workspace_bytes(int B, int N, int H, int K, int R) {
  const size_t cells = (size_t)(2 * R + 1) * (2 * R + 1);
  return (size_t)relpos_dtable_blocks(B, N, K) * H * cells * sizeof(float);
}

hipError_t launch_relpos_dtable(const RelposArgs& r, int B, int N, int H, int K, int dtype, const void* dbias,
                                float* dtable, void* workspace, hipStream_t stream) {
  const int cells = (2 * r.R + 1) * (2 * r.R + 1);
  const int blocks = relpos_dtable_blocks(B, N, K);
  const long long total = (long long)B * N * K;
  const long long per_block = (total + blocks - 1) / blocks;
  const size_t lds = (size_t)H * cells * sizeof(float);
  float* part = static_cast<float*>(workspace);
  if (dtype == 1)
    AFFMAE_LAUNCH("relpos_dtable_kernel", stream, relpos_dtable_part_kernel<bf16_t>, dim3(blocks),
                  dim3(kDtableThreads), lds, stream, r.coords, r.nbr_idx, (const bf16_t*)dbias, B, N, H, K, r.R,
                  r.rate, per_block, part);
  else
    AFFMAE_LAUNCH("relpos_dtable_kernel", stream, relpos_dtable_part_kernel<float>, dim3(blocks),
                  dim3(kDtableThreads), lds, stream, r.coords, r.nbr_idx, (const float*)dbias, B, N, H, K, r.R,
                  r.rate, per_block, part);
  AFFMAE_LAUNCH("relpos_dtable_sum_kernel", stream, relpos_dtable_sum_kernel, dim3((H * cells + 255) / 256), dim3(256),
                0, stream, part, blocks, H * cells, dtable);
  return hipGetLastError();
}

}  // namespace affmae
