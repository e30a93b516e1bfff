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
  const int cell = relpos_cell(cn, ci, rate, R);
  for (int h = 0; h < H; ++h) bias[(tok * H + h) * K + j] = table[(size_t)h * W * W + cell];
}

// K a multiple of 8, bf16: one thread per (token, 8 consecutive neighbours): two 16-byte index loads, eight
// coordinate gathers (the cost that remains), one 16-byte store per head.
__global__ __launch_bounds__(256) void relpos_bias8_kernel(const float* __restrict__ coords,
                                                           const int32_t* __restrict__ nbr_idx,
                                                           const bf16_t* __restrict__ table, int B, int N, int H,
                                                           int K, int R, float rate, bf16_t* __restrict__ bias) {
  const int chunks = K >> 3;
  const long long c = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= (long long)B * N * chunks) return;
  const long long tok = c / chunks;  // b * N + i
  const int j0 = (int)(c - tok * chunks) * 8;
  const int b = (int)(tok / N);
  const int4 n0 = *reinterpret_cast<const int4*>(nbr_idx + tok * K + j0);
  const int4 n1 = *reinterpret_cast<const int4*>(nbr_idx + tok * K + j0 + 4);
  const int nn[8] = {n0.x, n0.y, n0.z, n0.w, n1.x, n1.y, n1.z, n1.w};
  const float2 ci = reinterpret_cast<const float2*>(coords)[tok];
  const int W = 2 * R + 1;
  int cell[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float2 cn = reinterpret_cast<const float2*>(coords)[(long long)b * N + min(max(nn[e], 0), N - 1)];
    cell[e] = relpos_cell(cn, ci, rate, R);
  }
  for (int h = 0; h < H; ++h) {
    const bf16_t* t = table + (size_t)h * W * W;
    uint4 o;
    o.x = (uint32_t)t[cell[0]] | ((uint32_t)t[cell[1]] << 16);
    o.y = (uint32_t)t[cell[2]] | ((uint32_t)t[cell[3]] << 16);
    o.z = (uint32_t)t[cell[4]] | ((uint32_t)t[cell[5]] << 16);
    o.w = (uint32_t)t[cell[6]] | ((uint32_t)t[cell[7]] << 16);
    *reinterpret_cast<uint4*>(bias + (tok * H + h) * K + j0) = o;
  }
}

// Gradient of the table.  A workgroup adds the bias gradients of a slab of (token, neighbour) pairs into a table in
// LDS (the neighbours of one token have different offsets, so the lanes of a wave seldom meet in a bin; eight
// pairs per thread, their loads issued together), then stores its table; a second launch adds up the workgroups'
// tables, one workgroup per bin, in a fixed order.
// The tables in LDS are fp64 when they fit: on this chip an LDS atomic add of a double goes at the speed of an
// integer one, while ds_add_f32 takes about 3 cycles per lane (73 against 21 us for this kernel at the
// benchmark's shape) - and the sums come out more exact.
constexpr int kDtableThreads = 256;
constexpr int kDtableItems = 8;
template <typename T, typename A>
__global__ __launch_bounds__(kDtableThreads) void relpos_dtable_part_kernel(const float* __restrict__ coords,
                                                                           const int32_t* __restrict__ nbr_idx,
                                                                           const T* __restrict__ dbias, int B, int N,
                                                                           int H, int K, int R, float rate,
                                                                           uint32_t k_magic,
                                                                           float* __restrict__ part) {
  extern __shared__ __align__(8) unsigned char dtable_lds[];
  A* acc = reinterpret_cast<A*>(dtable_lds);  // [H][W*W]
  const int W = 2 * R + 1, cells = W * W;
  for (int i = threadIdx.x; i < H * cells; i += kDtableThreads) acc[i] = (A)0;
  __syncthreads();
  const int total = B * N * K;  // < 2^31
  const int lo = blockIdx.x * (kDtableThreads * kDtableItems);
  // (token, neighbour) of a pair: one division per workgroup, then a reciprocal multiplication on small numbers
  const int tok_lo = lo / K, rem_lo = lo - tok_lo * K;
  int tok[kDtableItems], j[kDtableItems], cell[kDtableItems];
  bool live[kDtableItems];
  int n[kDtableItems];
#pragma unroll
  for (int i = 0; i < kDtableItems; ++i) {
    const int e = lo + i * kDtableThreads + threadIdx.x;
    live[i] = e < total;
    const int ee = live[i] ? e : total - 1;
    const uint32_t o = (uint32_t)(rem_lo + (ee - lo));  // < 2048 + K
    const uint32_t dt = k_magic ? __umulhi(o, k_magic) : o;
    tok[i] = tok_lo + (int)dt;
    j[i] = (int)(o - dt * (uint32_t)K);
    n[i] = min(max(nbr_idx[ee], 0), N - 1);
  }
#pragma unroll
  for (int i = 0; i < kDtableItems; ++i) {
    const int b = tok[i] / N;
    const float2 ci = reinterpret_cast<const float2*>(coords)[tok[i]];
    const float2 cn = reinterpret_cast<const float2*>(coords)[b * N + n[i]];
    cell[i] = relpos_cell(cn, ci, rate, R);
  }
  for (int h = 0; h < H; ++h) {
    float g[kDtableItems];
#pragma unroll
    for (int i = 0; i < kDtableItems; ++i) g[i] = Elem<T>::load(dbias + ((size_t)tok[i] * H + h) * K + j[i]);
#pragma unroll
    for (int i = 0; i < kDtableItems; ++i)
      if (live[i]) atomicAdd(&acc[h * cells + cell[i]], (A)g[i]);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < H * cells; i += kDtableThreads) part[(size_t)blockIdx.x * H * cells + i] = (float)acc[i];
}

// The same for bf16 with K a multiple of 8: a thread takes two runs of 8 consecutive neighbours of a token
// (16-byte loads of the indices and of the bias gradients).
constexpr int kDtableChunks = 2;
template <typename A>
__global__ __launch_bounds__(kDtableThreads) void relpos_dtable_part8_kernel(const float* __restrict__ coords,
                                                                            const int32_t* __restrict__ nbr_idx,
                                                                            const bf16_t* __restrict__ dbias, int B,
                                                                            int N, int H, int K, int R, float rate,
                                                                            uint32_t c_magic,
                                                                            float* __restrict__ part) {
  extern __shared__ __align__(8) unsigned char dtable_lds[];
  A* acc = reinterpret_cast<A*>(dtable_lds);  // [H][W*W]
  const int W = 2 * R + 1, cells = W * W;
  for (int i = threadIdx.x; i < H * cells; i += kDtableThreads) acc[i] = (A)0;
  __syncthreads();
  const int chunks = K >> 3;
  const int total = B * N * chunks;
  const int lo = blockIdx.x * (kDtableThreads * kDtableChunks);
  const int tok_lo = lo / chunks, rem_lo = lo - tok_lo * chunks;
  int tok[kDtableChunks], j0[kDtableChunks], cell[kDtableChunks][8];
  bool live[kDtableChunks];
#pragma unroll
  for (int u = 0; u < kDtableChunks; ++u) {
    const int c = lo + u * kDtableThreads + threadIdx.x;
    live[u] = c < total;
    const int cc = live[u] ? c : total - 1;
    const uint32_t o = (uint32_t)(rem_lo + (cc - lo));
    const uint32_t dt = c_magic ? __umulhi(o, c_magic) : o;
    tok[u] = tok_lo + (int)dt;
    j0[u] = (int)(o - dt * (uint32_t)chunks) * 8;
    const int b = tok[u] / N;
    const int4 n0 = *reinterpret_cast<const int4*>(nbr_idx + (size_t)tok[u] * K + j0[u]);
    const int4 n1 = *reinterpret_cast<const int4*>(nbr_idx + (size_t)tok[u] * K + j0[u] + 4);
    const int nn[8] = {n0.x, n0.y, n0.z, n0.w, n1.x, n1.y, n1.z, n1.w};
    const float2 ci = reinterpret_cast<const float2*>(coords)[tok[u]];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float2 cn = reinterpret_cast<const float2*>(coords)[b * N + min(max(nn[e], 0), N - 1)];
      cell[u][e] = relpos_cell(cn, ci, rate, R);
    }
  }
  for (int h = 0; h < H; ++h) {
#pragma unroll
    for (int u = 0; u < kDtableChunks; ++u) {
      const uint4 g = *reinterpret_cast<const uint4*>(dbias + ((size_t)tok[u] * H + h) * K + j0[u]);
      const uint32_t w[4] = {g.x, g.y, g.z, g.w};
      if (live[u]) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          atomicAdd(&acc[h * cells + cell[u][2 * e]], (A)__uint_as_float(w[e] << 16));
          atomicAdd(&acc[h * cells + cell[u][2 * e + 1]], (A)__uint_as_float(w[e] & 0xffff0000u));
        }
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < H * cells; i += kDtableThreads) part[(size_t)blockIdx.x * H * cells + i] = (float)acc[i];
}

// dtable[i] = sum over the workgroups' tables of entry i: one workgroup per entry, fixed order
__global__ __launch_bounds__(256) void relpos_dtable_sum_kernel(const float* __restrict__ part, int blocks, int cells,
                                                                float* __restrict__ dtable) {
  __shared__ float wsum[4];
  const int i = blockIdx.x;
  float s = 0.f;
  for (int b = threadIdx.x; b < blocks; b += 256) s += part[(size_t)b * cells + i];
  s = wave_sum(s);
  if ((threadIdx.x & (kWave - 1)) == 0) wsum[threadIdx.x / kWave] = s;
  __syncthreads();
  if (threadIdx.x == 0) dtable[i] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

}  // namespace

hipError_t launch_relpos_bias(const RelposArgs& r, int B, int N, int H, int K, int dtype, void* bias,
                              hipStream_t stream) {
  const long long total = (long long)B * N * K;
  const dim3 grid((unsigned)((total + 255) / 256));
  if (dtype == 1 && K % 8 == 0 && reinterpret_cast<uintptr_t>(r.nbr_idx) % 16 == 0 &&
      reinterpret_cast<uintptr_t>(bias) % 16 == 0) {
    const long long chunks = total / 8;
    AFFMAE_LAUNCH("relpos_bias_kernel", stream, relpos_bias8_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256),
                  0, stream, r.coords, r.nbr_idx, (const bf16_t*)r.table, B, N, H, K, r.R, r.rate, (bf16_t*)bias);
  } else if (dtype == 1)
    AFFMAE_LAUNCH("relpos_bias_kernel", stream, relpos_bias_kernel<bf16_t>, grid, dim3(256), 0, stream, r.coords,
                  r.nbr_idx, (const bf16_t*)r.table, B, N, H, K, r.R, r.rate, (bf16_t*)bias);
  else
    AFFMAE_LAUNCH("relpos_bias_kernel", stream, relpos_bias_kernel<float>, grid, dim3(256), 0, stream, r.coords,
                  r.nbr_idx, (const float*)r.table, B, N, H, K, r.R, r.rate, (float*)bias);
  return hipGetLastError();
}

static bool relpos_chunked(int K, int dtype) { return dtype == 1 && K % 8 == 0; }
int relpos_dtable_blocks(int B, int N, int K) {
  // (the chunked kernel covers twice as many pairs per workgroup: this is an upper bound for it)
  const long long total = (long long)B * N * K;
  return (int)((total + kDtableThreads * kDtableItems - 1) / (kDtableThreads * kDtableItems));
}
size_t relpos_dtable_workspace_bytes(int B, int N, int H, int K, int R) {
  const size_t cells = (size_t)(2 * R + 1) * (2 * R + 1);
  return (size_t)relpos_dtable_blocks(B, N, K) * H * cells * sizeof(float);
}

hipError_t launch_relpos_dtable(const RelposArgs& r, int B, int N, int H, int K, int dtype, const void* dbias,
                                float* dtable, void* workspace, hipStream_t stream) {
  const int cells = (2 * r.R + 1) * (2 * r.R + 1);
  const int blocks = relpos_dtable_blocks(B, N, K);
  const bool wide = (size_t)H * cells * sizeof(double) <= 48 * 1024;  // fp64 tables fit
  const size_t lds = (size_t)H * cells * (wide ? sizeof(double) : sizeof(float));
  const uint32_t k_magic = K <= 1 ? 0u : (uint32_t)((1ull << 32) / (uint32_t)K) + 1u;
  float* part = static_cast<float*>(workspace);
  int used = blocks;
#define AFFMAE_DTABLE(KERNEL, GRID, ...) \
  AFFMAE_LAUNCH("relpos_dtable_kernel", stream, KERNEL, dim3(GRID), dim3(kDtableThreads), lds, stream, __VA_ARGS__)
  if (relpos_chunked(K, dtype) && reinterpret_cast<uintptr_t>(r.nbr_idx) % 16 == 0 &&
      reinterpret_cast<uintptr_t>(dbias) % 16 == 0) {
    const int chunks = K / 8;
    const long long tc = (long long)B * N * chunks;
    const int per = kDtableThreads * kDtableChunks;
    used = (int)((tc + per - 1) / per);
    const uint32_t c_magic = chunks <= 1 ? 0u : (uint32_t)((1ull << 32) / (uint32_t)chunks) + 1u;
    if (wide)
      AFFMAE_DTABLE(relpos_dtable_part8_kernel<double>, used, r.coords, r.nbr_idx, (const bf16_t*)dbias, B, N, H, K,
                    r.R, r.rate, c_magic, part);
    else
      AFFMAE_DTABLE(relpos_dtable_part8_kernel<float>, used, r.coords, r.nbr_idx, (const bf16_t*)dbias, B, N, H, K,
                    r.R, r.rate, c_magic, part);
  } else if (dtype == 1) {
    if (wide)
      AFFMAE_DTABLE((relpos_dtable_part_kernel<bf16_t, double>), blocks, r.coords, r.nbr_idx, (const bf16_t*)dbias, B,
                    N, H, K, r.R, r.rate, k_magic, part);
    else
      AFFMAE_DTABLE((relpos_dtable_part_kernel<bf16_t, float>), blocks, r.coords, r.nbr_idx, (const bf16_t*)dbias, B,
                    N, H, K, r.R, r.rate, k_magic, part);
  } else {
    if (wide)
      AFFMAE_DTABLE((relpos_dtable_part_kernel<float, double>), blocks, r.coords, r.nbr_idx, (const float*)dbias, B, N,
                    H, K, r.R, r.rate, k_magic, part);
    else
      AFFMAE_DTABLE((relpos_dtable_part_kernel<float, float>), blocks, r.coords, r.nbr_idx, (const float*)dbias, B, N,
                    H, K, r.R, r.rate, k_magic, part);
  }
#undef AFFMAE_DTABLE
  AFFMAE_LAUNCH("relpos_dtable_sum_kernel", stream, relpos_dtable_sum_kernel, dim3(H * cells), dim3(256), 0, stream,
                part, used, H * cells, dtable);
  return hipGetLastError();
}

hipError_t launch_relpos_table_sum(const float* part, int tables, int entries, float* dtable, hipStream_t stream) {
  AFFMAE_LAUNCH("relpos_dtable_sum_kernel", stream, relpos_dtable_sum_kernel, dim3(entries), dim3(256), 0, stream,
                part, tables, entries, dtable);
  return hipGetLastError();
}

}  // namespace affmae
