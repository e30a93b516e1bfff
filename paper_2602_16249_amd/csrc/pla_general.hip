// Local attention over arbitrary neighbour tables (paper, Sec. "Flash-style
// Cluster Attention and Fast Decoder KNN", the FlashNbhdAttn equation), gather
// formulation: one wave per token, rows fetched straight from global memory.
// This path makes no assumption about the table (any indices, repeats allowed)
// and serves fp32 storage; the cluster-tiled kernels cover the clustered bf16
// case.  Scores are never stored: per (token, head) the K logits live one per
// lane, the softmax runs on wave shuffles in fp32, and only the K probabilities
// pass through LDS to the channel-parallel accumulation phase.
#include "device_util.h"
#include "launch.h"
#include "timing.h"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace affmae {
namespace {

constexpr int kWavesPerBlock = 4;

template <typename T, int D>
__device__ __forceinline__ float dot_row(const float (&a)[D], const T* row) {
  float r[D];
  load_row<D>(row, r);
  float acc = 0.f;
#pragma unroll
  for (int t = 0; t < D; ++t) acc = fmaf(a[t], r[t], acc);
  return acc;
}

// LDS layout per wave: int nb[Kp]; float P[H][Kp]; (bwd) float dS[H][Kp]; (bwd, blank) float acc[2][C]
// with Kp = K + 1 (slot K = blank column).

template <typename T, int D>
__global__ __launch_bounds__(256) void pla_fwd_general_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const T* __restrict__ bias,
    const int32_t* __restrict__ nbr_idx, const T* __restrict__ k_blank, const T* __restrict__ v_blank,
    long long tokens, int N, int H, int K, float scale, T* __restrict__ out, float* __restrict__ lse) {
  extern __shared__ float smem[];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int Kp = K + 1;
  const int C = H * D;
  float* wbase = smem + (size_t)wave * (Kp + (size_t)H * Kp);
  int* nb = reinterpret_cast<int*>(wbase);
  float* P = wbase + Kp;

  for (long long tok = (long long)blockIdx.x * kWavesPerBlock + wave; tok < tokens;
       tok += (long long)gridDim.x * kWavesPerBlock) {
    const long long img_base = (tok / N) * N;  // first token of this image
    if (lane < K) nb[lane] = min(max(nbr_idx[tok * K + lane], 0), N - 1);
    wave_lds_sync();
    for (int h = 0; h < H; ++h) {
      float qr[D];
      load_row<D>(q + (tok * H + h) * D, qr);
      float s = -INFINITY;
      if (lane < K) {
        const T* krow = k + ((img_base + nb[lane]) * H + h) * D;
        s = scale * dot_row<T, D>(qr, krow);
        if (bias) s += Elem<T>::load(bias + (tok * H + h) * K + lane);
      }
      float sb = -INFINITY;
      if (k_blank) sb = scale * dot_row<T, D>(qr, k_blank + (size_t)h * D);
      const float m = fmaxf(wave_max(s), sb);
      const float e = (lane < K) ? expf(s - m) : 0.f;
      const float eb = k_blank ? expf(sb - m) : 0.f;
      const float z = wave_sum(e) + eb;
      if (lane < K) P[h * Kp + lane] = e / z;
      if (lane == 0) {
        P[h * Kp + K] = eb / z;
        lse[tok * H + h] = m + logf(z);
      }
    }
    wave_lds_sync();
    for (int c = lane; c < C; c += kWave) {
      const int h = c / D;
      float acc = 0.f;
      for (int j = 0; j < K; ++j) acc = fmaf(P[h * Kp + j], Elem<T>::load(v + (img_base + nb[j]) * C + c), acc);
      if (v_blank) acc = fmaf(P[h * Kp + K], Elem<T>::load(v_blank + c), acc);
      Elem<T>::store(out + tok * C + c, acc);
    }
    wave_lds_sync();
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void pla_bwd_general_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const T* __restrict__ bias,
    const int32_t* __restrict__ nbr_idx, const T* __restrict__ k_blank, const T* __restrict__ v_blank,
    const float* __restrict__ lse, const T* __restrict__ dout, long long tokens, int N, int H, int K, float scale,
    T* __restrict__ dq, float* __restrict__ dk_acc, float* __restrict__ dv_acc, T* __restrict__ dbias,
    float* __restrict__ dk_blank, float* __restrict__ dv_blank) {
  extern __shared__ float smem[];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int Kp = K + 1;
  const int C = H * D;
  const bool blank_grad = k_blank && dk_blank;
  const size_t per_wave = Kp + 2 * (size_t)H * Kp + (blank_grad ? 2 * (size_t)C : 0);
  float* wbase = smem + (size_t)wave * per_wave;
  int* nb = reinterpret_cast<int*>(wbase);
  float* P = wbase + Kp;
  float* dS = P + (size_t)H * Kp;
  float* bacc = dS + (size_t)H * Kp;  // [2][C] running blank-row gradients of this wave
  if (blank_grad)
    for (int c = lane; c < 2 * C; c += kWave) bacc[c] = 0.f;

  for (long long tok = (long long)blockIdx.x * kWavesPerBlock + wave; tok < tokens;
       tok += (long long)gridDim.x * kWavesPerBlock) {
    const long long img_base = (tok / N) * N;
    if (lane < K) nb[lane] = min(max(nbr_idx[tok * K + lane], 0), N - 1);
    wave_lds_sync();
    for (int h = 0; h < H; ++h) {
      float qr[D], gr[D];
      load_row<D>(q + (tok * H + h) * D, qr);
      load_row<D>(dout + (tok * H + h) * D, gr);
      const float l = lse[tok * H + h];
      float p = 0.f, dP = 0.f;
      if (lane < K) {
        const long long row = ((img_base + nb[lane]) * H + h) * D;
        float s = scale * dot_row<T, D>(qr, k + row);
        if (bias) s += Elem<T>::load(bias + (tok * H + h) * K + lane);
        p = expf(s - l);
        dP = dot_row<T, D>(gr, v + row);
      }
      float pb = 0.f, dPb = 0.f;
      if (k_blank) {
        pb = expf(scale * dot_row<T, D>(qr, k_blank + (size_t)h * D) - l);
        dPb = dot_row<T, D>(gr, v_blank + (size_t)h * D);
      }
      const float Dsum = wave_sum(p * dP) + pb * dPb;
      const float ds = p * (dP - Dsum);
      if (lane < K) {
        P[h * Kp + lane] = p;
        dS[h * Kp + lane] = ds;
        if (dbias) Elem<T>::store(dbias + (tok * H + h) * K + lane, ds);
      }
      if (lane == 0) {
        P[h * Kp + K] = pb;
        dS[h * Kp + K] = pb * (dPb - Dsum);
      }
    }
    wave_lds_sync();
    for (int c = lane; c < C; c += kWave) {
      const int h = c / D;
      const float qc = Elem<T>::load(q + tok * C + c);
      const float gc = Elem<T>::load(dout + tok * C + c);
      float acc = 0.f;
      for (int j = 0; j < K; ++j) {
        const long long row = (img_base + nb[j]) * C + c;
        const float ds = dS[h * Kp + j];
        acc = fmaf(ds, Elem<T>::load(k + row), acc);
        unsafeAtomicAdd(dk_acc + row, scale * ds * qc);
        unsafeAtomicAdd(dv_acc + row, P[h * Kp + j] * gc);
      }
      if (k_blank) {
        acc = fmaf(dS[h * Kp + K], Elem<T>::load(k_blank + c), acc);
        if (blank_grad) {
          bacc[c] += scale * dS[h * Kp + K] * qc;
          bacc[C + c] += P[h * Kp + K] * gc;
        }
      }
      Elem<T>::store(dq + tok * C + c, scale * acc);
    }
    wave_lds_sync();
  }
  if (blank_grad) {
    for (int c = lane; c < C; c += kWave) {
      unsafeAtomicAdd(dk_blank + c, bacc[c]);
      unsafeAtomicAdd(dv_blank + c, bacc[C + c]);
    }
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0.f;
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ a, bf16_t* __restrict__ o, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    o[i] = f32_to_bf16(a[i]);
}

int grid_for(size_t n, int per_block, int cap) {
  size_t g = (n + per_block - 1) / per_block;
  if (g < 1) g = 1;
  if (g > (size_t)cap) g = cap;
  return (int)g;
}

template <typename T, int D>
hipError_t fwd_impl(const PlaArgs& a, hipStream_t stream) {
  const long long tokens = (long long)a.B * a.N;
  const int Kp = a.K + 1;
  const size_t lds = kWavesPerBlock * (Kp + (size_t)a.H * Kp) * sizeof(float);
  const int grid = grid_for((size_t)tokens, kWavesPerBlock, 1 << 20);
  AFFMAE_LAUNCH("pla_fwd_general_kernel", stream, (pla_fwd_general_kernel<T, D>), dim3(grid), dim3(256), lds, stream, (const T*)a.q,
                     (const T*)a.k, (const T*)a.v, (const T*)a.bias, a.nbr_idx, (const T*)a.k_blank,
                     (const T*)a.v_blank, tokens, a.N, a.H, a.K, a.scale, (T*)a.out, a.lse);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t bwd_impl(const PlaArgs& a, hipStream_t stream) {
  const long long tokens = (long long)a.B * a.N;
  const size_t elems = (size_t)tokens * a.H * D;
  float *dk_acc, *dv_acc;
  if (a.dtype == 0) {  // fp32 storage: accumulate in place
    dk_acc = (float*)a.dk;
    dv_acc = (float*)a.dv;
  } else {
    dk_acc = (float*)a.workspace;
    dv_acc = dk_acc + elems;
  }
  const int zgrid = grid_for(elems, 256 * 8, 4096);
  AFFMAE_LAUNCH("fill_zero_kernel", stream, fill_zero_kernel, dim3(zgrid), dim3(256), 0, stream, dk_acc, elems);
  AFFMAE_LAUNCH("fill_zero_kernel", stream, fill_zero_kernel, dim3(zgrid), dim3(256), 0, stream, dv_acc, elems);
  const bool blank_grad = a.k_blank && a.dk_blank;
  if (blank_grad) {
    AFFMAE_LAUNCH("fill_zero_kernel", stream, fill_zero_kernel, dim3(1), dim3(256), 0, stream, a.dk_blank, (size_t)a.H * D);
    AFFMAE_LAUNCH("fill_zero_kernel", stream, fill_zero_kernel, dim3(1), dim3(256), 0, stream, a.dv_blank, (size_t)a.H * D);
  }
  const int Kp = a.K + 1;
  const size_t per_wave = Kp + 2 * (size_t)a.H * Kp + (blank_grad ? 2 * (size_t)a.H * D : 0);
  const size_t lds = kWavesPerBlock * per_wave * sizeof(float);
  // With blank gradients every wave keeps a running sum, so bound the grid.
  const int grid = grid_for((size_t)tokens, kWavesPerBlock, blank_grad ? 2048 : (1 << 20));
  AFFMAE_LAUNCH("pla_bwd_general_kernel", stream, (pla_bwd_general_kernel<T, D>), dim3(grid), dim3(256), lds, stream, (const T*)a.q,
                     (const T*)a.k, (const T*)a.v, (const T*)a.bias, a.nbr_idx, (const T*)a.k_blank,
                     (const T*)a.v_blank, a.lse, (const T*)a.dout, tokens, a.N, a.H, a.K, a.scale, (T*)a.dq, dk_acc,
                     dv_acc, (T*)a.dbias, a.dk_blank, a.dv_blank);
  if (a.dtype != 0) {
    const int cgrid = grid_for(elems, 256 * 8, 4096);
    AFFMAE_LAUNCH("cast_bf16_kernel", stream, cast_bf16_kernel, dim3(cgrid), dim3(256), 0, stream, dk_acc, (bf16_t*)a.dk, elems);
    AFFMAE_LAUNCH("cast_bf16_kernel", stream, cast_bf16_kernel, dim3(cgrid), dim3(256), 0, stream, dv_acc, (bf16_t*)a.dv, elems);
  }
  return hipGetLastError();
}

}  // namespace

size_t pla_bwd_general_workspace_bytes(int B, int N, int H, int d, int dtype) {
  if (dtype == 0) return 0;
  return 2 * (size_t)B * N * H * d * sizeof(float);
}

#define AFFMAE_DISPATCH(IMPL)                                            \
  if (a.dtype == 0) {                                                    \
    switch (a.d) {                                                       \
      case 16: return IMPL<float, 16>(a, stream);                        \
      case 32: return IMPL<float, 32>(a, stream);                        \
      case 64: return IMPL<float, 64>(a, stream);                        \
    }                                                                    \
  } else {                                                               \
    switch (a.d) {                                                       \
      case 16: return IMPL<bf16_t, 16>(a, stream);                       \
      case 32: return IMPL<bf16_t, 32>(a, stream);                       \
      case 64: return IMPL<bf16_t, 64>(a, stream);                       \
    }                                                                    \
  }                                                                      \
  return hipErrorInvalidValue;

hipError_t launch_pla_fwd_general(const PlaArgs& a, hipStream_t stream) { AFFMAE_DISPATCH(fwd_impl) }
hipError_t launch_pla_bwd_general(const PlaArgs& a, hipStream_t stream) { AFFMAE_DISPATCH(bwd_impl) }

}  // namespace affmae
