// Local attention over arbitrary neighbour tables (paper, Sec. "Flash-style
// Cluster Attention and Fast Decoder KNN", the FlashNbhdAttn equation), gather
// formulation: one wave per token, the neighbours' rows fetched straight from
// global memory.  This path makes no assumption about the table (any indices,
// repeats allowed: every slot is its own softmax column) and serves fp32 storage
// and every head size; the cluster-tiled kernels cover the clustered bf16 case.
//
// Lane layout, all three kernels: a head's row of D channels is PP = D / E pieces of 16 bytes (E = 4 fp32 or 8
// bf16 channels); lane (r, c) = (lane / PP, lane % PP) holds piece c of the r-th of the 64 / PP rows of a trip, so a
// load instruction fetches whole rows, PP lanes wide, and K neighbours take ceil(K * PP / 64) trips.  A dot product
// with the query's row is a partial sum per lane and an add over the PP lanes of the row; a weighted sum of rows
// is accumulated per lane and added over the rows at the end.  Scores are never stored.
// Backward: the query-side kernel writes dq and dbias and keeps p and dS of every (query, slot) pair; dk and dv are
// gathered, not scattered: the pairs are filed per neighbour token (the list builder shared with the decoder's and
// the merging backward) and a wave per token adds dS q and p dout over its list - no floating-point atomics.
#include "cluster_common.h"
#include "device_util.h"
#include "launch.h"
#include "select_util.h"
#include "timing.h"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace affmae {
namespace {

constexpr int kWavesPerBlock = 4;

// 16 bytes of a row as fp32 values (the first E of v)
template <typename T>
struct Piece;
template <>
struct Piece<float> {
  static constexpr int E = 4;
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
struct Piece<bf16_t> {
  static constexpr int E = 8;
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

// Sums and maxima over lanes whose numbers differ in the bits LO .. HI (powers of two), every lane receiving the
// result.  The exchanges run on the vector ALU (DPP patterns inside a row of 16 lanes, the row / half swaps across
// rows): a softmax row costs some fifty of them, and through the LDS crossbar they were most of the kernel's time.
// All lanes of the wave must be active.
template <int J>
__device__ __forceinline__ float lane_xor_f(float x, int lane) {
  return __uint_as_float(lane_xor_u32<J>(__float_as_uint(x), lane));
}
template <int LO, int HI>
__device__ __forceinline__ float sum_bits(float x, int lane) {
  if constexpr (LO <= HI) {
    x += lane_xor_f<LO>(x, lane);
    return sum_bits<LO * 2, HI>(x, lane);
  } else {
    return x;
  }
}
template <int LO, int HI>
__device__ __forceinline__ float max_bits(float x, int lane) {
  if constexpr (LO <= HI) {
    x = fmaxf(x, lane_xor_f<LO>(x, lane));
    return max_bits<LO * 2, HI>(x, lane);
  } else {
    return x;
  }
}
// sum over the PP lanes of a row / over the 64 / PP rows of a trip (same piece) / over the wave
template <int PP>
__device__ __forceinline__ float row_sum(float x, int lane) { return sum_bits<1, PP / 2>(x, lane); }
template <int PP, int E>
__device__ __forceinline__ void rows_sum(float (&a)[8], int lane) {
#pragma unroll
  for (int i = 0; i < E; ++i) a[i] = sum_bits<PP, 32>(a[i], lane);
}
__device__ __forceinline__ float all_sum(float x, int lane) { return sum_bits<1, 32>(x, lane); }
__device__ __forceinline__ float all_max(float x, int lane) { return max_bits<1, 32>(x, lane); }
// exp(x) for x <= 0 or so: the library routine for fp32 storage (1e-5 bar), the hardware exp2 for bf16 storage
template <typename T>
__device__ __forceinline__ float exp_for(float x) {
  if constexpr (sizeof(T) == 2) return __builtin_amdgcn_exp2f(x * 1.4426950408889634f);
  else return expf(x);
}

// <a, b> over the 16 bytes at pa and pb: fp32 pieces by fused multiply-adds, bf16 pieces by four two-element dot
// instructions on the packed values (no unpacking)
__device__ __forceinline__ float dot_raw(const float* pa, const float* pb) {
  const float4 a = *reinterpret_cast<const float4*>(pa), b = *reinterpret_cast<const float4*>(pb);
  return fmaf(a.w, b.w, fmaf(a.z, b.z, fmaf(a.y, b.y, a.x * b.x)));
}
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ float dot_raw(const uint4& a, const uint4& b) {
  float acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), 0.f, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), acc, false);
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), acc, false);
}
__device__ __forceinline__ float dot_raw(const bf16_t* pa, const bf16_t* pb) {
  return dot_raw(*reinterpret_cast<const uint4*>(pa), *reinterpret_cast<const uint4*>(pb));
}

template <int E>
__device__ __forceinline__ float dot_piece(const float (&a)[8], const float (&b)[8]) {
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < E; ++i) acc = fmaf(a[i], b[i], acc);
  return acc;
}

// The neighbour rows of this lane in every trip: element offset of its piece in head 0 of the row, and whether the
// trip's row is one of the K (a row past the end repeats the last neighbour and gets weight 0).
template <int TR>
struct LaneRows {
  size_t off[TR];
  bool valid[TR];
};
template <int PP, int E>
__device__ __forceinline__ LaneRows<PP> lane_rows(int mynb, long long img_base, int C, int K, int lane) {
  constexpr int RPT = kWave / PP;
  const int rl = lane / PP, pc = lane % PP;
  LaneRows<PP> r;
#pragma unroll
  for (int t = 0; t < PP; ++t) {
    const int j = t * RPT + rl;
    r.valid[t] = j < K;
    const int nbj = __shfl(mynb, min(j, K - 1));
    r.off[t] = (size_t)(img_base + nbj) * C + (size_t)(pc * E);
  }
  return r;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void pla_fwd_general_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const T* __restrict__ bias,
    const int32_t* __restrict__ nbr_idx, const T* __restrict__ k_blank, const T* __restrict__ v_blank,
    long long tokens, int N, int H, int K, float scale, T* __restrict__ out, float* __restrict__ lse) {
  constexpr int E = Piece<T>::E, PP = D / E, RPT = kWave / PP, TR = PP;  // K <= 64 = RPT * TR
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int rl = lane / PP, pc = lane % PP;
  const int C = H * D;
  const int trips = (K + RPT - 1) / RPT;
  for (long long tok = (long long)blockIdx.x * kWavesPerBlock + wave; tok < tokens;
       tok += (long long)gridDim.x * kWavesPerBlock) {
    const long long img_base = (tok / N) * N;  // first token of this image
    const int mynb = min(max(nbr_idx[tok * K + min(lane, K - 1)], 0), N - 1);
    const LaneRows<TR> rows = lane_rows<PP, E>(mynb, img_base, C, K, lane);
    for (int h = 0; h < H; ++h) {
      const T* qrow = q + (tok * H + h) * D + pc * E;
      float s[TR], smax = -INFINITY;
#pragma unroll
      for (int t = 0; t < TR; ++t) {
        s[t] = -INFINITY;
        if (t < trips) {
          const float dot = row_sum<PP>(dot_raw(qrow, k + rows.off[t] + (size_t)h * D), lane);
          const float bj = (bias && rows.valid[t]) ? Elem<T>::load(bias + (tok * H + h) * K + t * RPT + rl) : 0.f;
          s[t] = rows.valid[t] ? fmaf(scale, dot, bj) : -INFINITY;
          smax = fmaxf(smax, s[t]);
        }
      }
      float sb = -INFINITY, eb = 0.f;
      if (k_blank) {
        sb = scale * row_sum<PP>(dot_raw(qrow, k_blank + (size_t)h * D + pc * E), lane);
      }
      const float m = fmaxf(all_max(smax, lane), sb);
      float e[TR], zl = 0.f;
#pragma unroll
      for (int t = 0; t < TR; ++t) {
        e[t] = 0.f;
        if (t < trips) {
          e[t] = rows.valid[t] ? exp_for<T>(s[t] - m) : 0.f;
          zl += e[t];
        }
      }
      if (k_blank) eb = exp_for<T>(sb - m);
      const float z = all_sum(pc == 0 ? zl : 0.f, lane) + eb;  // every row once
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < TR; ++t) {
        if (t < trips) {
          float vp[8];
          Piece<T>::load(v + rows.off[t] + (size_t)h * D, vp);
#pragma unroll
          for (int i = 0; i < E; ++i) acc[i] = fmaf(e[t], vp[i], acc[i]);
        }
      }
      rows_sum<PP, E>(acc, lane);
      if (v_blank) {
        float vb[8];
        Piece<T>::load(v_blank + (size_t)h * D + pc * E, vb);
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = fmaf(eb, vb[i], acc[i]);
      }
      if (rl == 0) {
        const float inv = 1.f / z;
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] *= inv;
        Piece<T>::store(out + (tok * H + h) * D + pc * E, acc);
      }
      if (lane == 0) lse[tok * H + h] = m + logf(z);
    }
  }
}

// Query side of the backward: dq, dbias, and p / dS of every (query, slot) pair for the key side; also the global
// token of every pair and the lowest and highest of a query's K, for the list builder.
template <typename T, int D>
__global__ __launch_bounds__(256) void pla_bwd_general_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const T* __restrict__ bias,
    const int32_t* __restrict__ nbr_idx, const T* __restrict__ k_blank, const T* __restrict__ v_blank,
    const float* __restrict__ lse, const T* __restrict__ dout, long long tokens, int N, int H, int K, float scale,
    T* __restrict__ dq, T* __restrict__ dbias, float* __restrict__ pw, float* __restrict__ dsw,
    int32_t* __restrict__ pair_tok, int2* __restrict__ bounds, float* __restrict__ dk_blank,
    float* __restrict__ dv_blank) {
  constexpr int E = Piece<T>::E, PP = D / E, RPT = kWave / PP, TR = PP;
  extern __shared__ float smem[];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int rl = lane / PP, pc = lane % PP;
  const int C = H * D;
  const int trips = (K + RPT - 1) / RPT;
  const bool blank_grad = k_blank && dk_blank;
  float* bacc = smem + (size_t)wave * 2 * C;  // [2][C] running blank-row gradients of this wave
  if (blank_grad)
    for (int c = lane; c < 2 * C; c += kWave) bacc[c] = 0.f;

  for (long long tok = (long long)blockIdx.x * kWavesPerBlock + wave; tok < tokens;
       tok += (long long)gridDim.x * kWavesPerBlock) {
    const long long img_base = (tok / N) * N;
    const int mynb = min(max(nbr_idx[tok * K + min(lane, K - 1)], 0), N - 1);
    const LaneRows<TR> rows = lane_rows<PP, E>(mynb, img_base, C, K, lane);
    {
      const int gtok = (int)(img_base + mynb);  // lanes >= K repeat the last neighbour
      if (lane < K) pair_tok[tok * K + lane] = gtok;
      int tmin = gtok, tmax = gtok;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        tmin = min(tmin, __shfl_xor(tmin, o));
        tmax = max(tmax, __shfl_xor(tmax, o));
      }
      if (lane == 0) bounds[tok] = make_int2(tmin, tmax);
    }
    for (int h = 0; h < H; ++h) {
      const T* qrow = q + (tok * H + h) * D + pc * E;
      const T* grow = dout + (tok * H + h) * D + pc * E;
      const float l = lse[tok * H + h];
      float kp[TR][8], p[TR], dP[TR], Dl = 0.f;
#pragma unroll
      for (int t = 0; t < TR; ++t) {
        p[t] = 0.f;
        dP[t] = 0.f;
        if (t < trips) {
          Piece<T>::load(k + rows.off[t] + (size_t)h * D, kp[t]);
          const float dot = row_sum<PP>(dot_raw(qrow, k + rows.off[t] + (size_t)h * D), lane);
          dP[t] = row_sum<PP>(dot_raw(grow, v + rows.off[t] + (size_t)h * D), lane);
          const float bj = (bias && rows.valid[t]) ? Elem<T>::load(bias + (tok * H + h) * K + t * RPT + rl) : 0.f;
          p[t] = rows.valid[t] ? exp_for<T>(fmaf(scale, dot, bj) - l) : 0.f;
          Dl = fmaf(p[t], dP[t], Dl);
        }
      }
      float pb = 0.f, dPb = 0.f, kb[8];
      if (k_blank) {
        Piece<T>::load(k_blank + (size_t)h * D + pc * E, kb);
        pb = exp_for<T>(scale * row_sum<PP>(dot_raw(qrow, k_blank + (size_t)h * D + pc * E), lane) - l);
        dPb = row_sum<PP>(dot_raw(grow, v_blank + (size_t)h * D + pc * E), lane);
      }
      const float Dsum = all_sum(pc == 0 ? Dl : 0.f, lane) + pb * dPb;  // every row once
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int t = 0; t < TR; ++t) {
        if (t < trips) {
          const float ds = p[t] * (dP[t] - Dsum);
          if (pc == 0 && rows.valid[t]) {
            const long long at = (tok * H + h) * K + t * RPT + rl;
            pw[at] = p[t];
            dsw[at] = ds;
            if (dbias) Elem<T>::store(dbias + at, ds);
          }
#pragma unroll
          for (int i = 0; i < E; ++i) acc[i] = fmaf(ds, kp[t][i], acc[i]);
        }
      }
      rows_sum<PP, E>(acc, lane);
      const float dsb = pb * (dPb - Dsum);
      if (k_blank) {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = fmaf(dsb, kb[i], acc[i]);
      }
      if (rl == 0) {
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] *= scale;
        Piece<T>::store(dq + (tok * H + h) * D + pc * E, acc);
        if (blank_grad) {
          float qv[8], gv[8];
          Piece<T>::load(qrow, qv);
          Piece<T>::load(grow, gv);
#pragma unroll
          for (int i = 0; i < E; ++i) {
            bacc[h * D + pc * E + i] += scale * dsb * qv[i];
            bacc[C + h * D + pc * E + i] += pb * gv[i];
          }
        }
      }
    }
  }
  if (blank_grad) {
    wave_lds_sync();
    for (int c = lane; c < C; c += kWave) {
      unsafeAtomicAdd(dk_blank + c, bacc[c]);
      unsafeAtomicAdd(dv_blank + c, bacc[C + c]);
    }
  }
}

// Key side of the backward: dk[t] = scale * sum over the pairs (i, j) filed under token t of dS[i,j] q[i],
// dv[t] = sum of p[i,j] dout[i]; a pair id is i * K + j with i the query's global token.  Tokens that nobody lists get
// zero rows.
template <typename T, int D>
__global__ __launch_bounds__(256) void pla_bwd_general_key_kernel(
    const T* __restrict__ q, const T* __restrict__ dout, const float* __restrict__ pw, const float* __restrict__ dsw,
    const int32_t* __restrict__ offset, const int32_t* __restrict__ list, long long tokens, int H, int K,
    uint32_t k_magic, float scale, T* __restrict__ dk, T* __restrict__ dv) {
  constexpr int E = Piece<T>::E, PP = D / E, RPT = kWave / PP;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int rl = lane / PP, pc = lane % PP;
  for (long long tok = (long long)blockIdx.x * kWavesPerBlock + wave; tok < tokens;
       tok += (long long)gridDim.x * kWavesPerBlock) {
    const int lo = offset[tok], n = offset[tok + 1] - lo;
    for (int h = 0; h < H; ++h) {
      float ak[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, av[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int base = 0; base < n; base += RPT) {
        const int idx = base + rl;
        const bool on = idx < n;
        const int pair = list[lo + min(idx, n - 1)];  // a row past the end repeats the last pair with weight 0
        const int i = exact_div(pair, K, k_magic), j = pair - i * K;
        const long long at = ((long long)i * H + h) * K + j;
        const float ps = on ? pw[at] : 0.f, dss = on ? dsw[at] : 0.f;
        float qp[8], gp[8];
        Piece<T>::load(q + ((long long)i * H + h) * D + pc * E, qp);
        Piece<T>::load(dout + ((long long)i * H + h) * D + pc * E, gp);
#pragma unroll
        for (int c = 0; c < E; ++c) {
          ak[c] = fmaf(dss, qp[c], ak[c]);
          av[c] = fmaf(ps, gp[c], av[c]);
        }
      }
      rows_sum<PP, E>(ak, lane);
      rows_sum<PP, E>(av, lane);
      if (rl == 0) {
#pragma unroll
        for (int c = 0; c < E; ++c) ak[c] *= scale;
        Piece<T>::store(dk + (tok * H + h) * D + pc * E, ak);
        Piece<T>::store(dv + (tok * H + h) * D + pc * E, av);
      }
    }
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0.f;
}

int grid_for(size_t n, int per_block, int cap) {
  size_t g = (n + per_block - 1) / per_block;
  if (g < 1) g = 1;
  if (g > (size_t)cap) g = cap;
  return (int)g;
}

size_t general_align(size_t n) { return (n + 255) & ~(size_t)255; }
struct GeneralBwdLayout {
  size_t p_off, ds_off, pair_off, bounds_off, offset_off, list_off, total;
};
GeneralBwdLayout general_bwd_layout(int B, int N, int H, int K) {
  GeneralBwdLayout L;
  const size_t tokens = (size_t)B * N, pairs = tokens * K;
  size_t off = 0;
  L.p_off = off;      off += general_align(pairs * H * sizeof(float));
  L.ds_off = off;     off += general_align(pairs * H * sizeof(float));
  L.pair_off = off;   off += general_align(pairs * sizeof(int32_t));
  L.bounds_off = off; off += general_align(tokens * 2 * sizeof(int32_t));
  L.offset_off = off; off += general_align((tokens + 1) * sizeof(int32_t));
  L.list_off = off;   off += general_align(pairs * sizeof(int32_t));
  L.total = off;
  return L;
}

template <typename T, int D>
hipError_t fwd_impl(const PlaArgs& a, hipStream_t stream) {
  const long long tokens = (long long)a.B * a.N;
  const int grid = grid_for((size_t)tokens, kWavesPerBlock, 1 << 20);
  AFFMAE_LAUNCH("pla_fwd_general_kernel", stream, (pla_fwd_general_kernel<T, D>), dim3(grid), dim3(256), 0, stream, (const T*)a.q,
                     (const T*)a.k, (const T*)a.v, (const T*)a.bias, a.nbr_idx, (const T*)a.k_blank,
                     (const T*)a.v_blank, tokens, a.N, a.H, a.K, a.scale, (T*)a.out, a.lse);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t bwd_impl(const PlaArgs& a, hipStream_t stream) {
  const long long tokens = (long long)a.B * a.N;
  if (tokens * a.K >= (1ll << 31)) return hipErrorInvalidValue;  // pair ids are 32-bit
  const GeneralBwdLayout L = general_bwd_layout(a.B, a.N, a.H, a.K);
  char* ws = static_cast<char*>(a.workspace);
  float* pw = reinterpret_cast<float*>(ws + L.p_off);
  float* dsw = reinterpret_cast<float*>(ws + L.ds_off);
  int32_t* pair_tok = reinterpret_cast<int32_t*>(ws + L.pair_off);
  int2* bounds = reinterpret_cast<int2*>(ws + L.bounds_off);
  int32_t* offset = reinterpret_cast<int32_t*>(ws + L.offset_off);
  int32_t* list = reinterpret_cast<int32_t*>(ws + L.list_off);
  const bool blank_grad = a.k_blank && a.dk_blank;
  if (blank_grad) {
    AFFMAE_LAUNCH("fill_zero_kernel", stream, fill_zero_kernel, dim3(1), dim3(256), 0, stream, a.dk_blank, (size_t)a.H * D);
    AFFMAE_LAUNCH("fill_zero_kernel", stream, fill_zero_kernel, dim3(1), dim3(256), 0, stream, a.dv_blank, (size_t)a.H * D);
  }
  const size_t lds = blank_grad ? kWavesPerBlock * 2 * (size_t)a.H * D * sizeof(float) : 0;
  // With blank gradients every wave keeps a running sum, so bound the grid.
  const int grid = grid_for((size_t)tokens, kWavesPerBlock, blank_grad ? 2048 : (1 << 20));
  AFFMAE_LAUNCH("pla_bwd_general_kernel", stream, (pla_bwd_general_kernel<T, D>), dim3(grid), dim3(256), lds, stream, (const T*)a.q,
                     (const T*)a.k, (const T*)a.v, (const T*)a.bias, a.nbr_idx, (const T*)a.k_blank,
                     (const T*)a.v_blank, a.lse, (const T*)a.dout, tokens, a.N, a.H, a.K, a.scale, (T*)a.dq,
                     (T*)a.dbias, pw, dsw, pair_tok, bounds, a.dk_blank, a.dv_blank);
  const hipError_t e = launch_pair_lists(pair_tok, a.B, a.N, a.N * a.K, offset, list, stream,
                                         reinterpret_cast<const int32_t*>(bounds), a.K);
  if (e != hipSuccess) return e;
  const int kgrid = grid_for((size_t)tokens, kWavesPerBlock, 1 << 20);
  AFFMAE_LAUNCH("pla_bwd_general_key_kernel", stream, (pla_bwd_general_key_kernel<T, D>), dim3(kgrid), dim3(256), 0, stream,
                (const T*)a.q, (const T*)a.dout, pw, dsw, offset, list, tokens, a.H, a.K, div_magic(a.K), a.scale,
                (T*)a.dk, (T*)a.dv);
  return hipGetLastError();
}

}  // namespace

size_t pla_bwd_general_workspace_bytes(int B, int N, int H, int K) { return general_bwd_layout(B, N, H, K).total; }

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
