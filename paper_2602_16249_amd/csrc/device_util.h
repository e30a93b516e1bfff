// Internal device helpers shared by the HIP kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace affmae {

constexpr int kWave = 64;

typedef uint16_t bf16_t;  // bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

// Round to nearest, ties to even.  NaN stays NaN (quiet bit forced).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <>
struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Load D contiguous elements (row start aligned to 16 bytes) into fp32 registers.
template <int D>
__device__ __forceinline__ void load_row(const float* p, float (&r)[D]) {
  const float4* p4 = reinterpret_cast<const float4*>(p);
#pragma unroll
  for (int t = 0; t < D / 4; ++t) {
    float4 x = p4[t];
    r[4 * t + 0] = x.x;
    r[4 * t + 1] = x.y;
    r[4 * t + 2] = x.z;
    r[4 * t + 3] = x.w;
  }
}
template <int D>
__device__ __forceinline__ void load_row(const bf16_t* p, float (&r)[D]) {
  const uint4* p4 = reinterpret_cast<const uint4*>(p);
#pragma unroll
  for (int t = 0; t < D / 8; ++t) {
    uint4 x = p4[t];
    uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      r[8 * t + 2 * e + 0] = __uint_as_float(w[e] << 16);
      r[8 * t + 2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
  }
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// Orders LDS traffic between the lanes of one wave (no workgroup barrier).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// Cell of a relative-position table (paper, Sec. "AutoFocusFormer": relative position from the 2-D token
// coordinates): along each axis clamp(rint((nbr - query) * rate), -R, R), in fp32 one operation at a time, ties
// to even; cell = (by + R) * (2R + 1) + bx + R.  Every kernel that needs a cell calls this, so that all of them
// take the same integer decision.  The clamped offsets are small integers held in fp32, so combining them with
// one fused multiply-add is exact; a NaN offset lands on -R (the median instruction returns the minimum then).
__device__ __forceinline__ float relpos_axis(float nbr, float query, float rate, float Rf) {
#pragma clang fp contract(off)
  const float d = nbr - query;
  const float t = d * rate;
  return __builtin_amdgcn_fmed3f(__builtin_rintf(t), -Rf, Rf);
}
__device__ __forceinline__ int relpos_cell(float2 nbr, float2 query, float rate, int R) {
  const float Rf = (float)R;
  const float c = __builtin_fmaf(relpos_axis(nbr.y, query.y, rate, Rf), (float)(2 * R + 1),
                                 relpos_axis(nbr.x, query.x, rate, Rf));
  return (int)c + (R * (2 * R + 1) + R);
}

}  // namespace affmae
