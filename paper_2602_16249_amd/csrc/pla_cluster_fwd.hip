// Cluster-tiled local attention, forward (paper, Sec. "Flash-style Cluster
// Attention and Fast Decoder KNN": stream over tiles, never store the scores,
// fp32 softmax statistics; the equation is FlashNbhdAttn).
//
// Valid when tokens are stored in cluster order and every neighbour of a token
// lies in one of its cluster's M near clusters (the table affmae_knn builds), bf16
// storage, d = 32, S a multiple of 16.
//
// One workgroup per cluster, one wave per strip of 16 queries.  The K and V rows
// of the cluster's M*S candidate tokens are staged through LDS in chunks of 256
// candidates (V transposed, so that candidates are contiguous), shared by all
// strips.  Per strip and pair of 16-candidate tiles the scores of all 16x32
// (query, candidate) pairs come from two MFMAs, computed transposed (candidates x
// queries) so that the probabilities leave the softmax already in the operand
// layout of the P.V MFMAs.  A query only attends to its K neighbours: their
// bias values are scattered into a per-wave LDS tile that holds -inf everywhere
// else, which is added to the scores; candidate tiles that hold no neighbour of
// the strip are skipped altogether.
#include "device_util.h"
#include "launch.h"
#include "timing.h"

namespace affmae {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kD = 32;             // channels per head
constexpr int kChunk = 256;        // candidates staged at a time
constexpr int kKRow = kD + 8;      // bf16 per staged K row (80 B: conflict-free 16 B reads)
constexpr int kVRow = kChunk + 8;  // bf16 per staged V^T row
constexpr int kTilesPerChunk = kChunk / 16;
constexpr int kMaxEntries = 16;    // (16 queries * K <= 64 neighbours) / 64 lanes
constexpr uint32_t kNoPos = 0xffffu;

union Frag8 {
  bf16x8 v;
  uint4 u4;
  uint2 u2[2];
  uint32_t u[4];
  uint16_t h[8];
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

__device__ __forceinline__ uint32_t wave_or(uint32_t x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x |= __shfl_xor(x, o);
  return x;
}

struct FwdParams {
  const bf16_t *q, *k, *v, *bias;
  const int32_t* nbr_idx;
  const int32_t* near;
  const bf16_t *k_blank, *v_blank;
  int N, H, K, S, M, G;
  float scale;
  bf16_t* out;
  float* lse;
};

// Stage candidates [c0, c0 + kChunk) of the cluster's list: K rows as they are,
// V rows transposed.  Positions at or beyond Cn are zero-filled.
__device__ __forceinline__ void stage_chunk(const FwdParams& p, long long img_base, const int32_t* near_c, int c0,
                                            int Cn, int h, bf16_t* Ks, bf16_t* Vt) {
  const int C = p.H * kD;
  // K: thread -> (row, 16-byte piece)
  for (int w = threadIdx.x; w < kChunk * 4; w += blockDim.x) {
    const int row = w >> 2, piece = w & 3;
    const int pos = c0 + row;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (pos < Cn) {
      const int m = pos / p.S, r = pos - m * p.S;
      const int e = min(max(near_c[m], 0), p.G - 1);
      const long long tok = img_base + (long long)e * p.S + r;
      val = *reinterpret_cast<const uint4*>(p.k + tok * C + h * kD + piece * 8);
    }
    *reinterpret_cast<uint4*>(Ks + row * kKRow + piece * 8) = val;
  }
  // V: thread -> (group of 4 candidates, 8 channels); writes 8 transposed 4-vectors
  for (int w = threadIdx.x; w < (kChunk / 4) * 4; w += blockDim.x) {
    const int grp = w >> 2, oct = w & 3;
    uint4 rows[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int pos = c0 + grp * 4 + i;
      rows[i] = make_uint4(0, 0, 0, 0);
      if (pos < Cn) {
        const int m = pos / p.S, r = pos - m * p.S;
        const int e = min(max(near_c[m], 0), p.G - 1);
        const long long tok = img_base + (long long)e * p.S + r;
        rows[i] = *reinterpret_cast<const uint4*>(p.v + tok * C + h * kD + oct * 8);
      }
    }
    const uint32_t* r0 = reinterpret_cast<const uint32_t*>(&rows[0]);
    const uint32_t* r1 = reinterpret_cast<const uint32_t*>(&rows[1]);
    const uint32_t* r2 = reinterpret_cast<const uint32_t*>(&rows[2]);
    const uint32_t* r3 = reinterpret_cast<const uint32_t*>(&rows[3]);
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {  // channel pair 2*e2, 2*e2+1 of this octet
      uint2 lo, hi;
      lo.x = (r0[e2] & 0xffffu) | (r1[e2] << 16);
      lo.y = (r2[e2] & 0xffffu) | (r3[e2] << 16);
      hi.x = (r0[e2] >> 16) | (r1[e2] & 0xffff0000u);
      hi.y = (r2[e2] >> 16) | (r3[e2] & 0xffff0000u);
      const int ch = oct * 8 + e2 * 2;
      *reinterpret_cast<uint2*>(Vt + (ch + 0) * kVRow + grp * 4) = lo;
      *reinterpret_cast<uint2*>(Vt + (ch + 1) * kVRow + grp * 4) = hi;
    }
  }
}

__global__ __launch_bounds__(1024) void pla_fwd_cluster_kernel(FwdParams p) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem_raw);
  bf16_t* Vt = Ks + kChunk * kKRow;
  bf16_t* scratch_all = Vt + kD * kVRow;

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int g = lane >> 4, r = lane & 15;
  const int b = blockIdx.x / p.G, c = blockIdx.x % p.G;
  const long long img_base = (long long)b * p.N;
  const long long tok0 = img_base + (long long)c * p.S + wave * 16;  // first query of this strip
  const int32_t* near_c = p.near + ((size_t)b * p.G + c) * p.M;
  const int Cn = p.M * p.S;
  const int nchunks = (Cn + kChunk - 1) / kChunk;
  const int C = p.H * kD;
  const int K = p.K;
  bf16_t* scratch = scratch_all + (size_t)wave * kTilesPerChunk * 256;

  // Position of every (query, slot) of the strip in the cluster's candidate list.
  // Low 16 bits: the position (kNoPos if the promise is broken), bits 16..19: the query.
  uint32_t pos[kMaxEntries];
  const int nent = 16 * K;
#pragma unroll
  for (int t = 0; t < kMaxEntries; ++t) {
    pos[t] = kNoPos;
    const int e = t * kWave + lane;
    if (e < nent) {
      const int n = p.nbr_idx[tok0 * K + e];  // [16 queries][K] is contiguous
      const int ecl = n / p.S, rr = n - ecl * p.S;
      uint32_t where = kNoPos;
      for (int m = 0; m < p.M; ++m)
        if (near_c[m] == ecl && n >= 0) where = (uint32_t)(m * p.S + rr);
      pos[t] = where | ((uint32_t)(e / K) << 16);
    }
  }

  for (int h = 0; h < p.H; ++h) {
    // Q^T operand: lane (query r, channels 8g..8g+7)
    Frag8 qf;
    qf.u4 = *reinterpret_cast<const uint4*>(p.q + (tok0 + r) * C + h * kD + g * 8);
    uint16_t bias_bits[kMaxEntries];
#pragma unroll
    for (int t = 0; t < kMaxEntries; ++t) {
      bias_bits[t] = 0;
      const int e = t * kWave + lane;
      if (p.bias && e < nent) bias_bits[t] = p.bias[(tok0 * K + e) * p.H + h];
    }
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};

    for (int ch = 0; ch < nchunks; ++ch) {
      __syncthreads();
      stage_chunk(p, img_base, near_c, ch * kChunk, Cn, h, Ks, Vt);
      __syncthreads();

      // which 16-candidate tiles of this chunk hold a neighbour of the strip
      uint32_t tm = 0;
#pragma unroll
      for (int t = 0; t < kMaxEntries; ++t)
        if ((pos[t] & 0xffffu) != kNoPos && ((pos[t] & 0xffffu) >> 8) == (uint32_t)ch) tm |= 1u << ((pos[t] & 255) >> 4);
      tm = __builtin_amdgcn_readfirstlane(wave_or(tm));
      if (tm == 0) continue;
      // -inf everywhere in those tiles, then the bias of the real neighbours
      for (uint32_t rest = tm; rest; rest &= rest - 1) {
        const int tile = __builtin_ctz(rest);
        *reinterpret_cast<uint2*>(scratch + tile * 256 + lane * 4) =
            make_uint2(0xff80ff80u, 0xff80ff80u);
      }
      wave_lds_sync();
#pragma unroll
      for (int t = 0; t < kMaxEntries; ++t) {
        if ((pos[t] & 0xffffu) != kNoPos && ((pos[t] & 0xffffu) >> 8) == (uint32_t)ch) {
          const int qi = pos[t] >> 16;
          const int local = pos[t] & 255;
          scratch[(local >> 4) * 256 + qi * 16 + (local & 15)] = bias_bits[t];
        }
      }
      wave_lds_sync();

      for (int pair = 0; pair < kTilesPerChunk / 2; ++pair) {
        const uint32_t bits = (tm >> (2 * pair)) & 3u;
        if (bits == 0) continue;
        float s[8];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          if (bits & (1u << tt)) {
            const int tile = pair * 2 + tt;
            Frag8 kf;
            kf.u4 = *reinterpret_cast<const uint4*>(Ks + (tile * 16 + r) * kKRow + g * 8);
            f32x4 st = {0.f, 0.f, 0.f, 0.f};
            st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, qf.v, st, 0, 0, 0);
            const uint2 bm = *reinterpret_cast<const uint2*>(scratch + tile * 256 + r * 16 + g * 4);
            s[4 * tt + 0] = fmaf(st[0], p.scale, __uint_as_float(bm.x << 16));
            s[4 * tt + 1] = fmaf(st[1], p.scale, __uint_as_float(bm.x & 0xffff0000u));
            s[4 * tt + 2] = fmaf(st[2], p.scale, __uint_as_float(bm.y << 16));
            s[4 * tt + 3] = fmaf(st[3], p.scale, __uint_as_float(bm.y & 0xffff0000u));
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) s[4 * tt + i] = -INFINITY;
          }
        }
        float mx = s[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) mx = fmaxf(mx, s[i]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __expf(m_run - m_safe);
        float pr[8], psum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          pr[i] = __expf(s[i] - m_safe);
          psum += pr[i];
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[dt][i] *= alpha;
        Frag8 pf;  // P^T operand: k-slots 0..3 = tile 0 candidates 4g..4g+3, 4..7 = tile 1
        pf.u[0] = pack_bf16x2(pr[0], pr[1]);
        pf.u[1] = pack_bf16x2(pr[2], pr[3]);
        pf.u[2] = pack_bf16x2(pr[4], pr[5]);
        pf.u[3] = pack_bf16x2(pr[6], pr[7]);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          Frag8 vf;  // V^T operand: lane (channel dt*16 + r, the same candidates)
          const bf16_t* vrow = Vt + (dt * 16 + r) * kVRow + pair * 32 + g * 4;
          vf.u2[0] = *reinterpret_cast<const uint2*>(vrow);
          vf.u2[1] = *reinterpret_cast<const uint2*>(vrow + 16);
          acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pf.v, acc[dt], 0, 0, 0);
        }
      }
    }

    // The probabilities that entered the MFMAs were rounded to bf16; the
    // denominator uses the unrounded ones, as the definition does.
    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    float m_fin = m_run;
    if (p.k_blank) {
      Frag8 kb;
      kb.u4 = *reinterpret_cast<const uint4*>(p.k_blank + h * kD + g * 8);
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) part = fmaf(bf16_to_f32(qf.h[i]), bf16_to_f32(kb.h[i]), part);
      part += __shfl_xor(part, 16);
      part += __shfl_xor(part, 32);
      const float sb = p.scale * part;
      m_fin = fmaxf(m_run, sb);
      const float alpha = __expf(m_run - m_fin);
      const float pb = __expf(sb - m_fin);
      l_tot = l_tot * alpha + pb;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          acc[dt][i] = acc[dt][i] * alpha + pb * bf16_to_f32(p.v_blank[h * kD + dt * 16 + g * 4 + i]);
    }
    const float inv = 1.f / l_tot;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
      uint2 o;
      o.x = pack_bf16x2(acc[dt][0] * inv, acc[dt][1] * inv);
      o.y = pack_bf16x2(acc[dt][2] * inv, acc[dt][3] * inv);
      *reinterpret_cast<uint2*>(p.out + (tok0 + r) * C + h * kD + dt * 16 + g * 4) = o;
    }
    if (g == 0) p.lse[(tok0 + r) * p.H + h] = m_fin + __logf(l_tot);
  }
}

}  // namespace

bool pla_cluster_supported(const PlaArgs& a) {
  if (!a.near_clusters || a.dtype != 1 || a.d != kD) return false;
  if (a.S % 16 || a.S < 16 || a.S > 128) return false;  // one wave per 16 queries; LDS scratch per wave
  if (a.K > 64 || (long long)a.M * a.S > 65535 - 256) return false;
  return true;
}

size_t pla_fwd_cluster_lds_bytes(int S) {
  return (size_t)(kChunk * kKRow + kD * kVRow) * 2 + (size_t)(S / 16) * kTilesPerChunk * 256 * 2;
}

hipError_t launch_pla_fwd_cluster(const PlaArgs& a, hipStream_t stream) {
  FwdParams p;
  p.q = (const bf16_t*)a.q; p.k = (const bf16_t*)a.k; p.v = (const bf16_t*)a.v; p.bias = (const bf16_t*)a.bias;
  p.nbr_idx = a.nbr_idx; p.near = a.near_clusters;
  p.k_blank = (const bf16_t*)a.k_blank; p.v_blank = (const bf16_t*)a.v_blank;
  p.N = a.N; p.H = a.H; p.K = a.K; p.S = a.S; p.M = a.M; p.G = a.N / a.S;
  p.scale = a.scale;
  p.out = (bf16_t*)a.out; p.lse = a.lse;
  const size_t lds = pla_fwd_cluster_lds_bytes(a.S);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pla_fwd_cluster_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  AFFMAE_LAUNCH("pla_fwd_cluster_kernel", stream, pla_fwd_cluster_kernel, dim3(a.B * p.G), dim3(a.S / 16 * kWave),
                lds, stream, p);
  return hipGetLastError();
}

}  // namespace affmae
