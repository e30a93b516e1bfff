// Plan of the cluster-tiled attention kernels, built from the neighbour table
// (paper, Sec. "Limitations": neighbourhood tables are cached per encoder stage
// and reused by every block; the plan is such a table in the layout the tiled
// kernels read).  One wave per strip of 16 queries.
#include "cluster_common.h"
#include "launch.h"
#include "timing.h"

namespace affmae {
namespace {

struct PlanParams {
  const int32_t* nbr_idx;  // [B,N,K]
  const int32_t* near;     // [B,G,M]
  int N, K, S, M, G;
  uint32_t s_magic, k_magic;
  int strips, strips_per_image, slot_stride;
  uint16_t* slots;    // [strips][slot_stride]
  uint16_t* entries;  // [strips][16*K]
};

__device__ __forceinline__ unsigned long long wave_or64(unsigned long long x) {
  uint32_t lo = wave_or32((uint32_t)x), hi = wave_or32((uint32_t)(x >> 32));
  return ((unsigned long long)hi << 32) | lo;
}

__global__ __launch_bounds__(256) void pla_plan_kernel(PlanParams p) {
  const int lane = threadIdx.x & (kWave - 1);
  const int sg = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (sg >= p.strips) return;  // wave-uniform
  const int b = sg / p.strips_per_image;
  const int q0 = (sg - b * p.strips_per_image) * 16;  // first query, within the image
  const int c = fast_div(q0, p.s_magic);
  const int32_t* near_c = p.near + ((size_t)b * p.G + c) * p.M;
  const int tiles_per_cluster = p.S / 16;
  const int nent = 16 * p.K;
  const int32_t* nbr = p.nbr_idx + ((size_t)b * p.N + q0) * p.K;

  // candidate-list tile of every (query, slot): m * (S/16) + (token % S) / 16
  int ct[kMaxEntries], tok[kMaxEntries];
  unsigned long long mask = 0;
#pragma unroll
  for (int t = 0; t < kMaxEntries; ++t) {
    ct[t] = -1;
    tok[t] = 0;
    const int e = t * kWave + lane;
    if (e < nent) {
      const int n = nbr[e];
      const int nn = min(max(n, 0), p.N - 1);
      const int ecl = fast_div(nn, p.s_magic);
      int where = -1;
      for (int m = 0; m < p.M; ++m)
        if (near_c[m] == ecl) where = m;
      if (where >= 0 && n == nn) {
        ct[t] = where * tiles_per_cluster + ((nn - ecl * p.S) >> 4);
        tok[t] = nn;
        mask |= 1ull << ct[t];
      }
    }
  }
  mask = wave_or64(mask);
  uint16_t* ent = p.entries + (size_t)sg * nent;
#pragma unroll
  for (int t = 0; t < kMaxEntries; ++t) {
    const int e = t * kWave + lane;
    if (e < nent) {
      uint32_t off = kNoEntry;
      if (ct[t] >= 0) {
        const int slot = __popcll(mask & ((1ull << ct[t]) - 1ull));
        off = (uint32_t)(slot * 256 + fast_div(e, p.k_magic) * 16 + (tok[t] & 15));
      }
      ent[e] = (uint16_t)off;
    }
  }
  // slot table: count, then the token tile of every slot; padding repeats a valid tile
  uint16_t* sl = p.slots + (size_t)sg * p.slot_stride;
  const int count = __popcll(mask);
  int my_tile = -1;
  if ((mask >> lane) & 1ull) {
    const int m = lane / tiles_per_cluster, tt = lane - m * tiles_per_cluster;
    const int e = min(max(near_c[m], 0), p.G - 1);
    my_tile = e * tiles_per_cluster + tt;  // token tile within the image
    sl[1 + __popcll(mask & ((1ull << lane) - 1ull))] = (uint16_t)my_tile;
  }
  const int own_tile = q0 >> 4;
  if (lane == 0) sl[0] = (uint16_t)count;
  for (int s = count + lane; s < p.slot_stride - 1; s += kWave) sl[1 + s] = (uint16_t)own_tile;
}

}  // namespace

hipError_t launch_pla_plan(const int32_t* nbr_idx, const int32_t* near, int B, int N, int K, int S, int M, void* plan,
                           hipStream_t stream) {
  const PlanLayout L = make_plan_layout(B, N, K, S, M);
  PlanParams p;
  p.nbr_idx = nbr_idx; p.near = near;
  p.N = N; p.K = K; p.S = S; p.M = M; p.G = N / S;
  p.s_magic = div_magic(S); p.k_magic = div_magic(K);
  p.strips = L.strips; p.strips_per_image = N / 16; p.slot_stride = L.slot_stride;
  p.slots = reinterpret_cast<uint16_t*>(static_cast<char*>(plan) + L.slots_off);
  p.entries = reinterpret_cast<uint16_t*>(static_cast<char*>(plan) + L.entries_off);
  AFFMAE_LAUNCH("pla_plan_kernel", stream, pla_plan_kernel, dim3((L.strips + 3) / 4), dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace affmae
