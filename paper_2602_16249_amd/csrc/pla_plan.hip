// Plan of the cluster-tiled attention kernels, built from the neighbour table
// (paper, Sec. "Limitations": neighbourhood tables are cached per encoder stage
// and reused by every block; the plan is such a table in the layout the tiled
// kernels read).  Forward tables: one wave per strip of 16 queries.  Reverse
// tables (which strips touch a token tile): count, prefix sum, fill, sort.
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
  int strips, strips_per_image, slot_stride, max_slots;
  uint16_t* slots;    // [strips][slot_stride]
  uint16_t* entries;  // [strips][16*K]
  int32_t* rev_count;
  int32_t* rev_offset;
  int32_t* rev_cursor;
  unsigned long long* rev_list;
  uint16_t* sorted_pos;  // [strips][places]
  uint16_t* runs;        // [strips][runs_stride]
  int runs_stride, places;
};

__device__ __forceinline__ unsigned long long wave_or64(unsigned long long x) {
  uint32_t lo = wave_or32((uint32_t)x), hi = wave_or32((uint32_t)(x >> 32));
  return ((unsigned long long)hi << 32) | lo;
}

__global__ __launch_bounds__(256) void plan_zero_kernel(int32_t* a, int32_t* b, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    a[i] = 0;
    b[i] = 0;
  }
}

// NE = entries per lane: 16 K / 64 rounded up to a multiple of 4 (the loops over a lane's entries are unrolled)
template <int NE>
__global__ __launch_bounds__(256) void pla_plan_kernel(PlanParams p) {
  __shared__ uint16_t sorted_all[4][NE * kWave + kMaxSlots];
  __shared__ int slot_count_all[4][kMaxSlots];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform: keeps per-wave indices in SGPRs
  const int sg = blockIdx.x * (blockDim.x / kWave) + wave;
  if (sg >= p.strips) return;  // wave-uniform; no workgroup barrier below
  uint16_t* sorted = sorted_all[wave];
  int* slot_count = slot_count_all[wave];
  const int b = sg / p.strips_per_image;
  const int q0 = (sg - b * p.strips_per_image) * 16;  // first query, within the image
  const int c = fast_div(q0, p.s_magic);
  const int32_t* near_c = p.near + ((size_t)b * p.G + c) * p.M;
  const int tiles_per_cluster = p.S / 16;
  const int nent = 16 * p.K;
  const int nent_real = min(16, p.N - q0) * p.K;  // the image's last strip may hold fewer than 16 queries
  const int32_t* nbr = p.nbr_idx + ((size_t)b * p.N + q0) * p.K;

  // candidate-list tile of every (query, slot): m * (S/16) + (token % S) / 16
  const int near_v = (lane < p.M) ? near_c[lane] : -1;  // lane m: the m-th near cluster (M <= 64)
  int ct[NE], tok[NE], ecl[NE], where[NE];
  bool inr[NE];
#pragma unroll
  for (int t = 0; t < NE; ++t) {
    const int e = t * kWave + lane;
    const int n = (e < nent_real) ? nbr[e] : -1;  // queries past the end have no entries
    const int nn = min(max(n, 0), p.N - 1);
    inr[t] = e < nent && n == nn;
    tok[t] = nn;
    ecl[t] = fast_div(nn, p.s_magic);
    where[t] = -1;
  }
  for (int m = 0; m < p.M; ++m) {  // the last match wins, as a scan of the list would have it
    const int cl = __builtin_amdgcn_readlane(near_v, m);
#pragma unroll
    for (int t = 0; t < NE; ++t) where[t] = (ecl[t] == cl) ? m : where[t];
  }
  unsigned long long mask = 0;
#pragma unroll
  for (int t = 0; t < NE; ++t) {
    ct[t] = -1;
    if (inr[t] && where[t] >= 0) {
      ct[t] = where[t] * tiles_per_cluster + ((tok[t] - ecl[t] * p.S) >> 4);
      mask |= 1ull << ct[t];
    } else {
      tok[t] = 0;
    }
  }
  mask = wave_or64(mask);
  uint16_t* ent = p.entries + (size_t)sg * nent;
  uint32_t off[NE];
#pragma unroll
  for (int t = 0; t < NE; ++t) {
    const int e = t * kWave + lane;
    off[t] = kNoEntry;
    if (e < nent) {
      if (ct[t] >= 0) {
        const int slot = __popcll(mask & ((1ull << ct[t]) - 1ull));
        off[t] = (uint32_t)(slot * 256 + tile_cell(fast_div(e, p.k_magic), tok[t] & 15));
      }
      ent[e] = (uint16_t)off[t];
    }
  }
  // slot table: count, then the token tile of every slot; padding repeats a valid tile
  uint16_t* sl = p.slots + (size_t)sg * p.slot_stride;
  const int count = __popcll(mask);
  if ((mask >> lane) & 1ull) {
    const int m = lane / tiles_per_cluster, tt = lane - m * tiles_per_cluster;
    const int e = min(max(near_c[m], 0), p.G - 1);
    const int my_tile = e * tiles_per_cluster + tt;  // token tile within the image
    sl[1 + __popcll(mask & ((1ull << lane) - 1ull))] = (uint16_t)my_tile;
    atomicAdd(p.rev_count + (size_t)b * p.strips_per_image + my_tile, 1);
  }
  const int own_tile = q0 >> 4;
  if (lane == 0) sl[0] = (uint16_t)count;
  for (int s = count + lane; s < p.slot_stride - 1; s += kWave) sl[1 + s] = (uint16_t)own_tile;

  // runs: the valid entries grouped by slot, every run starting at an even place; assembled in LDS and written
  // out in rows.  Unused places hold kNoEntry.  Two sweeps over the lane's entries with LDS counters per slot:
  // count, then claim a place (the order inside a run is the order in which the wave's LDS atomics are served;
  // any order gives the same results downstream, where every entry is addressed by its own value).
  for (int w = lane; w < NE * kWave + kMaxSlots; w += kWave) sorted[w] = (uint16_t)kNoEntry;
  if (lane < kMaxSlots) slot_count[lane] = 0;
  wave_lds_sync();
#pragma unroll
  for (int t = 0; t < NE; ++t)
    if (off[t] != kNoEntry) atomicAdd(&slot_count[off[t] >> 8], 1);
  wave_lds_sync();
  uint16_t* runs = p.runs + (size_t)sg * p.runs_stride;
  // exclusive prefix over the slots, every start rounded up to an even place (lane s: slot s)
  int mine = (lane < count) ? slot_count[lane] : 0;
  mine = (mine + 1) & ~1;
  int incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  const int start = incl - mine;
  const int last_count = __shfl((lane < count) ? slot_count[lane] : 0, max(count - 1, 0));
  const int last_start = __shfl(start, max(count - 1, 0));
  int place = count > 0 ? last_start + last_count : 0;  // places used: the last run is not padded
  wave_lds_sync();
  if (lane < count) {
    runs[lane] = (uint16_t)start;
    slot_count[lane] = start;  // becomes the cursor of the slot
  }
  wave_lds_sync();
#pragma unroll
  for (int t = 0; t < NE; ++t)
    if (off[t] != kNoEntry) sorted[atomicAdd(&slot_count[off[t] >> 8], 1)] = (uint16_t)off[t];
  if (lane == 0) runs[count] = (uint16_t)place;
  wave_lds_sync();
  uint16_t* sp = p.sorted_pos + (size_t)sg * p.places;
  for (int w = lane; w < p.places; w += kWave) sp[w] = sorted[w];
}

// Exclusive prefix sum of rev_count.  Workgroup j owns elements [1024 j, 1024 j + 1024): it first adds up
// everything before them (coalesced reads of a few hundred KB at most, all from L2), then scans its own.
// No workgroup waits for another.
__global__ __launch_bounds__(256) void plan_scan_kernel(const int32_t* __restrict__ count, int32_t* __restrict__ offset,
                                                       int n) {
  __shared__ int32_t part[4];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int first = blockIdx.x * 1024;
  int before = 0;
  for (int i = tid * 4; i < first; i += 1024) {  // first is a multiple of 1024: whole 16-byte pieces
    const int4 v = *reinterpret_cast<const int4*>(count + i);
    before += v.x + v.y + v.z + v.w;
  }
  // this thread's four elements
  const int at = first + tid * 4;
  int c[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) c[i] = (at + i < n) ? count[at + i] : 0;
  const int mine = c[0] + c[1] + c[2] + c[3];
  // wave-inclusive scan of (mine) and wave sum of (before)
  int incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) before += __shfl_xor(before, o);
  if (lane == kWave - 1) part[wave] = incl;
  __shared__ int32_t before_all[4];
  if (lane == 0) before_all[wave] = before;
  __syncthreads();
  int base = before_all[0] + before_all[1] + before_all[2] + before_all[3];
  for (int w = 0; w < wave; ++w) base += part[w];
  int run = base + incl - mine;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (at + i < n) offset[at + i] = run;
    run += c[i];
  }
  if (at <= n - 1 && n - 1 < at + 4) offset[n] = run;  // the thread that owns the last element: run is the total
}

// Every strip appends itself to the list of each token tile it touches.
__global__ __launch_bounds__(256) void plan_fill_kernel(PlanParams p) {
  const int lane = threadIdx.x & (kWave - 1);
  const int sg = blockIdx.x * (blockDim.x / kWave) + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (sg >= p.strips) return;
  const int b = sg / p.strips_per_image;
  const int strip_in_image = sg - b * p.strips_per_image;
  const uint16_t* sl = p.slots + (size_t)sg * p.slot_stride;
  const int count = min((int)sl[0], p.max_slots);
  if (lane < count) {
    const size_t kt = (size_t)b * p.strips_per_image + sl[1 + lane];
    const int at = atomicAdd(p.rev_cursor + kt, 1);
    const uint16_t* runs = p.runs + (size_t)sg * p.runs_stride;
    const uint32_t start = runs[lane], len = (uint32_t)runs[lane + 1] - start;  // len may count one pad place
    p.rev_list[(size_t)p.rev_offset[kt] + at] =
        ((unsigned long long)(start | (len << 16)) << 32) | (((uint32_t)strip_in_image << 8) | (uint32_t)lane);
  }
}

// Sort every token tile's list ascending by (strip, slot): rank by counting (lists are short).
__global__ __launch_bounds__(256) void plan_sort_kernel(PlanParams p) {
  const int lane = threadIdx.x & (kWave - 1);
  const int kt = blockIdx.x * (blockDim.x / kWave) + __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (kt >= p.strips) return;
  const int lo = p.rev_offset[kt], n = p.rev_offset[kt + 1] - lo;
  unsigned long long* list = p.rev_list + lo;
  if (n <= kWave) {
    const unsigned long long mine = lane < n ? list[lane] : ~0ull;
    const uint32_t key = (uint32_t)mine;
    int rank = 0;
    for (int j = 0; j < n; ++j) rank += (__shfl(key, j) < key) ? 1 : 0;  // keys are distinct
    if (lane < n) list[rank] = mine;  // every lane has read its element before any write lands (one wave)
  } else if (lane == 0) {
    for (int i = 1; i < n; ++i) {  // insertion sort; only for unusually popular tiles
      const unsigned long long v = list[i];
      int j = i - 1;
      while (j >= 0 && (uint32_t)list[j] > (uint32_t)v) {
        list[j + 1] = list[j];
        --j;
      }
      list[j + 1] = v;
    }
  }
}

}  // namespace

hipError_t launch_pla_plan(const int32_t* nbr_idx, const int32_t* near, int B, int N, int K, int S, int M, void* plan,
                           hipStream_t stream) {
  const PlanLayout L = make_plan_layout(B, N, K, S, M);
  char* base = static_cast<char*>(plan);
  PlanParams p;
  p.nbr_idx = nbr_idx; p.near = near;
  p.N = N; p.K = K; p.S = S; p.M = M; p.G = (N + S - 1) / S;  // the last cluster may be short
  p.s_magic = div_magic(S); p.k_magic = div_magic(K);
  p.strips = L.strips; p.strips_per_image = (N + 15) / 16; p.slot_stride = L.slot_stride; p.max_slots = L.max_slots;
  p.slots = reinterpret_cast<uint16_t*>(base + L.slots_off);
  p.entries = reinterpret_cast<uint16_t*>(base + L.entries_off);
  p.rev_count = reinterpret_cast<int32_t*>(base + L.rev_count_off);
  p.rev_offset = reinterpret_cast<int32_t*>(base + L.rev_offset_off);
  p.rev_cursor = reinterpret_cast<int32_t*>(base + L.rev_cursor_off);
  p.rev_list = reinterpret_cast<unsigned long long*>(base + L.rev_list_off);
  p.sorted_pos = reinterpret_cast<uint16_t*>(base + L.sorted_pos_off);
  p.runs = reinterpret_cast<uint16_t*>(base + L.runs_off);
  p.runs_stride = L.runs_stride; p.places = L.places;
  const dim3 per_strip((L.strips + 3) / 4);
  AFFMAE_LAUNCH("plan_zero_kernel", stream, plan_zero_kernel, dim3((L.strips + 255) / 256), dim3(256), 0, stream,
                p.rev_count, p.rev_cursor, L.strips);
  const int ne = (16 * K + kWave - 1) / kWave;
  if (ne <= 4) AFFMAE_LAUNCH("pla_plan_kernel", stream, pla_plan_kernel<4>, per_strip, dim3(256), 0, stream, p);
  else if (ne <= 8) AFFMAE_LAUNCH("pla_plan_kernel", stream, pla_plan_kernel<8>, per_strip, dim3(256), 0, stream, p);
  else if (ne <= 12) AFFMAE_LAUNCH("pla_plan_kernel", stream, pla_plan_kernel<12>, per_strip, dim3(256), 0, stream, p);
  else AFFMAE_LAUNCH("pla_plan_kernel", stream, pla_plan_kernel<kMaxEntries>, per_strip, dim3(256), 0, stream, p);
  AFFMAE_LAUNCH("plan_scan_kernel", stream, plan_scan_kernel, dim3((L.strips + 1023) / 1024), dim3(256), 0, stream,
                p.rev_count, p.rev_offset, L.strips);
  AFFMAE_LAUNCH("plan_fill_kernel", stream, plan_fill_kernel, per_strip, dim3(256), 0, stream, p);
  AFFMAE_LAUNCH("plan_sort_kernel", stream, plan_sort_kernel, per_strip, dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace affmae
