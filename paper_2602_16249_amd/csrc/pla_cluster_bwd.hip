// Cluster-tiled local attention, backward (chain rule on the FlashNbhdAttn
// equation of Sec. "Flash-style Cluster Attention and Fast Decoder KNN"; the
// paper prints no backward).  Same preconditions and plan as the forward
// kernel.  Two kernels:
//
//  query-stationary (one wave per strip of 16 queries): recomputes the
//    probabilities p from lse tile by tile exactly as the forward pass forms the
//    scores, forms dP = V dO^T with MFMAs, dS = p (dP - D) with D = <dout, out>,
//    accumulates dQ^T = K^T dS^T (K^T read from the staged rows with the transposing LDS read),
//    and leaves what the other kernel needs in compact arrays: dS of the real (query, neighbour)
//    pairs in [token, head, slot] order is dbias; their p goes to the workspace in the plan's run
//    order (grouped by token tile), with D of every query.  With blank tokens the blank column joins
//    every query's softmax: its dS feeds dq, and the strip's sums for dk_blank / dv_blank go to
//    the workspace, to be added up over the strips in a fixed order by a last kernel;
//
//  key-stationary (one wave per tile of 16 tokens): walks the sorted list of
//    strips that touch the tile, reads each strip's run of p values for the
//    tile as one contiguous piece, spreads it over a 16x16 tile in LDS, forms
//    dS = p (dP - D) itself (one more MFMA on its own V rows: handing dS over as
//    well would cost 2 bytes per pair written and read again, and both kernels run
//    close to what the memory system delivers), and accumulates dK^T = Q^T dS and
//    dV^T = dO^T P in registers, so dk and dv are written once, without atomics and
//    in a fixed summation order.
#include "cluster_common.h"
#include "launch.h"
#include "timing.h"

namespace affmae {
namespace {

constexpr int kSlotCapB = 10;  // token tiles resident per wave: one tile of (p, dS) words each (10 KB); three workgroups per CU
static_assert(kSlotCapB % 2 == 0, "an odd pass uses one more tile for the second half of its last pair");
constexpr float kLog2e = 1.4426950408889634f;

struct BwdParams {
  const bf16_t *q, *k, *v, *bias, *out, *dout;
  const float* lse;
  const uint16_t *slots, *entries;
  const int32_t* rev_offset;
  const unsigned long long* rev_list;
  const uint16_t *sorted_pos, *runs;
  int N, H, K, strips, strips_per_image, slot_stride, max_slots, runs_stride, places;
  uint32_t k_magic, cq_magic;  // reciprocals of K and of K / 8
  uint32_t h_magic, spi_magic;  // ... of H and of strips_per_image
  int head_groups;              // key-stationary kernel: H / heads per wave
  uint32_t hgr_magic;           // ... its reciprocal
  float scale;
  bf16_t *dq, *dk, *dv;
  bf16_t* ds;    // [B,N,H,K] dS = dbias, or nullptr when the caller does not want it
  bf16_t* ph;    // workspace [strips][H][places]: p of every place of the plan's run order
  float* dsum;   // workspace [strips][H][16]: -D = -<dout, out> of the strip's queries
  const bf16_t *k_blank, *v_blank;  // [H,32] or nullptr
  float* blank_part;                // workspace [strips][H][2][32]: the strip's parts of dk_blank, dv_blank; or nullptr
  // bias from a relative-position table (REL kernels): token coordinates [B,N,2], table [H][2R+1][2R+1]
  const float* coords;
  const bf16_t* rel_table;
  int R;
  float rate;
  float* rel_part;  // workspace [strips][H][(2R+1)^2]: every wave's sums of dS per bin (needs (2R+1)^2 <= kRelCells),
                    // or nullptr: then dS goes out through `ds` for the stand-alone table-gradient kernel
};
constexpr int kRelCells = 128;  // bins of a wave's fp64 table: the third KB of its row tile, idle after the prologue

__device__ __forceinline__ f32x4 mfma32(const Frag8& a, const Frag8& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16(const Frag4& a, const Frag4& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a.v, b.v, c, 0, 0, 0);
}

__device__ __forceinline__ int xcd_contiguous_block() {
  // Workgroups are dealt round-robin to the 8 XCDs (one L2 each); neighbouring strips and tiles share
  // rows, so give every XCD a contiguous range.  The grid is a multiple of 8.
  const int per_xcd = gridDim.x >> 3;
  return (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
}

// ------------------------------------------------------------------------------------------------
// query-stationary kernel
// Items per lane as in the forward kernel: NT chunks of 8 slots (K % 8 == 0) or NT single entries.
// REL: the bias comes from the head's relative-position table as in the forward kernel (tile coordinates staged
// in the wave's row tile, bin per pair, value through the vector cache), and the table's gradient is summed per
// wave: each pair's dS is added to its bin in an fp64 table in LDS (ds_add_f64 runs at the speed of an integer
// LDS atomic on this chip; the fp32 form is several times slower) and the wave writes its table out at the end.
// RAG: N is not a multiple of 16 (only then do the row clamps and store tests below exist in the code).
template <int NT, bool VEC, bool REL, bool SUMS, bool RAG>
__device__ __forceinline__ void pla_bwd_query_body(const BwdParams& p) {
  static_assert(!SUMS || REL, "the table's gradient belongs to the table form");
  static_assert(!REL || VEC, "the table form is built for 16-byte items");
  // per wave and resident token tile, a 16 x 16 tile of words: the bias (low half) until the tile has been
  // processed, then p (low half) and dS (high half), the word that the key-stationary kernel is handed
  // + a spare cell: entries that are not of the pass (other passes, no neighbour, dead items) are steered to it
  // with one unsigned minimum - their offset relative to the pass is at least kSlotCapB * 256, wrapped around or
  // not, because every pass but the last is full.  Skipped bias values land in its low half; its high half stays
  // zero, which is what a skipped read of dS takes.
  __shared__ __align__(16) uint32_t pd_all[4][kSlotCapB * 256 + 4];
  __shared__ __align__(16) u32x4 kv_all[4][3 * 64];  // per wave: rows of two token tiles (K, then V), or the strip's q, dout, out
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform: keeps per-wave indices in SGPRs
  const int g = lane >> 4, r = lane & 15;
  const int lane_cell = tile_cell(r, 4 * g);  // the lane's piece of a 16 x 16 tile: row r, columns 4g..4g+3
  // one wave per (strip, head): the heads of a strip sit in neighbouring waves and share cache lines
  const int unit = xcd_contiguous_block() * 4 + wave;
  const int sg = exact_div(unit, p.H, p.h_magic);
  const int h = unit - sg * p.H;
  if (sg >= p.strips) return;  // wave-uniform; no workgroup barrier in this kernel
  uint32_t* pdtile = pd_all[wave];
  bf16_t* halves = reinterpret_cast<bf16_t*>(pdtile);  // [2 * cell] low half, [2 * cell + 1] high half
  constexpr uint32_t kSpare = kSlotCapB * 256u;
  if (lane == 0) pdtile[kSpare] = 0u;  // (ordered before its first read by the fences of the passes)
  const int b = exact_div(sg, p.strips_per_image, p.spi_magic);
  const long long img_base = (long long)b * p.N;
  const int q0 = (sg - b * p.strips_per_image) * 16;  // first query of the strip, within the image
  const long long tok0 = img_base + q0;
  // An image's last strip and last token tile may be short (N % 16 != 0): rows past the end are never addressed -
  // loads repeat the last real row (no plan entry refers to it, so p = dS = 0 there), stores are skipped.
  const int nq = RAG ? min(16, p.N - q0) : 16;
  const int C = p.H * kD;
  const int K = p.K;

  const uint16_t* sl = p.slots + (size_t)sg * p.slot_stride;
  const int cnt_raw = sl[0];
  const int my_tile = (lane < p.slot_stride - 1) ? (int)sl[1 + lane] : 0;
  constexpr int EW = VEC ? 4 : 1;  // 32-bit words per item
  uint32_t ent[NT][EW];
  uint32_t item_off[NT];  // element offset of the item's first value within head 0's [token, head, :] rows
  bool item_live[NT];
  const int items = VEC ? 2 * K : 16 * K;
  const int chunks_per_query = K >> 3;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int i = t * kWave + lane;
    const bool live = i < items;
    const int ii = live ? i : 0;
    int qi;
    if (VEC) {
      const uint4 w = *reinterpret_cast<const uint4*>(p.entries + (size_t)sg * 16 * K + (size_t)ii * 8);
      ent[t][0] = live ? w.x : 0xffffffffu;
      ent[t][EW > 1 ? 1 : 0] = live ? w.y : 0xffffffffu;
      ent[t][EW > 2 ? 2 : 0] = live ? w.z : 0xffffffffu;
      ent[t][EW > 3 ? 3 : 0] = live ? w.w : 0xffffffffu;
      qi = fast_div(ii, p.cq_magic);
      item_off[t] = (uint32_t)(qi * p.H * K + (ii - qi * chunks_per_query) * 8);
    } else {
      ent[t][0] = live ? (uint32_t)p.entries[(size_t)sg * 16 * K + ii] : kNoEntry;
      qi = fast_div(ii, p.k_magic);
      item_off[t] = (uint32_t)(qi * p.H * K + (ii - qi * K));
    }
    item_live[t] = live && (!RAG || qi < nq);  // items of queries past the image's end: no bias is read, no dbias written
  }
  const int ntiles = min((int)__builtin_amdgcn_readfirstlane(cnt_raw), kMaxSlots);
  const int tr_off[2] = {tile_tr_offset(g, r, 0), tile_tr_offset(g, r, 1)};
  // K/V rows cross through LDS: lane (row lane/4, 16-byte piece lane%4) loads 64 contiguous bytes per
  // quad (16 memory-pipeline cycles per load instead of the 64 of a load straight into the operand
  // layout, whose quads touch four rows), and each lane reads back the piece its operand needs; the
  // piece index is XOR-swizzled by the row so that writes and reads spread over all banks.
  const char* kimg = reinterpret_cast<const char*>(p.k + (size_t)img_base * C);
  const char* vimg = reinterpret_cast<const char*>(p.v + (size_t)img_base * C);
  const int la = lane >> 2, lc = lane & 3;
  const uint32_t lane_off_h = (uint32_t)(la * C * 2 + lc * 16 + h * kD * 2);  // the lane's piece of a tile's rows, head h
  const uint32_t tile_bytes = 16u * (uint32_t)C * 2u;
  const uint32_t lane_off_max = (uint32_t)(p.N - 1) * (uint32_t)C * 2u + (uint32_t)(lc * 16 + h * kD * 2);  // same piece of the image's last row
  u32x4* kv = kv_all[wave];
  const int wr_chunk = tile_chunk(la, lc);
  const int rd_chunk = tile_chunk(r, g);
  const size_t strip_rows = (size_t)tok0 * p.H * K;  // first element of the strip's [token, head, :] rows

  // entry values of the strip in run order, two consecutive places per lane and round (loaded late in each pass)
  constexpr int SR = VEC ? NT * 4 + 1 : NT / 2 + 1;
  {
    Frag8 qf, gf, of;  // lane (query r, channels 8g..8g+7) of q, dout, out
    {  // the strip's rows cross through LDS like the K/V rows
      const size_t qrow = (size_t)(tok0 + (RAG ? min(la, nq - 1) : la)) * C + h * kD + lc * 8;
      const u32x4 qraw = *reinterpret_cast<const u32x4*>(p.q + qrow);
      const u32x4 graw = *reinterpret_cast<const u32x4*>(p.dout + qrow);
      const u32x4 oraw = *reinterpret_cast<const u32x4*>(p.out + qrow);
      kv[0 * 64 + wr_chunk] = qraw;
      kv[1 * 64 + wr_chunk] = graw;
      kv[2 * 64 + wr_chunk] = oraw;
      wave_lds_sync();
      qf.x4 = kv[0 * 64 + rd_chunk];
      gf.x4 = kv[1 * 64 + rd_chunk];
      of.x4 = kv[2 * 64 + rd_chunk];
      wave_lds_sync();
    }
    double* tabw = reinterpret_cast<double*>(kv + 2 * 64);  // REL: [bin] sums of dS, this wave's
    constexpr bool rel_sum = SUMS;  // else dS goes out through p.ds (the table does not fit)
    if (rel_sum) kv[2 * 64 + lane] = u32x4{0u, 0u, 0u, 0u};
    uint32_t cells[SUMS ? NT : 1][SUMS ? 2 : 1];  // bins of this lane's pairs (< kRelCells <= 256), four per word
    if (SUMS) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 2; ++e) cells[t][e] = 0u;
    }
    const int RW = 2 * p.R + 1;
    float Dq = 0.f;  // D of query r
#pragma unroll
    for (int i = 0; i < 8; ++i) Dq = fmaf(bf16_to_f32(gf.h[i]), bf16_to_f32(of.h[i]), Dq);
    Dq = group_sum(Dq);
    if (g == 0) p.dsum[((size_t)sg * p.H + h) * 16 + r] = -Dq;  // the key-stationary kernel forms dS with it
    const float nl2 = -p.lse[(size_t)(tok0 + (RAG ? min(r, nq - 1) : r)) * p.H + h] * kLog2e;
    const size_t head_rows = strip_rows + (size_t)h * K;
    f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    if (p.k_blank) {
      // the blank column of query r: s = scale <q, k_blank>, p = exp(s - lse), dP = <dout, v_blank>, dS = p (dP - D)
      Frag8 kb, vb;  // channels 8g..8g+7 of the head's blank rows
      kb.u4 = *reinterpret_cast<const uint4*>(p.k_blank + h * kD + g * 8);
      vb.u4 = *reinterpret_cast<const uint4*>(p.v_blank + h * kD + g * 8);
      float sq = 0.f, gv = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        sq = fmaf(bf16_to_f32(qf.h[i]), bf16_to_f32(kb.h[i]), sq);
        gv = fmaf(bf16_to_f32(gf.h[i]), bf16_to_f32(vb.h[i]), gv);
      }
      sq = group_sum(sq);
      gv = group_sum(gv);
      const float pb = (!RAG || r < nq) ? __builtin_amdgcn_exp2f(fmaf(p.scale * sq, kLog2e, nl2)) : 0.f;  // no blank column for a query past the end
      const float dsb = pb * (gv - Dq);
      // dq^T[channel 16dt + 4g + i][query r] += dS k_blank (the scale is applied when dq is written)
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[dt][i] = fmaf(dsb, bf16_to_f32(p.k_blank[h * kD + dt * 16 + g * 4 + i]), acc[dt][i]);
      if (p.blank_part) {
        // the strip's parts: dk_blank[c] = scale sum_r dS_r q[r][c], dv_blank[c] = sum_r p_r dout[r][c]; lane (r, g)
        // holds channels 8g..8g+7 of query r, so the sum over r runs over the 16 lanes of a row of the wave
        float pk[8], pv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          pk[i] = p.scale * dsb * bf16_to_f32(qf.h[i]);
          pv[i] = pb * bf16_to_f32(gf.h[i]);
#pragma unroll
          for (int o = 8; o > 0; o >>= 1) {
            pk[i] += __shfl_xor(pk[i], o);
            pv[i] += __shfl_xor(pv[i], o);
          }
        }
        if (r == 0) {
          float* dst = p.blank_part + ((size_t)sg * p.H + h) * 2 * kD + g * 8;
          *reinterpret_cast<float4*>(dst) = make_float4(pk[0], pk[1], pk[2], pk[3]);
          *reinterpret_cast<float4*>(dst + 4) = make_float4(pk[4], pk[5], pk[6], pk[7]);
          *reinterpret_cast<float4*>(dst + kD) = make_float4(pv[0], pv[1], pv[2], pv[3]);
          *reinterpret_cast<float4*>(dst + kD + 4) = make_float4(pv[4], pv[5], pv[6], pv[7]);
        }
      }
    }
    uint32_t dacc[NT][EW];  // dS of this lane's items (packed bf16), gathered pass by pass
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int e = 0; e < EW; ++e) dacc[t][e] = 0u;
    bf16_t* ph_head = p.ph + ((size_t)sg * p.H + h) * p.places;

    for (int slot0 = 0; slot0 < ntiles; slot0 += kSlotCapB) {
      const int nsl = min(kSlotCapB, ntiles - slot0);
      const uint32_t lo = (uint32_t)slot0 * 256u, span = (uint32_t)nsl * 256u;
      {
        uint32_t bw[NT][EW];  // bias of this lane's items
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          if (VEC) {
            uint4 w = make_uint4(0, 0, 0, 0);
            if (REL) {  // the query's coordinates instead
              const int ii = item_live[t] ? t * kWave + lane : 0;  // (a live item's query is inside the image)
              const float2 c = (reinterpret_cast<const float2*>(p.coords) + tok0)[fast_div(ii, p.cq_magic)];
              w.x = __float_as_uint(c.x);
              w.y = __float_as_uint(c.y);
            } else if (p.bias && item_live[t]) {
              w = *reinterpret_cast<const uint4*>(p.bias + head_rows + item_off[t]);
            }
            bw[t][0] = w.x;
            bw[t][EW > 1 ? 1 : 0] = w.y;
            bw[t][EW > 2 ? 2 : 0] = w.z;
            bw[t][EW > 3 ? 3 : 0] = w.w;
          } else {
            bw[t][0] = (p.bias && item_live[t]) ? (uint32_t)p.bias[head_rows + item_off[t]] : 0u;
          }
        }
        // (an odd pass gets one more tile of -inf: the second half of its last pair, which repeats a tile)
        for (int s = 0; s < nsl + (nsl & 1); ++s)
          *reinterpret_cast<uint4*>(pdtile + s * 256 + lane * 4) = make_uint4(0xff80u, 0xff80u, 0xff80u, 0xff80u);
        const float2* cxy = reinterpret_cast<const float2*>(kv);  // REL: [slot of the pass][token of the tile]
        if (REL) {
          const float2* cimg = reinterpret_cast<const float2*>(p.coords) + img_base;
#pragma unroll
          for (int i = 0; i < (kSlotCapB * 16 + kWave - 1) / kWave; ++i) {
            const int tile = __shfl(my_tile, slot0 + min(4 * i + g, nsl - 1));
            reinterpret_cast<float2*>(kv)[i * kWave + lane] = cimg[(uint32_t)(RAG ? min(tile * 16 + r, p.N - 1) : tile * 16 + r)];
          }
        }
        wave_lds_sync();
        const bf16_t* tab = REL ? p.rel_table + h * RW * RW : nullptr;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
          for (int e = 0; e < (VEC ? 8 : 1); ++e) {
            const uint32_t off = VEC ? ((ent[t][e >> 1] >> (16 * (e & 1))) & 0xffffu) : (ent[t][0] & 0xffffu);
            const uint32_t rel = off - lo;  // other passes, kNoEntry and dead items fall outside [0, span)
            uint32_t bits;
            if (REL) {
              // (an entry outside the pass reads some coordinate pair of the tile area: any value gives a cell of the table)
              const float2 cn = cxy[((rel >> 4) & 0xf0u) | cell_token(rel)];
              const int cell = relpos_cell(cn, make_float2(__uint_as_float(bw[t][0]), __uint_as_float(bw[t][EW > 1 ? 1 : 0])), p.rate, p.R);
              bits = *reinterpret_cast<const bf16_t*>(reinterpret_cast<const char*>(tab) + (uint32_t)cell * 2u);
              if (SUMS) cells[SUMS ? t : 0][SUMS ? (e >> 2) : 0] |= (rel < span ? (uint32_t)cell : 0u) << (8 * (e & 3));
            } else {
              bits = VEC ? ((bw[t][e >> 1] >> (16 * (e & 1))) & 0xffffu) : bw[t][0];
            }
            halves[2u * min(rel, kSpare)] = (bf16_t)bits;
          }
        }
        wave_lds_sync();
      }

      const int npairs = (nsl + 1) >> 1;
      auto load_pair = [&](int pr, u32x4& k0, u32x4& v0, u32x4& k1, u32x4& v1) {
        // the image's rows as a scalar base + a 32-bit vector offset (an image is smaller than 4 GB): the tile's
        // byte offset is one scalar product, added to the lane's offset by one vector add per tile that serves the
        // K and the V load (64-bit scalar arithmetic per tile costs ten instructions, and a wave issues one
        // instruction per turn of whatever kind); made opaque, or the compiler rebuilds 64-bit vector addresses
        const uint32_t tile0 = (uint32_t)__builtin_amdgcn_readlane(my_tile, slot0 + min(2 * pr, nsl - 1));
        const uint32_t tile1 = (uint32_t)__builtin_amdgcn_readlane(my_tile, slot0 + min(2 * pr + 1, nsl - 1));
        uint32_t off0 = lane_off_h + tile0 * tile_bytes, off1 = lane_off_h + tile1 * tile_bytes;
        if (RAG) {
          off0 = min(off0, lane_off_max);
          off1 = min(off1, lane_off_max);
        }
        asm volatile("" : "+v"(off0), "+v"(off1));
        k0 = *reinterpret_cast<const u32x4*>(kimg + off0);
        v0 = *reinterpret_cast<const u32x4*>(vimg + off0);
        k1 = *reinterpret_cast<const u32x4*>(kimg + off1);
        v1 = *reinterpret_cast<const u32x4*>(vimg + off1);
      };
      // pieces as loaded -> LDS -> operand pieces
      auto stage_pair = [&](const u32x4& k0, const u32x4& v0, const u32x4& k1, const u32x4& v1, Frag8(&kf)[2],
                            Frag8(&vf)[2], Frag8(&kt)[2]) {
        kv[0 * 64 + wr_chunk] = k0;
        kv[1 * 64 + wr_chunk] = k1;
        wave_lds_sync();
        kf[0].x4 = kv[0 * 64 + rd_chunk];
        kf[1].x4 = kv[1 * 64 + rd_chunk];
        {
          // K^T operand, lane (channel 16dt + r, tokens 4g..4g+3 of both tiles), by the transposing LDS read
          const char* kbase = reinterpret_cast<const char*>(kv);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) {
            const uint2 a = lds_read_tr(kbase + 0 * 1024 + tr_off[dt]);
            const uint2 b = lds_read_tr(kbase + 1 * 1024 + tr_off[dt]);
            kt[dt].u[0] = a.x; kt[dt].u[1] = a.y; kt[dt].u[2] = b.x; kt[dt].u[3] = b.y;
          }
        }
        wave_lds_sync();
        kv[0 * 64 + wr_chunk] = v0;
        kv[1 * 64 + wr_chunk] = v1;
        wave_lds_sync();
        vf[0].x4 = kv[0 * 64 + rd_chunk];
        vf[1].x4 = kv[1 * 64 + rd_chunk];
      };
      auto compute_pair = [&](int pr, const Frag8(&kf)[2], const Frag8(&vf)[2], const Frag8(&kt)[2]) {
        // A pass with an odd number of tiles repeats its last tile in the second half of the last pair, under
        // a bias tile of -inf: p and dS come out 0 without a test.  The whole pair is one basic block.
        Frag8 dsf;  // dS^T operand: k-slots 0..3 = first tile's tokens 4g..4g+3, 4..7 = second tile's
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          {
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            const f32x4 st = mfma32(kf[tt], qf, z);   // <k[token 4g+i], q[query r]>
            const f32x4 dpt = mfma32(vf[tt], gf, z);  // <v[token 4g+i], dout[query r]>
            uint32_t* cell = pdtile + (2 * pr + tt) * 256 + lane_cell;
            const uint4 bm = *reinterpret_cast<const uint4*>(cell);
            float pv[4], dsv[4];
            pv[0] = __builtin_amdgcn_exp2f(fmaf(fmaf(st[0], p.scale, __uint_as_float(bm.x << 16)), kLog2e, nl2));
            pv[1] = __builtin_amdgcn_exp2f(fmaf(fmaf(st[1], p.scale, __uint_as_float(bm.y << 16)), kLog2e, nl2));
            pv[2] = __builtin_amdgcn_exp2f(fmaf(fmaf(st[2], p.scale, __uint_as_float(bm.z << 16)), kLog2e, nl2));
            pv[3] = __builtin_amdgcn_exp2f(fmaf(fmaf(st[3], p.scale, __uint_as_float(bm.w << 16)), kLog2e, nl2));
#pragma unroll
            for (int i = 0; i < 4; ++i) dsv[i] = pv[i] * (dpt[i] - Dq);
            // (p, dS) words replace the bias of these cells, which is no longer needed
            *reinterpret_cast<uint4*>(cell) = make_uint4(pack_bf16x2(pv[0], dsv[0]), pack_bf16x2(pv[1], dsv[1]),
                                                         pack_bf16x2(pv[2], dsv[2]), pack_bf16x2(pv[3], dsv[3]));
            dsf.u[2 * tt + 0] = pack_bf16x2(dsv[0], dsv[1]);
            dsf.u[2 * tt + 1] = pack_bf16x2(dsv[2], dsv[3]);
          }
        }
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) acc[dt] = mfma32(kt[dt], dsf, acc[dt]);  // dq^T[channel 16dt + 4g+i][query r]
      };
      // The loads of the next pair fly during this pair's math; every load in straight-line code (a load
      // under a condition makes the compiler wait for all outstanding loads where the paths join).
      u32x4 sk0, sv0, sk1, sv1;
      Frag8 kf[2], vf[2], kt[2];
      load_pair(0, sk0, sv0, sk1, sv1);
      for (int pr = 0; pr + 1 < npairs; ++pr) {
        stage_pair(sk0, sv0, sk1, sv1, kf, vf, kt);
        load_pair(pr + 1, sk0, sv0, sk1, sv1);
        compute_pair(pr, kf, vf, kt);
      }
      stage_pair(sk0, sv0, sk1, sv1, kf, vf, kt);
      // The run-order entry values are needed after the last pair only: their loads fly during its math, in
      // the registers that the staged K/V rows have just left.
      uint32_t sp[SR];
#pragma unroll
      for (int t = 0; t < SR; ++t) {
        const int w = t * 2 * kWave + 2 * lane;
        sp[t] = (w < p.places) ? *reinterpret_cast<const uint32_t*>(p.sorted_pos + (size_t)sg * p.places + w) : 0xffffffffu;
      }
      compute_pair(npairs - 1, kf, vf, kt);
      wave_lds_sync();
      // REL: dS of this pass's real pairs, added to their bins
      if (rel_sum) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t off = (ent[t][e >> 1] >> (16 * (e & 1))) & 0xffffu;
            const uint32_t rel = off - lo;
            if (rel < span) {
              const uint32_t cell = (cells[SUMS ? t : 0][SUMS ? (e >> 2) : 0] >> (8 * (e & 3))) & 0xffu;
              atomicAdd(&tabw[cell], (double)bf16_to_f32(halves[2u * rel + 1u]));
            }
          }
        }
      }
      // dS of this pass's real (query, neighbour) pairs in [token, head, slot] order (dbias)
      if (!SUMS && p.ds) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
          for (int e = 0; e < (VEC ? 8 : 1); ++e) {
            const uint32_t off = VEC ? ((ent[t][e >> 1] >> (16 * (e & 1))) & 0xffffu) : (ent[t][0] & 0xffffu);
            const uint32_t rel = off - lo;
            dacc[t][e >> 1] |= (uint32_t)halves[2u * min(rel, kSpare) + 1u] << (16 * (e & 1));
          }
        }
      }
      // p of this pass's slots in run order: consecutive places, so the stores are whole rows.
      // Runs start at even places: a pair of places belongs to one slot, or its second place is unused.
#pragma unroll
      for (int t = 0; t < SR; ++t) {
        const uint32_t rel0 = (sp[t] & 0xffffu) - lo, rel1 = (sp[t] >> 16) - lo;  // other passes and unused places
        const bool in0 = rel0 < span, in1 = rel1 < span;                         // fall outside [0, span)
        const uint32_t a0 = min(rel0, kSpare), a1 = min(rel1, kSpare);
        const uint32_t p0 = halves[2u * a0], p1 = halves[2u * a1];
        if (in0) *reinterpret_cast<uint32_t*>(ph_head + t * 2 * kWave + 2 * lane) = p0 | ((in1 ? p1 : 0u) << 16);
      }
      wave_lds_sync();
    }
    // dbias [token, head, slot]; whole 16-byte pieces when K is a multiple of 8
    if (!SUMS && p.ds) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        if (item_live[t]) {
          if (VEC)
            *reinterpret_cast<uint4*>(p.ds + head_rows + item_off[t]) =
                make_uint4(dacc[t][0], dacc[t][EW > 1 ? 1 : 0], dacc[t][EW > 2 ? 2 : 0], dacc[t][EW > 3 ? 3 : 0]);
          else
            p.ds[head_rows + item_off[t]] = (bf16_t)dacc[t][0];
        }
      }
    }
    if (rel_sum) {  // (the last pass ended with a wave_lds_sync)
      float* dst = p.rel_part + ((size_t)sg * p.H + h) * (RW * RW);
      for (int c = lane; c < RW * RW; c += kWave) dst[c] = (float)tabw[c];
    }
    // dq rows cross through LDS the other way: lane (query r, channels 16dt + 4g..+3) holds 8 bytes of
    // 16-byte piece 2dt + g/2 of row r; lane (row lane/4, piece lane%4) stores 16 bytes
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
      uint2 o;
      o.x = pack_bf16x2(acc[dt][0] * p.scale, acc[dt][1] * p.scale);
      o.y = pack_bf16x2(acc[dt][2] * p.scale, acc[dt][3] * p.scale);
      reinterpret_cast<uint2*>(kv)[tile_chunk(r, 2 * dt + (g >> 1)) * 2 + (g & 1)] = o;
    }
    wave_lds_sync();
    if (!RAG || la < nq) *reinterpret_cast<u32x4*>(p.dq + (size_t)(tok0 + la) * C + h * kD + lc * 8) = kv[wr_chunk];
    wave_lds_sync();
  }
}

template <int NT, bool RAG>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 3))) void pla_bwd_query_kernel(BwdParams p) {
  pla_bwd_query_body<NT, true, false, false, RAG>(p);
}
template <int NT, bool RAG>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void pla_bwd_query_rel_kernel(BwdParams p) {
  pla_bwd_query_body<NT, true, true, true, RAG>(p);
}
template <int NT, bool RAG>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 3))) void pla_bwd_query_rel_ds_kernel(BwdParams p) {
  pla_bwd_query_body<NT, true, true, false, RAG>(p);
}
template <int NT, bool RAG>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void pla_bwd_query_scalar_kernel(BwdParams p) {
  pla_bwd_query_body<NT, false, false, false, RAG>(p);
}

// ------------------------------------------------------------------------------------------------
// key-stationary kernel
template <int HG>
struct KeyItem {
  uint32_t w[2][HG];     // p of places 2*lane, 2*lane+1 (+128 in the second round) of the run, two bf16 halves
  uint32_t code[2];      // their entry values, two 16-bit halves
  uint32_t len;          // places in the run (wave-uniform)
};

// HG = heads handled by one wave's sweep over the tile's list (2 when H is even: one walk of the list, one load of
// the entry values and one pass over the q / dout rows serve both).  One wave per (token tile, group of HG heads),
// the groups of a tile in consecutive waves: they walk the same list over the same strips at the same time, so the
// strips' rows, the entry values and the list are fetched into the XCD's L2 once for all heads, and the rows that an
// XCD has in use at a time do not grow with the number of heads.
template <int HG, bool RAG>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 4))) void pla_bwd_key_kernel(BwdParams p) {
  __shared__ __align__(16) bf16_t tile_all[4][HG * 256];  // per wave and head: p[token][query]
  // per wave, twice (two incidences in flight): the strip's q rows, then its dout rows.  They come straight from
  // memory (global_load_lds: 16 bytes per lane, lane l's piece landing at 16 l; no registers, no LDS write
  // instructions), so each lane fetches the piece that belongs in its place of the swizzled tile.
  __shared__ __align__(16) u32x4 rows_all[4][2][2 * HG * 64];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform: keeps per-wave indices in SGPRs
  const int g = lane >> 4, r = lane & 15;
  const int lane_cell = tile_cell(r, 4 * g);  // the lane's piece of a 16 x 16 tile: row r, columns 4g..4g+3
  const int unit = xcd_contiguous_block() * 4 + wave;
  const int kt = exact_div(unit, p.head_groups, p.hgr_magic);  // token tile, global
  if (kt >= p.strips) return;
  const int hg = (unit - kt * p.head_groups) * HG;  // first head of the wave's group
  bf16_t* tile = tile_all[wave];
  u32x4* rows0 = rows_all[wave][0];
  u32x4* rows1 = rows_all[wave][1];
  const int b = exact_div(kt, p.strips_per_image, p.spi_magic);
  const int C = p.H * kD;
  const size_t strip_base = (size_t)b * p.strips_per_image;
  // rows of the image; its last token tile and last strip may be short (N % 16 != 0): loads past the end repeat the
  // last real row (its p is 0: no entry refers to it), stores past the end are skipped
  const size_t img_row0 = (size_t)b * p.N;
  const int t0 = (kt - b * p.strips_per_image) * 16;  // the tile's first token, within the image
  const int nt = RAG ? min(16, p.N - t0) : 16;
  const int lo = __builtin_amdgcn_readfirstlane(p.rev_offset[kt]);
  const int n = __builtin_amdgcn_readfirstlane(p.rev_offset[kt + 1]) - lo;
  // q / dout rows cross through LDS: a lane loads 16 contiguous bytes of a row so that a quad reads 64
  // contiguous bytes (a load straight into the operand layout puts a quad on four rows and costs four
  // times the memory-pipeline cycles); each lane then reads back the piece its operand needs.  The piece
  // index is XOR-swizzled by the row so that writes and reads spread over all banks.
  constexpr int PR = 4 * HG;  // 16-byte pieces per row of the head group
  const int la = lane / PR, lc = lane % PR;  // row within a load of 64 / PR rows, piece
  const uint32_t q_lane = (uint32_t)(la * C + lc * 8);  // per-lane part of the row addresses (elements)
  auto swz = [](int row) { return HG == 2 ? ((row & 7) ^ (row >> 3)) : (((row >> 1) & 3) ^ ((row >> 3) & 1)); };
  int wr_chunk[HG];
#pragma unroll
  for (int i = 0; i < HG; ++i) {
    const int row = i * (64 / PR) + la;
    wr_chunk[i] = row * PR + (lc ^ swz(row));
  }
  // element offset, within the strip's rows, of the piece this lane fetches in load i: row i * 64 / PR + la, and
  // the piece whose place in the tile is lc, i.e. piece lc ^ swz(row)
  uint32_t q_dma[HG], q_dma_row[HG], q_dma_piece[HG];  // whole offset (full strips); row and piece apart (RAG)
#pragma unroll
  for (int i = 0; i < HG; ++i) {
    const int row = i * (64 / PR) + la;
    q_dma_row[i] = (uint32_t)row;
    q_dma_piece[i] = (uint32_t)((lc ^ swz(row)) * 8);
    q_dma[i] = (uint32_t)(row * C) + q_dma_piece[i];
  }
  // what this lane gives to lds_read_tr to receive, for channel 16dt + r of head hh, the values of rows (queries)
  // 4g..4g+3: the quarter r % 4 of those 16 channels in row 4g + r / 4
  int tr_off[HG][2];
#pragma unroll
  for (int hh = 0; hh < HG; ++hh)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
      const int row = 4 * g + (r >> 2);
      tr_off[hh][dt] = (row * PR + ((4 * hh + 2 * dt + ((r & 3) >> 1)) ^ swz(row))) * 16 + (r & 1) * 8;
    }

  // where lane (query r, channels 8g..8g+7 of head hh) finds its piece of the staged dout rows
  int gf_chunk[HG];
#pragma unroll
  for (int hh = 0; hh < HG; ++hh) gf_chunk[hh] = HG * 64 + r * PR + ((4 * hh + g) ^ swz(r));

  {
    // The hand-over carries p only: dS = p (dP - D) is formed here, with dP - D = <dout[query], v[token]> - D from one
    // more MFMA on the tile's own V rows (operand: lane (token r, channels 8g..8g+7)) and the dout rows that
    // are staged anyway.  It comes out as lane (token r, queries 4g..4g+3), the operand layout of dK^T = Q^T dS.
    Frag8 vop[HG];
#pragma unroll
    for (int hh = 0; hh < HG; ++hh)
      vop[hh].u4 = *reinterpret_cast<const uint4*>(p.v + (img_row0 + t0 + (RAG ? min(r, nt - 1) : r)) * C + (size_t)((hg + hh) * kD) + g * 8);
    f32x4 dk[HG][2], dv[HG][2];
#pragma unroll
    for (int hh = 0; hh < HG; ++hh)
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        dk[hh][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        dv[hh][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    for (int base = 0; base < n; base += kWave) {
      const int nb = min(kWave, n - base);
      const unsigned long long mine = (lane < nb) ? p.rev_list[lo + base + lane] : 0ull;
      const uint32_t mine_lo = (uint32_t)mine, mine_hi = (uint32_t)(mine >> 32);
      // all loads of one item, nothing else: what is done with the words waits until compute(), so that
      // no use of a loaded value sits between the loads of one item and the math of the previous one
      auto fetch = [&](int i, KeyItem<HG>& it, u32x4* rows) {
        const uint32_t inc = __builtin_amdgcn_readlane(mine_lo, i);
        const uint32_t run = __builtin_amdgcn_readlane(mine_hi, i);
        const size_t sgq = strip_base + (inc >> 8);
        const uint32_t start = run & 0xffffu;
        it.len = run >> 16;
        const int sq0 = (int)(inc >> 8) * 16;  // the strip's first query, within the image
        const uint32_t last_q = (uint32_t)min(15, p.N - 1 - sq0);
        const size_t qbase = (img_row0 + sq0) * C + (size_t)(hg * kD);
        typedef const __attribute__((address_space(1))) void* gptr_t;
        typedef __attribute__((address_space(3))) void* lptr_t;
#pragma unroll
        for (int i = 0; i < HG; ++i) {  // load i: rows i * 64 / PR onwards
          const uint32_t at = RAG ? min(q_dma_row[i], last_q) * (uint32_t)C + q_dma_piece[i] : q_dma[i];
          __builtin_amdgcn_global_load_lds((gptr_t)(p.q + qbase + at), (lptr_t)(rows + i * 64), 16, 0, 0);
          __builtin_amdgcn_global_load_lds((gptr_t)(p.dout + qbase + at), (lptr_t)(rows + HG * 64 + i * 64), 16, 0, 0);
        }
        // runs start at even places and the rows hold an even number of places: aligned pairs
        const uint16_t* codes = p.sorted_pos + sgq * p.places + start;
        const bf16_t* words = p.ph + (sgq * p.H + hg) * p.places + start;
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
          const uint32_t e = (uint32_t)(rr * 2 * kWave + 2 * lane);
          const bool on = e < it.len;
          it.code[rr] = on ? *reinterpret_cast<const uint32_t*>(codes + e) : 0xffffffffu;
#pragma unroll
          for (int hh = 0; hh < HG; ++hh)
            it.w[rr][hh] = on ? *reinterpret_cast<const uint32_t*>(words + (size_t)hh * p.places + e) : 0u;
        }
      };
      // -D of the queries 4g..4g+3 of item i's strip: one copy only, loaded for the next item when the current one
      // has used its own (it is small and cached; a second copy would cost the kernel its fourth wave per SIMD)
      float4 dsum[HG];
      auto load_dsum = [&](int i) {
        const uint32_t inc = __builtin_amdgcn_readlane(mine_lo, min(i, nb - 1));
        const size_t sgq = strip_base + (inc >> 8);
#pragma unroll
        for (int hh = 0; hh < HG; ++hh)
          dsum[hh] = *reinterpret_cast<const float4*>(p.dsum + (sgq * p.H + hg + hh) * 16 + g * 4);
      };
      auto compute = [&](const KeyItem<HG>& it, const u32x4* rows, int next) {
        // spread the run over the tile: cell [token][query] <- p; unlisted cells stay 0 (hence dS = 0 there)
#pragma unroll
        for (int hh = 0; hh < HG; ++hh) *reinterpret_cast<uint2*>(tile + hh * 256 + lane * 4) = make_uint2(0u, 0u);
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const uint32_t c = (it.code[rr] >> (16 * half)) & 0xffffu;  // query * 16 + token % 16 in the low byte
            if (c != kNoEntry) {
              const uint32_t cell = (uint32_t)tile_cell((int)cell_token(c), (int)((c >> 4) & 15u));  // [token][query], same XOR
#pragma unroll
              for (int hh = 0; hh < HG; ++hh) tile[hh * 256 + cell] = (bf16_t)(half ? it.w[rr][hh] >> 16 : it.w[rr][hh] & 0xffffu);
            }
          }
        }
        wave_lds_sync();
#pragma unroll
        for (int hh = 0; hh < HG; ++hh) {
          Frag4 pf, df;  // operand B of the 16x16x16 MFMA: lane (token r, queries 4g..4g+3)
          const uint2 w = *reinterpret_cast<const uint2*>(tile + hh * 256 + lane_cell);  // p[token r][queries 4g..]
          pf.u[0] = w.x;
          pf.u[1] = w.y;
          Frag8 gf;  // lane (query r, channels 8g..8g+7) of dout
          gf.x4 = rows[gf_chunk[hh]];
          // <dout[query 4g+i], v[token r]> - D[query 4g+i]: the accumulator starts at -D
          const f32x4 nd = {dsum[hh].x, dsum[hh].y, dsum[hh].z, dsum[hh].w};
          const f32x4 dp = mfma32(gf, vop[hh], nd);
          df.u[0] = pack_bf16x2(__uint_as_float(w.x << 16) * dp[0], __uint_as_float(w.x & 0xffff0000u) * dp[1]);
          df.u[1] = pack_bf16x2(__uint_as_float(w.y << 16) * dp[2], __uint_as_float(w.y & 0xffff0000u) * dp[3]);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) {
            // operand A: lane (channel 16dt + r, queries 4g..4g+3) of q and dout, by the transposing LDS read
            const uint2 qw = lds_read_tr(reinterpret_cast<const char*>(rows) + tr_off[hh][dt]);
            const uint2 gw = lds_read_tr(reinterpret_cast<const char*>(rows + HG * 64) + tr_off[hh][dt]);
            Frag4 qT, gT;
            qT.u[0] = qw.x; qT.u[1] = qw.y;
            gT.u[0] = gw.x; gT.u[1] = gw.y;
            dk[hh][dt] = mfma16(qT, df, dk[hh][dt]);  // dk^T[channel 16dt + 4g+i][token r]
            dv[hh][dt] = mfma16(gT, pf, dv[hh][dt]);
          }
        }
        load_dsum(next);
        __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): every read of this item's rows has returned (they may be refilled)
        wave_lds_sync();  // the next item clears the tile
      };
      // Two items in flight.  Every load is issued unconditionally in straight-line code (an index past
      // the end repeats the last item): a load under a condition makes the compiler wait for all
      // outstanding loads where the paths join.
      KeyItem<HG> A, B;
      load_dsum(0);
      fetch(0, A, rows0);
      int i = 0;
      for (; i + 2 < nb; i += 2) {
        fetch(i + 1, B, rows1);
        compute(A, rows0, i + 1);
        fetch(i + 2, A, rows0);  // compute(A) has consumed every read of rows0 (its MFMAs are issued)
        compute(B, rows1, i + 2);
      }
      if (i + 1 < nb) {
        fetch(i + 1, B, rows1);
        compute(A, rows0, i + 1);
        compute(B, rows1, i + 2);
      } else {
        compute(A, rows0, i + 1);
      }
    }
    // dk / dv rows cross through LDS the other way: lane (token r, channels 16dt + 4g..+3 of head hh)
    // holds 8 bytes of 16-byte piece 4hh + 2dt + g/2 of row r; the loading pattern stores 16 bytes per lane
#pragma unroll
    for (int hh = 0; hh < HG; ++hh) {
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        const int at = (r * PR + ((4 * hh + 2 * dt + (g >> 1)) ^ swz(r))) * 2 + (g & 1);
        uint2 o;
        o.x = pack_bf16x2(dk[hh][dt][0] * p.scale, dk[hh][dt][1] * p.scale);
        o.y = pack_bf16x2(dk[hh][dt][2] * p.scale, dk[hh][dt][3] * p.scale);
        reinterpret_cast<uint2*>(rows0)[at] = o;
        o.x = pack_bf16x2(dv[hh][dt][0], dv[hh][dt][1]);
        o.y = pack_bf16x2(dv[hh][dt][2], dv[hh][dt][3]);
        reinterpret_cast<uint2*>(rows0 + HG * 64)[at] = o;
      }
    }
    wave_lds_sync();
#pragma unroll
    for (int i = 0; i < HG; ++i) {
      const size_t at = (img_row0 + t0 + i * (64 / PR)) * C + (size_t)(hg * kD) + q_lane;
      if (!RAG || i * (64 / PR) + la < nt) {
        *reinterpret_cast<u32x4*>(p.dk + at) = rows0[wr_chunk[i]];
        *reinterpret_cast<u32x4*>(p.dv + at) = rows0[HG * 64 + wr_chunk[i]];
      }
    }
    wave_lds_sync();
  }
}

// dk_blank, dv_blank [H,32] = sum over the strips of their parts, in a fixed order.  One workgroup per
// (head, which of the two): 32 groups of 32 lanes, group j adds strips j, j + 32, ...
__global__ __launch_bounds__(1024) void pla_blank_reduce_kernel(const float* __restrict__ part, int strips, int H,
                                                               float* __restrict__ dk_blank,
                                                               float* __restrict__ dv_blank) {
  __shared__ float acc[32][kD + 1];
  const int h = blockIdx.x >> 1, which = blockIdx.x & 1;
  const int c = threadIdx.x & 31, grp = threadIdx.x >> 5;
  float s = 0.f;
  for (int sg = grp; sg < strips; sg += 32) s += part[(((size_t)sg * H + h) * 2 + which) * kD + c];
  acc[grp][c] = s;
  __syncthreads();
  if (grp == 0) {
    float t = 0.f;
    for (int j = 0; j < 32; ++j) t += acc[j][c];
    (which ? dv_blank : dk_blank)[h * kD + c] = t;
  }
}

// First step of the sum of the waves' relative-position tables [strips][H][cells]: workgroup (head, part) adds
// its share of the strips, thread = (bin, one of the groups that fit 256 threads), and writes one table.
constexpr int kRelParts = 256;
__global__ __launch_bounds__(256) void pla_rel_reduce_kernel(const float* __restrict__ part, int strips, int H,
                                                             int cells, float* __restrict__ out) {
  __shared__ float acc[256];
  const int h = blockIdx.x / kRelParts, pt = blockIdx.x - h * kRelParts;
  const int groups = 256 / cells;  // cells <= 128: at least two
  const int c = threadIdx.x % cells, grp = threadIdx.x / cells;
  const int per = (strips + kRelParts - 1) / kRelParts;
  const int end = min(strips, (pt + 1) * per);
  float s = 0.f;
  if (grp < groups)
    for (int sg = pt * per + grp; sg < end; sg += groups) s += part[((size_t)sg * H + h) * cells + c];
  acc[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x < cells) {
    float t = 0.f;
    for (int j = 0; j < groups; ++j) t += acc[j * cells + threadIdx.x];
    out[((size_t)pt * H + h) * cells + threadIdx.x] = t;
  }
}

}  // namespace

size_t pla_bwd_cluster_rel_workspace_bytes(int B, int N, int H, int R) {
  // tables of the waves, then the tables of pla_rel_reduce_kernel
  const size_t cells = (size_t)(2 * R + 1) * (2 * R + 1);
  return plan_align((size_t)B * ((N + 15) / 16) * H * cells * sizeof(float)) + plan_align((size_t)kRelParts * H * cells * sizeof(float));
}
bool pla_bwd_cluster_rel_sums(int R) { return (2 * R + 1) * (2 * R + 1) <= kRelCells; }

size_t pla_bwd_cluster_workspace_bytes(int B, int N, int H, int K, int S, int M) {
  const PlanLayout L = make_plan_layout(B, N, K, S, M);
  return plan_align((size_t)L.strips * H * L.places * sizeof(bf16_t)) +  // p in run order
         plan_align((size_t)L.strips * H * 16 * sizeof(float)) +         // D of every query
         plan_align((size_t)L.strips * H * 2 * kD * sizeof(float));        // parts of the blank gradients
}

hipError_t launch_pla_bwd_cluster(const PlaArgs& a, const void* plan, void* workspace, hipStream_t stream) {
  const PlanLayout L = make_plan_layout(a.B, a.N, a.K, a.S, a.M);
  const char* base = static_cast<const char*>(plan);
  BwdParams p;
  p.q = (const bf16_t*)a.q; p.k = (const bf16_t*)a.k; p.v = (const bf16_t*)a.v; p.bias = (const bf16_t*)a.bias;
  p.out = (const bf16_t*)a.out; p.dout = (const bf16_t*)a.dout; p.lse = a.lse;
  p.slots = reinterpret_cast<const uint16_t*>(base + L.slots_off);
  p.entries = reinterpret_cast<const uint16_t*>(base + L.entries_off);
  p.rev_offset = reinterpret_cast<const int32_t*>(base + L.rev_offset_off);
  p.rev_list = reinterpret_cast<const unsigned long long*>(base + L.rev_list_off);
  p.sorted_pos = reinterpret_cast<const uint16_t*>(base + L.sorted_pos_off);
  p.runs = reinterpret_cast<const uint16_t*>(base + L.runs_off);
  p.runs_stride = L.runs_stride; p.places = L.places;
  p.N = a.N; p.H = a.H; p.K = a.K;
  p.strips = L.strips; p.strips_per_image = (a.N + 15) / 16; p.slot_stride = L.slot_stride; p.max_slots = L.max_slots;
  p.scale = a.scale;
  p.dq = (bf16_t*)a.dq; p.dk = (bf16_t*)a.dk; p.dv = (bf16_t*)a.dv;
  const size_t ph_bytes = plan_align((size_t)L.strips * a.H * L.places * sizeof(bf16_t));
  const size_t dsum_bytes = plan_align((size_t)L.strips * a.H * 16 * sizeof(float));
  p.ph = static_cast<bf16_t*>(workspace);
  p.dsum = reinterpret_cast<float*>(static_cast<char*>(workspace) + ph_bytes);
  p.ds = (bf16_t*)a.dbias;
  p.k_blank = (const bf16_t*)a.k_blank; p.v_blank = (const bf16_t*)a.v_blank;
  p.blank_part = (a.k_blank && a.dk_blank)
                     ? reinterpret_cast<float*>(static_cast<char*>(workspace) + ph_bytes + dsum_bytes)
                     : nullptr;

  p.coords = a.rel_coords; p.rel_table = (const bf16_t*)a.rel_table; p.R = a.rel_R; p.rate = a.rel_rate;
  p.rel_part = a.rel_part;
  const int key_hg = a.H % 2 == 0 ? 2 : 1;  // heads per wave of the key-stationary kernel
  p.head_groups = a.H / key_hg;
  p.hgr_magic = div_magic(p.head_groups);
  // one wave per (token tile, head group); multiple of 8 for the XCD-contiguous mapping
  const dim3 grid((((long long)L.strips * p.head_groups + 3) / 4 + 7) / 8 * 8);
  const dim3 grid_q((((long long)L.strips * a.H + 3) / 4 + 7) / 8 * 8);  // one wave per (strip, head)
  p.k_magic = div_magic(a.K);
  p.cq_magic = div_magic(a.K >= 8 ? a.K / 8 : 1);
  p.h_magic = div_magic(a.H);
  p.spi_magic = div_magic((a.N + 15) / 16);
  const bool vec = a.K % 8 == 0 && (!a.bias || reinterpret_cast<uintptr_t>(a.bias) % 16 == 0) &&
                   (!p.ds || reinterpret_cast<uintptr_t>(p.ds) % 16 == 0);
  const bool rag = a.N % 16 != 0;  // a short last strip / token tile per image: the variants with row clamps
#define AFFMAE_BWDQ(KERNEL, NT)                                                                              \
  do {                                                                                                       \
    if (rag) AFFMAE_LAUNCH("pla_bwd_query_kernel", stream, (KERNEL<NT, true>), grid_q, dim3(256), 0, stream, p);  \
    else AFFMAE_LAUNCH("pla_bwd_query_kernel", stream, (KERNEL<NT, false>), grid_q, dim3(256), 0, stream, p);     \
  } while (0)
  if (a.rel_table && a.rel_part) {  // callers check pla_cluster_relpos_supported first
    if (2 * a.K <= kWave) AFFMAE_BWDQ(pla_bwd_query_rel_kernel, 1); else AFFMAE_BWDQ(pla_bwd_query_rel_kernel, 2);
  } else if (a.rel_table) {
    if (2 * a.K <= kWave) AFFMAE_BWDQ(pla_bwd_query_rel_ds_kernel, 1); else AFFMAE_BWDQ(pla_bwd_query_rel_ds_kernel, 2);
  } else if (vec) {
    if (2 * a.K <= kWave) AFFMAE_BWDQ(pla_bwd_query_kernel, 1); else AFFMAE_BWDQ(pla_bwd_query_kernel, 2);
  } else {
    const int ent = (16 * a.K + kWave - 1) / kWave;
    if (ent <= 4) AFFMAE_BWDQ(pla_bwd_query_scalar_kernel, 4);
    else if (ent <= 8) AFFMAE_BWDQ(pla_bwd_query_scalar_kernel, 8);
    else if (ent <= 12) AFFMAE_BWDQ(pla_bwd_query_scalar_kernel, 12);
    else AFFMAE_BWDQ(pla_bwd_query_scalar_kernel, 16);
  }
#undef AFFMAE_BWDQ
  if (a.H % 2 == 0) {
    if (rag) AFFMAE_LAUNCH("pla_bwd_key_kernel", stream, (pla_bwd_key_kernel<2, true>), grid, dim3(256), 0, stream, p);
    else AFFMAE_LAUNCH("pla_bwd_key_kernel", stream, (pla_bwd_key_kernel<2, false>), grid, dim3(256), 0, stream, p);
  } else {
    if (rag) AFFMAE_LAUNCH("pla_bwd_key_kernel", stream, (pla_bwd_key_kernel<1, true>), grid, dim3(256), 0, stream, p);
    else AFFMAE_LAUNCH("pla_bwd_key_kernel", stream, (pla_bwd_key_kernel<1, false>), grid, dim3(256), 0, stream, p);
  }
  if (a.rel_table && a.rel_part) {
    const int cells = (2 * a.rel_R + 1) * (2 * a.rel_R + 1);
    float* second = reinterpret_cast<float*>(reinterpret_cast<char*>(a.rel_part) +
                                             plan_align((size_t)L.strips * a.H * cells * sizeof(float)));
    AFFMAE_LAUNCH("pla_rel_reduce_kernel", stream, pla_rel_reduce_kernel, dim3(a.H * kRelParts), dim3(256), 0, stream,
                  a.rel_part, L.strips, a.H, cells, second);
    const hipError_t e = launch_relpos_table_sum(second, kRelParts, a.H * cells, a.rel_dtable, stream);
    if (e != hipSuccess) return e;
  }
  if (p.blank_part)
    AFFMAE_LAUNCH("pla_blank_reduce_kernel", stream, pla_blank_reduce_kernel, dim3(2 * a.H), dim3(1024), 0, stream,
                  p.blank_part, L.strips, a.H, a.dk_blank, a.dv_blank);
  return hipGetLastError();
}

}  // namespace affmae
