// Cluster-tiled local attention, forward (paper, Sec. "Flash-style Cluster
// Attention and Fast Decoder KNN": stream over tiles, never store the scores,
// fp32 softmax statistics; the equation is FlashNbhdAttn).
//
// Valid when tokens are stored in cluster order and every neighbour of a token
// lies in one of its cluster's M near clusters (the table affmae_knn builds), bf16
// storage, d = 32, S a multiple of 16.  Driven by the plan of pla_plan.hip.
//
// One wave per (strip of 16 queries, head), no workgroup-level cooperation.  The strip's
// neighbours live in a few token tiles (16 consecutive tokens each).  Per pair of
// such tiles the scores of all 16 x 32 (query, token) pairs come from two MFMAs
// on K rows and the strip's Q rows; they are computed transposed (tokens x
// queries) so that the probabilities leave the softmax already in the operand
// layout of the P.V MFMAs.  A query attends only to its K neighbours: their bias
// values are scattered into a per-wave LDS tile that holds -inf everywhere else
// and is added to the scores.  Rows are loaded 64 contiguous bytes per quad and
// cross a per-wave LDS tile into the operand layout (see below); the transposed
// V operand that P.V needs is read from the same tile with the transposing LDS
// read.  No workgroup barrier anywhere; overlapping neighbourhoods share rows
// through L2.
#include "cluster_common.h"
#include "launch.h"
#include "timing.h"

namespace affmae {
namespace {

constexpr int kSlotCap = 10;  // token tiles whose bias tile is resident per wave (5 KB): four workgroups per CU
static_assert(kSlotCap % 2 == 0, "an odd pass uses one more tile for the second half of its last pair");
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 40.f;  // the softmax reference follows the running maximum in steps of at least this much

struct FwdParams {
  const bf16_t *q, *k, *v, *bias, *k_blank, *v_blank;
  const uint16_t *slots, *entries;
  int N, H, K, strips, strips_per_image, slot_stride;
  uint32_t k_magic, cq_magic;  // reciprocals of K and of K / 8
  uint32_t h_magic, spi_magic;  // ... of H and of strips_per_image
  float scale;
  // bias from a relative-position table (REL kernels): token coordinates [B,N,2], table [H][2R+1][2R+1]
  const float* coords;
  const bf16_t* rel_table;
  int R;
  float rate;
  bf16_t* out;
  float* lse;
};

__device__ __forceinline__ f32x4 mfma32(const Frag8& a, const Frag8& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}

// Per strip the plan holds 16*K entries, one per (query, neighbour slot), query-major; bias rows
// [token, head, :] hold the matching K values.  With K a multiple of 8 a lane owns NT chunks of 8
// consecutive slots of one query (16-byte loads of entries and of bias); otherwise NT single entries.
constexpr int kFwdWaves = 4;  // waves per workgroup; they share nothing but the launch
// REL: the bias of a (query, neighbour) pair is looked up in the head's relative-position table instead of being
// read from a tensor.  The coordinates of the pass's token tiles are staged once in the wave's K/V tile (free
// until the first pair is staged); a lane then reads the neighbour's coordinates by the entry's (slot, token)
// fields, takes the bin against its query's coordinates and fetches the table value through the vector cache.
// RAG: N is not a multiple of 16 (only then do the row clamps and store tests below exist in the code).
template <int NT, bool VEC, bool REL, bool RAG>
__device__ __forceinline__ void pla_fwd_cluster_body(const FwdParams& p) {
  static_assert(!REL || VEC, "the table form is built for 16-byte items");
  __shared__ __align__(16) bf16_t scratch_all[kFwdWaves][kSlotCap * 256 + 8];  // + a cell that absorbs skipped entries
  __shared__ __align__(16) u32x4 kv_all[kFwdWaves][4 * 64];  // K and V rows of one pair of token tiles, per wave
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform: keeps per-wave indices in SGPRs
  const int g = lane >> 4, r = lane & 15;
  // Consecutive strips share K/V rows; workgroups are dealt round-robin to the 8 XCDs (one L2
  // each), so give every XCD a contiguous range of strips.
  const int per_xcd = gridDim.x >> 3;
  const int blk = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  // one wave per (strip, head): the heads of a strip sit in neighbouring waves and share cache lines
  const int unit = blk * kFwdWaves + wave;
  const int sg = exact_div(unit, p.H, p.h_magic);
  const int h = unit - sg * p.H;
  if (sg >= p.strips) return;  // wave-uniform; the kernel has no workgroup barrier
  bf16_t* scratch = scratch_all[wave];
  const int b = exact_div(sg, p.strips_per_image, p.spi_magic);
  const long long img_base = (long long)b * p.N;
  const int q0 = (sg - b * p.strips_per_image) * 16;  // first query of the strip, within the image
  const long long tok0 = img_base + q0;
  // An image's last strip and last token tile may be short (N % 16 != 0): rows past the end are never addressed -
  // loads repeat the last real row (no plan entry refers to it, so it meets probability 0), stores are skipped.
  const int nq = RAG ? min(16, p.N - q0) : 16;
  const int C = p.H * kD;
  const int K = p.K;

  const uint16_t* sl = p.slots + (size_t)sg * p.slot_stride;
  const int cnt_raw = sl[0];
  const int my_tile = (lane < p.slot_stride - 1) ? (int)sl[1 + lane] : 0;

  // Plan entries of this lane and the matching bias values.  They are used only while a pass scatters its bias
  // tile; a later pass (rare) loads them again, so that they hold no registers during the tile loop.
  constexpr int EW = VEC ? 4 : 1;  // 32-bit words per item
  const int items = VEC ? 2 * K : 16 * K;  // chunks of 8, or single entries
  const int chunks_per_query = K >> 3;
  const bf16_t* bias_head = p.bias ? p.bias + (size_t)tok0 * p.H * K + (size_t)h * K : nullptr;
  auto load_items = [&](uint32_t (&ent)[NT][EW], uint32_t (&bw)[NT][EW]) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int i = t * kWave + lane;
      const bool live = i < items;
      const int ii = live ? i : 0;
      if (VEC) {
        const uint4 w = *reinterpret_cast<const uint4*>(p.entries + (size_t)sg * 16 * K + (size_t)ii * 8);
        ent[t][0] = live ? w.x : 0xffffffffu;
        ent[t][EW > 1 ? 1 : 0] = live ? w.y : 0xffffffffu;
        ent[t][EW > 2 ? 2 : 0] = live ? w.z : 0xffffffffu;
        ent[t][EW > 3 ? 3 : 0] = live ? w.w : 0xffffffffu;
        const int qi_raw = fast_div(ii, p.cq_magic), j0 = (ii - qi_raw * chunks_per_query) * 8;
        const int qi = RAG ? min(qi_raw, nq - 1) : qi_raw;
        uint4 bv = make_uint4(0, 0, 0, 0);
        if (REL) {  // the query's coordinates instead
          const float2 c = (reinterpret_cast<const float2*>(p.coords) + tok0)[qi];
          bv.x = __float_as_uint(c.x);
          bv.y = __float_as_uint(c.y);
        } else if (bias_head) {
          bv = *reinterpret_cast<const uint4*>(bias_head + (uint32_t)(qi * p.H * K + j0));
        }
        bw[t][0] = bv.x;
        bw[t][EW > 1 ? 1 : 0] = bv.y;
        bw[t][EW > 2 ? 2 : 0] = bv.z;
        bw[t][EW > 3 ? 3 : 0] = bv.w;
      } else {
        ent[t][0] = live ? (uint32_t)p.entries[(size_t)sg * 16 * K + ii] : kNoEntry;
        const int qi_raw = fast_div(ii, p.k_magic), qi = RAG ? min(qi_raw, nq - 1) : qi_raw;
        bw[t][0] = bias_head ? (uint32_t)bias_head[(uint32_t)(qi * p.H * K + (ii - qi_raw * K))] : 0u;
      }
    }
  };
  // K/V rows of a token tile come in through LDS.  The MFMA operand wants lane (row r, channels
  // 8g..8g+7), which puts the four lanes of a quad on four different rows, and the memory pipeline
  // serves one row segment per cycle: such a load costs 64 cycles against 16 for a load whose quads
  // read 64 contiguous bytes.  So lane (row lane/4, 16-byte piece lane%4) loads, the pieces cross
  // through a per-wave LDS tile, and each lane reads back the piece its operand needs.  The piece index
  // is XOR-swizzled by the row so that both the writes and the reads spread over all banks.
  const char* kimg = reinterpret_cast<const char*>(p.k + (size_t)img_base * C);
  const char* vimg = reinterpret_cast<const char*>(p.v + (size_t)img_base * C);
  const int la = lane >> 2, lc = lane & 3;
  const uint32_t lane_off_h = (uint32_t)(la * C * 2 + lc * 16 + h * kD * 2);  // the lane's piece of a tile's rows, head h
  const uint32_t tile_bytes = 16u * (uint32_t)C * 2u;
  const uint32_t lane_off_max = (uint32_t)(p.N - 1) * (uint32_t)C * 2u + (uint32_t)(lc * 16 + h * kD * 2);  // same piece of the image's last row
  u32x4* kv = kv_all[wave];
  const int wr_chunk = tile_chunk(la, lc);
  const int rd_chunk = tile_chunk(r, g);
  const int lane_cell = tile_cell(r, 4 * g);  // the lane's piece of a bias tile: query r, tokens 4g..4g+3
  // V^T operand of P.V, lane (channel 16 dt + r, tokens 4g..4g+3): read from the staged row-major V tile by the
  // transposing LDS read; this lane addresses the quarter (r % 4) of the 16 channels of token 4g + r / 4
  int vt_off[2];  // byte offsets inside a staged tile
#pragma unroll
  for (int dt = 0; dt < 2; ++dt) vt_off[dt] = tile_tr_offset(g, r, dt);
  {
    Frag8 qf;
    uint32_t ent[NT][EW], bw[NT][EW];
    load_items(ent, bw);
    // the Q^T operand: lane (query r, channels 8g..8g+7)
    const u32x4 qraw =
        *reinterpret_cast<const u32x4*>(p.q + ((size_t)tok0 * C + (size_t)(h * kD)) + (uint32_t)((RAG ? min(la, nq - 1) : la) * C + lc * 8));
    // first use of a loaded value: everything the strip streams in is in flight by now
    const int ntiles = min((int)__builtin_amdgcn_readfirstlane(cnt_raw), kMaxSlots);
    kv[wr_chunk] = qraw;  // the q rows cross through LDS like the K/V rows
    wave_lds_sync();
    qf.x4 = kv[rd_chunk];
    float m_run = -INFINITY, l_run = 0.f;
    f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};

    for (int slot0 = 0; slot0 < ntiles;) {
      const int nsl = min(kSlotCap, ntiles - slot0);
      // bias tile: -inf everywhere, then the bias of the real (query, neighbour) pairs
      // (an odd pass gets one more tile of -inf: the second half of its last pair, which repeats a tile)
      for (int s = 0; s < nsl + (nsl & 1); ++s)
        *reinterpret_cast<uint2*>(scratch + s * 256 + lane * 4) = make_uint2(0xff80ff80u, 0xff80ff80u);
      const float2* cxy = reinterpret_cast<const float2*>(kv);  // REL: [slot of the pass][token of the tile]
      if (REL) {
        const float2* cimg = reinterpret_cast<const float2*>(p.coords) + img_base;
#pragma unroll
        for (int i = 0; i < (kSlotCap * 16 + kWave - 1) / kWave; ++i) {
          const int tile = __shfl(my_tile, slot0 + min(4 * i + g, nsl - 1));
          reinterpret_cast<float2*>(kv)[i * kWave + lane] = cimg[(uint32_t)(RAG ? min(tile * 16 + r, p.N - 1) : tile * 16 + r)];
        }
      }
      wave_lds_sync();
      const uint32_t lo = (uint32_t)slot0 * 256u;
      const int RW = 2 * p.R + 1;
      const bf16_t* tab = REL ? p.rel_table + h * RW * RW : nullptr;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int e = 0; e < (VEC ? 8 : 1); ++e) {
          // entries of other passes, kNoEntry and dead items fall outside the pass: they go to the spare cell
          const uint32_t off = VEC ? ((ent[t][e >> 1] >> (16 * (e & 1))) & 0xffffu) : (ent[t][0] & 0xffffu);
          const uint32_t rel = off - lo;
          uint32_t bits;
          if (REL) {
            // (an entry outside the pass reads some coordinate pair of the tile area: any value gives a cell of the table)
            const float2 cn = cxy[((rel >> 4) & 0xf0u) | cell_token(rel)];
            const int cell = relpos_cell(cn, make_float2(__uint_as_float(bw[t][0]), __uint_as_float(bw[t][EW > 1 ? 1 : 0])), p.rate, p.R);
            bits = *reinterpret_cast<const bf16_t*>(reinterpret_cast<const char*>(tab) + (uint32_t)cell * 2u);
          } else {
            bits = VEC ? ((bw[t][e >> 1] >> (16 * (e & 1))) & 0xffffu) : bw[t][0];
          }
          // (every pass but the last is full, so an offset outside the pass is at least kSlotCap * 256 away,
          // wrapped around or not: one unsigned minimum steers it to the spare cell)
          scratch[min(rel, (uint32_t)kSlotCap * 256u)] = (bf16_t)bits;
        }
      }
      wave_lds_sync();

      const int npairs = (nsl + 1) >> 1;
      auto load_pair = [&](int pr, u32x4& k0, u32x4& v0, u32x4& k1, u32x4& v1) {
        // Address = the image's K (V) rows as a scalar base + a 32-bit vector offset (an image is smaller than
        // 4 GB): the tile's byte offset is one scalar product, broadcast and added to the lane's offset by ONE vector
        // add per tile, which serves the K and the V load.  (Folding the tile into the scalar base instead costs
        // ten scalar instructions of 64-bit arithmetic per tile, and a wave issues one instruction per turn of
        // whatever kind.)  The offsets are made opaque, or the compiler rebuilds 64-bit vector addresses.
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
                            Frag8(&vt)[2]) {
        kv[0 * 64 + wr_chunk] = k0;
        kv[1 * 64 + wr_chunk] = v0;
        kv[2 * 64 + wr_chunk] = k1;
        kv[3 * 64 + wr_chunk] = v1;
        wave_lds_sync();
        kf[0].x4 = kv[0 * 64 + rd_chunk];
        kf[1].x4 = kv[2 * 64 + rd_chunk];
        const char* vbase = reinterpret_cast<const char*>(kv);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {  // k-slots 0..3 = first tile's tokens 4g..4g+3, 4..7 = second tile's
          const uint2 a = lds_read_tr(vbase + 1 * 1024 + vt_off[dt]);
          const uint2 b = lds_read_tr(vbase + 3 * 1024 + vt_off[dt]);
          vt[dt].u[0] = a.x; vt[dt].u[1] = a.y; vt[dt].u[2] = b.x; vt[dt].u[3] = b.y;
        }
      };
      auto compute_pair = [&](int pr, const Frag8(&kf)[2], const Frag8(&vt)[2]) {
        // a pass with an odd number of tiles repeats its last tile in the second half of the last pair, under
        // a bias tile of -inf: its scores are -inf without a test.  The whole pair is one basic block.
        float s[8];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          f32x4 st = {0.f, 0.f, 0.f, 0.f};
          st = mfma32(kf[tt], qf, st);  // st[i] = <k[token 4g+i], q[query r]>
          const uint2 bm = *reinterpret_cast<const uint2*>(scratch + (2 * pr + tt) * 256 + lane_cell);
          s[4 * tt + 0] = fmaf(st[0], p.scale, __uint_as_float(bm.x << 16));
          s[4 * tt + 1] = fmaf(st[1], p.scale, __uint_as_float(bm.x & 0xffff0000u));
          s[4 * tt + 2] = fmaf(st[2], p.scale, __uint_as_float(bm.y << 16));
          s[4 * tt + 3] = fmaf(st[3], p.scale, __uint_as_float(bm.y & 0xffff0000u));
        }
        float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
        // Online softmax with a lazily moved reference: m_run (one value per query, the same in the four lanes
        // that share the query) only follows the maximum when some score rose more than kLazy above it, and only
        // then are the maxima of the lanes combined and the sums rescaled (wave-uniform test).  Probabilities are
        // relative to m_run and may reach e^kLazy; the fp32 sums and the bf16 operand (8 exponent bits) keep their
        // relative precision at that size.
        if (__ballot(mx > m_run + kLazy) != 0ull) {  // also the first finite score after -inf
          mx = group_max(mx);
          const bool move = mx > m_run + kLazy;
          const float m_new = move ? mx : m_run;
          const float alpha = move ? __builtin_amdgcn_exp2f((m_run - m_new) * kLog2e) : 1.f;  // exp2(-inf) = 0
          l_run *= alpha;
#pragma unroll
          for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[dt][i] *= alpha;
          m_run = m_new;
        }
        const float shift = (m_run == -INFINITY) ? 0.f : -m_run * kLog2e;
        float pr8[8], psum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          pr8[i] = __builtin_amdgcn_exp2f(fmaf(s[i], kLog2e, shift));
          psum += pr8[i];
        }
        l_run += psum;
        Frag8 pf;  // P^T operand: k-slots 0..3 = first tile's tokens 4g..4g+3, 4..7 = second tile's
        pf.u[0] = pack_bf16x2(pr8[0], pr8[1]);
        pf.u[1] = pack_bf16x2(pr8[2], pr8[3]);
        pf.u[2] = pack_bf16x2(pr8[4], pr8[5]);
        pf.u[3] = pack_bf16x2(pr8[6], pr8[7]);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) acc[dt] = mfma32(vt[dt], pf, acc[dt]);
      };
      // The loads of the next pair fly during this pair's math.  Every load sits in straight-line code: a
      // load under a condition would make the compiler wait for all outstanding loads where the paths join.
      u32x4 sk0, sv0, sk1, sv1;
      Frag8 kf[2], vt[2];
      load_pair(0, sk0, sv0, sk1, sv1);
      for (int pr = 0; pr + 1 < npairs; ++pr) {
        stage_pair(sk0, sv0, sk1, sv1, kf, vt);
        load_pair(pr + 1, sk0, sv0, sk1, sv1);
        compute_pair(pr, kf, vt);
      }
      stage_pair(sk0, sv0, sk1, sv1, kf, vt);
      compute_pair(npairs - 1, kf, vt);
      wave_lds_sync();  // the next pass overwrites the bias tile
      slot0 += kSlotCap;
      if (slot0 >= ntiles) break;
      load_items(ent, bw);
    }

    // The probabilities that entered the MFMAs were rounded to bf16; the
    // denominator uses the unrounded ones, as the definition does.
    float l_tot = group_sum(l_run);
    float m_fin = m_run;
    if (p.k_blank) {
      Frag8 kb;
      kb.u4 = *reinterpret_cast<const uint4*>(p.k_blank + h * kD + g * 8);
      float part = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) part = fmaf(bf16_to_f32(qf.h[i]), bf16_to_f32(kb.h[i]), part);
      part = group_sum(part);
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
    // out rows cross through LDS the other way: lane (query r, channels 16dt + 4g..+3) holds 8 bytes of
    // 16-byte piece 2dt + g/2 of row r; lane (row lane/4, piece lane%4) stores 16 bytes
    wave_lds_sync();
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
      uint2 o;
      o.x = pack_bf16x2(acc[dt][0] * inv, acc[dt][1] * inv);
      o.y = pack_bf16x2(acc[dt][2] * inv, acc[dt][3] * inv);
      reinterpret_cast<uint2*>(kv)[tile_chunk(r, 2 * dt + (g >> 1)) * 2 + (g & 1)] = o;
    }
    wave_lds_sync();
    if (!RAG || la < nq)
      *reinterpret_cast<u32x4*>(p.out + ((size_t)tok0 * C + (size_t)(h * kD)) + (uint32_t)(la * C + lc * 8)) = kv[wr_chunk];
    if (g == 0 && (!RAG || r < nq)) (p.lse + (size_t)tok0 * p.H + h)[(uint32_t)(r * p.H)] = m_fin + __logf(l_tot);
  }
}

// The 16-byte path keeps four waves per SIMD; the single-entry path (K not a multiple of 8) holds more
// per-lane state and is built for two.
template <int NT, bool RAG>
__global__ __launch_bounds__(kFwdWaves* kWave) __attribute__((amdgpu_waves_per_eu(4, 4))) void pla_fwd_cluster_kernel(FwdParams p) {
  pla_fwd_cluster_body<NT, true, false, RAG>(p);
}
template <int NT, bool RAG>
__global__ __launch_bounds__(kFwdWaves* kWave) __attribute__((amdgpu_waves_per_eu(4, 4))) void pla_fwd_cluster_rel_kernel(FwdParams p) {
  pla_fwd_cluster_body<NT, true, true, RAG>(p);
}
template <int NT, bool RAG>
__global__ __launch_bounds__(kFwdWaves* kWave) __attribute__((amdgpu_waves_per_eu(3, 4))) void pla_fwd_cluster_scalar_kernel(FwdParams p) {
  pla_fwd_cluster_body<NT, false, false, RAG>(p);
}

}  // namespace

bool pla_cluster_relpos_supported(const PlaArgs& a) {
  // the table form of the tiled kernels: 16-byte items, 8-byte coordinate pairs
  return pla_cluster_supported(a) && a.K % 8 == 0 && a.rel_coords && a.rel_table &&
         reinterpret_cast<uintptr_t>(a.rel_coords) % 8 == 0;
}

bool pla_cluster_supported(const PlaArgs& a) {
  if (!a.near_clusters || a.dtype != 1 || a.d != kD) return false;
  if (a.S % 16 || a.S < 16) return false;                         // token tiles never straddle clusters
  if (a.M > (a.N + a.S - 1) / a.S) return false;
  if ((long long)a.M * a.S / 16 > kMaxSlots) return false;        // tile set of a strip is a 64-bit mask
  if (a.K > 64 || (a.N + 15) / 16 > 65535) return false;          // 16-bit plan entries and tile ids
  if ((long long)a.N * a.S >= (1ll << 31)) return false;          // range of the reciprocal division
  if ((long long)a.N * a.H * kD * 2 >= (1ll << 32)) return false; // 32-bit byte offsets inside an image's K / V
  return true;
}

size_t pla_plan_bytes(int B, int N, int K, int S, int M) { return make_plan_layout(B, N, K, S, M).total; }

hipError_t launch_pla_fwd_cluster(const PlaArgs& a, const void* plan, hipStream_t stream) {
  const PlanLayout L = make_plan_layout(a.B, a.N, a.K, a.S, a.M);
  FwdParams p;
  p.q = (const bf16_t*)a.q; p.k = (const bf16_t*)a.k; p.v = (const bf16_t*)a.v; p.bias = (const bf16_t*)a.bias;
  p.k_blank = (const bf16_t*)a.k_blank; p.v_blank = (const bf16_t*)a.v_blank;
  p.slots = reinterpret_cast<const uint16_t*>(static_cast<const char*>(plan) + L.slots_off);
  p.entries = reinterpret_cast<const uint16_t*>(static_cast<const char*>(plan) + L.entries_off);
  p.N = a.N; p.H = a.H; p.K = a.K;
  p.strips = L.strips; p.strips_per_image = (a.N + 15) / 16; p.slot_stride = L.slot_stride;
  p.scale = a.scale;
  p.out = (bf16_t*)a.out; p.lse = a.lse;
  p.coords = a.rel_coords; p.rel_table = (const bf16_t*)a.rel_table; p.R = a.rel_R; p.rate = a.rel_rate;
  p.k_magic = div_magic(a.K);
  p.cq_magic = div_magic(a.K >= 8 ? a.K / 8 : 1);
  p.h_magic = div_magic(a.H);
  p.spi_magic = div_magic((a.N + 15) / 16);
  // the XCD-contiguous mapping needs a grid that is a multiple of 8; surplus waves exit at once
  const dim3 grid((((long long)L.strips * a.H + kFwdWaves - 1) / kFwdWaves + 7) / 8 * 8);
  const bool vec = a.K % 8 == 0 && (!a.bias || reinterpret_cast<uintptr_t>(a.bias) % 16 == 0);
  const bool rag = a.N % 16 != 0;  // a short last strip / token tile per image: the variants with row clamps
#define AFFMAE_FWD(KERNEL, NT)                                                                                   \
  do {                                                                                                           \
    if (rag)                                                                                                     \
      AFFMAE_LAUNCH("pla_fwd_cluster_kernel", stream, (KERNEL<NT, true>), grid, dim3(kFwdWaves * kWave), 0, stream, p);  \
    else                                                                                                         \
      AFFMAE_LAUNCH("pla_fwd_cluster_kernel", stream, (KERNEL<NT, false>), grid, dim3(kFwdWaves * kWave), 0, stream, p); \
  } while (0)
  if (a.rel_table) {  // callers check pla_cluster_relpos_supported first
    if (2 * a.K <= kWave) AFFMAE_FWD(pla_fwd_cluster_rel_kernel, 1); else AFFMAE_FWD(pla_fwd_cluster_rel_kernel, 2);
  } else if (vec) {
    if (2 * a.K <= kWave) AFFMAE_FWD(pla_fwd_cluster_kernel, 1); else AFFMAE_FWD(pla_fwd_cluster_kernel, 2);
  } else {
    const int ent = (16 * a.K + kWave - 1) / kWave;
    if (ent <= 4) AFFMAE_FWD(pla_fwd_cluster_scalar_kernel, 4);
    else if (ent <= 8) AFFMAE_FWD(pla_fwd_cluster_scalar_kernel, 8);
    else if (ent <= 12) AFFMAE_FWD(pla_fwd_cluster_scalar_kernel, 12);
    else AFFMAE_FWD(pla_fwd_cluster_scalar_kernel, 16);
  }
#undef AFFMAE_FWD
  return hipGetLastError();
}

}  // namespace affmae
