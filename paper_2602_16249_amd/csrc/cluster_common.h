// Shared definitions of the cluster-tiled attention kernels (bf16, d = 32).
//
// Tokens are handled in tiles of 16 consecutive tokens ("token tiles"); a strip
// is the token tile seen as 16 queries.  Because clusters hold a multiple of 16
// tokens in cluster order, a token tile never straddles clusters.
//
// The plan (built by pla_plan.hip from the neighbour table) describes, per
// strip, which token tiles hold at least one neighbour of one of its queries
// ("slots", at most kMaxSlots) and, for every (query, neighbour slot j), where
// that neighbour sits: entry = slot * 256 + tile_cell(query, token % 16) (see tile_cell below).
#pragma once

#include "device_util.h"

namespace affmae {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;  // 16 bytes on their way through registers

constexpr int kD = 32;                 // channels per head
constexpr int kMaxSlots = 64;          // token tiles one strip may touch (M*S/16 <= 64)
constexpr int kMaxEntries = 16;        // 16 queries * K (<= 64) neighbours / 64 lanes
constexpr uint32_t kNoEntry = 0xffffu;

union Frag8 {
  bf16x8 v;
  uint4 u4;
  u32x4 x4;
  uint2 u2[2];
  uint32_t u[4];
  uint16_t h[8];
};

union Frag4 {
  s16x4 v;
  uint2 u2;
  uint32_t u[2];
  uint16_t h[4];
};

// Layout of the plan buffer.  "Incidence" = (strip, slot): a strip and one of the token tiles it touches.
// Per strip the valid entries are also listed grouped by slot ("runs", ascending entry index inside a
// run): sorted_pos holds the entry values in that order and runs[s] the start of slot s's run, so the
// (p, dS) words that the backward pass leaves in run order can be read back per incidence as one
// contiguous piece.  The reverse tables list, per token tile, the incidences that touch it (sorted, so
// that sums formed along a list do not depend on scheduling), each with the place of its run.
struct PlanLayout {
  int strips;        // B * ceil(N / 16) (also the number of token tiles)
  int max_slots;     // M * S / 16
  int slot_stride;   // uint16 per strip in the slot table: [0] = count, [1 + s] = token tile of slot s
  int runs_stride;   // uint16 per strip in the run table: [s] = first place of slot s, [count] = places used
  int places;        // places per strip in run order: 16 * K entries + room to start every run at an even place
  int K;
  size_t slots_off;       // uint16 [strips][slot_stride]
  size_t entries_off;     // uint16 [strips][16 * K]
  size_t sorted_pos_off;  // uint16 [strips][places]   entry values grouped by slot; kNoEntry in unused places
  size_t runs_off;        // uint16 [strips][runs_stride]
  size_t rev_count_off;   // int32  [strips]      incidences per token tile
  size_t rev_offset_off;  // int32  [strips + 1]  exclusive prefix sum of rev_count
  size_t rev_cursor_off;  // int32  [strips]      build-time cursors
  size_t rev_list_off;    // uint64 [strips * max_slots]  low: (strip within image) << 8 | slot; high: run start | run length << 16
  size_t total;
};

inline size_t plan_align(size_t n) { return (n + 255) / 256 * 256; }

inline PlanLayout make_plan_layout(int B, int N, int K, int S, int M) {
  PlanLayout L;
  L.strips = (int)((long long)B * ((N + 15) / 16));  // the last strip / token tile of an image may be short
  int max_slots = (int)((long long)M * S / 16);
  L.max_slots = max_slots;
  L.slot_stride = 1 + max_slots + (max_slots & 1);  // room to pad to an even number of slots
  if (L.slot_stride & 1) L.slot_stride += 1;
  L.K = K;
  size_t off = 0;
  L.slots_off = off;
  off += plan_align((size_t)L.strips * L.slot_stride * sizeof(uint16_t));
  L.entries_off = off;
  off += plan_align((size_t)L.strips * 16 * K * sizeof(uint16_t));
  L.places = 16 * K + max_slots + (max_slots & 1);  // even
  L.sorted_pos_off = off;
  off += plan_align((size_t)L.strips * L.places * sizeof(uint16_t));
  L.runs_stride = max_slots + 2 + (max_slots & 1);
  L.runs_off = off;
  off += plan_align((size_t)L.strips * L.runs_stride * sizeof(uint16_t));
  L.rev_count_off = off;
  off += plan_align((size_t)L.strips * sizeof(int32_t));
  L.rev_offset_off = off;
  off += plan_align(((size_t)L.strips + 1) * sizeof(int32_t));
  L.rev_cursor_off = off;
  off += plan_align((size_t)L.strips * sizeof(int32_t));
  L.rev_list_off = off;
  off += plan_align((size_t)L.strips * max_slots * sizeof(uint64_t));
  L.total = off;
  return L;
}

// Cells of a 16 x 16 (query, token) tile in LDS sit at query * 16 + (token ^ (f(query) << 2)), f(q) = (q >> 1) & 3,
// and the plan's entries carry the cell in this form.  A lane of the MFMA layouts reads or writes the four cells of
// tokens 4g..4g+3 of query r as one piece of 8 bytes (bf16 cells) or 16 bytes (word cells); without the XOR the
// pieces of several queries start on the same banks (measured per 16-byte access of a wave, 16 waves per CU: write
// 32 cycles without, 13.6 with; read 8.2 without, 5.6 with this f, 8.2 with f = ((q >> 1) & 3) ^ (q >> 3)).  The
// XOR only permutes groups of four tokens, so a piece still holds tokens 4g'..4g'+3.
__device__ __forceinline__ int cell_group_swizzle(int q) { return (q >> 1) & 3; }  // q in 0..15
__device__ __forceinline__ int tile_cell(int q, int tok) { return q * 16 + (tok ^ (cell_group_swizzle(q) << 2)); }
// token of a cell value (low byte of an entry)
__device__ __forceinline__ uint32_t cell_token(uint32_t cell) {
  return (cell & 15u) ^ (((cell >> 5) & 3u) << 2);
}

// Division of a non-negative int by a small run-time constant through a 32-bit reciprocal (exact for the
// ranges used here: n * d < 2^31).  The reciprocal of 1 does not fit 32 bits: magic 0 stands for it.
__device__ __forceinline__ int fast_div(int n, uint32_t magic) {
  // (a sum, not a choice between the two: the choice on a uniform magic becomes a branch at every use)
  return (int)(__umulhi((uint32_t)n, magic) + (magic == 0u ? (uint32_t)n : 0u));
}
inline uint32_t div_magic(int d) { return d <= 1 ? 0u : (uint32_t)((1ull << 32) / (uint32_t)d) + 1u; }
// The same for any non-negative n and d >= 1: the reciprocal is rounded up, so the quotient it gives is at most
// one too large; one multiplication checks it.  (The compiler's own division by a run-time value is a chain of
// ~30 dependent instructions through the reciprocal unit, at the head of every wave.)
__device__ __forceinline__ int exact_div(int n, int d, uint32_t magic) {
  const uint32_t q = __umulhi((uint32_t)n, magic) + (magic == 0u ? (uint32_t)n : 0u);
  return (int)(q - (q * (uint32_t)d > (uint32_t)n ? 1u : 0u));
}

__device__ __forceinline__ uint32_t wave_or32(uint32_t x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x |= __shfl_xor(x, o);
  return x;
}

// Reductions over the four lanes that hold one query's values (lanes r, r+16, r+32, r+48), on the
// VALU lane-swap instructions of gfx950: no trip through the LDS crossbar.
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
__device__ __forceinline__ float group_max(float x) {
  u32x2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float m = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  u32x2 b = __builtin_amdgcn_permlane16_swap(__float_as_uint(m), __float_as_uint(m), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float group_sum(float x) {
  u32x2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  const float m = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  u32x2 b = __builtin_amdgcn_permlane16_swap(__float_as_uint(m), __float_as_uint(m), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Place, in 16-byte pieces, of piece `piece` (0..3) of row `row` (0..15) in a 1 KB LDS tile of 16 rows
// of 64 bytes.  The XOR spreads both access patterns of the kernels over the banks: lane (row lane/4, piece
// lane%4) writes (13.6 cycles per access whatever the XOR), lane (row lane%16, piece lane/16) reads (5.6 cycles
// with this XOR, 8.2 without).
__device__ __forceinline__ int tile_chunk(int row, int piece) {
  return row * 4 + (piece ^ ((row >> 1) & 3));
}

// ds_read_b64_tr_b16: inside a group of 16 lanes, lanes 4j..4j+3 address the four 8-byte quarters of a row j of
// 16 bf16 values (j = 0..3), and lane i of the group receives element i of rows 0..3: a 4 x 16 block read by
// columns.  With rows = tokens and columns = channels this is the transposed operand of an MFMA.
__device__ __forceinline__ uint2 lds_read_tr(const void* p) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  return __builtin_bit_cast(uint2, r);
}

// Byte offset, inside a staged 16 x 32 tile (layout of tile_chunk), that lane (r = lane % 16, g = lane / 16) gives
// to lds_read_tr to receive, for channel 16 dt + r, the values of rows 4g..4g+3: it addresses the quarter r % 4 of
// the 16 channels of row 4g + r / 4.
__device__ __forceinline__ int tile_tr_offset(int g, int r, int dt) {
  return tile_chunk(4 * g + (r >> 2), 2 * dt + ((r & 3) >> 1)) * 16 + (r & 1) * 8;
}

// Two fp32 -> packed bf16 (round to nearest even), low half first.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, b);
}

}  // namespace affmae
