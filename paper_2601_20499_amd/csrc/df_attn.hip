// df_attn_fwd / df_head_score: varlen-per-head flash-style attention for gfx950.
//
// Work decomposition.  A unit is one (head, 256-query tile): 8 wavefronts of 32
// queries each stream the head's visible keys - sink region, window region,
// current chunk, in this order (the concatenation order of Eq. 2) - in tiles of
// 64 keys.  A dummy head has an empty history, so its units iterate the current
// chunk only: no masked tile is ever issued.  Heads differ in length by the ratio
// of their contexts (3x between full and dummy heads, 20x with packed long
// contexts), so heads are not dealt out whole.  The key tiles of all heads,
// longest head first, are the "columns"; query tiles are taken in groups of
// team_size, and the line of (group, column) positions is cut into equal spans,
// one per TEAM of workgroups.  A team has one workgroup per query tile of a
// group: its members walk the same columns at the same time, each for its own
// 256 queries, so they share every K/V tile in L2 while it is hot, and every
// team does the same amount of work.  A unit that lies inside one span is
// finished in place.  A unit cut by span boundaries is put together by the
// workgroup that holds its last piece (the pieces lie with the same member of
// consecutive teams): every workgroup walks its span from the END, so a piece
// that does not end its unit is done early - its sums (m, l, region sums,
// unnormalised O in fp32) go to the workspace and a flag goes up - and the
// piece that ends a unit is the last thing a workgroup does: it waits for the
// flags of the earlier pieces, folds their sums and its own in key order and
// writes the result.  This
// needs every workgroup of the launch on the device at once; when the device
// cannot hold them all, the pieces are left in the workspace and a second kernel
// puts them together in the same order with the same arithmetic.  Teams are laid
// out XCD-major (workgroup id mod 8 selects the XCD), so a team sits on one or
// two XCDs.
//
// MFMA mapping.  Scores are computed transposed, S^T = K Q^T, with
// v_mfma_f32_32x32x16_bf16: the K tile is the A operand (ds_read_b128 from a
// row-major LDS tile), the wave's Q fragment is the B operand (registers, loaded
// once per unit).  In the 32x32 accumulator layout a lane owns ONE query
// (column lane%32) and 16 of the 32 keys of a block, so the softmax row
// reductions are in-lane except for one exchange with lane^32, and the
// probabilities are already in the register layout the second product needs
// as its B operand: O^T += V^T P^T.  V^T is the A operand and is read from a
// row-major V tile in LDS with the transposing ds_read_b64_tr_b16.
//
// Schedule.  The 8 waves form two groups of 4 (one wave of each group per
// SIMD).  Every tile iteration of a wave has an MFMA phase (S = K Q^T of tile t
// and O += V^T P^T of tile t-1) and a VALU/memory phase (online softmax of tile
// t, issue of the global loads of a later tile).  The workgroup meets at one
// barrier per iteration, which group 0 takes after its VALU phase and group 1
// after its MFMA phase: between two barriers group 0 runs MFMA(t), VALU(t) and
// group 1 runs VALU(t-1), MFMA(t), so on every SIMD one wave is in its MFMA
// phase while the other is in its VALU phase: the matrix core and the vector
// ALU overlap without relying on instruction scheduling.
//
// Staging.  K and V tiles go from global memory straight into LDS with
// buffer_load_dwordx4 ... lds (no registers, no LDS store instructions); rows
// past the end of a head's buffer read as zero through the buffer range check.
// One such instruction fills 1 KB of LDS contiguously, so a tile is stored as
// groups of rows {g, g+NG, g+2NG, ...} (NG = 16 groups for d = 128), each group
// 1 KB plus a small pad.  With 16 B of pad per K group the 32 rows a wavefront
// reads per ds_read_b128 fall into distinct banks, with 64 B per V group the
// four consecutive keys of a ds_read_b64_tr_b16 do, and every operand address
// is still "lane base + compile-time offset".  Tiles rotate through four LDS
// buffers each; loads are issued two to three iterations before their first use.
//
// Online softmax keeps a reference exponent m per row and per-lane partial row
// sums l in fp32.  m is the maximum of the row's first tile and is NOT raised
// tile by tile: exp2 of a logit above m simply exceeds one, which fp32 holds
// with room to spare.  Only when a row's sum passes 2^100 (or is no longer
// finite) is m raised to the row's current maximum plus the logarithm of the
// sum and O, l rescaled, so the per-tile work has no row maximum, no
// comparison against the old one and no rescaling; P is rounded to bf16 (RNE)
// before the second product; l sums the unrounded fp32 values.  The output is
// divided by l and rounded to bf16 once at the end.
//
// The frame attention score of Eq. 3 falls out of the same statistics: with the
// keys ordered sink | window | current, snapshots (m1,l1) after the sink region
// and (m2,l2) after the window region give a row's region masses as
// l1*2^(m1-m3)/l3, (l2*2^(m2-m3) - l1*2^(m1-m3))/l3 and the remainder.
#include <algorithm>
#include <cmath>
#include <atomic>
#include <cstdlib>
#include <mutex>
#include <numeric>
#include <type_traits>
#include <vector>

#include "df_internal.h"

namespace df {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16;

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kBQ = kWaves * 32;   // queries per workgroup
constexpr int kKT = 64;            // keys per LDS tile
constexpr int kNBuf = 4;           // LDS buffers per operand
constexpr float kSumLimit = 0x1p100f; // the reference of the exponentials is raised when a row's running sum passes this
constexpr int kXcd = 8;            // XCDs per device: consecutive workgroup ids go to consecutive XCDs
constexpr int kNumCU = 256;        // MI355X: one workgroup per CU (LDS-bound occupancy)
constexpr int kMinSpan = 8;        // do not cut the work finer than this many key tiles per team
constexpr int kSpinLimit = 1 << 22; // polls of a hand-over flag before a workgroup gives up (seconds; normally one poll)

struct AttnParams {
  const u16 *q, *k_cur, *v_cur, *k_hist, *v_hist;
  u16 *out;
  float *lse;          // [H, Nq] or null
  float *part;         // workspace: [H, n_qtiles, 4] partial score sums, or null
  int32_t *tickets;    // workspace: [H] counters of the merged units of a head (zeroed by the main kernel)
  unsigned long long *flags;   // workspace: one word per workgroup, = epoch once its hand-over sum is in memory
  unsigned long long epoch;    // this launch's flag value: random, so that memory never holds it by chance
  int32_t handoff;     // cut units are put together inside the main kernel (needs all workgroups on the device at once)
  float *slots;        // workspace: 2 partial-result slots per workgroup (see Slot)
  float *score;        // [H, 3] frame attention scores, or null
  int64_t q_st, q_sh, kc_st, kc_sh, o_st, o_sh;
  int32_t Nq, Nc, H, n_qtiles;
  int32_t team_size, n_teams, n_groups;   // members of a team, teams (= spans), groups of team_size query tiles
  int32_t total_cols;          // key tiles of all heads
  int64_t line_len;            // n_groups * total_cols: positions of the line the teams share out
  int16_t n_cut_units[kMaxHeads];   // units of a head that span boundaries cut (put together by the merge kernel)
  int32_t cum[kMaxHeads + 1];  // first column of the hh-th longest head
  uint32_t cur_bytes;  // addressable bytes of one head's current-chunk rows: ((Nc-1)*kc_st + d) * 2
  float c;             // softmax_scale * log2(e)
  float inv_c;         // 1 / c
  float scale;         // softmax_scale
  int64_t hist_off[kMaxHeads + 1];
  int32_t hist_len[kMaxHeads];   // rows of each head that hold keys (a prefix of its rows)
  int32_t sink_len[kMaxHeads];
  uint8_t order[kMaxHeads];    // heads sorted by descending key count
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ unsigned pack_bf16x2(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(unsigned, h);
}

// Both values of the lane pair (lane, lane^32): a = the lower lane's value, b = the upper lane's.
// v_permlane32_swap_b32 exchanges lanes 32..63 of its first operand with lanes 0..31 of its second.
__device__ __forceinline__ void pair_values(float x, float &a, float &b) {
  a = x;
  b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float pair_max(float x) { float a, b; pair_values(x, a, b); return fmaxf(a, b); }
__device__ __forceinline__ float pair_sum(float x) { float a, b; pair_values(x, a, b); return a + b; }

// Workgroup barrier that waits for this wave's LDS traffic only: global loads stay in flight.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Position, inside a 32-key block, of the key whose scores land in accumulator
// row i: bits 2 and 3 of i are exchanged.  With it, accumulator registers
// 8t..8t+7 of a lane in half hf hold the 8 consecutive keys 16t+8hf .. +7,
// which is exactly the k-slice that lane feeds to the second product.
__device__ __forceinline__ int key_of_row(int i) {
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}



// LDS layout of one 64-key tile (all sizes in bytes).  Row r lives in group r % NG at position
// r / NG; a group is the 1 KB one buffer_load ... lds instruction writes, followed by a pad.
template <int D>
struct TileLayout {
  static constexpr int ROWB = D * 2;            // bytes per row
  static constexpr int RPG = 1024 / ROWB;       // rows per group
  static constexpr int NG = kKT / RPG;          // groups per tile
  static constexpr int KGS = 1024 + 16;         // K group stride
  static constexpr int VGS = 1024 + 64;         // V group stride
  static constexpr int KTILE = NG * KGS, VTILE = NG * VGS;
  static constexpr int k_row(int r) { return (r % NG) * KGS + (r / NG) * ROWB; }
  static constexpr int v_row(int r) { return (r % NG) * VGS + (r / NG) * ROWB; }
};

__device__ __forceinline__ unsigned lds_address(const void *ptr) {
  return unsigned(reinterpret_cast<uintptr_t>(ptr));     // low half of a flat LDS address = LDS offset
}

// The MFMA phase of a wave (both products of one tile, LDS operand reads hand-ordered) as one asm block.
#include "df_attn_phase.inc"

typedef __attribute__((address_space(3))) void lds_void;

// Partial result of one piece of a unit, as the main kernel leaves it in the workspace and the
// merge kernel reads it back.  Both kernels use the same thread <-> element mapping, so the layout
// is simply "in register order": per thread (m, l, l_sink, l_sink+window) and D/8 vectors of 4
// consecutive output elements.
template <int D>
struct Slot {
  static constexpr int kStats = kThreads * 4;                   // floats
  static constexpr int kFloats = kStats + kThreads * (D / 8) * 4;
  __device__ static float *stats(float *slot, int tid) { return slot + 4 * tid; }
  __device__ static float *ovec(float *slot, int tid, int i) { return slot + kStats + (i * kThreads + tid) * 4; }
};

// A partial result may be handed from one workgroup to another while the kernel runs (see the piece
// loop).  The L2 caches of the eight XCDs are not kept coherent with each other for ordinary accesses,
// so this data is written and read with the cache-control bits of a system-scope atomic access (sc0
// sc1: stores write through to memory, loads are served from memory) - the same bits the compiler puts
// on a relaxed system-scope atomic, here on 16-byte accesses - instead of cache maintenance, which
// would also throw the K/V tiles the team shares out of L2.
__device__ __forceinline__ void store4_through(float *ptr, float a, float b, float c, float d) {
  const f32x4 v = {a, b, c, d};
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(ptr), "v"(v) : "memory");
}
// Four 16-byte loads at ptr + i * stride floats; returns when the data is in the registers.
__device__ __forceinline__ void load4x4_through(const float *ptr, int stride, f32x4 (&v)[4]) {
  const float *p1 = ptr + stride, *p2 = ptr + 2 * stride, *p3 = ptr + 3 * stride;
  asm volatile(
      "global_load_dwordx4 %0, %4, off sc0 sc1\n\t"
      "global_load_dwordx4 %1, %5, off sc0 sc1\n\t"
      "global_load_dwordx4 %2, %6, off sc0 sc1\n\t"
      "global_load_dwordx4 %3, %7, off sc0 sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
      : "v"(ptr), "v"(p1), "v"(p2), "v"(p3)
      : "memory");
}
__device__ __forceinline__ f32x4 load4_through(const float *ptr) {
  f32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(ptr) : "memory");
  return v;
}

// A whole slot (the thread's statistics and its N = D/8 vectors of O) with every load in flight at once and one
// wait: the slot's address is uniform, the thread's part of it is tid * 16 bytes, vectors are 8 KB apart.
template <int N>
__device__ __forceinline__ void load_slot_through(const float *slot, int tid, f32x4 &st, f32x4 (&v)[N]);
template <>
__device__ __forceinline__ void load_slot_through<16>(const float *slot, int tid, f32x4 &st, f32x4 (&v)[16]) {
  static_assert(Slot<128>::kStats * 4 == 0x2000 && kThreads * 16 == 0x2000, "offsets of the asm below");
  const unsigned vo = unsigned(tid) * 16u;
  unsigned t0, t1;
  asm volatile(
      "global_load_dwordx4 %[st], %[vo], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0x2000, %[vo]\n\t"
      "global_load_dwordx4 %[v0], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x4000, %[vo]\n\t"
      "global_load_dwordx4 %[v1], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0x6000, %[vo]\n\t"
      "global_load_dwordx4 %[v2], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x8000, %[vo]\n\t"
      "global_load_dwordx4 %[v3], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0xa000, %[vo]\n\t"
      "global_load_dwordx4 %[v4], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0xc000, %[vo]\n\t"
      "global_load_dwordx4 %[v5], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0xe000, %[vo]\n\t"
      "global_load_dwordx4 %[v6], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x10000, %[vo]\n\t"
      "global_load_dwordx4 %[v7], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0x12000, %[vo]\n\t"
      "global_load_dwordx4 %[v8], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x14000, %[vo]\n\t"
      "global_load_dwordx4 %[v9], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0x16000, %[vo]\n\t"
      "global_load_dwordx4 %[v10], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x18000, %[vo]\n\t"
      "global_load_dwordx4 %[v11], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0x1a000, %[vo]\n\t"
      "global_load_dwordx4 %[v12], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x1c000, %[vo]\n\t"
      "global_load_dwordx4 %[v13], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0x1e000, %[vo]\n\t"
      "global_load_dwordx4 %[v14], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x20000, %[vo]\n\t"
      "global_load_dwordx4 %[v15], %[t1], %[sb] sc0 sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : [st] "=&v"(st), [v0] "=&v"(v[0]), [v1] "=&v"(v[1]), [v2] "=&v"(v[2]), [v3] "=&v"(v[3]), [v4] "=&v"(v[4]), [v5] "=&v"(v[5]), [v6] "=&v"(v[6]), [v7] "=&v"(v[7]), [v8] "=&v"(v[8]), [v9] "=&v"(v[9]), [v10] "=&v"(v[10]), [v11] "=&v"(v[11]), [v12] "=&v"(v[12]), [v13] "=&v"(v[13]), [v14] "=&v"(v[14]), [v15] "=&v"(v[15]), [t0] "=&v"(t0), [t1] "=&v"(t1)
      : [vo] "v"(vo), [sb] "s"(slot)
      : "memory");
}
template <>
__device__ __forceinline__ void load_slot_through<8>(const float *slot, int tid, f32x4 &st, f32x4 (&v)[8]) {
  static_assert(Slot<64>::kStats * 4 == 0x2000 && kThreads * 16 == 0x2000, "offsets of the asm below");
  const unsigned vo = unsigned(tid) * 16u;
  unsigned t0, t1;
  asm volatile(
      "global_load_dwordx4 %[st], %[vo], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0x2000, %[vo]\n\t"
      "global_load_dwordx4 %[v0], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x4000, %[vo]\n\t"
      "global_load_dwordx4 %[v1], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0x6000, %[vo]\n\t"
      "global_load_dwordx4 %[v2], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x8000, %[vo]\n\t"
      "global_load_dwordx4 %[v3], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0xa000, %[vo]\n\t"
      "global_load_dwordx4 %[v4], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0xc000, %[vo]\n\t"
      "global_load_dwordx4 %[v5], %[t1], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t0], 0xe000, %[vo]\n\t"
      "global_load_dwordx4 %[v6], %[t0], %[sb] sc0 sc1\n\t"
      "v_add_u32 %[t1], 0x10000, %[vo]\n\t"
      "global_load_dwordx4 %[v7], %[t1], %[sb] sc0 sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : [st] "=&v"(st), [v0] "=&v"(v[0]), [v1] "=&v"(v[1]), [v2] "=&v"(v[2]), [v3] "=&v"(v[3]), [v4] "=&v"(v[4]), [v5] "=&v"(v[5]), [v6] "=&v"(v[6]), [v7] "=&v"(v[7]), [t0] "=&v"(t0), [t1] "=&v"(t1)
      : [vo] "v"(vo), [sb] "s"(slot)
      : "memory");
}

// Weighted sum of the earlier pieces' value and a later piece's, written out so that both places that
// put pieces together (in the main kernel and in the merge kernel) round in the same way.
__device__ __forceinline__ float fold(float earlier, float w_earlier, float later, float w_later) {
  return __fmaf_rn(earlier, w_earlier, __fmul_rn(later, w_later));
}

// Partial-result slot of (span, first or later piece of the span, member of the team).
__device__ __forceinline__ int64_t slot_index(const AttnParams &p, int span, int which, int member) {
  return int64_t(2 * span + which) * p.team_size + member;
}

// Where the work is cut.  The line has one position per (group of query tiles, column); span s covers
// positions [span_begin(s), span_begin(s+1)).  Host and device use the same arithmetic.
__host__ __device__ __forceinline__ int64_t span_begin(int64_t s, int64_t line_len, int64_t n_spans) {
  return (s * line_len) / n_spans;
}

// One piece of a span: the part of a unit (group of query tiles x head) that the span holds.  The same
// walk - from the span's end to its start - is taken by the kernel and by the host check of a plan.
struct Piece {
  int grp, hh;          // group of query tiles; head (index into the length-sorted order)
  int n_tiles;          // key tiles of the unit
  int t_begin, t_end;   // the piece: tiles [t_begin, t_end) of the unit
  int64_t unit_lo;      // line position of the unit's first tile
  int64_t pos;          // line position of the piece's first tile
};
// Head (index into the length-sorted order) that owns column `col`.
__host__ __device__ __forceinline__ int head_of_column(const AttnParams &p, int col) {
  int hh = 0;
  while (col >= p.cum[hh + 1]) ++hh;
  return hh;
}

// The piece of span [span_lo, ...) that ends at line position pos_end (span_lo < pos_end <= the span's end).
__host__ __device__ __forceinline__ Piece piece_ending_at(const AttnParams &p, int64_t span_lo, int64_t pos_end) {
  Piece c;
  c.grp = int((pos_end - 1) / p.total_cols);
  const int col = int((pos_end - 1) - int64_t(c.grp) * p.total_cols);
  c.hh = head_of_column(p, col);
  c.n_tiles = p.cum[c.hh + 1] - p.cum[c.hh];
  c.unit_lo = int64_t(c.grp) * p.total_cols + p.cum[c.hh];
  c.pos = span_lo > c.unit_lo ? span_lo : c.unit_lo;
  c.t_begin = int(c.pos - c.unit_lo);
  c.t_end = int(pos_end - c.unit_lo);
  return c;
}

// Normalise, round and store one thread's share of 32 output columns (block db) of a finished unit.
__device__ __forceinline__ void store_output_block(const AttnParams &p, int h, int row, int hf, int db, const f32x16 &o,
                                                   float inv) {
  u16 *dst = p.out + row * p.o_st + h * p.o_sh + 4 * hf + 32 * db;
#pragma unroll
  for (int cq = 0; cq < 4; ++cq) {
    uint2 w;
    w.x = pack_bf16x2(o[4 * cq] * inv, o[4 * cq + 1] * inv);
    w.y = pack_bf16x2(o[4 * cq + 2] * inv, o[4 * cq + 3] * inv);
    *reinterpret_cast<uint2 *>(dst + 8 * cq) = w;
  }
}
template <int D>
__device__ __forceinline__ void store_output(const AttnParams &p, int h, int row, int hf, const f32x16 (&o)[D / 32],
                                             float inv) {
#pragma unroll
  for (int db = 0; db < D / 32; ++db) store_output_block(p, h, row, hf, db, o[db], inv);
}

// Sum of the two region masses over the 256 rows of a unit, in a fixed order (deterministic): a
// butterfly over the 32 rows of every wave, then the 8 waves in order.  Both halves of a lane pair hold
// the same masses, so the butterfly stays inside one half.
__device__ __forceinline__ void reduce_masses(const AttnParams &p, float *lds_red, int h, int qt, int tid,
                                              float mass_a, float mass_b) {
  const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
  for (int m = 1; m < 32; m <<= 1) {
    mass_a += __shfl_xor(mass_a, m);
    mass_b += __shfl_xor(mass_b, m);
  }
  if (lane == 0) {
    lds_red[2 * wave] = mass_a;
    lds_red[2 * wave + 1] = mass_b;
  }
  __syncthreads();
  if (tid < 2) {
    float acc = 0.f;
    for (int w = 0; w < kWaves; ++w) acc += lds_red[2 * w + tid];
    p.part[(int64_t(h) * p.n_qtiles + qt) * 4 + tid] = acc;
  }
  __syncthreads();
}

// F[h] = (sum_a, sum_b - sum_a, n - sum_b) / n over the head's query tiles, in tile order.
__device__ __forceinline__ void finish_score(const AttnParams &p, int h) {
  float a = 0.f, b = 0.f;
  for (int t = 0; t < p.n_qtiles; ++t) {
    a += p.part[(int64_t(h) * p.n_qtiles + t) * 4];
    b += p.part[(int64_t(h) * p.n_qtiles + t) * 4 + 1];
  }
  const float inv = 1.f / float(p.Nq);
  p.score[3 * h] = a * inv;
  p.score[3 * h + 1] = (b - a) * inv;
  p.score[3 * h + 2] = (float(p.Nq) - b) * inv;
}

template <int D, bool SCORE_ONLY>
__global__ __launch_bounds__(kThreads) void df_attn_kernel(const AttnParams p) {
  constexpr int KS = D / 16;            // k-steps of the first product
  constexpr int DB = D / 32;            // 32-row blocks of O^T
  using L = TileLayout<D>;
  constexpr int GPW = L::NG / kWaves;   // row groups each wave loads per tile (2 for d=128, 1 for d=64)
  constexpr int kDmaPerPhase = GPW * (SCORE_ONLY ? 1 : 2);   // buffer loads a wave issues per VALU phase
  __shared__ __attribute__((aligned(16))) unsigned char lds_k[kNBuf * L::KTILE];
  __shared__ __attribute__((aligned(16))) unsigned char lds_v[SCORE_ONLY ? 16 : kNBuf * L::VTILE];
  __shared__ float lds_red[kWaves * 2];
  __shared__ int lds_ok;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int group = wave >> 2;
  const int j = lane & 31, hf = lane >> 5;

  // the merge kernel counts the merged units of a head: its counters start at zero (this kernel ends
  // before that one begins)
  if (blockIdx.x == 0 && p.tickets != nullptr && tid < p.H) p.tickets[tid] = 0;

  // ---- this workgroup's team (span of the line) and member index (query tile inside a group); XCD-major numbering
  const int n_slots_x = int(gridDim.x) / kXcd;
  const int wg = (gridDim.x % kXcd == 0) ? (blockIdx.x % kXcd) * n_slots_x + blockIdx.x / kXcd : blockIdx.x;
  const int span = wg / p.team_size, member = wg % p.team_size;
  if (span >= p.n_teams) return;
  const int64_t span_lo = span_begin(span, p.line_len, p.n_teams);
  const int64_t span_hi = span_begin(span + 1, p.line_len, p.n_teams);

  // per-lane LDS byte addresses of the MFMA A operands (buffer 0); see TileLayout for the row placement
  const int g16 = lane >> 4, i16 = lane & 15;
  const int krow = key_of_row(j);
  const int vrow = 8 * (g16 >> 1) + (i16 >> 2);
  const unsigned k_lane_addr = lds_address(lds_k) + (krow % L::NG) * L::KGS + (krow / L::NG) * L::ROWB + 16 * hf;
  const unsigned v_lane_addr = lds_address(lds_v) + (vrow % L::NG) * L::VGS + (vrow / L::NG) * L::ROWB +
                               32 * (g16 & 1) + 8 * (i16 & 3);
  // lane -> (row position inside the group, 16-byte chunk of the row) in the 1 KB a load writes
  const int dma_pos = (16 * lane) / L::ROWB, dma_chunk = (16 * lane) % L::ROWB;
  const uint32_t cur_stride_b = uint32_t(p.kc_st) * 2u;
  const int voff_hist = dma_pos * L::NG * L::ROWB + dma_chunk;
  const int voff_cur = dma_pos * L::NG * int(cur_stride_b) + dma_chunk;
  constexpr uint32_t kNoTile = 0x7ff00000u;      // beyond every descriptor (plus any lane offset): the load writes zeros
  const uint32_t lane_vo_hist = uint32_t(voff_hist) + uint32_t(wave) * L::ROWB;      // lane offset + this wave's first row group
  const uint32_t lane_vo_cur = uint32_t(voff_cur) + uint32_t(wave) * cur_stride_b;

  // The pieces of the span are taken from its end to its start.  A head that a span boundary cuts in two
  // is then begun by the workgroup that has it at the end of its span as the FIRST thing it does, and
  // completed by the workgroup that has the rest at the start of its span as the LAST thing it does: by
  // then the first part has long been in memory, and the second workgroup finishes the unit itself
  // (hand-over) instead of leaving a partial result to a second kernel.
#pragma unroll 1
  for (int64_t pos_end = span_hi; pos_end > span_lo;) {
    // ---- the piece that ends at `pos_end`: group of query tiles, head, first and last tile of this team's share
    const Piece piece = piece_ending_at(p, span_lo, pos_end);
    const int grp = piece.grp, hh = piece.hh;      // hh: index into the length-sorted head order
    const int h = p.order[hh];
    const int64_t hoff = p.hist_off[h];
    const int len_h = p.hist_len[h];
    const int sink = p.sink_len[h];
    const int nt0 = (sink + kKT - 1) / kKT;
    const int nt1 = (len_h - sink + kKT - 1) / kKT;
    const int nt2 = (p.Nc + kKT - 1) / kKT;
    const int n_tiles = piece.n_tiles;             // = nt0 + nt1 + nt2
    const int64_t unit_lo = piece.unit_lo;         // line position of the unit's first tile
    const int64_t piece_pos = piece.pos;
    const int t_begin = piece.t_begin, t_end = piece.t_end;
    pos_end = piece_pos;
    // Hand-over: a piece that does not end its unit leaves its partial sums in the workspace and raises a
    // flag; the piece that ends the unit (always the last thing its workgroup does) collects the sums of
    // all earlier pieces - they lie with the same member of the preceding teams - and finishes the unit.
    const bool give = p.handoff && t_end < n_tiles;
    const bool take = p.handoff && t_begin > 0 && t_end == n_tiles;
    const int qt = grp * p.team_size + member;     // this workgroup's query tile in this group
    if (qt >= p.n_qtiles) continue;                // the last group may have fewer tiles than the team has members
    const int q0 = qt * kBQ + wave * 32;
    // a wave whose 32 rows all lie past the last query (tail of the last query tile) moves tiles and keeps
    // the barriers, but computes nothing
    const bool wave_live = q0 < p.Nq;

    // ---- global -> LDS: buffer descriptors of this head's history and current-chunk rows.  A load
    // past the end of the descriptor returns zeros, which is how partial and absent tiles are padded.
    const int hist_bytes = len_h * L::ROWB;
    const __amdgpu_buffer_rsrc_t rs_kh = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16 *>(p.k_hist) + hoff * D, 0, hist_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_kc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16 *>(p.k_cur) + h * p.kc_sh, 0, int(p.cur_bytes), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_vh = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16 *>(SCORE_ONLY ? p.k_hist : p.v_hist) + hoff * D, 0, hist_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_vc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u16 *>(SCORE_ONLY ? p.k_cur : p.v_cur) + h * p.kc_sh, 0, int(p.cur_bytes), 0x00020000);
    // Issue this wave's share of tile t (zeros if the piece does not reach it) into LDS buffer `slot`.
    // The whole byte offset travels in the VGPR offset, the only part of a buffer address that the
    // hardware checks against the descriptor's size (the SGPR offset is not range-checked).
    auto dma_tile = [&](int t, int slot, bool is_v) {
      bool cur = false;
      uint32_t toff = kNoTile;
      uint32_t stride_b = L::ROWB;
      if (t >= t_end) toff = kNoTile;
      else if (t < nt0) toff = uint32_t(t * kKT) * L::ROWB;
      else if (t < nt0 + nt1) toff = uint32_t(sink + (t - nt0) * kKT) * L::ROWB;
      else { cur = true; stride_b = cur_stride_b; toff = uint32_t((t - nt0 - nt1) * kKT) * cur_stride_b; }
      unsigned char *dst = is_v ? lds_v + slot * L::VTILE : lds_k + slot * L::KTILE;
      const int gs = is_v ? L::VGS : L::KGS;
#pragma unroll
      for (int i = 0; i < GPW; ++i) {
        const int g = wave + kWaves * i;
        lds_void *d = (lds_void *)(dst + g * gs);
        const int vo = int(toff + uint32_t(g) * stride_b + uint32_t(cur ? voff_cur : voff_hist));
        if (cur) __builtin_amdgcn_raw_ptr_buffer_load_lds(is_v ? rs_vc : rs_kc, d, 16, vo, 0, 0, 0);
        else __builtin_amdgcn_raw_ptr_buffer_load_lds(is_v ? rs_vh : rs_kh, d, 16, vo, 0, 0, 0);
      }
    };

    // Inside the tile loop the loads follow two cursors (K three tiles ahead, V two), advanced by one
    // tile per iteration: byte offset += keys per tile * row stride, LDS buffer rotated, and only at
    // the few tiles where a cursor enters the window region, the current chunk or the end of the piece
    // are offset, step and descriptor worked out again.  That keeps the scalar work per iteration
    // to a handful of instructions.
    struct Cursor {
      int t, next_event;            // tile under the cursor; first tile at which step/descriptor change
      uint32_t vo;                  // per lane: byte offset of this lane's 16 bytes of the wave's first row group
      uint32_t step, step_g;        // bytes per tile; bytes between the wave's row groups (kWaves rows apart)
    };
    // the descriptor each cursor currently reads through (the history's or the current chunk's); kept outside
    // the struct and changed only where a cursor crosses into another region, not selected per tile
    __amdgpu_buffer_rsrc_t rs_k_now = rs_kh, rs_v_now = rs_vh;
    auto relocate = [&](Cursor &c, bool is_v) {
      const int t = c.t;
      bool cur = true;
      if (t >= t_end) {             // absent tile: out of range for every lane, the loads write zeros
        c.vo = kNoTile; c.step = 0; c.step_g = 0; c.next_event = INT32_MAX;
      } else if (t < nt0 + nt1) {
        const uint32_t row0 = t < nt0 ? uint32_t(t * kKT) : uint32_t(sink + (t - nt0) * kKT);
        c.vo = lane_vo_hist + row0 * L::ROWB; c.step = kKT * L::ROWB; c.step_g = kWaves * L::ROWB;
        c.next_event = min(t < nt0 ? nt0 : nt0 + nt1, t_end);
        cur = false;
      } else {
        c.vo = lane_vo_cur + uint32_t((t - nt0 - nt1) * kKT) * cur_stride_b;
        c.step = kKT * cur_stride_b; c.step_g = kWaves * cur_stride_b; c.next_event = t_end;
      }
      if (is_v) rs_v_now = cur ? rs_vc : rs_vh;
      else rs_k_now = cur ? rs_kc : rs_kh;
    };
    // one tile on: next tile's bytes; then this wave's share of that tile goes out into LDS buffer `slot`
    // (a compile-time number: the tile loop is unrolled over the four buffers)
    auto advance_and_load = [&](Cursor &c, bool is_v, int slot) {
      const unsigned tile_b = is_v ? L::VTILE : L::KTILE, gs = is_v ? L::VGS : L::KGS;
      const unsigned dst = (is_v ? lds_address(lds_v) : lds_address(lds_k)) + wave * gs + slot * tile_b;
      ++c.t;
      c.vo += c.step;
      if (c.t == c.next_event) relocate(c, is_v);
#pragma unroll
      for (int i = 0; i < GPW; ++i) {
        lds_void *d = (lds_void *)(uintptr_t)(dst + kWaves * i * gs);
        const int vo = int(c.vo + uint32_t(i) * c.step_g);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(is_v ? rs_v_now : rs_k_now, d, 16, vo, 0, 0, 0);
      }
    };

    // ---- Q fragment: B operand of S^T = K Q^T.  Lane (j, hf) holds, for query j,
    // elements 16*ks + 8*hf .. +7 of every k-step.
    bf16x8 qf[KS];
    {
      int row = q0 + j;
      row = row < p.Nq ? row : p.Nq - 1;          // tail rows re-read the last query; never stored
      const u16 *src = p.q + row * p.q_st + h * p.q_sh + 8 * hf;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
    }

    // ---- piece prologue: its first three K tiles and first two V tiles on their way into LDS; the
    // spare V buffer, which the first MFMA phase multiplies with P = 0, is cleared
    dma_tile(t_begin, 0, false);
    dma_tile(t_begin + 1, 1, false);
    dma_tile(t_begin + 2, 2, false);
    if (!SCORE_ONLY) {
      dma_tile(t_begin, 0, true);
      dma_tile(t_begin + 1, 1, true);
      for (int i = tid; i < L::VTILE / 16; i += kThreads) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4 *>(lds_v + (kNBuf - 1) * L::VTILE + 16 * i) = z;
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m = -INFINITY;
    float l = 0.f;                           // this lane's share of the row sum, relative to m
    float nmc = INFINITY;                    // -m * c
    float snap_m0 = -INFINITY, snap_l0 = 0.f, snap_m1 = -INFINITY, snap_l1 = 0.f;
    f32x16 s[2];
    bf16x8 pb[2][2];                         // P^T of the previous tile, [key block][16-key step]
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int ts = 0; ts < 2; ++ts)
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[kb][ts][e] = (__bf16)0.f;
    // the cursors start on the last tiles the prologue has issued (K: t_begin + 2 in buffer 2, V: t_begin + 1 in buffer 1)
    Cursor kc, vc;
    kc.t = t_begin + 2;
    relocate(kc, false);
    vc.t = t_begin + 1;
    relocate(vc, true);

    const int seg_end0 = nt0 - 1, seg_end1 = nt0 + nt1 - 1;
    // last tile of the segment that tile t lies in (empty segments have no tiles)
    auto seg_end_from = [&](int t) { return t < nt0 ? seg_end0 : (t < nt0 + nt1 ? seg_end1 : n_tiles - 1); };
    int next_seg_end = seg_end_from(t_begin);
    // P^T of the tile in s against the reference -nmc/c: bf16 operands of the second product into pb, and
    // the sum of the unrounded values over this lane's 32 keys (four independent chains)
    auto exp_tile = [&](float nmc_) {
      float c4[4];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) {
          unsigned w[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float e0 = fast_exp2(__builtin_fmaf(s[kb][8 * ts + 2 * e], p.c, nmc_));
            const float e1 = fast_exp2(__builtin_fmaf(s[kb][8 * ts + 2 * e + 1], p.c, nmc_));
            w[e] = pack_bf16x2(e0, e1);
            if (kb == 0 && ts == 0) c4[e] = e0 + e1;
            else c4[e] += e0 + e1;   // plain adds: the dot-product instructions share the matrix core and stall its MFMAs
          }
          u32x4 u = {w[0], w[1], w[2], w[3]};
          pb[kb][ts] = __builtin_bit_cast(bf16x8, u);
        }
      return (c4[0] + c4[1]) + (c4[2] + c4[3]);
    };
    // One tile iteration; SLOT = LDS buffer of K(t), a compile-time number (the loop below is unrolled over
    // the four buffers, so no buffer address is computed at run time).  V(t-1) is in buffer SLOT + 3, the
    // loads of this iteration fill K(t+3) into buffer SLOT + 3 and V(t+2) into buffer SLOT + 2 (mod 4).
    int t = t_begin;
    auto iteration = [&](auto slot_c) {
      constexpr int SLOT = decltype(slot_c)::value;
      int n_valid_t = kKT;                    // real keys in tile t: only a segment's last tile can be partial
      bool seg_last = false;                  // tile t ends the sink or the window region (or the unit)
      if (t == next_seg_end) {
        seg_last = true;
        if (t == seg_end0) n_valid_t = sink - (nt0 - 1) * kKT;
        else if (t == seg_end1) n_valid_t = len_h - sink - (nt1 - 1) * kKT;
        else n_valid_t = p.Nc - (nt2 - 1) * kKT;
        next_seg_end = seg_end_from(t + 1);
      }
      // ================= MFMA phase =================
      // Always both products: at the first tile the second one multiplies P = 0 with the zero-filled
      // spare V buffer, after the last tile the first one computes scores of a stale tile that nobody reads.
      if (wave_live)
        MfmaPhase<D, !SCORE_ONLY>::run(k_lane_addr + SLOT * L::KTILE, v_lane_addr + ((SLOT + 3) & 3) * L::VTILE, qf, pb, s, o);
      // One workgroup barrier per iteration, taken by group 1 here and by group 0 after its VALU
      // phase: between two barriers group 0 runs MFMA(t), VALU(t) and group 1 runs VALU(t-1), MFMA(t),
      // so the two waves of a SIMD are in opposite phases without being locked phase by phase.
      // Before a barrier a wave waits for those of its loads that the MFMA phases behind that barrier read.
      // Tile K(t+3) / V(t+2), issued in VALU phase t, is first read in MFMA phase t+3, which begins behind
      // barrier t+2 (barrier n = the one group 0 takes after VALU(n) and group 1 after MFMA(n)).  Group 0
      // issues it before barrier t and may leave the loads of its latest two phases in flight; group 1
      // issues it behind barrier t and may leave those of its latest phase in flight.  Either way a load has
      // about two iterations to land.  Behind a barrier every wave has finished MFMA(t-1), whose tiles'
      // buffers the next VALU phases overwrite.
      if (group == 1) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kDmaPerPhase) : "memory");
        lds_barrier();
      }
      // ================= VALU / memory phase =================
      // every wave issues the same number of loads once per VALU phase (absent tiles load zeros), so
      // the s_waitcnt counts hold
      advance_and_load(kc, false, (SLOT + 3) & 3);
      if (!SCORE_ONLY) advance_and_load(vc, true, (SLOT + 2) & 3);
      if (t < t_end && wave_live) {
        if (n_valid_t < kKT) {                // keys past the end of the segment
          const int key0 = 8 * hf;
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v)      // key = key0 + 32 kb + 16 (v / 8) + v % 8
              if (key0 >= n_valid_t - (32 * kb + 16 * (v >> 3) + (v & 7))) s[kb][v] = -INFINITY;
        }
        // P = 2^(c s - c m) against the reference m the row already has, its sum in four chains
        float ts = exp_tile(nmc);
        float l_new = l + ts;
        // No row maximum is taken on the common path.  m is only a reference: what has to hold is
        // that nothing overflows, and any P beyond the limit (or infinite, or the NaN of an all-masked
        // start) shows in the row's sum.  Rare: the first tile of a piece, and rows that outgrow 2^100.
        if (__any(!(l_new <= kSumLimit))) {
          float a = s[0][0];
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) a = fmaxf(a, s[kb][v]);
          const float mx = pair_max(a);       // exact row maximum of the tile: the new P are at most 1
          // the reference also absorbs the size of the sum so far (l becomes O(1)); -inf while l = 0
          const float m_new = fmaxf(fmaxf(m, mx), m + __builtin_amdgcn_logf(pair_sum(l)) * p.inv_c);
          const float alpha = fast_exp2((m - m_new) * p.c);
          m = m_new;
          nmc = -m * p.c;
          l *= alpha;
          if (!SCORE_ONLY) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
              for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
          }
          ts = exp_tile(nmc);
          l_new = l + ts;
        }
        l = l_new;
        if (seg_last) {                       // rare: keep the bookkeeping out of the common path
          if (t == seg_end0) { snap_m0 = m; snap_l0 = l; }
          if (t == seg_end1) { snap_m1 = m; snap_l1 = l; }
        }
      }
      if (group == 0) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kDmaPerPhase) : "memory");
        lds_barrier();
      }
    };
#pragma unroll 1
    for (;;) {
      iteration(std::integral_constant<int, 0>{});
      if (++t > t_end) break;
      iteration(std::integral_constant<int, 1>{});
      if (++t > t_end) break;
      iteration(std::integral_constant<int, 2>{});
      if (++t > t_end) break;
      iteration(std::integral_constant<int, 3>{});
      if (++t > t_end) break;
    }
    // no load of this piece may land in the next one's tiles, and no wave may still be reading them
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    lds_barrier();
    // Region sums of this piece: a region that ended before the piece began contributes nothing, a
    // region the piece ends in (or before) contains everything the piece has summed.
    const float l_piece = l;
    if (seg_end0 >= t_end) { snap_m0 = m; snap_l0 = l_piece; }
    if (seg_end1 >= t_end) { snap_m1 = m; snap_l1 = l_piece; }

    // ---- piece epilogue
    const float lt = pair_sum(l_piece);
    const float l1 = pair_sum(snap_l0 * fast_exp2((snap_m0 - m) * p.c));   // sink region, relative to m
    const float l2 = pair_sum(snap_l1 * fast_exp2((snap_m1 - m) * p.c));   // sink + window regions
    const int row = q0 + j;
    const bool valid = row < p.Nq;
    float m_u = m, lt_u = lt, l1_u = l1, l2_u = l2;
    if (take) {
      // The earlier pieces were written when their workgroups began their spans (a piece that fills a whole
      // span: when that workgroup ended), i.e. long ago or at about this time.  Wait until every flag says
      // its piece is in memory; the wait is bounded so that a workgroup that never runs cannot hang the
      // device: the rows then come out as NaN.
      int s_first = span - 1;                      // span that holds the unit's first tile
      while (s_first > 0 && span_begin(s_first, p.line_len, p.n_teams) > unit_lo) --s_first;
      if (tid == 0) {
        int all = 1;
        for (int sp = s_first; sp < span; ++sp) {
          unsigned long long *flag = p.flags + sp * p.team_size + member;
          int ok = 0;
          for (int spin = 0; spin < kSpinLimit && !ok; ++spin) {
            ok = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) == p.epoch;
            if (!ok) __builtin_amdgcn_s_sleep(16);
          }
          // a flag has one reader: put it back, so that a replay of this launch (same epoch) starts clean
          __hip_atomic_store(flag, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
          all &= ok;
        }
        lds_ok = all;
      }
      __syncthreads();
      const float poison = lds_ok ? 0.f : NAN;
      // earlier pieces first, this one last: the same order and arithmetic as the merge kernel
      if (s_first == span - 1) {
        // the common case, one earlier piece: all of it is loaded with one wait (folding it into an empty sum
        // would give back the same numbers)
        const int which = unit_lo > span_begin(s_first, p.line_len, p.n_teams) ? 1 : 0;
        const float *slot = p.slots + slot_index(p, s_first, which, member) * Slot<D>::kFloats;
        f32x4 st, v[D / 8];
        if constexpr (SCORE_ONLY) st = load4_through(Slot<D>::stats(const_cast<float *>(slot), tid));
        else load_slot_through<D / 8>(slot, tid, st, v);
        const float m_new = fmaxf(st[0], m);
        const float w_h = (st[0] == m_new) ? 1.f : fast_exp2((st[0] - m_new) * p.c);
        const float w_t = (m == m_new) ? 1.f : fast_exp2((m - m_new) * p.c);
        m_u = m_new + poison;
        lt_u = fold(st[1], w_h, lt, w_t);
        l1_u = fold(st[2], w_h, l1, w_t);
        l2_u = fold(st[3], w_h, l2, w_t);
        if (!SCORE_ONLY) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int cq = 0; cq < 4; ++cq)
#pragma unroll
              for (int e = 0; e < 4; ++e) o[db][4 * cq + e] = fold(v[db * 4 + cq][e], w_h, o[db][4 * cq + e], w_t);
        }
      } else {
        float M = -INFINITY, Lt = 0.f, La = 0.f, Lb = 0.f;
        f32x16 acc[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
#pragma unroll 1
        for (int sp = s_first; sp < span; ++sp) {
          const int which = unit_lo > span_begin(sp, p.line_len, p.n_teams) ? 1 : 0;
          const float *slot = p.slots + slot_index(p, sp, which, member) * Slot<D>::kFloats;
          const f32x4 st = load4_through(Slot<D>::stats(const_cast<float *>(slot), tid));
          const float m_new = fmaxf(M, st[0]);
          const float w_old = (M == m_new) ? 1.f : fast_exp2((M - m_new) * p.c);
          const float w_new = (st[0] == m_new) ? 1.f : fast_exp2((st[0] - m_new) * p.c);
          M = m_new;
          Lt = fold(Lt, w_old, st[1], w_new);
          La = fold(La, w_old, st[2], w_new);
          Lb = fold(Lb, w_old, st[3], w_new);
          if (!SCORE_ONLY) {
#pragma unroll
            for (int db = 0; db < DB; ++db) {
              f32x4 v[4];
              load4x4_through(Slot<D>::ovec(const_cast<float *>(slot), tid, db * 4), kThreads * 4, v);
#pragma unroll
              for (int cq = 0; cq < 4; ++cq)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[db][4 * cq + e] = fold(acc[db][4 * cq + e], w_old, v[cq][e], w_new);
            }
          }
        }
        const float m_new = fmaxf(M, m);
        const float w_h = (M == m_new) ? 1.f : fast_exp2((M - m_new) * p.c);
        const float w_t = (m == m_new) ? 1.f : fast_exp2((m - m_new) * p.c);
        m_u = m_new + poison;
        lt_u = fold(Lt, w_h, lt, w_t);
        l1_u = fold(La, w_h, l1, w_t);
        l2_u = fold(Lb, w_h, l2, w_t);
        if (!SCORE_ONLY) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] = fold(acc[db][v], w_h, o[db][v], w_t);
        }
      }
      __syncthreads();                             // lds_ok is free again
    }
    if (t_end == n_tiles && (t_begin == 0 || take)) {
      // the unit is complete
      const float inv = 1.f / lt_u;
      if (!SCORE_ONLY && valid) {
        store_output<D>(p, h, row, hf, o, inv);
        if (p.lse != nullptr && hf == 0) p.lse[int64_t(h) * p.Nq + row] = m_u * p.scale + __logf(lt_u);
      }
      if (p.part != nullptr)
        reduce_masses(p, lds_red, h, qt, tid, valid ? l1_u * inv : 0.f, valid ? l2_u * inv : 0.f);
    } else {
      // a piece that starts at the span's first position uses the span's slot 0, a later one slot 1
      float *slot = p.slots + slot_index(p, span, piece_pos == span_lo ? 0 : 1, member) * Slot<D>::kFloats;
      store4_through(Slot<D>::stats(slot, tid), m_u, lt_u, l1_u, l2_u);
      if (!SCORE_ONLY) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int cq = 0; cq < 4; ++cq)
            store4_through(Slot<D>::ovec(slot, tid, db * 4 + cq), o[db][4 * cq], o[db][4 * cq + 1], o[db][4 * cq + 2],
                           o[db][4 * cq + 3]);
      }
      if (give) {
        // each thread's stores are in memory when its counter reaches zero; after the barrier all are
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0)
          __hip_atomic_store(p.flags + span * p.team_size + member, p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
  }
}

// Second kernel.  Workgroup (k, member; db) looks at the boundary between spans k-1 and k: if it falls
// inside a head (not on its first column), the unit (group, head, member's query tile) was cut there
// and is put together from the partial results of its pieces, in key order, with the usual
// log-sum-exp weights; a unit cut by several boundaries is handled at the first of them.  blockIdx.y
// = db selects 32 of the D output columns, so that a unit is spread over D/32 workgroups (the kernel
// is a pure data mover and wants many loads in flight).  When scores are wanted, the db = 0 workgroup
// that completes the last unit of a head (counted per head) sums the head's per-tile masses in tile
// order; heads that were not cut anywhere get a workgroup of their own for that
// (blockIdx.x >= (n_teams - 1) * team_size).
template <int D, bool SCORE_ONLY>
__global__ __launch_bounds__(kThreads) void df_attn_merge_kernel(const AttnParams p) {
  __shared__ float lds_red[kWaves * 2];
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, j = lane & 31, hf = lane >> 5;
  const int db = int(blockIdx.y);
  const int n_merge = p.handoff ? 0 : (p.n_teams - 1) * p.team_size;
  if (int(blockIdx.x) >= n_merge) {                // score of a head no boundary cuts
    const int h = int(blockIdx.x) - n_merge;
    if (db == 0 && tid == 0 && p.n_cut_units[h] == 0) finish_score(p, h);
    return;
  }
  const int k = int(blockIdx.x) / p.team_size + 1, member = int(blockIdx.x) % p.team_size;
  const int64_t cut = span_begin(k, p.line_len, p.n_teams);
  const int grp = int(cut / p.total_cols);
  const int col = int(cut - int64_t(grp) * p.total_cols);
  const int hh = head_of_column(p, col);
  if (col == p.cum[hh]) return;                    // the boundary coincides with the head's first column
  const int64_t u_lo = int64_t(grp) * p.total_cols + p.cum[hh], u_hi = u_lo + (p.cum[hh + 1] - p.cum[hh]);
  if (k >= 2 && span_begin(k - 1, p.line_len, p.n_teams) > u_lo) return;   // an earlier boundary cuts the same unit
  const int qt = grp * p.team_size + member;
  if (qt >= p.n_qtiles) return;
  const int h = p.order[hh];
  const int s_lo = k - 1;                          // span that holds the unit's first column
  int s_hi = k;
  while (span_begin(s_hi + 1, p.line_len, p.n_teams) < u_hi) ++s_hi;

  float M = -INFINITY, Lt = 0.f, La = 0.f, Lb = 0.f;
  f32x16 o;
#pragma unroll
  for (int v = 0; v < 16; ++v) o[v] = 0.f;
#pragma unroll 1
  for (int sp = s_lo; sp <= s_hi; ++sp) {
    const int64_t b = span_begin(sp, p.line_len, p.n_teams);
    const float *slot = p.slots + slot_index(p, sp, u_lo > b ? 1 : 0, member) * Slot<D>::kFloats;
    const float4 st = *reinterpret_cast<const float4 *>(Slot<D>::stats(const_cast<float *>(slot), tid));
    const float m_new = fmaxf(M, st.x);
    // a piece of a wave that computes nothing (rows past the last query) has m = -inf throughout
    const float w_old = (M == m_new) ? 1.f : fast_exp2((M - m_new) * p.c);
    const float w_new = (st.x == m_new) ? 1.f : fast_exp2((st.x - m_new) * p.c);
    M = m_new;
    Lt = fold(Lt, w_old, st.y, w_new);
    La = fold(La, w_old, st.z, w_new);
    Lb = fold(Lb, w_old, st.w, w_new);
    if (!SCORE_ONLY) {
#pragma unroll
      for (int cq = 0; cq < 4; ++cq) {
        const float4 v4 = *reinterpret_cast<const float4 *>(Slot<D>::ovec(const_cast<float *>(slot), tid, db * 4 + cq));
        o[4 * cq] = fold(o[4 * cq], w_old, v4.x, w_new);
        o[4 * cq + 1] = fold(o[4 * cq + 1], w_old, v4.y, w_new);
        o[4 * cq + 2] = fold(o[4 * cq + 2], w_old, v4.z, w_new);
        o[4 * cq + 3] = fold(o[4 * cq + 3], w_old, v4.w, w_new);
      }
    }
  }
  const float inv = 1.f / Lt;
  const int row = qt * kBQ + wave * 32 + j;
  const bool valid = row < p.Nq;
  if (!SCORE_ONLY && valid) {
    store_output_block(p, h, row, hf, db, o, inv);
    if (db == 0 && p.lse != nullptr && hf == 0) p.lse[int64_t(h) * p.Nq + row] = M * p.scale + __logf(Lt);
  }
  if (db == 0 && p.part != nullptr) {
    reduce_masses(p, lds_red, h, qt, tid, valid ? La * inv : 0.f, valid ? Lb * inv : 0.f);
    // the unit's masses are out; whoever completes the head's last merged unit sums the head
    if (tid == 0) {
      __threadfence();
      const int done = __hip_atomic_fetch_add(p.tickets + h, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (done == p.n_cut_units[h] - 1) {
        __threadfence();
        finish_score(p, h);
      }
    }
  }
}

constexpr int64_t kMaxBufferBytes = 0x7ff00000;   // one head's rows must stay below the "no tile" offset
constexpr int kMinQTile = 128;   // smallest query tile any kernel variant uses (sizes the workspace)

// Workspace layout: [score partials: H * ceil(Nq/128) * 4 floats, rounded up to 256 B]
//                   [unit counters of the merge kernel: 256 B]
//                   [hand-over flags: one 8-byte word per workgroup]
//                   [partial-result slots: 2 per workgroup, kNumCU workgroups at most]
static size_t part_bytes(int H, int Nq) {
  const size_t tiles = (size_t(Nq) + kMinQTile - 1) / kMinQTile;
  return ((size_t(H) * tiles * 4 * sizeof(float) + 255) / 256) * 256;
}
constexpr size_t kTicketBytes = 256;
static_assert(kMaxHeads * sizeof(int32_t) <= kTicketBytes, "one counter per head");
static size_t slot_bytes(int d) {
  return size_t(d == 128 ? Slot<128>::kFloats : Slot<64>::kFloats) * sizeof(float);
}
constexpr size_t kFlagBytes = kNumCU * sizeof(unsigned long long);
static size_t workspace_bytes(int H, int d, int Nq) {
  return part_bytes(H, Nq) + kTicketBytes + kFlagBytes + 2 * size_t(kNumCU) * slot_bytes(d);
}

// The decomposition of a launch (A4).  Columns = key tiles of all heads, longest head first.  Query tiles
// are taken in groups of `team_size`; the line has one position per (group, column) and is cut into
// equal spans, one per team.  A team has one workgroup per query tile of a group; its members walk the
// same columns at the same time.  team_size is chosen so that as many of the kNumCU workgroups as
// possible have a query tile in every group: when the number of query tiles does not divide the
// number of compute units, smaller teams (more groups) fill the machine better than one team member per
// query tile.
static df_status plan(AttnParams &p) {
  p.n_qtiles = (p.Nq + kBQ - 1) / kBQ;
  int64_t total = 0;
  for (int hh = 0; hh < p.H; ++hh) {
    const int h = p.order[hh];
    const int64_t len = p.hist_len[h];
    const int64_t sink = p.sink_len[h];
    p.cum[hh] = int32_t(total);
    total += (sink + kKT - 1) / kKT + (len - sink + kKT - 1) / kKT + (p.Nc + kKT - 1) / kKT;
    if (total > INT32_MAX / 2) return DF_ERR_RANGE;
  }
  p.cum[p.H] = int32_t(total);
  p.total_cols = int32_t(total);
  // busy share of the machine for a team size s: workgroups launched x tiles present in the average group
  auto teams_of = [&](int s) {
    const int64_t groups = (p.n_qtiles + s - 1) / s;
    return int64_t(std::max<int64_t>(1, std::min<int64_t>(kNumCU / s, groups * total / kMinSpan)));
  };
  auto busy = [&](int s) {
    const int64_t groups = (p.n_qtiles + s - 1) / s;
    return double(teams_of(s) * s) / kNumCU * double(p.n_qtiles) / double(groups * s);
  };
  const int s_max = std::min(p.n_qtiles, kNumCU);
  double best = 0.0;
  for (int s = 1; s <= s_max; ++s) best = std::max(best, busy(s));
  // Larger teams share every K/V tile among more workgroups while it is hot in L2, so the largest team
  // that keeps 95 % of the machine busy (or the best there is) wins.
  const double want = std::min(best, 0.95);
  int team = s_max;
  while (team > 1 && busy(team) < want) --team;
  p.team_size = team;
  p.n_groups = (p.n_qtiles + team - 1) / team;
  p.n_teams = int32_t(teams_of(team));
  p.line_len = int64_t(p.n_groups) * total;
  // units cut by a span boundary (the same walk as the merge kernel's); with hand-over none is left to it
  for (int h = 0; h < p.H; ++h) p.n_cut_units[h] = 0;
  for (int k = 1; k < p.n_teams && !p.handoff; ++k) {
    const int64_t cut = span_begin(k, p.line_len, p.n_teams);
    const int grp = int(cut / total);
    const int col = int(cut - int64_t(grp) * total);
    const int hh = head_of_column(p, col);
    if (col == p.cum[hh]) continue;
    const int64_t u_lo = int64_t(grp) * total + p.cum[hh];
    if (k >= 2 && span_begin(k - 1, p.line_len, p.n_teams) > u_lo) continue;
    p.n_cut_units[p.order[hh]] += std::min(team, p.n_qtiles - grp * team);
  }
  return DF_OK;
}

// Whether the workgroups of a launch can hand partial results to each other while it runs: every one of
// them must be on the device at the same time, i.e. the device must have a compute unit for each (one
// workgroup fills a compute unit's LDS).  DF_ATTN_HANDOVER=0 in the environment selects the two-kernel
// path regardless (a process whose queues are restricted to a subset of the compute units needs it).
static bool handover_possible(int n_wg) {
  const char *e = std::getenv("DF_ATTN_HANDOVER");   // looked at on every call
  if (e && e[0] == '0') return false;
  static std::mutex mu;
  static int cus[64] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    (void)hipGetLastError();
    return false;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (cus[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
      (void)hipGetLastError();
      n = -1;
    }
    cus[dev] = n > 0 ? n : -1;
  }
  return cus[dev] >= n_wg;
}

// A flag value that neither stale workspace contents nor an earlier launch hold: a counter run through a
// 64-bit mixer, never zero.
static unsigned long long next_epoch() {
  static std::atomic<unsigned long long> counter{0x9e3779b97f4a7c15ull ^ (unsigned long long)(uintptr_t)&counter};
  unsigned long long z = counter.fetch_add(0x9e3779b97f4a7c15ull) + 0x9e3779b97f4a7c15ull;
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  z ^= z >> 31;
  return z ? z : 1ull;
}

template <int D, bool SCORE_ONLY>
static df_status launch(AttnParams &p, void *workspace, float *score_out, hipStream_t st) {
  p.handoff = 0;
  if (df_status s = plan(p)) return s;
  if (p.n_teams > 1 && handover_possible(p.n_teams * p.team_size)) {
    p.handoff = 1;
    for (int h = 0; h < p.H; ++h) p.n_cut_units[h] = 0;
    p.epoch = next_epoch();
  }
  char *ws = static_cast<char *>(workspace);
  p.part = score_out ? reinterpret_cast<float *>(ws) : nullptr;
  p.tickets = score_out ? reinterpret_cast<int32_t *>(ws + part_bytes(p.H, p.Nq)) : nullptr;
  p.flags = reinterpret_cast<unsigned long long *>(ws + part_bytes(p.H, p.Nq) + kTicketBytes);
  p.slots = reinterpret_cast<float *>(ws + part_bytes(p.H, p.Nq) + kTicketBytes + kFlagBytes);
  p.score = score_out;
  const int n_wg = p.n_teams * p.team_size;
  const int grid = n_wg >= kXcd ? (n_wg + kXcd - 1) / kXcd * kXcd : n_wg;   // XCD-major numbering needs a multiple of 8
  hipLaunchKernelGGL((df_attn_kernel<D, SCORE_ONLY>), dim3(grid), dim3(kThreads), 0, st, p);
  if (df_status s = launch_status()) return s;
  // second launch: units cut by span boundaries (unless they were handed over), and the per-head score sums
  const int n_merge = (p.handoff ? 0 : (p.n_teams - 1) * p.team_size) + (score_out ? p.H : 0);
  if (n_merge > 0) {
    hipLaunchKernelGGL((df_attn_merge_kernel<D, SCORE_ONLY>), dim3(n_merge, (SCORE_ONLY || p.handoff) ? 1 : D / 32),
                       dim3(kThreads), 0, st, p);
    if (df_status s = launch_status()) return s;
  }
  return DF_OK;
}

// Checks shared by both entry points; fills the per-head tables of `p`.
static df_status fill_heads(AttnParams &p, int H, int d, int Nq, int Nc, const int64_t *hist_off,
                            const int32_t *sink_len, const int32_t *hist_len, bool need_sink, const void *k_hist,
                            const void *v_hist, bool need_v) {
  if (H <= 0 || Nq <= 0 || Nc <= 0) return DF_ERR_SHAPE;
  if (H > kMaxHeads || (d != 64 && d != 128)) return DF_ERR_UNSUPPORTED;
  if (!hist_off) return DF_ERR_NULL;
  if (need_sink && !sink_len) return DF_ERR_NULL;
  if (hist_off[0] != 0) return DF_ERR_RANGE;
  int64_t any = 0;
  for (int h = 0; h < H; ++h) {
    const int64_t rows = hist_off[h + 1] - hist_off[h];
    if (rows < 0 || rows * d * 2 >= kMaxBufferBytes) return DF_ERR_RANGE;
    const int64_t len = hist_len ? hist_len[h] : rows;
    if (len < 0 || len > rows) return DF_ERR_RANGE;
    const int32_t sl = sink_len ? sink_len[h] : 0;
    if (sl < 0 || sl > len) return DF_ERR_RANGE;
    p.hist_off[h] = hist_off[h];
    p.hist_len[h] = int32_t(len);
    p.sink_len[h] = sl;
    any += len;
  }
  p.hist_off[H] = hist_off[H];
  if (any > 0) {
    if (!k_hist || (need_v && !v_hist)) return DF_ERR_NULL;
    if (!aligned16(k_hist) || (need_v && !aligned16(v_hist))) return DF_ERR_ALIGN;
  }
  int idx[kMaxHeads];
  std::iota(idx, idx + H, 0);
  std::stable_sort(idx, idx + H, [&](int a, int b) { return p.hist_len[a] > p.hist_len[b]; });
  for (int h = 0; h < H; ++h) p.order[h] = uint8_t(idx[h]);
  p.H = H;
  p.Nq = Nq;
  p.Nc = Nc;
  return DF_OK;
}

}  // namespace df

using namespace df;

extern "C" size_t df_attn_workspace_bytes(int32_t H, int32_t d, int32_t Nq) {
  if (H <= 0 || Nq <= 0 || (d != 64 && d != 128)) return 0;
  return workspace_bytes(H, d, Nq);
}

extern "C" df_status df_attn_plan(int32_t H, int32_t Nq, int32_t Nc, const int32_t *hist_len,
                                  const int32_t *hist_sink_len, df_attn_plan_info *out) {
  if (!hist_len || !out) return DF_ERR_NULL;
  if (H <= 0 || Nq <= 0 || Nc <= 0) return DF_ERR_SHAPE;
  if (H > kMaxHeads) return DF_ERR_UNSUPPORTED;
  AttnParams p{};
  int idx[kMaxHeads];
  for (int h = 0; h < H; ++h) {
    const int32_t sl = hist_sink_len ? hist_sink_len[h] : 0;
    if (hist_len[h] < 0 || sl < 0 || sl > hist_len[h]) return DF_ERR_RANGE;
    p.hist_len[h] = hist_len[h];
    p.sink_len[h] = sl;
    idx[h] = h;
  }
  std::stable_sort(idx, idx + H, [&](int a, int b) { return p.hist_len[a] > p.hist_len[b]; });
  for (int h = 0; h < H; ++h) p.order[h] = uint8_t(idx[h]);
  p.H = H;
  p.Nq = Nq;
  p.Nc = Nc;
  if (df_status s = plan(p)) return s;
  out->n_qtiles = p.n_qtiles;
  out->team_size = p.team_size;
  out->n_groups = p.n_groups;
  out->n_teams = p.n_teams;
  out->workgroups = p.n_teams * p.team_size;
  out->cut_units = 0;
  for (int h = 0; h < H; ++h) out->cut_units += p.n_cut_units[h];
  out->total_cols = p.total_cols;
  out->line_len = p.line_len;
  out->span_min = INT64_MAX;
  out->span_max = 0;
  for (int t = 0; t < p.n_teams; ++t) {
    const int64_t len = span_begin(t + 1, p.line_len, p.n_teams) - span_begin(t, p.line_len, p.n_teams);
    out->span_min = std::min(out->span_min, len);
    out->span_max = std::max(out->span_max, len);
  }
  out->busy = double(out->workgroups) / kNumCU * double(p.n_qtiles) / double(int64_t(p.n_groups) * p.team_size);
  // Walk every span the way the kernel does and check what the hand-over relies on: the pieces of a span
  // tile it, the pieces of a unit are consecutive, lie in consecutive spans and cover the unit, and a span
  // holds at most one piece that leaves its sums for a later span and at most one that collects earlier ones.
  out->pieces = out->gives = out->takes = out->max_pieces_per_unit = 0;
  out->consistent = 1;
  int64_t expect_unit = -1;        // unit_lo of the unit whose next piece the walk must meet, or -1
  int expect_t = 0, unit_pieces = 0, first_span = 0;
  for (int span = 0; span < p.n_teams; ++span) {
    const int64_t lo = span_begin(span, p.line_len, p.n_teams), hi = span_begin(span + 1, p.line_len, p.n_teams);
    // the kernel walks from the end; collect, then check in line order
    std::vector<Piece> list;
    for (int64_t pos_end = hi; pos_end > lo;) {
      const Piece c = piece_ending_at(p, lo, pos_end);
      if (c.pos >= pos_end || c.pos < lo) { out->consistent = 0; break; }
      list.push_back(c);
      pos_end = c.pos;
    }
    const int n = int(list.size());
    int gives = 0, takes = 0;
    int64_t at = lo;
    for (int i = n - 1; i >= 0; --i) {
      const Piece &c = list[i];
      if (c.pos != at || c.t_begin < 0 || c.t_end > c.n_tiles || c.t_begin >= c.t_end) out->consistent = 0;
      at = c.pos + (c.t_end - c.t_begin);
      if (c.t_begin == 0) {
        if (expect_unit != -1) out->consistent = 0;          // the unit before was left unfinished
        unit_pieces = 0;
        first_span = span;
      } else if (expect_unit != c.unit_lo || expect_t != c.t_begin || i != n - 1) {
        out->consistent = 0;                                  // a continued unit is the first piece of its span
      }
      ++unit_pieces;
      if (c.t_end < c.n_tiles) {
        ++gives;
        expect_unit = c.unit_lo;
        expect_t = c.t_end;
        if (i != 0) out->consistent = 0;                      // an unfinished unit is the last piece of its span
      } else {
        expect_unit = -1;
        if (c.t_begin > 0) {
          ++takes;
          // the kernel finds the span of the unit's first piece by stepping back from its own
          int s_first = span - 1;
          while (s_first > 0 && span_begin(s_first, p.line_len, p.n_teams) > c.unit_lo) --s_first;
          if (s_first != first_span || unit_pieces != span - first_span + 1) out->consistent = 0;
        }
        out->max_pieces_per_unit = std::max(out->max_pieces_per_unit, unit_pieces);
      }
    }
    if (at != hi || gives > 1 || takes > 1) out->consistent = 0;
    out->pieces += n;
    out->gives += gives;
    out->takes += takes;
  }
  if (expect_unit != -1) out->consistent = 0;
  return DF_OK;
}

// df_attn_fwd with the workspace given separately: the caller's (df_attn_fwd) or the library's static
// scratch (df_attn_fwd_static).
static df_status attn_fwd(const df_attn_args *a, void *stream, void *workspace, size_t workspace_size) {
  if (!a) return DF_ERR_NULL;
  if (!a->q || !a->k_cur || !a->v_cur || !a->out) return DF_ERR_NULL;
  AttnParams p{};
  if (df_status s = fill_heads(p, a->H, a->d, a->Nq, a->Nc, a->hist_off, a->hist_sink_len, a->hist_len,
                               a->score_out != nullptr, a->k_hist, a->v_hist, true))
    return s;
  if (!aligned16(a->q) || !aligned16(a->k_cur) || !aligned16(a->v_cur) || !aligned16(a->out))
    return DF_ERR_ALIGN;
  const bool multi = a->H > 1;
  if (!stride_ok(a->q_stride_tok) || !stride_ok(a->kc_stride_tok) || !stride_ok(a->o_stride_tok) ||
      (multi && (!stride_ok(a->q_stride_head) || !stride_ok(a->kc_stride_head) || !stride_ok(a->o_stride_head))))
    return DF_ERR_ALIGN;
  if (!(a->softmax_scale > 0.f) || !std::isfinite(a->softmax_scale)) return DF_ERR_RANGE;
  if (!workspace || workspace_size < workspace_bytes(a->H, a->d, a->Nq)) return DF_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return DF_ERR_ALIGN;
  p.q = static_cast<const u16 *>(a->q);
  p.k_cur = static_cast<const u16 *>(a->k_cur);
  p.v_cur = static_cast<const u16 *>(a->v_cur);
  p.k_hist = static_cast<const u16 *>(a->k_hist);
  p.v_hist = static_cast<const u16 *>(a->v_hist);
  p.out = static_cast<u16 *>(a->out);
  p.lse = a->lse_out;
  p.q_st = a->q_stride_tok; p.q_sh = a->q_stride_head;
  p.kc_st = a->kc_stride_tok; p.kc_sh = a->kc_stride_head;
  p.o_st = a->o_stride_tok; p.o_sh = a->o_stride_head;
  if ((int64_t(a->Nc - 1) * a->kc_stride_tok + a->d) * 2 >= kMaxBufferBytes || a->kc_stride_tok >= (1 << 24))
    return DF_ERR_RANGE;
  p.cur_bytes = uint32_t((int64_t(a->Nc - 1) * a->kc_stride_tok + a->d) * 2);
  p.scale = a->softmax_scale;
  p.c = a->softmax_scale * 1.4426950408889634f;
  p.inv_c = 1.f / p.c;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (a->d == 128) return launch<128, false>(p, workspace, a->score_out, st);
  return launch<64, false>(p, workspace, a->score_out, st);
}

extern "C" df_status df_attn_fwd(const df_attn_args *a, void *stream) {
  if (!a) return DF_ERR_NULL;
  return attn_fwd(a, stream, a->workspace, a->workspace_bytes);
}

// ---- df_attn_fwd_static: the same call for callers that cannot allocate (see df.h) -------------------
// The workspace is a file-scope device array.  Its name is only a host-side handle: the device address
// is looked up once per device and kept, and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[DF_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, or null if the runtime cannot provide it.
void *static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" df_status df_attn_fwd_static(const df_attn_args *a, void *stream) {
  if (!a) return DF_ERR_NULL;
  // sizes first: nothing else is looked at when the launch cannot fit the static scratch
  if (a->H <= 0 || a->Nq <= 0 || a->Nc <= 0) return DF_ERR_SHAPE;
  if (a->H > kMaxHeads || (a->d != 64 && a->d != 128)) return DF_ERR_UNSUPPORTED;
  if (workspace_bytes(a->H, a->d, a->Nq) > size_t(DF_STATIC_SCRATCH_BYTES)) return DF_ERR_WORKSPACE;
  void *ws = static_scratch();
  if (!ws) return DF_ERR_LAUNCH;
  return attn_fwd(a, stream, ws, size_t(DF_STATIC_SCRATCH_BYTES));
}

extern "C" df_status df_head_score(const df_score_args *a, void *stream) {
  if (!a) return DF_ERR_NULL;
  if (!a->q || !a->k_cur || !a->score_out) return DF_ERR_NULL;
  AttnParams p{};
  if (df_status s = fill_heads(p, a->H, a->d, a->Nq, a->Nc, a->hist_off, a->hist_sink_len, a->hist_len, true,
                               a->k_hist, nullptr, false))
    return s;
  if (a->q_sample_stride < 1 || a->q_offset < 0 || a->q_offset >= a->q_sample_stride || a->q_offset >= a->Nq)
    return DF_ERR_RANGE;
  if (!aligned16(a->q) || !aligned16(a->k_cur)) return DF_ERR_ALIGN;
  const bool multi = a->H > 1;
  if (!stride_ok(a->q_stride_tok) || !stride_ok(a->kc_stride_tok) ||
      (multi && (!stride_ok(a->q_stride_head) || !stride_ok(a->kc_stride_head))))
    return DF_ERR_ALIGN;
  if (!(a->softmax_scale > 0.f) || !std::isfinite(a->softmax_scale)) return DF_ERR_RANGE;
  if (!a->workspace || a->workspace_bytes < workspace_bytes(a->H, a->d, a->Nq)) return DF_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(a->workspace) & 255u) return DF_ERR_ALIGN;
  // the sampled queries are a strided view of Q
  const int n_samp = (a->Nq - a->q_offset + a->q_sample_stride - 1) / a->q_sample_stride;
  p.q = static_cast<const u16 *>(a->q) + int64_t(a->q_offset) * a->q_stride_tok;
  p.q_st = a->q_stride_tok * a->q_sample_stride;
  p.q_sh = a->q_stride_head;
  p.Nq = n_samp;
  p.k_cur = static_cast<const u16 *>(a->k_cur);
  p.v_cur = nullptr;
  p.k_hist = static_cast<const u16 *>(a->k_hist);
  p.v_hist = nullptr;
  p.out = nullptr;
  p.lse = nullptr;
  p.kc_st = a->kc_stride_tok; p.kc_sh = a->kc_stride_head;
  if ((int64_t(a->Nc - 1) * a->kc_stride_tok + a->d) * 2 >= kMaxBufferBytes || a->kc_stride_tok >= (1 << 24))
    return DF_ERR_RANGE;
  p.cur_bytes = uint32_t((int64_t(a->Nc - 1) * a->kc_stride_tok + a->d) * 2);
  p.scale = a->softmax_scale;
  p.c = a->softmax_scale * 1.4426950408889634f;
  p.inv_c = 1.f / p.c;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (a->d == 128) return launch<128, true>(p, a->workspace, a->score_out, st);
  return launch<64, true>(p, a->workspace, a->score_out, st);
}
