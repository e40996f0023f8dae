// df_attn_fwd / df_head_score: varlen-per-head flash-style attention for gfx950.
//
// Work decomposition.  One workgroup of 8 wavefronts owns one (head, 256-query
// tile) unit; each wavefront owns 32 queries and streams the head's visible
// keys - sink region, window region, current chunk, in this order (the
// concatenation order of Eq. 2) - in tiles of 64 keys.  A dummy head has an
// empty history, so its units iterate the current chunk only: no masked tile
// is ever issued.  Units are ordered longest head first and laid out so that
// the workgroups of one XCD (workgroup id mod 8) work on neighbouring query
// tiles of the same head and share its K/V tiles in that XCD's L2.
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
// t, LDS stores of the staged tile, global loads of a later tile), separated
// by workgroup barriers.  Group 1 starts one barrier late, so on every SIMD one
// wave is in its MFMA phase while the other is in its VALU phase: the matrix
// core and the vector ALU overlap without relying on instruction scheduling.
// K and V tiles rotate through three LDS buffers each; with the one-phase
// stagger a buffer is rewritten only after both groups have finished reading it.
//
// Online softmax keeps a running row maximum m and per-lane partial row sums
// l in fp32.  The maximum is only raised (and O, l rescaled) when some row of
// the wave exceeds it by more than 2^8, which keeps P within bf16/fp32 range
// and makes rescaling rare; P is rounded to bf16 (RNE) before the second
// product; l sums the fp32 values.  The output is divided by l and
// rounded to bf16 once at the end.
//
// The frame attention score of Eq. 3 falls out of the same statistics: with the
// keys ordered sink | window | current, snapshots (m1,l1) after the sink region
// and (m2,l2) after the window region give a row's region masses as
// l1*2^(m1-m3)/l3, (l2*2^(m2-m3) - l1*2^(m1-m3))/l3 and the remainder.
#include <algorithm>
#include <cmath>
#include <numeric>

#include "df_internal.h"

namespace df {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16;

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kBQ = kWaves * 32;   // queries per workgroup
constexpr int kKT = 64;            // keys per LDS tile
constexpr int kNBuf = 3;           // LDS buffers per operand
constexpr float kRescaleLog2 = 8.f;  // raise the running maximum only beyond this many powers of two
constexpr int kXcd = 8;            // XCDs per device: consecutive workgroup ids go to consecutive XCDs

struct AttnParams {
  const u16 *q, *k_cur, *v_cur, *k_hist, *v_hist;
  u16 *out;
  float *lse;          // [H, Nq] or null
  float *part;         // workspace: [H, n_qtiles, 4] partial score sums, or null
  int64_t q_st, q_sh, kc_st, kc_sh, o_st, o_sh;
  int32_t Nq, Nc, H, n_qtiles, n_units, units_per_xcd;
  float c;             // softmax_scale * log2(e)
  float scale;         // softmax_scale
  int64_t hist_off[kMaxHeads + 1];
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

// One key tile of a head: where its rows live and how many of the 64 are real.
struct Tile {
  const u16 *k, *v;
  int64_t stride;
  int n_valid;
};

template <int D, bool SCORE_ONLY>
__global__ __launch_bounds__(kThreads) void df_attn_kernel(const AttnParams p) {
  constexpr int KS = D / 16;            // k-steps of the first product
  constexpr int DB = D / 32;            // 32-row blocks of O^T
  constexpr int KROW = D + 8;           // K tile row, +16 B: conflict-free ds_read_b128 of 32 rows
  constexpr int VROW = D + 32;          // V tile row, +64 B: conflict-free ds_read_b64_tr_b16
  constexpr int KTILE = kKT * KROW, VTILE = kKT * VROW;
  constexpr int VEC_PER_ROW = D / 8;    // 16-byte vectors per row
  constexpr int ROWS_PER_PASS = kThreads / VEC_PER_ROW;
  constexpr int NPASS = kKT / ROWS_PER_PASS;   // 2 for D=128, 1 for D=64
  __shared__ __attribute__((aligned(16))) u16 lds_k[kNBuf * KTILE];
  __shared__ __attribute__((aligned(16))) u16 lds_v[SCORE_ONLY ? 8 : kNBuf * VTILE];
  __shared__ float lds_red[kBQ * 2];

  // ---- which unit: XCD x (= workgroup id mod 8) takes logical units [x*upx, (x+1)*upx)
  const int logical = (blockIdx.x % kXcd) * p.units_per_xcd + blockIdx.x / kXcd;
  if (logical >= p.n_units) return;
  const int h = p.order[logical / p.n_qtiles];
  const int qt = logical % p.n_qtiles;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int group = wave >> 2;
  const int j = lane & 31, hf = lane >> 5;
  const int q0 = qt * kBQ + wave * 32;

  // ---- tiles of this head: three segments, each cut into 64-key tiles
  const int64_t hoff = p.hist_off[h];
  const int len_h = int(p.hist_off[h + 1] - hoff);
  const int sink = p.sink_len[h];
  const int nt0 = (sink + kKT - 1) / kKT;
  const int nt1 = (len_h - sink + kKT - 1) / kKT;
  const int nt2 = (p.Nc + kKT - 1) / kKT;
  const int n_tiles = nt0 + nt1 + nt2;
  auto tile_at = [&](int t) -> Tile {
    Tile r;
    if (t < nt0) {
      const int k0 = t * kKT;
      r.k = p.k_hist + (hoff + k0) * D; r.v = p.v_hist + (hoff + k0) * D; r.stride = D; r.n_valid = min(kKT, sink - k0);
    } else if (t < nt0 + nt1) {
      const int k0 = (t - nt0) * kKT;
      r.k = p.k_hist + (hoff + sink + k0) * D; r.v = p.v_hist + (hoff + sink + k0) * D; r.stride = D;
      r.n_valid = min(kKT, len_h - sink - k0);
    } else {
      const int k0 = (t - nt0 - nt1) * kKT;
      r.k = p.k_cur + h * p.kc_sh + k0 * p.kc_st; r.v = p.v_cur + h * p.kc_sh + k0 * p.kc_st; r.stride = p.kc_st;
      r.n_valid = min(kKT, p.Nc - k0);
    }
    return r;
  };

  // ---- global -> register -> LDS staging of one tile (rows past n_valid are zero-filled)
  const int st_col = tid % VEC_PER_ROW, st_row = tid / VEC_PER_ROW;
  auto load_tile = [&](const u16 *base, int64_t stride, int n_valid, u32x4 (&reg)[NPASS]) {
#pragma unroll
    for (int i = 0; i < NPASS; ++i) {
      const int r = st_row + i * ROWS_PER_PASS;
      u32x4 z = {0u, 0u, 0u, 0u};
      reg[i] = z;
      if (r < n_valid) reg[i] = *reinterpret_cast<const u32x4 *>(base + r * stride + 8 * st_col);
    }
  };
  auto store_tile = [&](u16 *lds, int row_len, const u32x4 (&reg)[NPASS]) {
#pragma unroll
    for (int i = 0; i < NPASS; ++i) {
      const int r = st_row + i * ROWS_PER_PASS;
      *reinterpret_cast<u32x4 *>(lds + r * row_len + 8 * st_col) = reg[i];
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

  // ---- prologue: K(0), V(0), K(1) into LDS; K(2) and V(1) staged in registers
  u32x4 kreg[NPASS], vreg[NPASS];
  {
    Tile t0 = tile_at(0);
    load_tile(t0.k, t0.stride, t0.n_valid, kreg);
    store_tile(lds_k, KROW, kreg);
    if (!SCORE_ONLY) {
      load_tile(t0.v, t0.stride, t0.n_valid, vreg);
      store_tile(lds_v, VROW, vreg);
    }
    if (n_tiles > 1) {
      Tile t1 = tile_at(1);
      load_tile(t1.k, t1.stride, t1.n_valid, kreg);
      store_tile(lds_k + KTILE, KROW, kreg);
      if (!SCORE_ONLY) load_tile(t1.v, t1.stride, t1.n_valid, vreg);
    }
    if (n_tiles > 2) {
      Tile t2 = tile_at(2);
      load_tile(t2.k, t2.stride, t2.n_valid, kreg);
    }
  }
  lds_barrier();
  if (group == 1) lds_barrier();          // stagger: group 1 runs one phase behind group 0

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  float m = -INFINITY, l = 0.f;
  float snap_m0 = -INFINITY, snap_l0 = 0.f, snap_m1 = -INFINITY, snap_l1 = 0.f;
  f32x16 s[2];
  bf16x8 pb[2][2];                         // P^T of the previous tile, [key block][16-key step]

  // per-lane LDS offsets (elements) of the MFMA A operands
  const int a_k = key_of_row(j) * KROW + 8 * hf;
  const int g16 = lane >> 4, i16 = lane & 15;
  const int a_v = (8 * (g16 >> 1) + (i16 >> 2)) * VROW + 16 * (g16 & 1) + 4 * (i16 & 3);

#pragma unroll 1
  for (int t = 0; t <= n_tiles; ++t) {
    // ================= MFMA phase =================
    if (t < n_tiles) {
      const u16 *kt = lds_k + (t % kNBuf) * KTILE + a_k;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kt + 32 * kb * KROW + 16 * ks);
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb], 0, 0, 0);
        }
    }
    if (!SCORE_ONLY && t > 0) {
      const u16 *vt = lds_v + ((t - 1) % kNBuf) * VTILE + a_v;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int ts = 0; ts < 2; ++ts)
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const u16 *src = vt + (32 * kb + 16 * ts) * VROW + 32 * db;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3))) *)(src));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3))) *)(src + 4 * VROW));
            const short a8 __attribute__((ext_vector_type(8))) = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a8), pb[kb][ts], o[db], 0, 0, 0);
          }
    }
    lds_barrier();
    // ================= VALU / memory phase =================
    // staged tiles K(t+2), V(t+1) -> LDS; then fetch K(t+3), V(t+2)
    if (t + 2 < n_tiles) store_tile(lds_k + ((t + 2) % kNBuf) * KTILE, KROW, kreg);
    if (!SCORE_ONLY && t + 1 < n_tiles) store_tile(lds_v + ((t + 1) % kNBuf) * VTILE, VROW, vreg);
    if (t + 3 < n_tiles) {
      Tile nx = tile_at(t + 3);
      load_tile(nx.k, nx.stride, nx.n_valid, kreg);
    }
    if (!SCORE_ONLY && t + 2 < n_tiles) {
      Tile nx = tile_at(t + 2);
      load_tile(nx.v, nx.stride, nx.n_valid, vreg);
    }
    if (t < n_tiles) {
      const int seg_end0 = nt0 - 1, seg_end1 = nt0 + nt1 - 1;
      int n_valid = kKT;
      if (t == seg_end0) n_valid = sink - (nt0 - 1) * kKT;
      else if (t == seg_end1) n_valid = len_h - sink - (nt1 - 1) * kKT;
      else if (t == n_tiles - 1) n_valid = p.Nc - (nt2 - 1) * kKT;
      if (n_valid < kKT) {                  // keys past the end of the segment
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = 32 * kb + 16 * (v >> 3) + 8 * hf + (v & 7);
            if (key >= n_valid) s[kb][v] = -INFINITY;
          }
      }
      float mx = s[0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
      mx = pair_max(mx);
      // raise the running maximum only when some row of the wave outgrew it by 2^kRescaleLog2
      if (__any((mx - m) * p.c > kRescaleLog2)) {
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2((m - m_new) * p.c);
        m = m_new;
        l *= alpha;
        if (!SCORE_ONLY) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
        }
      }
      const float nmc = -m * p.c;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) {
          unsigned w[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float e0 = fast_exp2(__builtin_fmaf(s[kb][8 * ts + 2 * e], p.c, nmc));
            const float e1 = fast_exp2(__builtin_fmaf(s[kb][8 * ts + 2 * e + 1], p.c, nmc));
            w[e] = pack_bf16x2(e0, e1);
            l += e0 + e1;
          }
          u32x4 u = {w[0], w[1], w[2], w[3]};
          pb[kb][ts] = __builtin_bit_cast(bf16x8, u);
        }
      if (t == seg_end0) { snap_m0 = m; snap_l0 = l; }
      if (t == seg_end1) { snap_m1 = m; snap_l1 = l; }
    }
    lds_barrier();
  }
  if (group == 0) lds_barrier();          // matches group 1's extra barrier at the start
  if (nt0 == 0) { snap_m0 = -INFINITY; snap_l0 = 0.f; }
  if (nt1 == 0) { snap_m1 = snap_m0; snap_l1 = snap_l0; }

  // ---- epilogue: normalise, store, optional lse and score partials
  const float lt = pair_sum(l);
  const float inv = 1.f / lt;
  const int row = q0 + j;
  const bool valid = row < p.Nq;
  const float l1 = pair_sum(snap_l0 * fast_exp2((snap_m0 - m) * p.c));
  const float l2 = pair_sum(snap_l1 * fast_exp2((snap_m1 - m) * p.c));
  const float mass_a = valid ? l1 * inv : 0.f;     // row mass on the sink region
  const float mass_b = valid ? l2 * inv : 0.f;     // row mass on sink + window
  if (!SCORE_ONLY && valid) {
    u16 *dst = p.out + row * p.o_st + h * p.o_sh + 4 * hf;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int cq = 0; cq < 4; ++cq) {
        uint2 w;
        w.x = pack_bf16x2(o[db][4 * cq] * inv, o[db][4 * cq + 1] * inv);
        w.y = pack_bf16x2(o[db][4 * cq + 2] * inv, o[db][4 * cq + 3] * inv);
        *reinterpret_cast<uint2 *>(dst + 32 * db + 8 * cq) = w;
      }
    if (p.lse != nullptr && hf == 0) p.lse[int64_t(h) * p.Nq + row] = m * p.scale + __logf(lt);
  }
  if (p.part != nullptr) {
    // deterministic block reduction: one slot per query, summed in index order by two threads
    if (hf == 0) {
      lds_red[2 * (wave * 32 + j)] = mass_a;
      lds_red[2 * (wave * 32 + j) + 1] = mass_b;
    }
    __syncthreads();
    if (tid < 2) {
      float acc = 0.f;
      for (int qi = 0; qi < kBQ; ++qi) acc += lds_red[2 * qi + tid];
      p.part[(int64_t(h) * p.n_qtiles + qt) * 4 + tid] = acc;
    }
  }
}

// F[h] = (sum_a, sum_b - sum_a, n - sum_b) / n over the head's query tiles, in tile order.
__global__ void df_score_finish_kernel(const float *part, float *score, int n_qtiles, int n_rows) {
  const int h = blockIdx.x;
  if (threadIdx.x != 0) return;
  float a = 0.f, b = 0.f;
  for (int t = 0; t < n_qtiles; ++t) {
    a += part[(int64_t(h) * n_qtiles + t) * 4];
    b += part[(int64_t(h) * n_qtiles + t) * 4 + 1];
  }
  const float inv = 1.f / float(n_rows);
  score[3 * h] = a * inv;
  score[3 * h + 1] = (b - a) * inv;
  score[3 * h + 2] = (float(n_rows) - b) * inv;
}

constexpr int kMinQTile = 128;   // smallest query tile any kernel variant uses (sizes the workspace)

static size_t workspace_bytes(int H, int Nq) {
  const size_t tiles = (size_t(Nq) + kMinQTile - 1) / kMinQTile;
  return ((size_t(H) * tiles * 4 * sizeof(float) + 255) / 256) * 256 + 256;
}

template <int D, bool SCORE_ONLY>
static df_status launch(AttnParams &p, float *score_out, hipStream_t st) {
  p.n_qtiles = (p.Nq + kBQ - 1) / kBQ;
  p.n_units = p.n_qtiles * p.H;
  p.units_per_xcd = (p.n_units + kXcd - 1) / kXcd;
  dim3 grid(p.units_per_xcd * kXcd);
  hipLaunchKernelGGL((df_attn_kernel<D, SCORE_ONLY>), grid, dim3(kThreads), 0, st, p);
  if (df_status s = launch_status()) return s;
  if (score_out) {
    hipLaunchKernelGGL(df_score_finish_kernel, dim3(p.H), dim3(64), 0, st, p.part, score_out, p.n_qtiles, p.Nq);
    if (df_status s = launch_status()) return s;
  }
  return DF_OK;
}

// Checks shared by both entry points; fills the per-head tables of `p`.
static df_status fill_heads(AttnParams &p, int H, int d, int Nq, int Nc, const int64_t *hist_off,
                            const int32_t *sink_len, bool need_sink, const void *k_hist, const void *v_hist,
                            bool need_v) {
  if (H <= 0 || Nq <= 0 || Nc <= 0) return DF_ERR_SHAPE;
  if (H > kMaxHeads || (d != 64 && d != 128)) return DF_ERR_UNSUPPORTED;
  if (!hist_off) return DF_ERR_NULL;
  if (need_sink && !sink_len) return DF_ERR_NULL;
  if (hist_off[0] != 0) return DF_ERR_RANGE;
  for (int h = 0; h < H; ++h) {
    const int64_t len = hist_off[h + 1] - hist_off[h];
    if (len < 0 || len > INT32_MAX) return DF_ERR_RANGE;
    const int32_t sl = sink_len ? sink_len[h] : 0;
    if (sl < 0 || sl > len) return DF_ERR_RANGE;
    p.hist_off[h] = hist_off[h];
    p.sink_len[h] = sl;
  }
  p.hist_off[H] = hist_off[H];
  if (hist_off[H] > 0) {
    if (!k_hist || (need_v && !v_hist)) return DF_ERR_NULL;
    if (!aligned16(k_hist) || (need_v && !aligned16(v_hist))) return DF_ERR_ALIGN;
  }
  int idx[kMaxHeads];
  std::iota(idx, idx + H, 0);
  std::stable_sort(idx, idx + H, [&](int a, int b) {
    return hist_off[a + 1] - hist_off[a] > hist_off[b + 1] - hist_off[b];
  });
  for (int h = 0; h < H; ++h) p.order[h] = uint8_t(idx[h]);
  p.H = H;
  p.Nq = Nq;
  p.Nc = Nc;
  return DF_OK;
}

}  // namespace df

using namespace df;

extern "C" size_t df_attn_workspace_bytes(int32_t H, int32_t d, int32_t Nq) {
  (void)d;
  if (H <= 0 || Nq <= 0) return 0;
  return workspace_bytes(H, Nq);
}

extern "C" df_status df_attn_fwd(const df_attn_args *a, void *stream) {
  if (!a) return DF_ERR_NULL;
  if (!a->q || !a->k_cur || !a->v_cur || !a->out) return DF_ERR_NULL;
  AttnParams p{};
  if (df_status s = fill_heads(p, a->H, a->d, a->Nq, a->Nc, a->hist_off, a->hist_sink_len,
                               a->score_out != nullptr, a->k_hist, a->v_hist, true))
    return s;
  if (!aligned16(a->q) || !aligned16(a->k_cur) || !aligned16(a->v_cur) || !aligned16(a->out))
    return DF_ERR_ALIGN;
  const bool multi = a->H > 1;
  if (!stride_ok(a->q_stride_tok) || !stride_ok(a->kc_stride_tok) || !stride_ok(a->o_stride_tok) ||
      (multi && (!stride_ok(a->q_stride_head) || !stride_ok(a->kc_stride_head) || !stride_ok(a->o_stride_head))))
    return DF_ERR_ALIGN;
  if (!(a->softmax_scale > 0.f) || !std::isfinite(a->softmax_scale)) return DF_ERR_RANGE;
  if (a->score_out) {
    if (!a->workspace) return DF_ERR_WORKSPACE;
    if (a->workspace_bytes < workspace_bytes(a->H, a->Nq)) return DF_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(a->workspace) & 255u) return DF_ERR_ALIGN;
  }
  p.q = static_cast<const u16 *>(a->q);
  p.k_cur = static_cast<const u16 *>(a->k_cur);
  p.v_cur = static_cast<const u16 *>(a->v_cur);
  p.k_hist = static_cast<const u16 *>(a->k_hist);
  p.v_hist = static_cast<const u16 *>(a->v_hist);
  p.out = static_cast<u16 *>(a->out);
  p.lse = a->lse_out;
  p.part = a->score_out ? static_cast<float *>(a->workspace) : nullptr;
  p.q_st = a->q_stride_tok; p.q_sh = a->q_stride_head;
  p.kc_st = a->kc_stride_tok; p.kc_sh = a->kc_stride_head;
  p.o_st = a->o_stride_tok; p.o_sh = a->o_stride_head;
  p.scale = a->softmax_scale;
  p.c = a->softmax_scale * 1.4426950408889634f;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (a->d == 128) return launch<128, false>(p, a->score_out, st);
  return launch<64, false>(p, a->score_out, st);
}

extern "C" df_status df_head_score(const df_score_args *a, void *stream) {
  if (!a) return DF_ERR_NULL;
  if (!a->q || !a->k_cur || !a->score_out) return DF_ERR_NULL;
  AttnParams p{};
  if (df_status s = fill_heads(p, a->H, a->d, a->Nq, a->Nc, a->hist_off, a->hist_sink_len, true,
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
  if (!a->workspace || a->workspace_bytes < workspace_bytes(a->H, a->Nq)) return DF_ERR_WORKSPACE;
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
  p.part = static_cast<float *>(a->workspace);
  p.kc_st = a->kc_stride_tok; p.kc_sh = a->kc_stride_head;
  p.scale = a->softmax_scale;
  p.c = a->softmax_scale * 1.4426950408889634f;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (a->d == 128) return launch<128, true>(p, a->score_out, st);
  return launch<64, true>(p, a->score_out, st);
}
