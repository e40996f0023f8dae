// df_attn_fwd / df_head_score: varlen-per-head flash-style attention for gfx950.
//
// One workgroup (4 wavefronts of 64 lanes) owns one (head, query tile) unit and
// streams that head's visible keys - sink region, window region, current chunk,
// in this order (the concatenation order of Eq. 2) - through LDS in tiles of 64
// keys.  A dummy head has an empty history, so its units iterate the current
// chunk only: no masked tile is ever issued.  Units are launched longest head
// first so that the hardware dispatcher back-fills short (dummy) units.
//
// Per wavefront the scores are computed transposed, S^T = K Q^T, with
// v_mfma_f32_32x32x16_bf16: the K tile is the A operand (read from LDS), the
// wave's Q fragment is the B operand (held in registers for the whole unit).
// In the 32x32 accumulator layout each lane then owns ONE query (column
// lane%32) and 16 of the 32 keys of a block, so the softmax row reductions are
// in-lane except for one exchange with lane^32, and the probabilities are
// already in the register layout the second product needs as its B operand:
// O^T += V^T P^T, with V^T tiles read from LDS as the A operand.
//
// Online softmax keeps a running row maximum m and per-lane partial row sums l
// in fp32; P is rounded to bf16 (RNE) before the second product; the output is
// divided by l and rounded to bf16 once at the end.
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
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16;

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kKT = 64;      // keys per LDS tile
constexpr int kPad = 8;      // bf16 elements of row padding in LDS (16 bytes)

struct AttnParams {
  const u16 *q, *k_cur, *v_cur, *k_hist, *v_hist;
  u16 *out;
  float *lse;          // [H, Nq] or null
  float *part;         // workspace: [H, n_qtiles, 4] partial score sums, or null
  int64_t q_st, q_sh, kc_st, kc_sh, o_st, o_sh;
  int32_t Nq, Nc, H, n_qtiles;
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

// Position, inside a 32-key block, of the key whose scores land in accumulator
// row i: bits 2 and 3 of i are exchanged.  With it, accumulator registers
// 8t..8t+7 of a lane in half hf hold the 8 consecutive keys 16t+8hf .. +7,
// which is exactly the k-slice that lane feeds to the second product.
__device__ __forceinline__ int key_of_row(int i) {
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}

template <int D, int QB, bool SCORE_ONLY>
__global__ __launch_bounds__(kThreads) void df_attn_kernel(const AttnParams p) {
  constexpr int BQ = kWaves * 32 * QB;
  constexpr int KS = D / 16;           // k-steps of the first product
  constexpr int DB = D / 32;           // 32-row blocks of O^T
  constexpr int KROW = D + kPad;       // LDS row length of the K tile   [kKT][KROW]
  constexpr int VROW = kKT + kPad;     // LDS row length of the V^T tile [D][VROW]
  __shared__ __attribute__((aligned(16))) u16 lds_k[kKT * KROW];
  __shared__ __attribute__((aligned(16))) u16 lds_vt[SCORE_ONLY ? 8 : D * VROW];
  __shared__ float lds_red[BQ * 2];

  const int unit = blockIdx.x;
  const int h = p.order[unit / p.n_qtiles];
  const int qt = unit % p.n_qtiles;
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int j = lane & 31, hf = lane >> 5;
  const int q0 = qt * BQ + wave * 32 * QB;

  // ---- Q fragment: B operand of S^T = K Q^T.  Lane (j, hf) holds, for query j of each
  // 32-query block, elements 16*ks + 8*hf .. +7 of every k-step.
  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int row = q0 + 32 * qb + j;
    row = row < p.Nq ? row : p.Nq - 1;           // tail rows re-read the last query; never stored
    const u16 *src = p.q + row * p.q_st + h * p.q_sh + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[qb][ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
  }

  f32x16 o[DB][QB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[db][qb][v] = 0.f;
  float m[QB], l[QB], snap_m[2][QB], snap_l[2][QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { m[qb] = -INFINITY; l[qb] = 0.f; }

  const int64_t hoff = p.hist_off[h];
  const int len_h = int(p.hist_off[h + 1] - hoff);
  const int sink = p.sink_len[h];

#pragma unroll 1
  for (int seg = 0; seg < 3; ++seg) {
    // segment = (base pointers, row stride, number of keys)
    const u16 *kbase, *vbase;
    int64_t rstride;
    int n_keys;
    if (seg == 0)      { kbase = p.k_hist + hoff * D;          vbase = p.v_hist + hoff * D;          rstride = D; n_keys = sink; }
    else if (seg == 1) { kbase = p.k_hist + (hoff + sink) * D; vbase = p.v_hist + (hoff + sink) * D; rstride = D; n_keys = len_h - sink; }
    else               { kbase = p.k_cur + h * p.kc_sh;        vbase = p.v_cur + h * p.kc_sh;        rstride = p.kc_st; n_keys = p.Nc; }

#pragma unroll 1
    for (int k0 = 0; k0 < n_keys; k0 += kKT) {
      const int n_valid = min(kKT, n_keys - k0);
      __syncthreads();                             // previous tile fully consumed
      // ---- stage the K tile (row-major) and the V tile (transposed) in LDS
      {
        constexpr int VEC_PER_ROW = D / 8;
        constexpr int ROWS_PER_PASS = kThreads / VEC_PER_ROW;
        const int cv = tid % VEC_PER_ROW, r0 = tid / VEC_PER_ROW;
#pragma unroll
        for (int r = r0; r < kKT; r += ROWS_PER_PASS) {
          uint4 kv = {0u, 0u, 0u, 0u}, vv = {0u, 0u, 0u, 0u};
          if (r < n_valid) {
            kv = *reinterpret_cast<const uint4 *>(kbase + (k0 + r) * rstride + 8 * cv);
            if (!SCORE_ONLY) vv = *reinterpret_cast<const uint4 *>(vbase + (k0 + r) * rstride + 8 * cv);
          }
          *reinterpret_cast<uint4 *>(&lds_k[r * KROW + 8 * cv]) = kv;
          if (!SCORE_ONLY) {
            const unsigned w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              lds_vt[(8 * cv + 2 * e) * VROW + r] = u16(w[e] & 0xffffu);
              lds_vt[(8 * cv + 2 * e + 1) * VROW + r] = u16(w[e] >> 16);
            }
          }
        }
      }
      __syncthreads();

      // ---- S^T = K Q^T for 2 key blocks x QB query blocks
      f32x16 s[2][QB];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int v = 0; v < 16; ++v) s[kb][qb][v] = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const u16 *arow = &lds_k[(32 * kb + key_of_row(j)) * KROW + 8 * hf];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 a = *reinterpret_cast<const bf16x8 *>(arow + 16 * ks);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            s[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][ks], s[kb][qb], 0, 0, 0);
        }
      }
      // ---- mask the keys past the end of the segment (last tile only)
      if (n_valid < kKT) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = 32 * kb + 16 * (v >> 3) + 8 * hf + (v & 7);
            if (key >= n_valid) {
#pragma unroll
              for (int qb = 0; qb < QB; ++qb) s[kb][qb][v] = -INFINITY;
            }
          }
      }
      // ---- online softmax, one query per lane pair (lane, lane^32)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float mx = s[0][qb][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][qb][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m[qb], mx);
        const float alpha = fast_exp2((m[qb] - m_new) * p.c);
        const float nmc = -m_new * p.c;
        m[qb] = m_new;
        float rs = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float e = fast_exp2(__builtin_fmaf(s[kb][qb][v], p.c, nmc));
            s[kb][qb][v] = e;
            rs += e;
          }
        l[qb] = l[qb] * alpha + rs;
        if (!SCORE_ONLY) {
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][qb][v] *= alpha;
        }
      }
      // ---- O^T += V^T P^T
      if (!SCORE_ONLY) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            bf16x8 pb[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
              unsigned w[4];
#pragma unroll
              for (int e = 0; e < 4; ++e)
                w[e] = pack_bf16x2(s[kb][qb][8 * t + 2 * e], s[kb][qb][8 * t + 2 * e + 1]);
              uint4 u = {w[0], w[1], w[2], w[3]};
              pb[qb] = __builtin_bit_cast(bf16x8, u);
            }
#pragma unroll
            for (int db = 0; db < DB; ++db) {
              const bf16x8 a = *reinterpret_cast<const bf16x8 *>(
                  &lds_vt[(32 * db + j) * VROW + 32 * kb + 16 * t + 8 * hf]);
#pragma unroll
              for (int qb = 0; qb < QB; ++qb)
                o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb], o[db][qb], 0, 0, 0);
            }
          }
      }
    }
    if (seg < 2) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) { snap_m[seg][qb] = m[qb]; snap_l[seg][qb] = l[qb]; }
    }
  }

  // ---- epilogue: normalise, store, optional lse and score partials
  float mass_a[QB], mass_b[QB];     // row mass on sink, on sink+window
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float lt = l[qb] + __shfl_xor(l[qb], 32, 64);
    const float inv = 1.f / lt;
    const int row = q0 + 32 * qb + j;
    const bool valid = row < p.Nq;
    float l1 = snap_l[0][qb] * fast_exp2((snap_m[0][qb] - m[qb]) * p.c);
    float l2 = snap_l[1][qb] * fast_exp2((snap_m[1][qb] - m[qb]) * p.c);
    l1 += __shfl_xor(l1, 32, 64);
    l2 += __shfl_xor(l2, 32, 64);
    mass_a[qb] = valid ? l1 * inv : 0.f;
    mass_b[qb] = valid ? l2 * inv : 0.f;
    if (!SCORE_ONLY && valid) {
      u16 *dst = p.out + row * p.o_st + h * p.o_sh + 4 * hf;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int cq = 0; cq < 4; ++cq) {
          uint2 w;
          w.x = pack_bf16x2(o[db][qb][4 * cq] * inv, o[db][qb][4 * cq + 1] * inv);
          w.y = pack_bf16x2(o[db][qb][4 * cq + 2] * inv, o[db][qb][4 * cq + 3] * inv);
          *reinterpret_cast<uint2 *>(dst + 32 * db + 8 * cq) = w;
        }
      if (p.lse != nullptr && hf == 0)
        p.lse[int64_t(h) * p.Nq + row] = m[qb] * p.scale + __logf(lt);
    }
  }
  if (p.part != nullptr) {
    // deterministic block reduction: one slot per query, summed in index order by two threads
    if (hf == 0) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const int qi = wave * 32 * QB + 32 * qb + j;
        lds_red[2 * qi] = mass_a[qb];
        lds_red[2 * qi + 1] = mass_b[qb];
      }
    }
    __syncthreads();
    if (tid < 2) {
      float acc = 0.f;
      for (int qi = 0; qi < BQ; ++qi) acc += lds_red[2 * qi + tid];
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

template <int D, int QB, bool SCORE_ONLY>
static df_status launch(AttnParams &p, float *score_out, hipStream_t st) {
  constexpr int BQ = kWaves * 32 * QB;
  p.n_qtiles = (p.Nq + BQ - 1) / BQ;
  dim3 grid(p.n_qtiles * p.H);
  hipLaunchKernelGGL((df_attn_kernel<D, QB, SCORE_ONLY>), grid, dim3(kThreads), 0, st, p);
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
  if (a->d == 128) return launch<128, 1, false>(p, a->score_out, st);
  return launch<64, 1, false>(p, a->score_out, st);
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
  if (a->d == 128) return launch<128, 1, true>(p, a->score_out, st);
  return launch<64, 1, true>(p, a->score_out, st);
}
