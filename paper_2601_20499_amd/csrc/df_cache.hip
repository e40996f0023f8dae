// df_kv_append / df_pack_context: HBM-bound row movers for the per-head
// sliding-window cache (fixed sink + ring of recent tokens, Sec. 3.1).
//
// Both entry points resolve, on the host, one small plan per head that keeps
// rows (dummy heads have none and never reach the GPU), then launch one kernel
// that moves K and V rows with 128-bit accesses: 16 lanes cover one 256-byte
// row of d=128, so every wavefront reads and writes whole contiguous rows.
#include <algorithm>

#include "df_internal.h"

namespace df {

typedef unsigned vec16 __attribute__((ext_vector_type(4)));   // one 128-bit access

// One head's share of a copy.  Logical row i in [0, n_a + n_b):
//   i <  n_a : src row a_src + i,                        dst row a_dst + i
//   i >= n_a : j = i - n_a
//     append : src row b_src + j,                        dst row ring_base + (ring_start + j) % ring_cap
//     pack   : src row ring_base + (ring_start + j) % ring_cap,  dst row b_dst + j
struct HeadPlan {
  int64_t a_src, a_dst;     // part A: straight run (sink region)
  int64_t b_lin;            // part B: linear side (source token for append, destination row for pack)
  int64_t ring_base;        // part B: first row of the head's ring
  int32_t n_a, n_b;
  int32_t ring_start, ring_cap;
  int32_t head;             // head index (selects the strided source column in append)
  int32_t pad_;
};

struct CopyParams {
  const vec16 *src_k, *src_v;
  vec16 *dst_k, *dst_v;
  int64_t src_stride_tok;   // in 16-byte units; append: token stride of k_new; pack: row stride of the cache
  int64_t src_stride_head;  // in 16-byte units; append only
  int32_t row_vec;          // 16-byte vectors per row = d / 8
  int32_t n_plans;
  HeadPlan plan[kMaxHeads];
};

constexpr int kCopyThreads = 256;
constexpr int kVecPerBlock = 512;      // 16-byte vectors per workgroup: 2 per thread, 32 rows of d = 128

// RV = 16-byte vectors per row (d / 8), a template parameter so that row/column come from shifts
template <bool APPEND, int RV>
__global__ __launch_bounds__(kCopyThreads) void df_rows_kernel(const CopyParams p) {
  const HeadPlan &pl = p.plan[blockIdx.y];
  constexpr int rv = RV;
  const int n_vec = (pl.n_a + pl.n_b) * rv;
  const int block_v0 = int(blockIdx.x) * kVecPerBlock;
  if (block_v0 >= n_vec) return;
  const int v0 = block_v0 + int(threadIdx.x);
  const vec16 *__restrict__ src = blockIdx.z ? p.src_v : p.src_k;
  vec16 *__restrict__ dst = blockIdx.z ? p.dst_v : p.dst_k;
  constexpr int kPer = kVecPerBlock / kCopyThreads;
  vec16 val[kPer];
  int64_t daddr[kPer];
#pragma unroll
  for (int it = 0; it < kPer; ++it) {
    const int v = v0 + it * kCopyThreads;
    daddr[it] = -1;
    if (v < n_vec) {
      const int i = v / rv, col = v - i * rv;
      int64_t s_row, d_row;
      if (i < pl.n_a) {
        s_row = pl.a_src + i;
        d_row = pl.a_dst + i;
      } else {
        const int j = i - pl.n_a;
        int slot = pl.ring_start + j;
        if (slot >= pl.ring_cap) slot -= pl.ring_cap;
        if (APPEND) { s_row = pl.b_lin + j; d_row = pl.ring_base + slot; }
        else        { s_row = pl.ring_base + slot; d_row = pl.b_lin + j; }
      }
      const int64_t saddr = APPEND ? s_row * p.src_stride_tok + int64_t(pl.head) * p.src_stride_head + col
                                   : s_row * int64_t(rv) + col;
      val[it] = src[saddr];
      daddr[it] = d_row * int64_t(rv) + col;
    }
  }
#pragma unroll
  for (int it = 0; it < kPer; ++it)
    // written once and not read again by this kernel: non-temporal stores leave the cache to the reads
    if (daddr[it] >= 0) __builtin_nontemporal_store(val[it], &dst[daddr[it]]);
}

static df_status check_cache(const df_cache *c) {
  if (!c) return DF_ERR_NULL;
  if (!c->head_row_off || !c->sink_cap || !c->win_cap || !c->sink_len || !c->win_len || !c->win_pos)
    return DF_ERR_NULL;
  if (c->H <= 0) return DF_ERR_SHAPE;
  if (c->H > kMaxHeads || (c->d != 64 && c->d != 128)) return DF_ERR_UNSUPPORTED;
  if (c->head_row_off[0] != 0) return DF_ERR_RANGE;
  for (int h = 0; h < c->H; ++h) {
    if (c->sink_cap[h] < 0 || c->win_cap[h] < 0) return DF_ERR_SHAPE;
    const int64_t rows = c->head_row_off[h + 1] - c->head_row_off[h];
    if (rows < 0 || rows < int64_t(c->sink_cap[h]) + c->win_cap[h]) return DF_ERR_RANGE;
    if (c->sink_len[h] < 0 || c->sink_len[h] > c->sink_cap[h]) return DF_ERR_RANGE;
    if (c->win_len[h] < 0 || c->win_len[h] > c->win_cap[h]) return DF_ERR_RANGE;
    if (c->win_pos[h] < 0 || (c->win_cap[h] > 0 ? c->win_pos[h] >= c->win_cap[h] : c->win_pos[h] != 0))
      return DF_ERR_RANGE;
  }
  if (c->head_row_off[c->H] > 0) {
    if (!c->k_cache || !c->v_cache) return DF_ERR_NULL;
    if (!aligned16(c->k_cache) || !aligned16(c->v_cache)) return DF_ERR_ALIGN;
  }
  return DF_OK;
}

}  // namespace df

using namespace df;

extern "C" df_status df_kv_append(const df_append_args *a, void *stream) {
  if (!a) return DF_ERR_NULL;
  if (df_status s = check_cache(a->cache)) return s;
  const df_cache *c = a->cache;
  if (!a->k_new || !a->v_new) return DF_ERR_NULL;
  if (a->Nc <= 0) return DF_ERR_SHAPE;
  if (!aligned16(a->k_new) || !aligned16(a->v_new) || !stride_ok(a->stride_tok) ||
      (c->H > 1 && !stride_ok(a->stride_head)))
    return DF_ERR_ALIGN;

  CopyParams p{};
  p.src_k = static_cast<const vec16 *>(a->k_new);
  p.src_v = static_cast<const vec16 *>(a->v_new);
  p.dst_k = static_cast<vec16 *>(c->k_cache);
  p.dst_v = static_cast<vec16 *>(c->v_cache);
  p.row_vec = c->d / 8;
  p.src_stride_tok = a->stride_tok / 8;
  p.src_stride_head = a->stride_head / 8;
  int32_t new_sink[kMaxHeads], new_len[kMaxHeads], new_pos[kMaxHeads];
  int max_rows = 0, np = 0;
  for (int h = 0; h < c->H; ++h) {
    const int32_t room = c->sink_cap[h] - c->sink_len[h];
    const int32_t to_sink = std::min(room, a->Nc);
    const int32_t rest = a->Nc - to_sink;                  // tokens that go to the window
    const int32_t cap = c->win_cap[h];
    const int32_t kept = std::min(rest, cap);              // only the newest `cap` of them survive
    const int32_t skipped = rest - kept;
    new_sink[h] = c->sink_len[h] + to_sink;
    new_len[h] = std::min<int64_t>(cap, int64_t(c->win_len[h]) + rest);
    // the ring advances by every window-bound token, stored or not, so that slot order stays chronological
    new_pos[h] = cap > 0 ? int32_t((int64_t(c->win_pos[h]) + rest) % cap) : 0;
    if (to_sink + kept == 0) continue;
    HeadPlan &pl = p.plan[np++];
    pl.head = h;
    pl.n_a = to_sink;
    pl.a_src = 0;
    pl.a_dst = c->head_row_off[h] + c->sink_len[h];
    pl.n_b = kept;
    pl.b_lin = to_sink + skipped;
    pl.ring_base = c->head_row_off[h] + c->sink_cap[h];
    pl.ring_cap = std::max(cap, 1);
    pl.ring_start = cap > 0 ? int32_t((int64_t(c->win_pos[h]) + skipped) % cap) : 0;
    max_rows = std::max(max_rows, to_sink + kept);
  }
  p.n_plans = np;
  if (np > 0) {
    dim3 grid((max_rows * p.row_vec + kVecPerBlock - 1) / kVecPerBlock, np, 2);
    if (p.row_vec == 16)
      hipLaunchKernelGGL((df_rows_kernel<true, 16>), grid, dim3(kCopyThreads), 0, static_cast<hipStream_t>(stream), p);
    else
      hipLaunchKernelGGL((df_rows_kernel<true, 8>), grid, dim3(kCopyThreads), 0, static_cast<hipStream_t>(stream), p);
    if (df_status s = launch_status()) return s;
  }
  for (int h = 0; h < c->H; ++h) {
    c->sink_len[h] = new_sink[h];
    c->win_len[h] = new_len[h];
    c->win_pos[h] = new_pos[h];
  }
  return DF_OK;
}

extern "C" df_status df_pack_context(const df_pack_args *a, void *stream) {
  if (!a) return DF_ERR_NULL;
  if (df_status s = check_cache(a->cache)) return s;
  const df_cache *c = a->cache;
  if (!a->take_sink || !a->take_win || !a->hist_off_out || !a->sink_len_out) return DF_ERR_NULL;
  if (a->out_capacity_rows < 0) return DF_ERR_SHAPE;

  CopyParams p{};
  p.src_k = static_cast<const vec16 *>(c->k_cache);
  p.src_v = static_cast<const vec16 *>(c->v_cache);
  p.dst_k = static_cast<vec16 *>(a->k_out);
  p.dst_v = static_cast<vec16 *>(a->v_out);
  p.row_vec = c->d / 8;
  int64_t off[kMaxHeads + 1];
  int32_t sl[kMaxHeads];
  off[0] = 0;
  int max_rows = 0, np = 0;
  for (int h = 0; h < c->H; ++h) {
    if (a->take_sink[h] < 0 || a->take_win[h] < 0) return DF_ERR_SHAPE;
    const int32_t ts = std::min(a->take_sink[h], c->sink_len[h]);
    const int32_t tw = std::min(a->take_win[h], c->win_len[h]);
    sl[h] = ts;
    off[h + 1] = off[h] + ts + tw;
    if (ts + tw == 0) continue;
    const int32_t cap = c->win_cap[h];
    HeadPlan &pl = p.plan[np++];
    pl.head = h;
    pl.n_a = ts;
    pl.a_src = c->head_row_off[h];
    pl.a_dst = off[h];
    pl.n_b = tw;
    pl.b_lin = off[h] + ts;
    pl.ring_base = c->head_row_off[h] + c->sink_cap[h];
    pl.ring_cap = std::max(cap, 1);
    pl.ring_start = cap > 0 ? int32_t(((int64_t(c->win_pos[h]) - tw) % cap + cap) % cap) : 0;
    max_rows = std::max(max_rows, ts + tw);
  }
  if (off[c->H] > a->out_capacity_rows) return DF_ERR_RANGE;
  if (off[c->H] > 0) {
    if (!a->k_out || !a->v_out) return DF_ERR_NULL;
    if (!aligned16(a->k_out) || !aligned16(a->v_out)) return DF_ERR_ALIGN;
  }
  p.n_plans = np;
  if (np > 0) {
    dim3 grid((max_rows * p.row_vec + kVecPerBlock - 1) / kVecPerBlock, np, 2);
    if (p.row_vec == 16)
      hipLaunchKernelGGL((df_rows_kernel<false, 16>), grid, dim3(kCopyThreads), 0, static_cast<hipStream_t>(stream), p);
    else
      hipLaunchKernelGGL((df_rows_kernel<false, 8>), grid, dim3(kCopyThreads), 0, static_cast<hipStream_t>(stream), p);
    if (df_status s = launch_status()) return s;
  }
  for (int h = 0; h <= c->H; ++h) a->hist_off_out[h] = off[h];
  for (int h = 0; h < c->H; ++h) a->sink_len_out[h] = sl[h];
  return DF_OK;
}
