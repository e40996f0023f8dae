/*
 * df.h - C ABI of the Dummy Forcing attention hot path for AMD MI355X (gfx950).
 *
 * The library computes, for one transformer layer and one chunk of query
 * frames, self-attention against a head-heterogeneous KV cache: every head
 * attends to its own slice of history (sink frames, a recent window, or
 * nothing) followed by the keys of the current chunk.  It also scores heads by
 * where their attention mass falls, classifies them, and maintains the
 * per-head sliding-window cache.
 *
 * Conventions
 *   - "DEVICE" pointers address GPU memory of the current HIP device; "HOST"
 *     pointers address ordinary process memory.  The library never allocates or
 *     frees device memory and keeps no state between calls: the caller owns
 *     every buffer, including the workspace.
 *   - Tensors are bf16 (IEEE bfloat16 bit patterns) with the head dimension d
 *     contiguous.  Strides are given in elements.  d is 64 or 128.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Device work is enqueued asynchronously; host arrays passed to a call
 *     are read (and, where stated, written) before the call returns.
 *   - Every entry point validates its arguments on the host before touching
 *     the GPU and returns a df_status; on error nothing has been launched or
 *     written.  Nothing throws and nothing aborts.
 *   - Calls that share a workspace or an output buffer must be ordered by the
 *     caller (same stream or explicit dependencies).
 */
#ifndef DF_H_
#define DF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t df_status;

enum {
  DF_OK = 0,
  DF_ERR_NULL = 1,        /* a required pointer is NULL                                  */
  DF_ERR_SHAPE = 2,       /* a size is non-positive or inconsistent                      */
  DF_ERR_UNSUPPORTED = 3, /* d not in {64,128}, H > DF_MAX_HEADS, unknown mode/type      */
  DF_ERR_ALIGN = 4,       /* a device pointer or stride breaks the 16-byte row alignment */
  DF_ERR_WORKSPACE = 5,   /* workspace missing or too small                              */
  DF_ERR_RANGE = 6,       /* offsets not monotone, length beyond capacity, N out of range*/
  DF_ERR_LAUNCH = 7       /* the HIP runtime refused the launch                          */
};

#define DF_MAX_HEADS 64

/* Head types.  FULL is the baseline window of Eq. 2 (sink + L-1 neighbour
 * frames + current); SINK, NEIGHBOR and DUMMY are the three types of Eq. 5;
 * PACK_DUMMY is the dummy head with a one-frame packing context of Eq. 8. */
enum {
  DF_HEAD_FULL = 0,
  DF_HEAD_SINK = 1,
  DF_HEAD_NEIGHBOR = 2,
  DF_HEAD_DUMMY = 3,
  DF_HEAD_PACK_DUMMY = 4
};

/* Classification modes of df_classify. */
enum {
  DF_CLASSIFY_TWO_CLASS = 0, /* Observation 1: N largest alpha^current -> DUMMY, rest FULL    */
  DF_CLASSIFY_DHP = 1        /* Eq. 6-7 greedy rule: N smallest max(F0,F1) -> DUMMY, rest
                                SINK if F0 >= F1 else NEIGHBOR                                */
};

const char *df_status_string(df_status s);

/* Visible history of one head type in tokens (Sec. 3.1, Eq. 2, Eq. 5, Eq. 8).
 * T = tokens per frame, sink_frames/window_frames = size of the cache window
 * (window_frames = L-1).  Writes *n_sink and *n_win (HOST).  Pure host code. */
df_status df_head_context(int32_t head_type, int32_t T, int32_t sink_frames,
                          int32_t window_frames, int32_t *n_sink, int32_t *n_win);

/* ------------------------------------------------------------------------
 * df_attn_fwd: out_h = softmax(scale * Q_h [K_hist_h ; K_cur_h]^T) [V_hist_h ; V_cur_h]
 * for every head h (Eq. 2 / Eq. 5 / Eq. 8, depending on what history the caller
 * packed for the head).  Every query of the chunk sees every key of the chunk
 * and all of the head's packed history; a head with no history (dummy head)
 * runs over the current chunk only and issues no history tiles.
 *
 * Optionally also returns, per head, the frame attention score of Eq. 3 under
 * the head's own visibility: the mean over all Nq queries of the attention
 * mass on (sink region, neighbour region, current chunk).
 *
 * Launches: one kernel, plus a small second one when score_out is given.  The
 * keys of a (head, query tile) unit may be split between workgroups; when the
 * device has a compute unit for every workgroup of the launch (it has on the
 * part this library is written for) the partial sums go through the workspace
 * while the kernel runs and the workgroup with a unit's last keys collects
 * them, with a bounded wait: should a workgroup never get to run
 * (compute units taken away from the process), the rows concerned come out as
 * NaN after some seconds instead of hanging the device.  DF_ATTN_HANDOVER=0 in
 * the environment (read at every call) selects the other path, in which a
 * second kernel puts those units together; the results are the same bit for bit.
 * Two calls that use the same workspace must not overlap on the device.
 *
 * Under HIP graph capture: the call records kernels only (no memset, no copy),
 * but everything the host passes by value is frozen into them - shapes,
 * strides, pointers and the per-head tables hist_off / hist_sink_len /
 * hist_len.  A captured graph therefore stays valid only while the cache state
 * it was captured in holds (same head types, same per-head lengths, same
 * buffers); the data in the buffers may change.  After df_cache_append has
 * changed a length, or df_cache_pack has re-typed the heads, capture again.
 * ---------------------------------------------------------------------- */
typedef struct df_attn_args {
  const void *q;            /* DEVICE bf16, element (u,h,c) at q[u*q_stride_tok + h*q_stride_head + c] */
  int64_t q_stride_tok, q_stride_head;
  const void *k_cur;        /* DEVICE bf16, current chunk keys, Nc tokens, same addressing scheme      */
  const void *v_cur;        /* DEVICE bf16, current chunk values (same strides as k_cur)               */
  int64_t kc_stride_tok, kc_stride_head;
  const void *k_hist;       /* DEVICE bf16 [hist_off[H], d] row-major: head h owns rows
                               [hist_off[h], hist_off[h+1]), sink-region rows first.  May be NULL
                               when hist_off[H] == 0.                                                  */
  const void *v_hist;       /* DEVICE bf16, same layout                                                */
  const int64_t *hist_off;  /* HOST [H+1], hist_off[0] == 0, non-decreasing                            */
  const int32_t *hist_sink_len; /* HOST [H] or NULL: how many of head h's history rows form the sink
                               region (0 <= . <= len_h).  Required when score_out != NULL.             */
  const int32_t *hist_len;  /* HOST [H] or NULL: len_h, the rows of head h that hold keys, counted from
                               hist_off[h] (0 <= . <= hist_off[h+1]-hist_off[h]).  NULL = all of them.
                               With it k_hist/v_hist may be the df_cache buffers themselves, read in
                               place (hist_off = head_row_off, hist_sink_len = sink_len,
                               hist_len = sink_len + win_len): a head's filled rows are a prefix of its
                               rows, and the order of the window keys does not change the result.    */
  void *out;                /* DEVICE bf16, (u,h,c) at out[u*o_stride_tok + h*o_stride_head + c]       */
  int64_t o_stride_tok, o_stride_head;
  float *lse_out;           /* DEVICE fp32 [H, Nq] natural-log sum-exp of the scaled logits, or NULL   */
  float *score_out;         /* DEVICE fp32 [H, 3] = (sink, neighbour, current) mass, or NULL           */
  int32_t H, d, Nq, Nc;     /* heads, head dim, queries, current-chunk keys (all > 0)                  */
  float softmax_scale;      /* the paper's equations omit it; pass 1/sqrt(d) for standard attention    */
  void *workspace;          /* DEVICE, required: >= df_attn_workspace_bytes(H, d, Nq) bytes, 256-byte
                               aligned.  Holds the partial results of units whose keys are split
                               between workgroups and the per-tile score sums; contents are scratch.  */
  size_t workspace_bytes;
} df_attn_args;

size_t df_attn_workspace_bytes(int32_t H, int32_t d, int32_t Nq);
df_status df_attn_fwd(const df_attn_args *args, void *stream);

/* df_attn_fwd_static: df_attn_fwd for callers that cannot allocate device memory (code under HIP graph
 * capture, serving loops and harnesses that forbid hipMalloc).  args->workspace and
 * args->workspace_bytes are ignored: the workspace is a device array of DF_STATIC_SCRATCH_BYTES bytes
 * inside the library, which every GPU the library runs on holds until the process ends.  Same
 * kernels, same results bit for bit, same validation and error codes as df_attn_fwd, plus
 * DF_ERR_WORKSPACE when df_attn_workspace_bytes(H, d, Nq) exceeds DF_STATIC_SCRATCH_BYTES (with d = 128
 * that is H * ceil(Nq / 128) > 130928, i.e. more than 261760 queries at H = 64) and DF_ERR_LAUNCH when
 * the runtime cannot give the array's address.  The call allocates nothing.  All calls on one GPU share the array: calls that
 * may overlap on one GPU (different streams, different threads) race and must be ordered by the
 * caller; nothing in it has to be cleared between calls. */
#define DF_STATIC_SCRATCH_BYTES (70u << 20)
df_status df_attn_fwd_static(const df_attn_args *args, void *stream);

/* df_attn_plan: how df_attn_fwd / df_head_score share a launch out over the GPU's 256 compute units
 * (the head-type-driven scheduling: heads differ in context length by Eq. 5 / Eq. 8, so work is cut by
 * key tiles, not by heads).  Pure host code, launches nothing; for callers and tests that want to see
 * the decomposition.  Queries are taken in tiles of 256, keys in tiles of 64 per region (sink, window,
 * current chunk); the tiles of all heads, longest head first, form a line of columns; query tiles are
 * walked in groups of team_size; the line of (group, column) positions is cut into n_teams equal spans;
 * team t's member m handles query tile group*team_size + m over span t.
 * hist_len[h] = history keys of head h (>= 0), hist_sink_len[h] = how many of them are the sink region
 * (NULL = 0).  Errors: DF_ERR_NULL, DF_ERR_SHAPE (H, Nq, Nc <= 0), DF_ERR_UNSUPPORTED (H > DF_MAX_HEADS),
 * DF_ERR_RANGE (sink > len, or more than 2^30 key tiles). */
typedef struct df_attn_plan_info {
  int32_t n_qtiles;    /* ceil(Nq / 256)                                                        */
  int32_t team_size;   /* workgroups of a team: query tiles that walk the same key tiles together */
  int32_t n_groups;    /* ceil(n_qtiles / team_size)                                            */
  int32_t n_teams;     /* spans of the line                                                     */
  int32_t workgroups;  /* n_teams * team_size, at most 256                                      */
  int32_t cut_units;   /* (head, query tile) units split by a span boundary (put together by the last
                          piece's workgroup, or by a second kernel on the two-kernel path)      */
  int64_t total_cols;  /* key tiles of all heads                                                */
  int64_t line_len;    /* n_groups * total_cols                                                 */
  int64_t span_min, span_max; /* shortest and longest span, in key tiles                        */
  double busy;         /* share of the 256 workgroup slots that hold a query tile, averaged over the line */
  /* the walk over all spans that the kernel takes, checked on the host (per member of a team): */
  int32_t pieces;      /* parts of units that the spans hold                                     */
  int32_t gives;       /* pieces that do not end their unit (their sums are left for a later span) */
  int32_t takes;       /* pieces that end a unit begun in an earlier span (they collect those sums) */
  int32_t max_pieces_per_unit;
  int32_t consistent;  /* 1 if the pieces tile every span, the pieces of every unit are consecutive, lie
                          in consecutive spans and cover it, and no span gives or takes more than once  */
} df_attn_plan_info;

df_status df_attn_plan(int32_t H, int32_t Nq, int32_t Nc, const int32_t *hist_len,
                       const int32_t *hist_sink_len, df_attn_plan_info *out);

/* ------------------------------------------------------------------------
 * df_head_score: the global frame attention score F[h] = (alpha^sink,
 * alpha^neighbour, alpha^current) of Eq. 3 for every head, estimated on the
 * uniformly strided query sample u = q_offset, q_offset + q_sample_stride, ...
 * against all keys the caller packed (Dynamic Head Programming paragraph and
 * App. C: 25% of the queries, i.e. q_sample_stride = 4).  Only QK^T and the
 * softmax statistics are computed; V is never read.  F stays on the device.
 * ---------------------------------------------------------------------- */
typedef struct df_score_args {
  const void *q;  int64_t q_stride_tok, q_stride_head;          /* DEVICE bf16, as in df_attn_args */
  const void *k_cur; int64_t kc_stride_tok, kc_stride_head;     /* DEVICE bf16                     */
  const void *k_hist;               /* DEVICE bf16 ragged history keys, as in df_attn_args          */
  const int64_t *hist_off;          /* HOST [H+1]                                                   */
  const int32_t *hist_sink_len;     /* HOST [H], required                                           */
  const int32_t *hist_len;          /* HOST [H] or NULL, as in df_attn_args                         */
  float *score_out;                 /* DEVICE fp32 [H, 3]                                           */
  int32_t H, d, Nq, Nc;
  int32_t q_sample_stride, q_offset; /* stride >= 1, 0 <= q_offset < min(stride, Nq)                */
  float softmax_scale;
  void *workspace; size_t workspace_bytes; /* >= df_attn_workspace_bytes(H, d, Nq)                  */
} df_score_args;

df_status df_head_score(const df_score_args *args, void *stream);

/* ------------------------------------------------------------------------
 * df_classify: head types from frame attention scores (pure host code).
 *   F_host        HOST fp32 [n,3] rows (sink, neighbour, current)
 *   n_dummy       how many heads must become dummy (0 <= n_dummy <= n)
 *   mode          DF_CLASSIFY_TWO_CLASS or DF_CLASSIFY_DHP
 *   type_out_host HOST [n]   receives DF_HEAD_* per head
 *   key_out_host  HOST [n] or NULL: receives the sort key (history mass F0+F1
 *                 or max(F0,F1)) in fp32
 * Heads are sorted by ascending (key, index); n may span all layers' heads.
 * ---------------------------------------------------------------------- */
df_status df_classify(const float *F_host, int32_t n, int32_t n_dummy, int32_t mode,
                      uint8_t *type_out_host, float *key_out_host);

/* ------------------------------------------------------------------------
 * Per-head sliding-window KV cache with a fixed sink (Sec. 3.1) and
 * heterogeneous memory allocation: head h owns rows
 * [head_row_off[h], head_row_off[h+1]) of the cache buffers, laid out as
 * sink_cap[h] sink rows followed by a ring of win_cap[h] window rows.  A head
 * with both capacities zero (dummy head) owns no rows.  The first sink_cap[h]
 * tokens ever appended stay in the sink region for good; the window ring
 * keeps the most recent win_cap[h] later tokens.
 * The three state arrays are HOST memory owned by the caller and updated by
 * df_kv_append; a fresh cache has them all zero.
 * ---------------------------------------------------------------------- */
typedef struct df_cache {
  void *k_cache;               /* DEVICE bf16 [head_row_off[H], d] */
  void *v_cache;               /* DEVICE bf16, same layout         */
  const int64_t *head_row_off; /* HOST [H+1], head_row_off[h+1]-head_row_off[h] >= sink_cap[h]+win_cap[h] */
  const int32_t *sink_cap;     /* HOST [H] tokens                  */
  const int32_t *win_cap;      /* HOST [H] tokens                  */
  int32_t *sink_len;           /* HOST [H] in/out: filled sink rows */
  int32_t *win_len;            /* HOST [H] in/out: valid ring rows  */
  int32_t *win_pos;            /* HOST [H] in/out: ring slot the next token goes to */
  int32_t H, d;
} df_cache;

/* df_kv_append: append the finished chunk's keys/values (Nc tokens, in
 * chronological order) to every head's cache.  Heads without capacity are
 * skipped and cost no traffic; a head whose window is smaller than the chunk
 * (PACK_DUMMY keeps one frame) stores only the chunk's last win_cap tokens. */
typedef struct df_append_args {
  const df_cache *cache;
  const void *k_new;  /* DEVICE bf16, (t,h,c) at k_new[t*stride_tok + h*stride_head + c] */
  const void *v_new;
  int64_t stride_tok, stride_head;
  int32_t Nc;
} df_append_args;

df_status df_kv_append(const df_append_args *args, void *stream);

/* df_pack_context: gather, per head, [first take_sink[h] sink tokens | most
 * recent take_win[h] window tokens, oldest first] into the contiguous ragged
 * buffers df_attn_fwd / df_head_score read (the head indexing step of the
 * Heterogeneous Memory Allocation paragraph).  Requests beyond what is cached
 * are clipped.  Writes hist_off_out[H+1] and sink_len_out[H] (HOST). */
typedef struct df_pack_args {
  const df_cache *cache;
  const int32_t *take_sink;   /* HOST [H] tokens */
  const int32_t *take_win;    /* HOST [H] tokens */
  void *k_out;                /* DEVICE bf16 [out_capacity_rows, d] */
  void *v_out;
  int64_t out_capacity_rows;
  int64_t *hist_off_out;      /* HOST [H+1] */
  int32_t *sink_len_out;      /* HOST [H]   */
} df_pack_args;

df_status df_pack_context(const df_pack_args *args, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DF_H_ */
