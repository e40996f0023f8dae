"""ctypes binding of include/df.h: argument marshalling only.

Every function here has the name of the C entry point it calls and does no
arithmetic of its own: tensors are passed as raw device pointers plus sizes,
host bookkeeping arrays as ctypes arrays.  There is no CPU fallback: if the
HIP library is missing the import of this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

PKG = os.path.dirname(os.path.abspath(__file__))
# DF_HIP_LIBRARY names another build of the same sources (the host-sanitizer build of the tests)
LIB_PATH = os.environ.get("DF_HIP_LIBRARY") or os.path.join(PKG, "libdf_hip.so")

DF_OK = 0
(DF_ERR_NULL, DF_ERR_SHAPE, DF_ERR_UNSUPPORTED, DF_ERR_ALIGN, DF_ERR_WORKSPACE, DF_ERR_RANGE,
 DF_ERR_LAUNCH) = range(1, 8)
DF_MAX_HEADS = 64
DF_HEAD_FULL, DF_HEAD_SINK, DF_HEAD_NEIGHBOR, DF_HEAD_DUMMY, DF_HEAD_PACK_DUMMY = range(5)
DF_CLASSIFY_TWO_CLASS, DF_CLASSIFY_DHP = 0, 1

EXPORTS = ["df_status_string", "df_head_context", "df_attn_workspace_bytes", "df_attn_fwd", "df_attn_fwd_static", "df_attn_plan",
           "df_head_score", "df_classify", "df_kv_append", "df_pack_context"]


class DfError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


class df_attn_args(C.Structure):
    _fields_ = [("q", C.c_void_p), ("q_stride_tok", C.c_int64), ("q_stride_head", C.c_int64),
                ("k_cur", C.c_void_p), ("v_cur", C.c_void_p),
                ("kc_stride_tok", C.c_int64), ("kc_stride_head", C.c_int64),
                ("k_hist", C.c_void_p), ("v_hist", C.c_void_p),
                ("hist_off", C.POINTER(C.c_int64)), ("hist_sink_len", C.POINTER(C.c_int32)),
                ("hist_len", C.POINTER(C.c_int32)),
                ("out", C.c_void_p), ("o_stride_tok", C.c_int64), ("o_stride_head", C.c_int64),
                ("lse_out", C.c_void_p), ("score_out", C.c_void_p),
                ("H", C.c_int32), ("d", C.c_int32), ("Nq", C.c_int32), ("Nc", C.c_int32),
                ("softmax_scale", C.c_float),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class df_score_args(C.Structure):
    _fields_ = [("q", C.c_void_p), ("q_stride_tok", C.c_int64), ("q_stride_head", C.c_int64),
                ("k_cur", C.c_void_p), ("kc_stride_tok", C.c_int64), ("kc_stride_head", C.c_int64),
                ("k_hist", C.c_void_p),
                ("hist_off", C.POINTER(C.c_int64)), ("hist_sink_len", C.POINTER(C.c_int32)),
                ("hist_len", C.POINTER(C.c_int32)),
                ("score_out", C.c_void_p),
                ("H", C.c_int32), ("d", C.c_int32), ("Nq", C.c_int32), ("Nc", C.c_int32),
                ("q_sample_stride", C.c_int32), ("q_offset", C.c_int32),
                ("softmax_scale", C.c_float),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class df_attn_plan_info(C.Structure):
    _fields_ = [("n_qtiles", C.c_int32), ("team_size", C.c_int32), ("n_groups", C.c_int32), ("n_teams", C.c_int32),
                ("workgroups", C.c_int32), ("cut_units", C.c_int32),
                ("total_cols", C.c_int64), ("line_len", C.c_int64), ("span_min", C.c_int64), ("span_max", C.c_int64),
                ("busy", C.c_double),
                ("pieces", C.c_int32), ("gives", C.c_int32), ("takes", C.c_int32), ("max_pieces_per_unit", C.c_int32),
                ("consistent", C.c_int32)]


class df_cache(C.Structure):
    _fields_ = [("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
                ("head_row_off", C.POINTER(C.c_int64)),
                ("sink_cap", C.POINTER(C.c_int32)), ("win_cap", C.POINTER(C.c_int32)),
                ("sink_len", C.POINTER(C.c_int32)), ("win_len", C.POINTER(C.c_int32)),
                ("win_pos", C.POINTER(C.c_int32)),
                ("H", C.c_int32), ("d", C.c_int32)]


class df_append_args(C.Structure):
    _fields_ = [("cache", C.POINTER(df_cache)), ("k_new", C.c_void_p), ("v_new", C.c_void_p),
                ("stride_tok", C.c_int64), ("stride_head", C.c_int64), ("Nc", C.c_int32)]


class df_pack_args(C.Structure):
    _fields_ = [("cache", C.POINTER(df_cache)),
                ("take_sink", C.POINTER(C.c_int32)), ("take_win", C.POINTER(C.c_int32)),
                ("k_out", C.c_void_p), ("v_out", C.c_void_p), ("out_capacity_rows", C.c_int64),
                ("hist_off_out", C.POINTER(C.c_int64)), ("sink_len_out", C.POINTER(C.c_int32))]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                          "(python paper_2601_20499_amd/build.py); there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    lib.df_status_string.restype = C.c_char_p
    lib.df_status_string.argtypes = [C.c_int32]
    lib.df_head_context.restype = C.c_int32
    lib.df_head_context.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                    C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.df_attn_workspace_bytes.restype = C.c_size_t
    lib.df_attn_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
    lib.df_attn_fwd.restype = C.c_int32
    lib.df_attn_fwd.argtypes = [C.POINTER(df_attn_args), C.c_void_p]
    lib.df_attn_fwd_static.restype = C.c_int32
    lib.df_attn_fwd_static.argtypes = [C.POINTER(df_attn_args), C.c_void_p]
    lib.df_attn_plan.restype = C.c_int32
    lib.df_attn_plan.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                 C.POINTER(df_attn_plan_info)]
    lib.df_head_score.restype = C.c_int32
    lib.df_head_score.argtypes = [C.POINTER(df_score_args), C.c_void_p]
    lib.df_classify.restype = C.c_int32
    lib.df_classify.argtypes = [C.POINTER(C.c_float), C.c_int32, C.c_int32, C.c_int32,
                                C.POINTER(C.c_uint8), C.POINTER(C.c_float)]
    lib.df_kv_append.restype = C.c_int32
    lib.df_kv_append.argtypes = [C.POINTER(df_append_args), C.c_void_p]
    lib.df_pack_context.restype = C.c_int32
    lib.df_pack_context.argtypes = [C.POINTER(df_pack_args), C.c_void_p]
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.df_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != DF_OK:
        raise DfError(status, where)


def _i64(xs: Sequence[int]):
    return (C.c_int64 * len(xs))(*[int(x) for x in xs])


def _i32(xs: Sequence[int]):
    return (C.c_int32 * len(xs))(*[int(x) for x in xs])


def df_attn_plan(Nq: int, Nc: int, hist_len: Sequence[int], hist_sink_len: Optional[Sequence[int]] = None) -> dict:
    """The launch decomposition df_attn_fwd would use for these per-head history lengths (host only)."""
    info = df_attn_plan_info()
    H = len(hist_len)
    _check(lib.df_attn_plan(H, int(Nq), int(Nc), _i32(hist_len),
                            _i32(hist_sink_len) if hist_sink_len is not None else None, C.byref(info)), "df_attn_plan")
    return {name: getattr(info, name) for name, _ in df_attn_plan_info._fields_}


def _ptr(t) -> Optional[int]:
    """Raw device (or host) address of a torch tensor, None for a missing or empty tensor."""
    if t is None or t.numel() == 0:
        return None
    return t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    if isinstance(stream, int):          # raw hipStream_t value; 0 = the default stream
        return stream or None
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def df_head_context(head_type: int, T: int, sink_frames: int, window_frames: int):
    ns, nw = C.c_int32(), C.c_int32()
    _check(lib.df_head_context(head_type, T, sink_frames, window_frames, C.byref(ns), C.byref(nw)),
           "df_head_context")
    return ns.value, nw.value


def df_attn_workspace_bytes(H: int, d: int, Nq: int) -> int:
    return int(lib.df_attn_workspace_bytes(H, d, Nq))


DF_STATIC_SCRATCH_BYTES = 70 << 20


def df_attn_fwd_static(q, k_cur, v_cur, k_hist, v_hist, hist_off, hist_sink_len, out, softmax_scale,
                       lse_out=None, score_out=None, stream=None, hist_len=None):
    """df_attn_fwd on the library's static device scratch: no workspace argument, nothing allocated."""
    df_attn_fwd(q, k_cur, v_cur, k_hist, v_hist, hist_off, hist_sink_len, out, softmax_scale, lse_out=lse_out,
                score_out=score_out, workspace=None, stream=stream, hist_len=hist_len, _entry="df_attn_fwd_static")


def df_attn_fwd(q, k_cur, v_cur, k_hist, v_hist, hist_off, hist_sink_len, out, softmax_scale,
                lse_out=None, score_out=None, workspace=None, stream=None, hist_len=None, _entry="df_attn_fwd"):
    """q/out: [Nq, H, d] and k_cur/v_cur: [Nc, H, d] bf16 device tensors (any token/head strides,
    d contiguous); k_hist/v_hist: [hist_off[-1], d] bf16; hist_off/hist_sink_len/hist_len: python ints."""
    a = df_attn_args()
    a.q, a.q_stride_tok, a.q_stride_head = _ptr(q), q.stride(0), q.stride(1)
    a.k_cur, a.v_cur = _ptr(k_cur), _ptr(v_cur)
    a.kc_stride_tok, a.kc_stride_head = k_cur.stride(0), k_cur.stride(1)
    assert v_cur.stride() == k_cur.stride()
    a.k_hist, a.v_hist = _ptr(k_hist), _ptr(v_hist)
    off = _i64(hist_off)
    a.hist_off = off
    sl = _i32(hist_sink_len) if hist_sink_len is not None else None
    a.hist_sink_len = sl
    hl = _i32(hist_len) if hist_len is not None else None
    a.hist_len = hl
    a.out, a.o_stride_tok, a.o_stride_head = _ptr(out), out.stride(0), out.stride(1)
    a.lse_out, a.score_out = _ptr(lse_out), _ptr(score_out)
    a.H, a.d, a.Nq, a.Nc = q.shape[1], q.shape[2], q.shape[0], k_cur.shape[0]
    a.softmax_scale = softmax_scale
    a.workspace = _ptr(workspace)
    a.workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(getattr(lib, _entry)(C.byref(a), _stream_handle(stream)), _entry)


def df_head_score(q, k_cur, k_hist, hist_off, hist_sink_len, score_out, softmax_scale,
                  q_sample_stride=4, q_offset=0, workspace=None, stream=None, hist_len=None):
    a = df_score_args()
    a.q, a.q_stride_tok, a.q_stride_head = _ptr(q), q.stride(0), q.stride(1)
    a.k_cur, a.kc_stride_tok, a.kc_stride_head = _ptr(k_cur), k_cur.stride(0), k_cur.stride(1)
    a.k_hist = _ptr(k_hist)
    off, sl = _i64(hist_off), _i32(hist_sink_len)
    a.hist_off, a.hist_sink_len = off, sl
    hl = _i32(hist_len) if hist_len is not None else None
    a.hist_len = hl
    a.score_out = _ptr(score_out)
    a.H, a.d, a.Nq, a.Nc = q.shape[1], q.shape[2], q.shape[0], k_cur.shape[0]
    a.q_sample_stride, a.q_offset = q_sample_stride, q_offset
    a.softmax_scale = softmax_scale
    a.workspace = _ptr(workspace)
    a.workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.df_head_score(C.byref(a), _stream_handle(stream)), "df_head_score")


def df_classify(F_host, n_dummy: int, mode: int):
    """F_host: sequence of n rows (sink, neighbour, current) in fp32.  Returns (types, keys)."""
    rows = [[float(x) for x in r] for r in F_host]
    n = len(rows)
    flat = (C.c_float * (3 * n))(*[x for r in rows for x in r])
    types = (C.c_uint8 * n)()
    keys = (C.c_float * n)()
    _check(lib.df_classify(flat, n, n_dummy, mode, types, keys), "df_classify")
    return list(types), list(keys)


class Cache:
    """Owner of the host-side state arrays of a df_cache plus references to its device buffers."""

    def __init__(self, k_cache, v_cache, head_row_off, sink_cap, win_cap, d: int):
        H = len(sink_cap)
        self.k_cache, self.v_cache = k_cache, v_cache
        self.head_row_off = _i64(head_row_off)
        self.sink_cap, self.win_cap = _i32(sink_cap), _i32(win_cap)
        self.sink_len, self.win_len, self.win_pos = _i32([0] * H), _i32([0] * H), _i32([0] * H)
        self.c = df_cache()
        self.c.k_cache, self.c.v_cache = _ptr(k_cache), _ptr(v_cache)
        self.c.head_row_off = self.head_row_off
        self.c.sink_cap, self.c.win_cap = self.sink_cap, self.win_cap
        self.c.sink_len, self.c.win_len, self.c.win_pos = self.sink_len, self.win_len, self.win_pos
        self.c.H, self.c.d = H, d
        self.H, self.d = H, d

    def in_place(self):
        """(k_hist, v_hist, hist_off, hist_sink_len, hist_len) for reading the cache without packing:
        the filled rows of a head are a prefix of its rows (sink rows, then the ring)."""
        H = self.H
        return (self.k_cache, self.v_cache, [int(self.head_row_off[h]) for h in range(H + 1)],
                [int(self.sink_len[h]) for h in range(H)],
                [int(self.sink_len[h]) + int(self.win_len[h]) for h in range(H)])


def df_kv_append(cache: Cache, k_new, v_new, stream=None):
    a = df_append_args()
    a.cache = C.pointer(cache.c)
    a.k_new, a.v_new = _ptr(k_new), _ptr(v_new)
    a.stride_tok, a.stride_head = k_new.stride(0), k_new.stride(1)
    assert v_new.stride() == k_new.stride()
    a.Nc = k_new.shape[0]
    _check(lib.df_kv_append(C.byref(a), _stream_handle(stream)), "df_kv_append")


def df_pack_context(cache: Cache, take_sink, take_win, k_out, v_out, stream=None):
    """Returns (hist_off [H+1], sink_len [H]) as python lists."""
    a = df_pack_args()
    a.cache = C.pointer(cache.c)
    ts, tw = _i32(take_sink), _i32(take_win)
    a.take_sink, a.take_win = ts, tw
    a.k_out, a.v_out = _ptr(k_out), _ptr(v_out)
    a.out_capacity_rows = k_out.shape[0]
    off = (C.c_int64 * (cache.H + 1))()
    sl = (C.c_int32 * cache.H)()
    a.hist_off_out, a.sink_len_out = off, sl
    _check(lib.df_pack_context(C.byref(a), _stream_handle(stream)), "df_pack_context")
    return list(off), list(sl)


def prepared_pack(cache: Cache, take_sink, take_win, k_out, v_out, stream=None):
    """df_pack_context with the arguments marshalled once: returns a function that issues the call.
    For loops in which the Python-side marshalling would otherwise be the slower part."""
    a = df_pack_args()
    a.cache = C.pointer(cache.c)
    ts, tw = _i32(take_sink), _i32(take_win)
    a.take_sink, a.take_win = ts, tw
    a.k_out, a.v_out = _ptr(k_out), _ptr(v_out)
    a.out_capacity_rows = k_out.shape[0]
    off = (C.c_int64 * (cache.H + 1))()
    sl = (C.c_int32 * cache.H)()
    a.hist_off_out, a.sink_len_out = off, sl
    keep = (a, ts, tw, off, sl, k_out, v_out, cache)
    handle = _stream_handle(stream)

    def call(_keep=keep):
        _check(lib.df_pack_context(C.byref(a), handle), "df_pack_context")
    return call


def prepared_append(cache: Cache, k_new, v_new, stream=None):
    """df_kv_append with the arguments marshalled once (the cache state still advances per call)."""
    a = df_append_args()
    a.cache = C.pointer(cache.c)
    a.k_new, a.v_new = _ptr(k_new), _ptr(v_new)
    a.stride_tok, a.stride_head = k_new.stride(0), k_new.stride(1)
    assert v_new.stride() == k_new.stride()
    a.Nc = k_new.shape[0]
    keep = (a, k_new, v_new, cache)
    handle = _stream_handle(stream)

    def call(_keep=keep):
        _check(lib.df_kv_append(C.byref(a), handle), "df_kv_append")
    return call
