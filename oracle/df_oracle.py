"""CPU oracle for the Dummy Forcing attention hot path.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain, fp64 statement of what the HIP library must
compute.  It is imported only by the tests, by the smoke check and by the
benchmark's cpu_baseline leg; the product path never calls it, and it shares
no code with the HIP kernels or their host glue.

Every function is the paper's definition written out with numpy in float64:
no tiling, no online rescaling, no fusion.  Callers widen the bf16 inputs the
GPU sees to float64 exactly before calling in.

Pins (tests/test_oracle_*.py, all CPU): brute-force python loops on tiny
shapes, closed forms (uniform softmax, constant V, two-key sigmoid), the
block-causal identity for all-FULL heads, dummy == current-chunk-only
attention, row sums of the attention map, an independent library softmax
attention on the special cases, exhaustive search for the classification
objective (Eq. 6-7 and the appendix' closed form V*), and the cache-ratio
arithmetic printed with Tab. 9.  The paper prints no worked numeric example
of an attention output or of a frame attention score, so no golden value of
those exists; the pins above stand in for it.
"""
from __future__ import annotations

import numpy as np

# Head types.  FULL is the baseline of Eq. 2 (sink + L-1 neighbours + current);
# SINK / NEIGHBOR / DUMMY are the three types of Eq. 5; PACK_DUMMY is Eq. 8.
HEAD_FULL = 0
HEAD_SINK = 1
HEAD_NEIGHBOR = 2
HEAD_DUMMY = 3
HEAD_PACK_DUMMY = 4

# Classification modes.
MODE_TWO_CLASS = 0   # Observation 1: top-N alpha^current are dummy, the rest stay FULL
MODE_DHP = 1         # Dynamic Head Programming, Eq. 6-7 and the greedy rule after them


# --------------------------------------------------------------------------
# Visible context per head type (Sec. 3.1 sliding window, Eq. 2, Eq. 5, Eq. 8)
# --------------------------------------------------------------------------
def head_context_tokens(head_type: int, T: int, sink_frames: int, window_frames: int):
    """(n_sink, n_win) in tokens for one head.

    The cache window holds `sink_frames` sink frames and `window_frames`
    (= L-1) neighbour frames of T tokens each (Sec. 3.1).  FULL sees both
    (Eq. 2); a sink head sees the sink only, a neighbour head the recent
    window only, a dummy head no history (Eq. 5); a packed dummy head sees
    the single most recent frame (Eq. 8).
    """
    if head_type == HEAD_FULL:
        return sink_frames * T, window_frames * T
    if head_type == HEAD_SINK:
        return sink_frames * T, 0
    if head_type == HEAD_NEIGHBOR:
        return 0, window_frames * T
    if head_type == HEAD_DUMMY:
        return 0, 0
    if head_type == HEAD_PACK_DUMMY:
        return 0, T
    raise ValueError(f"unknown head type {head_type}")


def visible_history(Nh: int, n_sink: int, n_win: int):
    """Index sets (sink_idx, win_idx) into a chronological history of Nh tokens.

    Sink region: the first min(n_sink, Nh) tokens.  Window region: the last
    n_win tokens that are not already in the sink region (the regions
    partition the visible keys, as the index sets J_r of Eq. 3 do).
    """
    ns = min(int(n_sink), int(Nh))
    w0 = max(ns, int(Nh) - int(n_win))
    return np.arange(0, ns, dtype=np.int64), np.arange(w0, Nh, dtype=np.int64)


# --------------------------------------------------------------------------
# Attention (Eq. 2 / 5 / 8) and the attention map used by Eq. 3
# --------------------------------------------------------------------------
def attention_map(q: np.ndarray, k: np.ndarray, scale: float):
    """Row-softmax of scale * q k^T.  Returns (A, lse): A[u, v] >= 0, rows sum to 1;
    lse[u] = log sum_v exp(scale * q_u . k_v)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    s = scale * (q @ k.T)
    m = s.max(axis=1, keepdims=True)
    p = np.exp(s - m)
    l = p.sum(axis=1, keepdims=True)
    return p / l, (m + np.log(l))[:, 0]


def head_attention(q, k_hist, v_hist, k_cur, v_cur, n_sink: int, n_win: int, scale: float):
    """One head of the heterogeneous attention.

    q            [Nq, d]  queries of the current chunk
    k_hist/v_hist[Nh, d]  this head's cached history, chronological (Nh may be 0)
    k_cur/v_cur  [Nc, d]  keys/values of the current chunk (all visible to all queries)
    n_sink/n_win          visible sink / window tokens (see head_context_tokens)

    Returns out [Nq, d], mass [Nq, 3] (per-row attention mass on the sink,
    neighbour and current regions: the inner sum of Eq. 3) and lse [Nq].
    Keys are concatenated in the order [sink, window, current] as in Eq. 2.
    """
    q = np.asarray(q, dtype=np.float64)
    k_hist = np.asarray(k_hist, dtype=np.float64).reshape(-1, q.shape[1])
    v_hist = np.asarray(v_hist, dtype=np.float64).reshape(-1, q.shape[1])
    k_cur = np.asarray(k_cur, dtype=np.float64)
    v_cur = np.asarray(v_cur, dtype=np.float64)
    sink_idx, win_idx = visible_history(k_hist.shape[0], n_sink, n_win)
    k = np.concatenate([k_hist[sink_idx], k_hist[win_idx], k_cur], axis=0)
    v = np.concatenate([v_hist[sink_idx], v_hist[win_idx], v_cur], axis=0)
    A, lse = attention_map(q, k, scale)
    out = A @ v
    a, b = len(sink_idx), len(sink_idx) + len(win_idx)
    mass = np.stack([A[:, :a].sum(axis=1), A[:, a:b].sum(axis=1), A[:, b:].sum(axis=1)], axis=1)
    return out, mass, lse


def frame_attention_score(mass: np.ndarray, q_offset: int = 0, q_stride: int = 1):
    """Eq. 3: alpha^r = mean over the scored query rows of the row mass on region r.

    The scored rows are u = q_offset, q_offset + q_stride, ... (the uniform
    query sample of the Dynamic Head Programming paragraph; stride 1 = all rows).
    """
    return np.asarray(mass, dtype=np.float64)[q_offset::q_stride].mean(axis=0)


def layer_attention(q, k_hist_list, v_hist_list, k_cur, v_cur, n_sink, n_win, scale,
                    rows=None):
    """All heads of one layer.  q, k_cur, v_cur: [N, H, d]; k_hist_list[h]: [Nh_h, d].
    `rows` optionally restricts the computed query rows (rows are independent).
    Returns out [len(rows), H, d], mass [H, len(rows), 3], lse [H, len(rows)]."""
    q = np.asarray(q, dtype=np.float64)
    H = q.shape[1]
    rows = np.arange(q.shape[0]) if rows is None else np.asarray(rows)
    outs, masses, lses = [], [], []
    for h in range(H):
        o, ms, ls = head_attention(q[rows, h, :], k_hist_list[h], v_hist_list[h],
                                   np.asarray(k_cur)[:, h, :], np.asarray(v_cur)[:, h, :],
                                   n_sink[h], n_win[h], scale)
        outs.append(o)
        masses.append(ms)
        lses.append(ls)
    return np.stack(outs, axis=1), np.stack(masses, axis=0), np.stack(lses, axis=0)


# --------------------------------------------------------------------------
# Head classification (Observation 1; Eq. 6-7 and the greedy rule)
# --------------------------------------------------------------------------
def dhp_value(F: np.ndarray, types) -> float:
    """Objective of Eq. 6 with the value function of Eq. 7."""
    F = np.asarray(F, dtype=np.float64)
    total = 0.0
    for h, c in enumerate(types):
        if c == HEAD_SINK:
            total += F[h, 0] + F[h, 2]
        elif c == HEAD_NEIGHBOR:
            total += F[h, 1] + F[h, 2]
        elif c == HEAD_DUMMY:
            total += F[h, 2]
        else:
            raise ValueError("Eq. 7 is defined for sink / neighbour / dummy only")
    return float(total)


def classify(F: np.ndarray, N: int, mode: int):
    """Head types from the global frame attention scores F [n, 3].

    MODE_DHP: l_h = max(F_h0, F_h1); the N smallest l_h become dummy; of the
    rest, sink if F_h0 >= F_h1 else neighbour (greedy rule after Eq. 7).
    MODE_TWO_CLASS: the N largest alpha^current = the N smallest history
    mass F_h0 + F_h1 become dummy, the others stay FULL (Observation 1).
    Ties in the sort are broken by the lower head index.
    Returns (types uint8 [n], key float64 [n]) where key is the sorted score.
    """
    F = np.asarray(F, dtype=np.float64)
    n = F.shape[0]
    if not 0 <= N <= n:
        raise ValueError("N out of range")
    if mode == MODE_DHP:
        key = np.maximum(F[:, 0], F[:, 1])
    elif mode == MODE_TWO_CLASS:
        key = F[:, 0] + F[:, 1]
    else:
        raise ValueError("unknown mode")
    order = sorted(range(n), key=lambda h: (key[h], h))
    types = np.zeros(n, dtype=np.uint8)
    dummy = set(order[:N])
    for h in range(n):
        if h in dummy:
            types[h] = HEAD_DUMMY
        elif mode == MODE_TWO_CLASS:
            types[h] = HEAD_FULL
        else:
            types[h] = HEAD_SINK if F[h, 0] >= F[h, 1] else HEAD_NEIGHBOR
    return types, key


# --------------------------------------------------------------------------
# KV cache: sliding window with a fixed sink (Sec. 3.1) as plain lists
# --------------------------------------------------------------------------
class CacheModel:
    """Per-head logical cache: `sink[h]` keeps the first sink_cap[h] tokens ever
    appended and never changes afterwards; `win[h]` keeps the most recent
    win_cap[h] of all later tokens, oldest first.  A head with both
    capacities zero keeps nothing (dummy heads drop their cache, Observation 3).
    Rows are stored as whatever dtype the caller passes (bit patterns stay exact)."""

    def __init__(self, H: int, d: int, sink_cap, win_cap, dtype=np.uint16):
        self.H, self.d = H, d
        self.sink_cap = [int(x) for x in sink_cap]
        self.win_cap = [int(x) for x in win_cap]
        self.k_sink = [np.zeros((0, d), dtype=dtype) for _ in range(H)]
        self.v_sink = [np.zeros((0, d), dtype=dtype) for _ in range(H)]
        self.k_win = [np.zeros((0, d), dtype=dtype) for _ in range(H)]
        self.v_win = [np.zeros((0, d), dtype=dtype) for _ in range(H)]

    def append(self, k_new: np.ndarray, v_new: np.ndarray):
        """k_new, v_new: [Nc, H, d] in chronological token order."""
        for h in range(self.H):
            room = self.sink_cap[h] - self.k_sink[h].shape[0]
            take = max(0, min(room, k_new.shape[0]))
            self.k_sink[h] = np.concatenate([self.k_sink[h], k_new[:take, h]], axis=0)
            self.v_sink[h] = np.concatenate([self.v_sink[h], v_new[:take, h]], axis=0)
            kw = np.concatenate([self.k_win[h], k_new[take:, h]], axis=0)
            vw = np.concatenate([self.v_win[h], v_new[take:, h]], axis=0)
            keep = self.win_cap[h]
            self.k_win[h] = kw[kw.shape[0] - min(keep, kw.shape[0]):]
            self.v_win[h] = vw[vw.shape[0] - min(keep, vw.shape[0]):]

    def pack(self, take_sink, take_win):
        """Ragged per-head context [sink[:take_sink] | last take_win window tokens],
        heads concatenated.  Returns (Kp, Vp, hist_off [H+1], sink_len [H])."""
        ks, vs, off, sl = [], [], [0], []
        for h in range(self.H):
            a = min(int(take_sink[h]), self.k_sink[h].shape[0])
            w = min(int(take_win[h]), self.k_win[h].shape[0])
            nwin = self.k_win[h].shape[0]
            ks += [self.k_sink[h][:a], self.k_win[h][nwin - w:]]
            vs += [self.v_sink[h][:a], self.v_win[h][nwin - w:]]
            off.append(off[-1] + a + w)
            sl.append(a)
        return (np.concatenate(ks, axis=0), np.concatenate(vs, axis=0),
                np.asarray(off, dtype=np.int64), np.asarray(sl, dtype=np.int32))


def cache_kept_fraction(per_head_frames, baseline_frames: float) -> float:
    """Mean cached frames per head over a baseline window (the accounting behind Tab. 9)."""
    return float(np.mean(np.asarray(per_head_frames, dtype=np.float64)) / baseline_frames)
