"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *draws tensors and describes shapes*; it holds none of the
method's arithmetic (no softmax, no scores, no classification, no cache
logic) and is the one module shared by the tests of the CPU oracle and by the
callers of the HIP library.  All tensors are created on the CPU from a seeded
torch.Generator and rounded to bf16 once, so that the oracle and the GPU see
identical bit patterns.

Shapes follow the Self Forcing geometry the paper evaluates (Sec. 4.1, Tab. 2,
Tab. 4, App. C): 12 heads of width 128 per layer, 30 layers (360 heads), a
chunk of 3 latent frames, 1560 tokens per 832x480 latent frame and 3600 per
1280x720 frame, a cache window of one sink frame plus L-1 neighbour frames.
Real activations are not available; element-wise Gaussians with a per-head
query mean stand in for them, and "current-frame-focused" heads are planted by
shifting the current chunk's keys along that query mean.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch

HEAD_FULL, HEAD_SINK, HEAD_NEIGHBOR, HEAD_DUMMY, HEAD_PACK_DUMMY = 0, 1, 2, 3, 4


@dataclass
class Workload:
    name: str
    H: int
    d: int
    T: int                      # tokens per latent frame
    chunk_frames: int           # frames per query chunk
    hist_frames: int            # frames of history every head could see (sink first)
    sink_frames: int
    scale: float                # softmax scale
    seed: int
    head_type: List[int]        # per head, one of HEAD_*
    n_sink: List[int]           # visible sink tokens per head
    n_win: List[int]            # visible window tokens per head
    planted: List[int] = field(default_factory=list)   # heads biased towards the current chunk
    roles: List[str] = field(default_factory=list)     # planted role per head, where a generator sets one
    q: Optional[torch.Tensor] = None        # [Nq, H, d] bf16
    k_cur: Optional[torch.Tensor] = None    # [Nc, H, d] bf16
    v_cur: Optional[torch.Tensor] = None
    k_hist: Optional[torch.Tensor] = None   # [Nh, H, d] bf16, chronological, sink frame first
    v_hist: Optional[torch.Tensor] = None

    @property
    def Nq(self) -> int:
        return self.chunk_frames * self.T

    @property
    def Nc(self) -> int:
        return self.chunk_frames * self.T

    @property
    def Nh(self) -> int:
        return self.hist_frames * self.T

    def visible_len(self, h: int) -> int:
        ns = min(self.n_sink[h], self.Nh)
        return ns + (self.Nh - max(ns, self.Nh - self.n_win[h]))

    def attn_flop(self) -> float:
        """Algorithmic FLOP of one chunk-layer: QK^T and PV over visible keys only."""
        return sum(4.0 * self.Nq * (self.visible_len(h) + self.Nc) * self.d for h in range(self.H))

    def score_flop(self, q_stride: int = 4) -> float:
        nu = (self.Nq + q_stride - 1) // q_stride
        return 2.0 * nu * (self.Nh + self.Nc) * self.d * self.H


def _context(head_type: int, T: int, sink_frames: int, window_frames: int):
    # token counts of the visible sink / window region per head type (Eq. 2, 5, 8)
    table = {
        HEAD_FULL: (sink_frames * T, window_frames * T),
        HEAD_SINK: (sink_frames * T, 0),
        HEAD_NEIGHBOR: (0, window_frames * T),
        HEAD_DUMMY: (0, 0),
        HEAD_PACK_DUMMY: (0, T),
    }
    return table[head_type]


def _gauss(gen, shape, std=1.0, dtype=torch.float32):
    # drawn in slabs so that the largest configurations stay within a few GB of host memory
    out = torch.empty(shape, dtype=dtype)
    flat = out.view(-1)
    step = 1 << 24
    for s in range(0, flat.numel(), step):
        n = min(step, flat.numel() - s)
        flat[s:s + n] = (torch.randn(n, generator=gen, dtype=torch.float32) * std).to(dtype)
    return out


def _draw(w: Workload, planted: List[int], bias: float = 2.0, weak_bias: Optional[List[float]] = None,
          q_mean_std: float = 0.4, fp32: bool = False, sink_bias: Optional[List[float]] = None):
    """Q = G + mu_h with mu_h ~ q_mean_std * N(0, I); K, V element-wise N(0,1).
    Planted heads get K_cur += bias * mean_u(Q_h); other heads optionally a weak bias.
    sink_bias[h] != 0 shifts the keys of head h's sink frame(s) the same way (a sink-focused head)."""
    g = torch.Generator().manual_seed(w.seed)
    H, d = w.H, w.d
    dt = torch.float32
    q = _gauss(g, (w.Nq, H, d), dtype=dt)
    mu = torch.randn(H, d, generator=g) * q_mean_std
    q += mu[None]
    k_cur = _gauss(g, (w.Nc, H, d), dtype=dt)
    v_cur = _gauss(g, (w.Nc, H, d), dtype=dt)
    q_mean = q.mean(dim=0)                               # [H, d]
    for h in range(H):
        b = bias if h in planted else (weak_bias[h] if weak_bias is not None else 0.0)
        if b != 0.0:
            k_cur[:, h, :] += b * q_mean[h]
    store = torch.float32 if fp32 else torch.bfloat16
    w.q, w.k_cur, w.v_cur = q.to(store), k_cur.to(store), v_cur.to(store)
    if sink_bias is None:
        w.k_hist = _gauss(g, (w.Nh, H, d), dtype=store)
    else:
        k_hist = _gauss(g, (w.Nh, H, d), dtype=dt)
        ns = min(w.sink_frames * w.T, w.Nh)
        for h in range(H):
            if sink_bias[h] != 0.0:
                k_hist[:ns, h, :] += sink_bias[h] * q_mean[h]
        w.k_hist = k_hist.to(store)
    w.v_hist = _gauss(g, (w.Nh, H, d), dtype=store)
    w.planted = list(planted)
    return w


def _typed(name, H, d, T, chunk_frames, hist_frames, types, seed, scale=None, sink_frames=1):
    sink_frames = min(sink_frames, hist_frames)
    window_frames = hist_frames - sink_frames
    ctx = [_context(t, T, sink_frames, window_frames) for t in types]
    return Workload(name=name, H=H, d=d, T=T, chunk_frames=chunk_frames, hist_frames=hist_frames,
                    sink_frames=sink_frames, scale=(1.0 / math.sqrt(d)) if scale is None else scale,
                    seed=seed, head_type=list(types), n_sink=[c[0] for c in ctx], n_win=[c[1] for c in ctx])


def config1(fp32: bool = False) -> Workload:
    """Tiny plumbing case: 4 heads of width 64, 64 tokens per frame, one-frame chunk, 3 past
    frames (sink = frame 0), heads 0-2 full and head 3 dummy, plain N(0,1) tensors, seed 0."""
    w = _typed("config1_tiny", 4, 64, 64, 1, 3, [HEAD_FULL] * 3 + [HEAD_DUMMY], seed=0)
    return _draw(w, planted=[], q_mean_std=0.0, fp32=fp32)


def config2(dummy_heads=(2, 5, 9)) -> Workload:
    """Wan-1.3B-shaped layer at 832x480: 12 heads x 128, 1560 tokens per frame, 3-frame chunk
    (4680 queries), 1 sink + 5 recent frames of history; 3 planted dummy heads."""
    types = [HEAD_DUMMY if h in dummy_heads else HEAD_FULL for h in range(12)]
    w = _typed("config2_wan1.3b_480p", 12, 128, 1560, 3, 6, types, seed=1)
    return _draw(w, planted=list(dummy_heads))


def config3_layer(layer: int, T: int = 1560, hist_frames: int = 21) -> Workload:
    """One layer of the 30-layer stack: config-2 shapes with a 21-frame history; a seeded 2-4
    heads are planted per layer, the others get distinct weak biases so that their scores
    separate.  Head types are left FULL: they come from the classification under test."""
    g = torch.Generator().manual_seed(1000 + layer)
    n_plant = int(torch.randint(2, 5, (1,), generator=g))
    planted = sorted(torch.randperm(12, generator=g)[:n_plant].tolist())
    weak = (torch.rand(12, generator=g) * 0.5).tolist()
    w = _typed(f"config3_layer{layer}", 12, 128, T, 3, hist_frames, [HEAD_FULL] * 12, seed=2 + layer)
    return _draw(w, planted=planted, weak_bias=weak)


def config4(dummy_heads=(0, 6, 7)) -> Workload:
    """720P chunk: 3600 tokens per frame, 10800 queries, 12-frame history, 3 dummy heads."""
    types = [HEAD_DUMMY if h in dummy_heads else HEAD_FULL for h in range(12)]
    w = _typed("config4_720p", 12, 128, 3600, 3, 12, types, seed=3)
    return _draw(w, planted=list(dummy_heads))


def config5(T: int = 1560, hist_frames: int = 60) -> Workload:
    """Long-video context: 60 past frames cached, half of the heads dummy, the others see a
    one-frame sink plus a seeded window so that their history spans 3..60 frames, with both
    extremes present."""
    g = torch.Generator().manual_seed(4)
    perm = torch.randperm(12, generator=g).tolist()
    dummy = sorted(perm[:6])
    keep = sorted(perm[6:])
    frames = torch.randint(3, hist_frames + 1, (len(keep),), generator=g).tolist()
    frames[0], frames[-1] = 3, hist_frames
    types = [HEAD_DUMMY if h in dummy else HEAD_FULL for h in range(12)]
    w = _typed("config5_long_context", 12, 128, T, 3, hist_frames, types, seed=4)
    for h, f in zip(keep, frames):
        w.n_sink[h] = T
        w.n_win[h] = (f - 1) * T
    return _draw(w, planted=dummy)


def dhp3_layer(layer: int, T: int = 1560, hist_frames: int = 6, d: int = 128, H: int = 12) -> Workload:
    """One layer of a 30-layer stack for the paper's full method (Sec. 3.3: sink / neighbour /
    dummy heads, half of all heads dummy, classified globally over all layers' heads): config-2
    geometry (1 sink + hist_frames-1 recent frames, 3-frame chunk); every head gets a seeded role
    and strength: about half lean on the current chunk, about a fifth on the sink frame, the others
    keep the spread-out profile of plain Gaussians (most mass on the recent frames).  Head types are
    left FULL: they come from the classification under test.  `roles[h]` in {"current", "sink",
    "neighbor"} records what was planted."""
    g = torch.Generator().manual_seed(5000 + layer)
    u = torch.rand(H, generator=g).tolist()
    strength = torch.rand(H, generator=g).tolist()
    cur_bias, snk_bias, roles = [0.0] * H, [0.0] * H, []
    for h in range(H):
        if u[h] < 0.5:
            roles.append("current")
            cur_bias[h] = 1.0 + 1.5 * strength[h]
        elif u[h] < 0.7:
            roles.append("sink")
            snk_bias[h] = 1.5 + 1.5 * strength[h]
        else:
            roles.append("neighbor")
            cur_bias[h] = 0.4 * strength[h]
    w = _typed(f"dhp3_layer{layer}_T{T}", H, d, T, 3, hist_frames, [HEAD_FULL] * H, seed=7000 + layer)
    _draw(w, planted=[], weak_bias=cur_bias, sink_bias=snk_bias)
    w.planted = [h for h in range(H) if roles[h] == "current"]
    w.roles = roles
    return w


def long_context_layer(window_frames: int = 237, n_neighbor: int = 2, n_sink: int = 4, T: int = 1560) -> Workload:
    """Long-context reallocation (Sec. 4.4, the long-context table): the cache budget saved on dummy
    and sink heads goes to the neighbour heads, which see `window_frames` past frames; the other heads
    keep one frame (packing frame or sink).  12 heads: n_neighbor neighbour, n_sink sink, the rest
    packed dummy; the dummy heads are the planted ones."""
    H = 12
    types = [HEAD_NEIGHBOR] * n_neighbor + [HEAD_SINK] * n_sink + [HEAD_PACK_DUMMY] * (H - n_neighbor - n_sink)
    g = torch.Generator().manual_seed(11)
    types = [types[i] for i in torch.randperm(H, generator=g).tolist()]
    w = _typed(f"long_context_{window_frames}f", H, 128, T, 3, window_frames + 1, types, seed=12)
    return _draw(w, planted=[h for h, t in enumerate(types) if t == HEAD_PACK_DUMMY])


def res1080p(dummy_heads=(1, 4, 5, 8, 9, 11)) -> Workload:
    """1920x1088 chunk (Sec. 4.3): 8160 tokens per latent frame, 24480 queries, 1 sink + 5 recent
    frames of history, half of the heads packed dummy, the others full."""
    types = [HEAD_PACK_DUMMY if h in dummy_heads else HEAD_FULL for h in range(12)]
    w = _typed("res1080p", 12, 128, 8160, 3, 6, types, seed=13)
    return _draw(w, planted=list(dummy_heads))


def small_ragged(seed: int, H: int = 3, d: int = 128, T: int = 37, chunk_frames: int = 3,
                 hist_frames: int = 5, types=None, q_mean_std: float = 0.4, planted=()) -> Workload:
    """Small case with sizes that are multiples of no tile: used for element-wise parity."""
    types = list(types) if types is not None else [HEAD_FULL, HEAD_DUMMY, HEAD_NEIGHBOR][:H]
    w = _typed(f"small_T{T}_H{H}_d{d}_s{seed}", H, d, T, chunk_frames, hist_frames, types, seed=seed)
    return _draw(w, planted=list(planted), q_mean_std=q_mean_std)


# ---- views used by callers -------------------------------------------------
def visible_history_rows(w: Workload, h: int) -> torch.Tensor:
    """Row indices of head h's visible history inside the chronological history (sink first)."""
    ns = min(w.n_sink[h], w.Nh)
    w0 = max(ns, w.Nh - w.n_win[h])
    return torch.cat([torch.arange(0, ns), torch.arange(w0, w.Nh)])


def packed_history(w: Workload):
    """Ragged per-head history [sum_h len_h, d] as the attention entry point takes it,
    plus hist_off [H+1] and sink_len [H] (plain row selection, no arithmetic)."""
    ks, vs, off, sl = [], [], [0], []
    for h in range(w.H):
        rows = visible_history_rows(w, h)
        ks.append(w.k_hist[rows, h, :])
        vs.append(w.v_hist[rows, h, :])
        off.append(off[-1] + rows.numel())
        sl.append(min(w.n_sink[h], w.Nh))
    d = w.d
    k = torch.cat(ks, 0) if off[-1] else torch.zeros(0, d, dtype=w.q.dtype)
    v = torch.cat(vs, 0) if off[-1] else torch.zeros(0, d, dtype=w.q.dtype)
    return k.contiguous(), v.contiguous(), off, sl
