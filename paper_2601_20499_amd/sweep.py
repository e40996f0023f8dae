"""Single-layer attention time against context length and against the number of dummy heads
(the two per-layer curves of the paper: runtime vs context length, and vs the dummy-head count),
dense sliding-window attention against the head-heterogeneous contexts, on the same kernel.

    python -m paper_2601_20499_amd.sweep [--T 1560] [--reps 20]

Random bf16 tensors of the Wan-1.3B layer geometry (12 heads x 128, 3-frame chunk); only shapes
matter for the time.  Prints two markdown tables.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as df

H, D, CHUNK = 12, 128, 3


def time_attn(T, frames_per_head, sink_frames_per_head, reps, dev, H=H):
    """frames_per_head[h] = history frames head h sees; returns (ms, GFLOP)."""
    Nq = CHUNK * T
    lens = [f * T for f in frames_per_head]
    off = [0]
    for n in lens:
        off.append(off[-1] + n)
    sl = [min(s * T, n) for s, n in zip(sink_frames_per_head, lens)]
    g = torch.Generator(device=dev).manual_seed(0)
    mk = lambda *shape: torch.randn(*shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q, kc, vc = mk(Nq, H, D), mk(Nq, H, D), mk(Nq, H, D)
    kh, vh = mk(max(off[-1], 1), D), mk(max(off[-1], 1), D)
    out = torch.empty_like(q)
    ws = torch.empty(df.df_attn_workspace_bytes(H, D, Nq), dtype=torch.uint8, device=dev)
    call = lambda: df.df_attn_fwd(q, kc, vc, kh, vh, off, sl, out, D ** -0.5, workspace=ws)
    for _ in range(3):
        call()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        call()
    e1.record()
    torch.cuda.synchronize()
    flop = sum(4.0 * Nq * (n + Nq) * D for n in lens)
    return e0.elapsed_time(e1) / reps, flop / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--T", type=int, default=1560, help="tokens per latent frame")
    ap.add_argument("--reps", type=int, default=20)
    a = ap.parse_args()
    assert torch.cuda.is_available(), "needs a GPU"
    dev = torch.device("cuda:0")

    print(f"### attention ms per chunk-layer vs cached frames (T = {a.T}, 12 heads, 3-frame chunk)")
    print("| cached frames L (1 sink + L-1 recent) | dense ms | TFLOP/s | 6 packed dummy + 2 sink + 4 neighbour ms | TFLOP/s | speedup |")
    print("|---|---|---|---|---|---|")
    for L in (3, 6, 9, 12, 15, 21, 30):
        dense_ms, dense_gf = time_attn(a.T, [L] * H, [1] * H, a.reps, dev)
        frames = [1] * 6 + [1] * 2 + [L - 1] * 4            # packing frame | sink frame | L-1 recent frames
        sinks = [0] * 6 + [1] * 2 + [0] * 4
        m_ms, m_gf = time_attn(a.T, frames, sinks, a.reps, dev)
        print(f"| {L} | {dense_ms:.3f} | {dense_gf / dense_ms:.0f} | {m_ms:.3f} | {m_gf / m_ms:.0f} | {dense_ms / m_ms:.2f}x |", flush=True)

    print()
    print(f"### attention ms vs number of dummy heads N (T = {a.T}, 1 sink + 5 recent frames cached)")
    print("| N | full + dummy ms | speedup | full + packed dummy ms | speedup | sink/neighbour (1:2) + packed dummy ms | speedup |")
    print("|---|---|---|---|---|---|---|")
    L = 6
    base_ms = None
    for N in (0, 3, 6, 9, 12):
        keep = H - N
        two = time_attn(a.T, [0] * N + [L] * keep, [0] * N + [1] * keep, a.reps, dev)[0]
        packed = time_attn(a.T, [1] * N + [L] * keep, [0] * N + [1] * keep, a.reps, dev)[0]
        n_sink = keep // 3
        three = time_attn(a.T, [1] * N + [1] * n_sink + [L - 1] * (keep - n_sink),
                          [0] * N + [1] * n_sink + [0] * (keep - n_sink), a.reps, dev)[0]
        base_ms = two if base_ms is None else base_ms
        print(f"| {N} | {two:.3f} | {base_ms / two:.2f}x | {packed:.3f} | {base_ms / packed:.2f}x | {three:.3f} | {base_ms / three:.2f}x |", flush=True)

    print()
    print(f"### long context (T = {a.T}): sliding window of 36 frames, no window (237 frames for every head), "
          "and 237 frames for the neighbour heads only")
    print("| contexts of the 12 heads | cached frames / head | GFLOP | ms | TFLOP/s | vs 237-frame dense |")
    print("|---|---|---|---|---|---|")
    rows = [("dense, 36 frames (sliding window)", [36] * H, [1] * H),
            ("dense, 237 frames (no window)", [237] * H, [1] * H),
            ("6 packed dummy + 4 sink + 2 neighbour x 237 frames", [1] * 6 + [1] * 4 + [237] * 2, [0] * 6 + [1] * 4 + [0] * 2),
            ("6 packed dummy + 2 sink + 4 neighbour x 237 frames", [1] * 6 + [1] * 2 + [237] * 4, [0] * 6 + [1] * 2 + [0] * 4)]
    res = [(n, f, time_attn(a.T, f, sk, max(3, a.reps // 4), dev)) for n, f, sk in rows]
    ref_ms = res[1][2][0]
    for n, f, (ms, gf) in res:
        print(f"| {n} | {sum(f) / H:.1f} | {gf:.0f} | {ms:.3f} | {gf / ms:.0f} | {ref_ms / ms:.2f}x |", flush=True)

    print()
    print("### 1920x1088 chunk (8160 tokens per frame, 24480 queries, 1 sink + 5 recent frames cached)")
    print("| contexts of the 12 heads | GFLOP | ms | TFLOP/s | speedup |")
    print("|---|---|---|---|---|")
    rows = [("dense", [6] * H, [1] * H),
            ("6 full + 6 packed dummy", [1] * 6 + [6] * 6, [0] * 6 + [1] * 6),
            ("6 packed dummy + 2 sink + 4 neighbour", [1] * 6 + [1] * 2 + [5] * 4, [0] * 6 + [1] * 2 + [0] * 4)]
    res = [(n, time_attn(8160, f, sk, max(3, a.reps // 4), dev)) for n, f, sk in rows]
    for n, (ms, gf) in res:
        print(f"| {n} | {gf:.0f} | {ms:.3f} | {gf / ms:.0f} | {res[0][1][0] / ms:.2f}x |", flush=True)

    print()
    print(f"### 40 heads per layer (14B-class geometry, T = {a.T}, 1 sink + 5 recent frames cached)")
    print("| contexts of the 40 heads | GFLOP | ms | TFLOP/s | speedup |")
    print("|---|---|---|---|---|")
    rows = [("dense", [6] * 40, [1] * 40),
            ("20 packed dummy + 7 sink + 13 neighbour", [1] * 20 + [1] * 7 + [5] * 13, [0] * 20 + [1] * 7 + [0] * 13)]
    res = [(n, time_attn(a.T, f, sk, max(3, a.reps // 2), dev, H=40)) for n, f, sk in rows]
    for n, (ms, gf) in res:
        print(f"| {n} | {gf:.0f} | {ms:.3f} | {gf / ms:.0f} | {res[0][1][0] / ms:.2f}x |", flush=True)


if __name__ == "__main__":
    main()
