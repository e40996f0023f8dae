"""The entry points only enqueue kernels (no allocation, no memset, no host synchronisation), so a
chunk-layer step can be captured in a HIP graph.  Replays are interleaved with eager work and
synchronisations and every replay is compared with the eager result."""
import numpy as np
import pytest
import torch

from paper_2601_20499_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def df():
    from paper_2601_20499_amd import binding
    return binding


def test_pack_attention_append_in_a_graph(df):
    d = gu.dev()
    w = wl.small_ragged(55, H=5, d=128, T=70, hist_frames=5,
                        types=[wl.HEAD_FULL, wl.HEAD_SINK, wl.HEAD_NEIGHBOR, wl.HEAD_PACK_DUMMY, wl.HEAD_DUMMY], planted=[3, 4])
    H, dd = w.H, w.d
    sink_cap = [min(w.n_sink[h], w.Nh) for h in range(H)]
    win_cap = [w.visible_len(h) - sink_cap[h] for h in range(H)]
    off = np.concatenate([[0], np.cumsum([s + x for s, x in zip(sink_cap, win_cap)])]).tolist()

    def fresh_cache():
        c = df.Cache(torch.zeros(off[-1], dd, dtype=torch.bfloat16, device=d),
                     torch.zeros(off[-1], dd, dtype=torch.bfloat16, device=d), off, sink_cap, win_cap, dd)
        kh, vh = w.k_hist.to(d), w.v_hist.to(d)
        for s in range(0, w.Nh, w.Nc):
            df.df_kv_append(c, kh[s:s + w.Nc], vh[s:s + w.Nc])
        return c

    cache, twin = fresh_cache(), fresh_cache()
    q, kc, vc = w.q.to(d), w.k_cur.to(d), w.v_cur.to(d)
    k_pack = torch.zeros(off[-1], dd, dtype=torch.bfloat16, device=d)
    v_pack = torch.zeros_like(k_pack)
    out = torch.zeros(w.Nq, H, dd, dtype=torch.bfloat16, device=d)
    F = torch.zeros(H, 3, dtype=torch.float32, device=d)
    ws = torch.empty(df.df_attn_workspace_bytes(H, dd, w.Nq), dtype=torch.uint8, device=d)
    state = (list(twin.sink_len), list(twin.win_len), list(twin.win_pos))

    def step():
        for h in range(H):      # the appended-to cache starts every step from the same host-side state
            twin.sink_len[h], twin.win_len[h], twin.win_pos[h] = state[0][h], state[1][h], state[2][h]
        p_off, p_sl = df.df_pack_context(cache, sink_cap, win_cap, k_pack, v_pack)
        df.df_attn_fwd(q, kc, vc, k_pack, v_pack, p_off, p_sl, out, w.scale, score_out=F, workspace=ws)
        df.df_kv_append(twin, kc, vc)

    step()                                             # eager reference
    torch.cuda.synchronize()
    ref_out, ref_F, ref_k = out.clone(), F.clone(), twin.k_cache.clone()
    ref, _, _ = gu.oracle_rows(w)
    gu.check_out(ref_out.float().cpu().double().numpy(), ref, "eager step")

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                         # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(4):
        out.fill_(7.0); F.fill_(7.0); k_pack.fill_(3.0); v_pack.fill_(3.0)
        twin.k_cache.copy_(cache.k_cache)              # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out), replay       # same kernels, same order: bitwise equal
        assert torch.equal(F, ref_F), replay
        assert torch.equal(twin.k_cache, ref_k), replay


def test_one_graph_per_ring_phase_across_successive_appends(df):
    """A captured step holds the host-side cache state (ring positions, lengths) of the moment of capture, so
    an autoregressive loop needs one graph per ring phase, captured with the host state advanced by the caller.
    Here the ring holds two chunks: two graphs, replayed alternately over four steps with new chunk data each
    step, against the same four steps run eagerly (outputs, scores and cache contents bit for bit)."""
    d = gu.dev()
    H, dd, T, Nc = 3, 128, 48, 96
    sink_cap, win_cap = [T, 0, 0], [2 * Nc, 2 * Nc, 0]         # sink + ring, ring only, dummy
    off = np.concatenate([[0], np.cumsum([s + x for s, x in zip(sink_cap, win_cap)])]).tolist()
    g = torch.Generator().manual_seed(77)
    mk = lambda *s: torch.randn(*s, generator=g).to(torch.bfloat16)
    hist_k, hist_v = mk(T + 2 * Nc, H, dd).to(d), mk(T + 2 * Nc, H, dd).to(d)
    steps = [(mk(Nc, H, dd).to(d), mk(Nc, H, dd).to(d), mk(Nc, H, dd).to(d)) for _ in range(4)]
    q, kc, vc = (torch.zeros(Nc, H, dd, dtype=torch.bfloat16, device=d) for _ in range(3))
    cache = df.Cache(torch.zeros(off[-1], dd, dtype=torch.bfloat16, device=d),
                     torch.zeros(off[-1], dd, dtype=torch.bfloat16, device=d), off, sink_cap, win_cap, dd)
    df.df_kv_append(cache, hist_k[:T], hist_v[:T])
    df.df_kv_append(cache, hist_k[T:T + Nc], hist_v[T:T + Nc])
    df.df_kv_append(cache, hist_k[T + Nc:], hist_v[T + Nc:])     # the ring is full from here on
    torch.cuda.synchronize()
    k0, v0 = cache.k_cache.clone(), cache.v_cache.clone()
    host0 = (list(cache.sink_len), list(cache.win_len), list(cache.win_pos))
    k_pack = torch.zeros(off[-1], dd, dtype=torch.bfloat16, device=d)
    v_pack = torch.zeros_like(k_pack)
    out = torch.zeros(Nc, H, dd, dtype=torch.bfloat16, device=d)
    F = torch.zeros(H, 3, dtype=torch.float32, device=d)
    ws = torch.empty(df.df_attn_workspace_bytes(H, dd, Nc), dtype=torch.uint8, device=d)

    def step():
        p_off, p_sl = df.df_pack_context(cache, sink_cap, win_cap, k_pack, v_pack)
        df.df_attn_fwd(q, kc, vc, k_pack, v_pack, p_off, p_sl, out, dd ** -0.5, score_out=F, workspace=ws)
        df.df_kv_append(cache, kc, vc)

    def restore():
        cache.k_cache.copy_(k0); cache.v_cache.copy_(v0)
        for h in range(H):
            cache.sink_len[h], cache.win_len[h], cache.win_pos[h] = host0[0][h], host0[1][h], host0[2][h]

    eager = []
    for qi, ki, vi in steps:                                   # the eager sequence
        q.copy_(qi); kc.copy_(ki); vc.copy_(vi)
        step()
        torch.cuda.synchronize()
        eager.append((out.clone(), F.clone(), cache.k_cache.clone(), cache.v_cache.clone()))
    assert list(cache.win_pos) == host0[2] and list(cache.win_len) == host0[1]   # four chunks = two turns of the ring
    assert not torch.equal(eager[0][0], eager[1][0])

    restore()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                              # warm-up on the capture stream (two steps: back in phase 0)
        step(); step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    restore()
    graphs = []
    for phase in range(2):                                     # capturing a step advances the host state to the next phase
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=side):
            step()
        graphs.append(gr)
    assert list(cache.win_pos) == host0[2]
    torch.cuda.synchronize()
    restore()
    for i, (qi, ki, vi) in enumerate(steps):
        q.copy_(qi); kc.copy_(ki); vc.copy_(vi)
        out.fill_(7.0); F.fill_(7.0)
        torch.cuda.synchronize()
        graphs[i % 2].replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager[i][0]), i
        assert torch.equal(F, eager[i][1]), i
        assert torch.equal(cache.k_cache, eager[i][2]) and torch.equal(cache.v_cache, eager[i][3]), i
