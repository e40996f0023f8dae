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
