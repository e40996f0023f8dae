"""Bit-exact parity of df_kv_append / df_pack_context with the oracle's cache model, and the
append -> pack -> attention chain over several autoregressive steps."""
import numpy as np
import pytest
import torch

from oracle import df_oracle as orc
from paper_2601_20499_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def df():
    from paper_2601_20499_amd import binding
    return binding


def bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def make_cache(df, H, d, sink_cap, win_cap, slack=3):
    rows = [s + w + (slack if s + w else 0) for s, w in zip(sink_cap, win_cap)]
    off = np.concatenate([[0], np.cumsum(rows)]).tolist()
    k = torch.full((off[-1], d), -1.0, dtype=torch.bfloat16, device=gu.dev())
    v = torch.full((off[-1], d), -1.0, dtype=torch.bfloat16, device=gu.dev())
    return df.Cache(k, v, off, sink_cap, win_cap, d)


@pytest.mark.parametrize("d,head_major", [(128, False), (64, True)])
def test_append_and_pack_bit_exact(df, d, head_major):
    H, T = 6, 23
    sink_cap = [T, T, 0, 0, 0, 2 * T]
    win_cap = [5 * T, 0, 4 * T, 0, T, 70]                 # full, sink, neighbour, dummy, pack-dummy, odd sizes
    cache = make_cache(df, H, d, sink_cap, win_cap)
    model = orc.CacheModel(H, d, sink_cap, win_cap, dtype=np.uint16)
    g = torch.Generator().manual_seed(3)
    for step, Nc in enumerate([3 * T, 3 * T, 5, 1, 3 * T, 9 * T, 3 * T, 64, 200]):
        k_new = torch.randn(Nc, H, d, generator=g).to(torch.bfloat16)
        v_new = torch.randn(Nc, H, d, generator=g).to(torch.bfloat16)
        if head_major:
            kd = k_new.permute(1, 0, 2).contiguous().to(gu.dev()).permute(1, 0, 2)
            vd = v_new.permute(1, 0, 2).contiguous().to(gu.dev()).permute(1, 0, 2)
        else:
            kd, vd = k_new.to(gu.dev()), v_new.to(gu.dev())
        df.df_kv_append(cache, kd, vd)
        model.append(bits(k_new), bits(v_new))
        for h in range(H):
            assert cache.sink_len[h] == model.k_sink[h].shape[0]
            assert cache.win_len[h] == model.k_win[h].shape[0]
        for take_sink, take_win in [(sink_cap, win_cap), ([T] * H, [2 * T] * H), ([0, 7, 3, 0, 0, 1], [11, 0, 1, 5, 0, 70])]:
            Kp, Vp, off, sl = model.pack(take_sink, take_win)
            cap_rows = int(off[-1]) + 4
            k_out = torch.full((cap_rows, d), 9.0, dtype=torch.bfloat16, device=gu.dev())
            v_out = torch.full((cap_rows, d), 9.0, dtype=torch.bfloat16, device=gu.dev())
            g_off, g_sl = df.df_pack_context(cache, take_sink, take_win, k_out, v_out)
            torch.cuda.synchronize()
            assert g_off == off.tolist() and g_sl == sl.tolist(), (step, g_off, off)
            n = int(off[-1])
            assert np.array_equal(bits(k_out[:n]), Kp) and np.array_equal(bits(v_out[:n]), Vp), step
            assert (k_out[n:] == 9.0).all() and (v_out[n:] == 9.0).all()      # nothing written past the end
    # slack rows between heads were never touched
    kc = cache.k_cache.float().cpu().numpy()
    for h in range(H):
        lo = cache.head_row_off[h] + sink_cap[h] + win_cap[h]
        assert (kc[lo:cache.head_row_off[h + 1]] == -1.0).all()


def test_append_pack_attention_chain(df):
    """Four autoregressive steps of a small layer: attention with the packed context of the
    cache, then append of the chunk, against the oracle doing the same with plain arrays."""
    H, d, T, C = 4, 128, 40, 3
    types = [wl.HEAD_FULL, wl.HEAD_NEIGHBOR, wl.HEAD_DUMMY, wl.HEAD_PACK_DUMMY]
    L_minus_1 = 4
    ctx = [df.df_head_context(t, T, 1, L_minus_1) for t in types]
    sink_cap, win_cap = [c[0] for c in ctx], [c[1] for c in ctx]
    cache = make_cache(df, H, d, sink_cap, win_cap, slack=0)
    g = torch.Generator().manual_seed(9)
    hist_k = [np.zeros((0, d)) for _ in range(H)]
    hist_v = [np.zeros((0, d)) for _ in range(H)]
    scale = 1 / np.sqrt(d)
    cap_rows = sum(sink_cap) + sum(win_cap)
    k_out = torch.zeros(cap_rows, d, dtype=torch.bfloat16, device=gu.dev())
    v_out = torch.zeros(cap_rows, d, dtype=torch.bfloat16, device=gu.dev())
    ws = torch.empty(df.df_attn_workspace_bytes(H, d, C * T), dtype=torch.uint8, device=gu.dev())
    for step in range(4):
        q = (torch.randn(C * T, H, d, generator=g) + 0.3).to(torch.bfloat16)
        kc = torch.randn(C * T, H, d, generator=g).to(torch.bfloat16)
        vc = torch.randn(C * T, H, d, generator=g).to(torch.bfloat16)
        off, sl = df.df_pack_context(cache, sink_cap, win_cap, k_out, v_out)
        out = torch.empty(C * T, H, d, dtype=torch.bfloat16, device=gu.dev())
        df.df_attn_fwd(q.to(gu.dev()), kc.to(gu.dev()), vc.to(gu.dev()), k_out, v_out, off, sl, out, scale, workspace=ws)
        df.df_kv_append(cache, kc.to(gu.dev()), vc.to(gu.dev()))
        torch.cuda.synchronize()
        ref, _, _ = orc.layer_attention(q.double().numpy(), hist_k, hist_v, kc.double().numpy(), vc.double().numpy(),
                                        sink_cap, win_cap, scale)
        gu.check_out(out.float().cpu().double().numpy(), ref, f"chain step {step}")
        for h in range(H):          # the oracle keeps the full chronological history; visibility does the rest
            hist_k[h] = np.concatenate([hist_k[h], kc[:, h].double().numpy()])
            hist_v[h] = np.concatenate([hist_v[h], vc[:, h].double().numpy()])


def test_attention_reads_the_rolling_cache_in_place(df):
    """Six autoregressive steps (the window ring wraps twice): attention straight on the cache
    buffers (hist_len = filled rows per head, window keys in ring order) against the oracle, and
    against attention on the packed, chronologically ordered context; also the fused scores, whose
    sink / window split must not depend on the ring's rotation."""
    H, d, T, C = 5, 128, 33, 3
    types = [wl.HEAD_FULL, wl.HEAD_NEIGHBOR, wl.HEAD_DUMMY, wl.HEAD_PACK_DUMMY, wl.HEAD_SINK]
    ctx = [df.df_head_context(t, T, 1, 4) for t in types]
    sink_cap, win_cap = [c[0] for c in ctx], [c[1] for c in ctx]
    cache = make_cache(df, H, d, sink_cap, win_cap, slack=5)
    g = torch.Generator().manual_seed(10)
    hist_k = [np.zeros((0, d)) for _ in range(H)]
    hist_v = [np.zeros((0, d)) for _ in range(H)]
    scale = 1 / np.sqrt(d)
    cap_rows = sum(sink_cap) + sum(win_cap)
    k_out = torch.zeros(cap_rows, d, dtype=torch.bfloat16, device=gu.dev())
    v_out = torch.zeros(cap_rows, d, dtype=torch.bfloat16, device=gu.dev())
    ws = torch.empty(df.df_attn_workspace_bytes(H, d, C * T), dtype=torch.uint8, device=gu.dev())
    for step in range(6):
        q = (torch.randn(C * T, H, d, generator=g) + 0.3).to(torch.bfloat16).to(gu.dev())
        kc = torch.randn(C * T, H, d, generator=g).to(torch.bfloat16)
        vc = torch.randn(C * T, H, d, generator=g).to(torch.bfloat16)
        kcd, vcd = kc.to(gu.dev()), vc.to(gu.dev())
        out_a = torch.empty(C * T, H, d, dtype=torch.bfloat16, device=gu.dev())
        out_b = torch.empty_like(out_a)
        F_a = torch.empty(H, 3, dtype=torch.float32, device=gu.dev())
        F_b = torch.empty_like(F_a)
        kh, vh, off, sl, hl = cache.in_place()
        assert all(n <= off[h + 1] - off[h] for h, n in enumerate(hl))
        df.df_attn_fwd(q, kcd, vcd, kh, vh, off, sl, out_a, scale, score_out=F_a, workspace=ws, hist_len=hl)
        p_off, p_sl = df.df_pack_context(cache, sink_cap, win_cap, k_out, v_out)
        assert [p_off[h + 1] - p_off[h] for h in range(H)] == hl and p_sl == sl
        df.df_attn_fwd(q, kcd, vcd, k_out, v_out, p_off, p_sl, out_b, scale, score_out=F_b, workspace=ws)
        df.df_kv_append(cache, kcd, vcd)
        torch.cuda.synchronize()
        ref, mass, _ = orc.layer_attention(q.cpu().double().numpy(), hist_k, hist_v, kc.double().numpy(),
                                           vc.double().numpy(), sink_cap, win_cap, scale)
        a, b = out_a.float().cpu().double().numpy(), out_b.float().cpu().double().numpy()
        gu.check_out(a, ref, f"in place, step {step}")
        assert np.abs(a - b).max() <= 2 ** -6, np.abs(a - b).max()      # same keys in another order: a bf16 ulp or two
        np.testing.assert_allclose(F_a.cpu().numpy(), mass.mean(axis=1), atol=gu.F_ABS)
        np.testing.assert_allclose(F_a.cpu().numpy(), F_b.cpu().numpy(), atol=2e-5)
        for h in range(H):
            hist_k[h] = np.concatenate([hist_k[h], kc[:, h].double().numpy()])
            hist_v[h] = np.concatenate([hist_v[h], vc[:, h].double().numpy()])
