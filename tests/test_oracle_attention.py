"""Pins for the oracle's attention and frame-attention-score functions (CPU only).

Each test checks oracle/df_oracle.py against something that is not the oracle:
pure-python brute force, closed forms, a library softmax-attention on the
special cases, and the structural identities of Eq. 2 / 5 / 8 / 3.
"""
import math

import numpy as np
import pytest
import torch

from oracle import df_oracle as orc


def _rand(rng, *shape):
    return rng.standard_normal(shape)


# ---------------------------------------------------------------- brute force
def _brute_head(q, kh, vh, kc, vc, n_sink, n_win, scale):
    """Python-float loops, keys enumerated one by one from the definition of the visible set."""
    Nq, d = len(q), len(q[0])
    Nh = len(kh)
    vis = []            # (region, k row, v row)
    for j in range(Nh):
        in_sink = j < n_sink
        in_win = (j >= Nh - n_win) and not in_sink
        if in_sink:
            vis.append((0, kh[j], vh[j]))
        elif in_win:
            vis.append((1, kh[j], vh[j]))
    for j in range(len(kc)):
        vis.append((2, kc[j], vc[j]))
    out = [[0.0] * d for _ in range(Nq)]
    mass = [[0.0] * 3 for _ in range(Nq)]
    for u in range(Nq):
        logits = [scale * sum(q[u][c] * kr[c] for c in range(d)) for (_, kr, _) in vis]
        mx = max(logits)
        w = [math.exp(s - mx) for s in logits]
        z = sum(w)
        for (r, _, vr), wi in zip(vis, w):
            a = wi / z
            mass[u][r] += a
            for c in range(d):
                out[u][c] += a * vr[c]
    return np.array(out), np.array(mass)


@pytest.mark.parametrize("Nq,Nh,Nc,d,n_sink,n_win", [
    (3, 7, 3, 4, 2, 3),     # sink + window with a gap of hidden tokens
    (2, 5, 4, 3, 2, 9),     # window would overlap the sink: union without duplicates
    (4, 6, 2, 5, 0, 4),     # neighbour-like: no sink
    (3, 6, 3, 2, 2, 0),     # sink-like: no window
    (5, 4, 5, 3, 0, 0),     # dummy: history invisible
    (2, 0, 3, 4, 3, 3),     # no history at all (first autoregressive step)
    (3, 3, 2, 2, 8, 1),     # sink capacity larger than the history
])
def test_head_attention_matches_brute_force(Nq, Nh, Nc, d, n_sink, n_win):
    rng = np.random.default_rng(Nq * 100 + Nh * 10 + Nc)
    q, kh, vh = _rand(rng, Nq, d), _rand(rng, Nh, d), _rand(rng, Nh, d)
    kc, vc = _rand(rng, Nc, d), _rand(rng, Nc, d)
    scale = 0.7
    out, mass, lse = orc.head_attention(q, kh, vh, kc, vc, n_sink, n_win, scale)
    bo, bm = _brute_head(q.tolist(), kh.tolist(), vh.tolist(), kc.tolist(), vc.tolist(), n_sink, n_win, scale)
    np.testing.assert_allclose(out, bo, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(mass, bm, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(mass.sum(axis=1), 1.0, rtol=0, atol=1e-13)


def test_config1_shape_brute_force_two_rows():
    """Config-1 geometry (64 tokens/frame, 3 past frames, d=64) on a few rows per head."""
    from paper_2601_20499_amd import workloads as wl
    w = wl.config1()
    rows = [0, 63]
    for h in range(w.H):
        q = w.q[rows, h].double().numpy()
        kh, vh = w.k_hist[:, h].double().numpy(), w.v_hist[:, h].double().numpy()
        kc, vc = w.k_cur[:, h].double().numpy(), w.v_cur[:, h].double().numpy()
        out, mass, _ = orc.head_attention(q, kh, vh, kc, vc, w.n_sink[h], w.n_win[h], w.scale)
        bo, bm = _brute_head(q.tolist(), kh.tolist(), vh.tolist(), kc.tolist(), vc.tolist(),
                             w.n_sink[h], w.n_win[h], w.scale)
        np.testing.assert_allclose(out, bo, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(mass, bm, rtol=1e-11, atol=1e-13)
        assert (w.visible_len(h) + w.Nc) == (64 if h == 3 else 256)


# ---------------------------------------------------------------- closed forms
def test_two_keys_is_a_sigmoid():
    # one query, d = 1, one history key and one current key: a_current = sigmoid(scale*q*(kc-kh))
    q, kh, kc, vh, vc, scale = 1.3, -0.4, 0.9, 2.0, -5.0, 0.5
    out, mass, lse = orc.head_attention([[q]], [[kh]], [[vh]], [[kc]], [[vc]], 1, 0, scale)
    sig = 1.0 / (1.0 + math.exp(-scale * q * (kc - kh)))
    assert mass[0, 2] == pytest.approx(sig, abs=1e-15)
    assert mass[0, 0] == pytest.approx(1 - sig, abs=1e-15)
    assert mass[0, 1] == 0.0
    assert out[0, 0] == pytest.approx(sig * vc + (1 - sig) * vh, abs=1e-14)
    assert lse[0] == pytest.approx(math.log(math.exp(scale * q * kh) + math.exp(scale * q * kc)), abs=1e-14)


def test_identical_keys_give_uniform_weights_and_count_ratios():
    rng = np.random.default_rng(3)
    d, Nh, Nc, Nq = 8, 40, 12, 5
    krow = _rand(rng, 1, d)
    kh, kc = np.repeat(krow, Nh, 0), np.repeat(krow, Nc, 0)
    vh, vc = _rand(rng, Nh, d), _rand(rng, Nc, d)
    q = _rand(rng, Nq, d)
    n_sink, n_win = 10, 17          # 13 history tokens hidden
    out, mass, _ = orc.head_attention(q, kh, vh, kc, vc, n_sink, n_win, 0.3)
    vis_v = np.concatenate([vh[:10], vh[Nh - 17:], vc])
    np.testing.assert_allclose(out, np.repeat(vis_v.mean(0, keepdims=True), Nq, 0), atol=1e-14)
    n = 10 + 17 + 12
    np.testing.assert_allclose(mass, np.repeat([[10 / n, 17 / n, 12 / n]], Nq, 0), atol=1e-15)
    F = orc.frame_attention_score(mass, 1, 2)
    np.testing.assert_allclose(F, [10 / n, 17 / n, 12 / n], atol=1e-15)


def test_zero_queries_and_constant_values():
    rng = np.random.default_rng(4)
    d = 6
    kh, vh, kc, vc = _rand(rng, 9, d), _rand(rng, 9, d), _rand(rng, 4, d), _rand(rng, 4, d)
    out, _, _ = orc.head_attention(np.zeros((3, d)), kh, vh, kc, vc, 9, 0, 1.0)
    np.testing.assert_allclose(out, np.repeat(np.concatenate([vh, vc]).mean(0, keepdims=True), 3, 0), atol=1e-14)
    const = np.full((9, d), 2.5), np.full((4, d), 2.5)
    out, _, _ = orc.head_attention(_rand(rng, 3, d), kh, const[0], kc, const[1], 3, 4, 1.0)
    np.testing.assert_allclose(out, 2.5, atol=1e-14)


def test_dominant_logit_selects_its_value_row():
    rng = np.random.default_rng(5)
    d = 4
    q = np.array([[1.0, 0, 0, 0]])
    kh = _rand(rng, 6, d) * 0.01
    kh[4] = [60.0, 0, 0, 0]                      # history token 4 dominates
    vh, kc, vc = _rand(rng, 6, d), _rand(rng, 3, d) * 0.01, _rand(rng, 3, d)
    out, mass, _ = orc.head_attention(q, kh, vh, kc, vc, 0, 3, 1.0)   # window = tokens 3,4,5
    np.testing.assert_allclose(out[0], vh[4], atol=1e-12)
    assert mass[0, 1] == pytest.approx(1.0, abs=1e-12)
    out, mass, _ = orc.head_attention(q, kh, vh, kc, vc, 2, 1, 1.0)   # token 4 hidden now
    assert mass[0, 1] < 0.5 and not np.allclose(out[0], vh[4])


# ---------------------------------------------------------------- invariances
def test_permutation_shift_and_split_merge_invariance():
    rng = np.random.default_rng(6)
    d, Nq, Nh, Nc = 5, 4, 11, 6
    q, kh, vh, kc, vc = (_rand(rng, Nq, d), _rand(rng, Nh, d), _rand(rng, Nh, d),
                         _rand(rng, Nc, d), _rand(rng, Nc, d))
    base, bmass, blse = orc.head_attention(q, kh, vh, kc, vc, 3, 5, 0.4)
    # joint permutation of K/V rows inside the window region and inside the current chunk
    ph = np.arange(Nh); ph[6:] = ph[6:][rng.permutation(5)]
    pc = rng.permutation(Nc)
    o2, m2, _ = orc.head_attention(q, kh[ph], vh[ph], kc[pc], vc[pc], 3, 5, 0.4)
    np.testing.assert_allclose(o2, base, atol=1e-14)
    np.testing.assert_allclose(m2, bmass, atol=1e-14)
    # adding one vector to every key shifts each row's logits by a constant
    delta = _rand(rng, 1, d)
    o3, m3, _ = orc.head_attention(q, kh + delta, vh, kc + delta, vc, 3, 5, 0.4)
    np.testing.assert_allclose(o3, base, atol=1e-13)
    np.testing.assert_allclose(m3, bmass, atol=1e-13)
    # attending to history and current separately and merging by log-sum-exp
    oh, _, lh = orc.head_attention(q, kh[:0], vh[:0], np.concatenate([kh[:3], kh[6:]]),
                                   np.concatenate([vh[:3], vh[6:]]), 0, 0, 0.4)
    oc, _, lc = orc.head_attention(q, kh[:0], vh[:0], kc, vc, 0, 0, 0.4)
    wh = 1 / (1 + np.exp(lc - lh))
    np.testing.assert_allclose(wh[:, None] * oh + (1 - wh)[:, None] * oc, base, atol=1e-13)
    np.testing.assert_allclose(1 - wh, bmass[:, 2], atol=1e-13)
    np.testing.assert_allclose(np.logaddexp(lh, lc), blse, atol=1e-13)


# ------------------------------------------- library cross-checks (special cases)
def _sdpa(q, k, v, scale, mask=None):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a))[None]
    return torch.nn.functional.scaled_dot_product_attention(
        t(q), t(k), t(v), attn_mask=None if mask is None else torch.from_numpy(mask)[None],
        scale=scale)[0].numpy()


def test_all_full_heads_equal_block_causal_attention():
    """Eq. 2 with a window that covers everything: rows of chunk i of a block-causal attention
    over the whole sequence (mask at chunk granularity)."""
    rng = np.random.default_rng(7)
    T, C, n_chunks, d = 5, 2, 4, 8
    N = T * C * n_chunks
    q, k, v = _rand(rng, N, d), _rand(rng, N, d), _rand(rng, N, d)
    chunk = np.arange(N) // (T * C)
    mask = chunk[:, None] >= chunk[None, :]
    ref = _sdpa(q, k, v, 0.35, mask)
    for i in range(n_chunks):
        lo, hi = i * T * C, (i + 1) * T * C
        out, _, _ = orc.head_attention(q[lo:hi], k[:lo], v[:lo], k[lo:hi], v[lo:hi], T, lo, 0.35)
        np.testing.assert_allclose(out, ref[lo:hi], atol=1e-12)


def test_sliding_window_types_against_masked_library_attention():
    """Single-frame steps: Eq. 2 (sink + L-1 neighbours + current), Eq. 5 (sink / neighbour /
    dummy) and Eq. 8 (packing frame i-1) as explicit frame masks over the full sequence."""
    rng = np.random.default_rng(8)
    T, n_frames, d, L = 4, 7, 6, 4              # window: 1 sink + (L-1)=3 neighbours
    N = T * n_frames
    q, k, v = _rand(rng, N, d), _rand(rng, N, d), _rand(rng, N, d)
    frame = np.arange(N) // T
    i = n_frames - 1                              # current frame
    rows = frame == i
    sink = frame == 0
    neigh = (frame >= i - (L - 1)) & (frame <= i - 1)
    cur = frame == i
    masks = {
        orc.HEAD_FULL: sink | neigh | cur,
        orc.HEAD_SINK: sink | cur,
        orc.HEAD_NEIGHBOR: neigh | cur,
        orc.HEAD_DUMMY: cur,
        orc.HEAD_PACK_DUMMY: (frame == i - 1) | cur,
    }
    for typ, keymask in masks.items():
        ref = _sdpa(q[rows], k, v, 0.5, np.repeat(keymask[None], T, 0))
        n_sink, n_win = orc.head_context_tokens(typ, T, 1, L - 1)
        out, mass, _ = orc.head_attention(q[rows], k[~cur], v[~cur], k[cur], v[cur], n_sink, n_win, 0.5)
        np.testing.assert_allclose(out, ref, atol=1e-12, err_msg=f"type {typ}")
        if typ == orc.HEAD_DUMMY:
            np.testing.assert_array_equal(mass[:, :2], 0.0)
            np.testing.assert_allclose(mass[:, 2], 1.0, rtol=0, atol=1e-15)
            np.testing.assert_allclose(out, _sdpa(q[rows], k[cur], v[cur], 0.5), atol=1e-12)


def test_frame_attention_score_index_sets():
    """Eq. 3 literally: A in R^{HW x (L+1)HW}, J_sink=[0,HW), J_neighbour=[HW,L*HW),
    J_current=[L*HW,(L+1)HW); sum over the columns of a region, mean over rows."""
    rng = np.random.default_rng(9)
    HW, L, d = 6, 3, 4
    q = _rand(rng, HW, d)
    keys = _rand(rng, (L + 1) * HW, d)
    vals = _rand(rng, (L + 1) * HW, d)
    A = torch.softmax(torch.from_numpy(0.6 * q @ keys.T), dim=1).numpy()
    alpha = [A[:, 0:HW].sum(1).mean(), A[:, HW:L * HW].sum(1).mean(), A[:, L * HW:].sum(1).mean()]
    _, mass, _ = orc.head_attention(q, keys[:L * HW], vals[:L * HW], keys[L * HW:], vals[L * HW:],
                                    HW, (L - 1) * HW, 0.6)
    F = orc.frame_attention_score(mass)
    np.testing.assert_allclose(F, alpha, atol=1e-14)
    assert F.sum() == pytest.approx(1.0, abs=1e-14)
    # sampled rows: every 4th query from offset 1
    Fs = orc.frame_attention_score(mass, 1, 4)
    np.testing.assert_allclose(Fs, [A[1::4, 0:HW].sum(1).mean(), A[1::4, HW:L * HW].sum(1).mean(),
                                    A[1::4, L * HW:].sum(1).mean()], atol=1e-14)


def test_attention_map_rows_and_lse():
    rng = np.random.default_rng(10)
    q, k = _rand(rng, 7, 5) * 3, _rand(rng, 13, 5) * 3
    A, lse = orc.attention_map(q, k, 0.9)
    np.testing.assert_allclose(A.sum(1), 1.0, atol=1e-14)
    assert (A >= 0).all()
    np.testing.assert_allclose(lse, torch.logsumexp(torch.from_numpy(0.9 * q @ k.T), 1).numpy(), atol=1e-13)
    # transposed operands or a sign error would break this asymmetric check
    s = 0.9 * q @ k.T
    np.testing.assert_allclose(np.log(A[2, 5] / A[2, 8]), s[2, 5] - s[2, 8], atol=1e-12)


def test_layer_attention_rows_subset():
    from paper_2601_20499_amd import workloads as wl
    w = wl.small_ragged(seed=11, H=3, d=64, T=9, hist_frames=4)
    kh = [w.k_hist[:, h].double().numpy() for h in range(w.H)]
    vh = [w.v_hist[:, h].double().numpy() for h in range(w.H)]
    args = (w.q.double().numpy(), kh, vh, w.k_cur.double().numpy(), w.v_cur.double().numpy(),
            w.n_sink, w.n_win, w.scale)
    full, fm, fl = orc.layer_attention(*args)
    rows = np.array([0, 5, 26])
    sub, sm, sl = orc.layer_attention(*args, rows=rows)
    np.testing.assert_array_equal(sub, full[rows])
    np.testing.assert_array_equal(sm, fm[:, rows])
    assert full.shape == (w.Nq, w.H, w.d) and fm.shape == (w.H, w.Nq, 3)


def test_planted_heads_put_most_mass_on_the_current_chunk():
    """The synthetic recipe reproduces Observation 1's signature on a reduced shape:
    planted heads put > 80% of their attention on the current chunk, the others
    split it roughly by key count."""
    from paper_2601_20499_amd import workloads as wl
    w = wl.small_ragged(seed=12, H=4, d=128, T=60, chunk_frames=3, hist_frames=6,
                        types=[wl.HEAD_FULL] * 4, planted=[1])
    for h in range(4):
        _, mass, _ = orc.head_attention(w.q[::7, h].double().numpy(), w.k_hist[:, h].double().numpy(),
                                        w.v_hist[:, h].double().numpy(), w.k_cur[:, h].double().numpy(),
                                        w.v_cur[:, h].double().numpy(), w.n_sink[h], w.n_win[h], w.scale)
        F = orc.frame_attention_score(mass)
        if h == 1:
            assert F[2] > 0.8
        else:
            np.testing.assert_allclose(F, [1 / 9, 5 / 9, 3 / 9], atol=0.06)


# ------------------------------------------- layer_attention: head slicing, pinned head by head
def _brute_lse(q, kh, kc, n_sink, n_win, scale):
    """log sum_v exp(scale q.k_v) over the visible keys, python floats, from the definition."""
    Nh = len(kh)
    keys = [kh[j] for j in range(Nh) if j < n_sink or j >= Nh - n_win] + list(kc)
    out = []
    for qu in q:
        logits = [scale * sum(a * b for a, b in zip(qu, kr)) for kr in keys]
        mx = max(logits)
        out.append(mx + math.log(sum(math.exp(s - mx) for s in logits)))
    return np.array(out)


def _distinct_heads_case():
    """Four heads that differ in everything layer_attention has to route per head: Q, K, V of the
    current chunk, history length and content, n_sink, n_win; head 2 has no history at all."""
    rng = np.random.default_rng(77)
    Nq, Nc, H, d = 5, 4, 4, 3
    q, kc, vc = _rand(rng, Nq, H, d), _rand(rng, Nc, H, d), _rand(rng, Nc, H, d)
    q *= np.array([0.5, 1.0, 2.0, 3.0])[None, :, None]          # heads differ in scale as well
    Nh = [7, 5, 0, 9]
    kh = [_rand(rng, n, d) for n in Nh]
    vh = [_rand(rng, n, d) + 3.0 * h for h, n in enumerate(Nh)]  # a per-head offset: a V mix-up cannot hide
    vc = vc + np.array([10.0, -10.0, 20.0, -20.0])[None, :, None]
    n_sink, n_win = [2, 0, 3, 4], [3, 4, 2, 0]
    return q, kh, vh, kc, vc, n_sink, n_win, 0.6


def _check_layer_against_brute(layer_fn):
    q, kh, vh, kc, vc, n_sink, n_win, scale = _distinct_heads_case()
    H = q.shape[1]
    for rows in (None, np.array([4, 0, 2])):
        out, mass, lse = layer_fn(q, kh, vh, kc, vc, n_sink, n_win, scale, rows=rows)
        sel = np.arange(q.shape[0]) if rows is None else rows
        assert out.shape == (len(sel), H, q.shape[2]) and mass.shape == (H, len(sel), 3) and lse.shape == (H, len(sel))
        for h in range(H):
            bo, bm = _brute_head(q[sel, h].tolist(), kh[h].tolist(), vh[h].tolist(), kc[:, h].tolist(),
                                 vc[:, h].tolist(), n_sink[h], n_win[h], scale)
            bl = _brute_lse(q[sel, h].tolist(), kh[h].tolist(), kc[:, h].tolist(), n_sink[h], n_win[h], scale)
            np.testing.assert_allclose(out[:, h], bo, rtol=1e-12, atol=1e-12, err_msg=f"out, head {h}")
            np.testing.assert_allclose(mass[h], bm, rtol=1e-12, atol=1e-13, err_msg=f"mass, head {h}")
            np.testing.assert_allclose(lse[h], bl, rtol=1e-12, atol=1e-12, err_msg=f"lse, head {h}")


def test_layer_attention_distinct_heads_against_brute_force():
    """layer_attention is what every GPU parity test calls: out, region masses and LSE of every
    head against the python-float brute force run head by head, with and without a row subset."""
    _check_layer_against_brute(orc.layer_attention)


@pytest.mark.parametrize("old,new", [
    ("np.asarray(v_cur)[:, h, :]", "np.asarray(v_cur)[:, 0, :]"),          # wrong head of V_cur
    ("np.asarray(k_cur)[:, h, :]", "np.asarray(k_cur)[:, (h + 1) % H, :]"),  # wrong head of K_cur
    ("v_hist_list[h]", "v_hist_list[min(h, 1)]"),                          # wrong head's cached values
    ("q[rows, h, :]", "q[rows, H - 1 - h, :]"),                            # wrong head of Q
    ("n_sink[h], n_win[h]", "n_win[h], n_sink[h]"),                        # sink / window swapped
])
def test_the_layer_pin_catches_planted_head_index_mistakes(old, new):
    """The pin above must fail on a scratch copy of the oracle with one routing mistake planted."""
    import inspect
    import types
    src = inspect.getsource(orc)
    assert src.count(old) == 1, old
    mutant = types.ModuleType("df_oracle_mutant")
    exec(compile(src.replace(old, new), "df_oracle_mutant", "exec"), mutant.__dict__)
    with pytest.raises((AssertionError, ValueError, IndexError)):
        _check_layer_against_brute(mutant.layer_attention)
