"""Parity of df_attn_fwd (through the C ABI) with the fp64 oracle on identical seeded inputs."""
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


def _full_parity(df, w, layout="thd"):
    out, score, lse = gu.run_attn(df, w, layout=layout)
    ref, mass, rlse = gu.oracle_rows(w)
    gu.check_out(out, ref, w.name)
    F = mass.mean(axis=1)
    assert np.abs(score - F).max() <= gu.F_ABS, (score, F)
    assert np.abs(score.sum(1) - 1).max() <= 1e-5
    assert np.abs(lse - rlse).max() <= gu.LSE_ABS
    return out, score


def test_config1_tiny(df):
    w = wl.config1()
    out, score = _full_parity(df, w)
    assert out.shape == (64, 4, 64)
    # the dummy head sees the current frame only: its score is exactly (0, 0, 1)
    np.testing.assert_array_equal(score[3], [0.0, 0.0, 1.0])
    # reported, not part of the bar: distance to the oracle run on the raw fp32 inputs
    w32 = wl.config1(fp32=True)
    ref32, _, _ = __import__("oracle.df_oracle", fromlist=["x"]).layer_attention(
        w32.q.double().numpy(), [w32.k_hist[:, h].double().numpy() for h in range(4)],
        [w32.v_hist[:, h].double().numpy() for h in range(4)], w32.k_cur.double().numpy(),
        w32.v_cur.double().numpy(), w32.n_sink, w32.n_win, w32.scale)
    print("config1 vs fp32-input oracle: max|err| = %.3e" % np.abs(out - ref32).max())


@pytest.mark.parametrize("seed,H,d,T,hist_frames,types", [
    (21, 3, 128, 97, 5, [wl.HEAD_FULL, wl.HEAD_DUMMY, wl.HEAD_NEIGHBOR]),       # 291 queries: ragged q tail, 8 key tiles
    (22, 5, 128, 37, 4, [wl.HEAD_FULL, wl.HEAD_SINK, wl.HEAD_NEIGHBOR, wl.HEAD_DUMMY, wl.HEAD_PACK_DUMMY]),
    (23, 4, 64, 50, 6, [wl.HEAD_SINK, wl.HEAD_PACK_DUMMY, wl.HEAD_FULL, wl.HEAD_DUMMY]),
    (24, 2, 64, 129, 3, [wl.HEAD_NEIGHBOR, wl.HEAD_FULL]),
    (25, 1, 128, 64, 2, [wl.HEAD_FULL]),                                         # everything a multiple of the tiles
    (26, 2, 128, 1, 3, [wl.HEAD_FULL, wl.HEAD_DUMMY]),                           # one token per frame
])
def test_small_ragged_all_head_types(df, seed, H, d, T, hist_frames, types):
    w = wl.small_ragged(seed, H=H, d=d, T=T, hist_frames=hist_frames, types=types, planted=[0])
    _full_parity(df, w)


def test_head_major_strides(df):
    w = wl.small_ragged(27, H=3, d=128, T=70, hist_frames=3)
    _full_parity(df, w, layout="htd")


def test_no_history_first_step(df):
    w = wl.small_ragged(28, H=3, d=128, T=45, hist_frames=0, types=[wl.HEAD_FULL, wl.HEAD_SINK, wl.HEAD_DUMMY])
    assert w.Nh == 0
    out, score = _full_parity(df, w)
    np.testing.assert_array_equal(score, np.repeat([[0.0, 0.0, 1.0]], 3, 0))


def test_structured_values_and_peaked_softmax(df):
    """Cases where the absolute tolerance bites: values with an O(1) per-head mean, and logits
    with a standard deviation of about 4 (a handful of keys carry each row)."""
    w = wl.small_ragged(29, H=2, d=128, T=80, hist_frames=4, types=[wl.HEAD_FULL, wl.HEAD_FULL])
    g = torch.Generator().manual_seed(5)
    shift = torch.randn(2, 128, generator=g)
    w.v_cur = (w.v_cur.float() + shift[None]).to(torch.bfloat16)
    w.v_hist = (w.v_hist.float() + shift[None]).to(torch.bfloat16)
    _full_parity(df, w)
    w2 = wl.small_ragged(30, H=2, d=128, T=80, hist_frames=4, types=[wl.HEAD_FULL, wl.HEAD_NEIGHBOR], q_mean_std=0.0)
    w2.scale = 4.0 / (128 ** 0.5)
    _full_parity(df, w2)


def test_bitwise_determinism_and_no_out_of_bounds_writes(df):
    w = wl.small_ragged(31, H=3, d=128, T=97, hist_frames=5)
    d = gu.dev()
    kp, vp, off, sl = wl.packed_history(w)
    q = w.q.to(d)
    pad = 5
    big = torch.full((w.Nq + 2 * pad, w.H, w.d), 7.0, dtype=torch.bfloat16, device=d)
    outs = []
    ws = torch.empty(df.df_attn_workspace_bytes(w.H, w.d, w.Nq), dtype=torch.uint8, device=d)
    for _ in range(2):
        big.fill_(7.0)
        ws.fill_(0xAB)
        df.df_attn_fwd(q, w.k_cur.to(d), w.v_cur.to(d), kp.to(d), vp.to(d), off, sl, big[pad:pad + w.Nq], w.scale,
                       workspace=ws)
        torch.cuda.synchronize()
        outs.append(big.clone())
    assert torch.equal(outs[0], outs[1])
    assert (outs[0][:pad] == 7.0).all() and (outs[0][pad + w.Nq:] == 7.0).all()


def _sampled_parity(df, w, n_rows, seed):
    out, score, _ = gu.run_attn(df, w, want_lse=False)
    rows = gu.sample_rows(w.Nq, n_rows, seed)
    ref, mass, _ = gu.oracle_rows(w, rows=rows)
    gu.check_out(out[rows], ref, w.name)
    # properties that hold at any size
    assert np.isfinite(out).all()
    assert np.abs(score.sum(1) - 1).max() <= 1e-5
    for h in range(w.H):
        if w.visible_len(h) == 0:
            np.testing.assert_array_equal(score[h], [0.0, 0.0, 1.0])
    # fused score with the same rows on both sides: a launch on the sampled queries alone, all keys
    sub = gu.fused_score_on_rows(df, w, rows)
    print(f"{w.name}: fused F on the sampled rows, max err {np.abs(sub - mass.mean(axis=1)).max():.2e}", flush=True)
    np.testing.assert_allclose(sub, mass.mean(axis=1), atol=gu.F_ABS)
    return out, score, rows, mass


def test_config2_wan_shape_every_row(df):
    """The headline workload against the oracle on all 4680 rows of all 12 heads: outputs, LSE and the
    fused frame attention scores (Eq. 3 over every query) to the same bars as the small cases."""
    w = wl.config2()
    assert w.attn_flop() == pytest.approx(336.4e9, rel=1e-3)
    out, score, lse = gu.run_attn(df, w)
    ref, mass, rlse = gu.oracle_rows(w)
    gu.check_out(out, ref, w.name)
    F = mass.mean(axis=1)
    print(f"config2 fused F max err {np.abs(score - F).max():.2e}, lse max err {np.abs(lse - rlse).max():.2e}", flush=True)
    assert np.abs(score - F).max() <= gu.F_ABS, (score, F)
    assert np.abs(lse - rlse).max() <= gu.LSE_ABS
    assert np.abs(score.sum(1) - 1).max() <= 1e-5
    # the recipe's bands: planted heads concentrate on the current chunk, the others split by key count
    for h in range(w.H):
        if h in w.planted:
            np.testing.assert_array_equal(score[h], [0.0, 0.0, 1.0])      # typed dummy: sees the chunk only
        else:
            np.testing.assert_allclose(F[h], [1 / 9, 5 / 9, 3 / 9], atol=0.03)


def test_config4_720p_sampled_rows(df):
    w = wl.config4()
    _sampled_parity(df, w, 96, seed=4)


def test_config5_long_context_sampled_rows(df):
    w = wl.config5()
    lens = sorted(w.visible_len(h) for h in range(w.H))
    assert lens[0] == 0 and lens[6] == 4680 and lens[-1] == 93600
    _sampled_parity(df, w, 64, seed=5)


def test_two_kernel_path_without_hand_over(df, monkeypatch):
    """DF_ATTN_HANDOVER=0 leaves the units that span boundaries cut to the second kernel instead of handing
    their partial sums from workgroup to workgroup.  Same pieces, same order of the same arithmetic: the
    two paths agree to the last bit, and both meet the oracle (multi-tile heads cut once and several times)."""
    w = wl.small_ragged(31, H=5, d=128, T=300, hist_frames=6,
                        types=[wl.HEAD_FULL, wl.HEAD_SINK, wl.HEAD_NEIGHBOR, wl.HEAD_DUMMY, wl.HEAD_FULL], planted=[0])
    plan = df.df_attn_plan(w.Nq, w.Nq, [w.visible_len(h) for h in range(w.H)])
    assert plan["n_teams"] > 2 and plan["cut_units"] > 0, plan
    out_a, score_a, lse_a = gu.run_attn(df, w)
    monkeypatch.setenv("DF_ATTN_HANDOVER", "0")
    out_b, score_b, lse_b = gu.run_attn(df, w)
    monkeypatch.delenv("DF_ATTN_HANDOVER")
    np.testing.assert_array_equal(out_a, out_b)
    np.testing.assert_array_equal(lse_a, lse_b)
    np.testing.assert_array_equal(score_a, score_b)
    ref, mass, rlse = gu.oracle_rows(w)
    gu.check_out(out_b, ref, w.name)
    assert np.abs(score_b - mass.mean(axis=1)).max() <= gu.F_ABS
    assert np.abs(lse_b - rlse).max() <= gu.LSE_ABS


def _direct(df, q, kc, vc, kh, vh, off, sl, scale, want_score=True):
    """df_attn_fwd on explicit tensors (queries and current keys may differ in number)."""
    d = gu.dev()
    H, dd = q.shape[1], q.shape[2]
    out = torch.full(q.shape, float("nan"), dtype=torch.bfloat16, device=d)
    score = torch.full((H, 3), float("nan"), dtype=torch.float32, device=d) if want_score else None
    ws = torch.empty(df.df_attn_workspace_bytes(H, dd, q.shape[0]), dtype=torch.uint8, device=d)
    df.df_attn_fwd(q.to(d), kc.to(d), vc.to(d), kh.to(d), vh.to(d), off, sl, out, scale, score_out=score, workspace=ws)
    torch.cuda.synchronize()
    return out.float().cpu().double().numpy(), (None if score is None else score.cpu().double().numpy())


def _oracle_direct(q, kc, vc, kh_list, vh_list, n_sink, n_win, scale, rows=None):
    from oracle import df_oracle as orc
    b = lambda t: t.double().numpy()
    return orc.layer_attention(b(q), [b(x) for x in kh_list], [b(x) for x in vh_list], b(kc), b(vc),
                               n_sink, n_win, scale, rows=rows)


def test_more_query_tiles_than_compute_units(df):
    """65 797 queries = 258 query tiles > 256 CUs: a team then passes over the query tiles in rounds.
    Few keys (30 of history, 40 current), so the oracle covers every row."""
    g = torch.Generator().manual_seed(21)
    Nq, Nc, Nh, H, d = 256 * 257 + 5, 40, 30, 2, 64
    mk = lambda *s: torch.randn(*s, generator=g).to(torch.bfloat16)
    q, kc, vc = mk(Nq, H, d), mk(Nc, H, d), mk(Nc, H, d)
    kh, vh = mk(Nh, H, d), mk(Nh, H, d)
    # head 0 sees 10 sink + 20 window keys, head 1 nothing but the current keys
    k_p, v_p = kh[:, 0].contiguous(), vh[:, 0].contiguous()
    out, score = _direct(df, q, kc, vc, k_p, v_p, [0, Nh, Nh], [10, 0], d ** -0.5)
    ref, mass, _ = _oracle_direct(q, kc, vc, [kh[:, 0], kh[:, 1]], [vh[:, 0], vh[:, 1]], [10, 0], [20, 0], d ** -0.5)
    gu.check_out(out, ref, "258 query tiles")
    np.testing.assert_allclose(score, mass.mean(axis=1), atol=gu.F_ABS)


def test_sixty_four_heads_and_a_single_query(df):
    """The most heads a call takes (DF_MAX_HEADS) and the fewest queries and current keys (one each)."""
    g = torch.Generator().manual_seed(22)
    H, d, Nh = 64, 128, 70
    mk = lambda *s: torch.randn(*s, generator=g).to(torch.bfloat16)
    q, kc, vc = mk(1, H, d), mk(1, H, d), mk(1, H, d)
    kh, vh = mk(Nh, H, d), mk(Nh, H, d)
    lens = [(h * 7) % (Nh + 1) for h in range(H)]            # 0 .. 70 keys of history, odd lengths
    sinks = [min(n, h % 5) for h, n in enumerate(lens)]
    off = [0]
    for n in lens:
        off.append(off[-1] + n)
    # head h keeps its first sinks[h] rows and its last lens[h]-sinks[h] rows
    rows = [torch.cat([torch.arange(0, s), torch.arange(Nh - (n - s), Nh)]) for n, s in zip(lens, sinks)]
    k_p = torch.cat([kh[r, h] for h, r in enumerate(rows)])
    v_p = torch.cat([vh[r, h] for h, r in enumerate(rows)])
    out, score = _direct(df, q, kc, vc, k_p, v_p, off, sinks, d ** -0.5)
    ref, mass, _ = _oracle_direct(q, kc, vc, [kh[:, h] for h in range(H)], [vh[:, h] for h in range(H)],
                                  sinks, [n - s for n, s in zip(lens, sinks)], d ** -0.5)
    gu.check_out(out, ref, "64 heads, one query")
    np.testing.assert_allclose(score, mass.mean(axis=1), atol=gu.F_ABS)
    with pytest.raises(df.DfError) as e:                       # one head more is refused, nothing launched
        q65 = mk(1, 65, d)
        _direct(df, q65, q65, q65, k_p, v_p, off + [off[-1]], sinks + [0], d ** -0.5)
    assert e.value.status == df.DF_ERR_UNSUPPORTED


def _random_case(rng):
    """A seeded random head mix: any number of heads, empty to multi-tile histories with any sink split, query
    and current-key counts that are multiples of nothing, either head dimension."""
    H = int(rng.choice([1, 2, 3, 5, 8, 12]))
    d = int(rng.choice([64, 128]))
    Nq = int(rng.choice([1, 31, 257, 700, 1283, 2049]))
    Nc = int(rng.choice([1, 63, 65, 300, Nq]))
    lens = [int(rng.choice([0, 0, 1, 64, 65, 130, 777, 2500])) for _ in range(H)]
    sinks = [int(rng.integers(0, n + 1)) for n in lens]
    return H, d, Nq, Nc, lens, sinks


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_against_the_oracle(df, seed):
    rng = np.random.default_rng(3000 + seed)
    H, d, Nq, Nc, lens, sinks = _random_case(rng)
    g = torch.Generator().manual_seed(3000 + seed)
    mk = lambda *s: torch.randn(*s, generator=g).to(torch.bfloat16)
    q, kc, vc = mk(Nq, H, d) + 0.25, mk(Nc, H, d), mk(Nc, H, d)
    q = q.to(torch.bfloat16)
    kh = [mk(n, d) for n in lens]
    vh = [mk(n, d) for n in lens]
    off = [0]
    for n in lens:
        off.append(off[-1] + n)
    k_p = torch.cat(kh) if off[-1] else torch.zeros(0, d, dtype=torch.bfloat16)
    v_p = torch.cat(vh) if off[-1] else torch.zeros(0, d, dtype=torch.bfloat16)
    print(f"seed {seed}: H={H} d={d} Nq={Nq} Nc={Nc} lens={lens} sinks={sinks} plan={df.df_attn_plan(Nq, Nc, lens, sinks)}",
          flush=True)
    out, score = _direct(df, q, kc, vc, k_p, v_p, off, sinks, d ** -0.5)
    # the packed rows of a head are its sink rows followed by its window rows: the oracle sees them as a history
    # of exactly that length with n_sink sink keys and the rest as window
    ref, mass, _ = _oracle_direct(q, kc, vc, kh, vh, sinks, [n - s for n, s in zip(lens, sinks)], d ** -0.5)
    gu.check_out(out, ref, f"random shape {seed}")
    np.testing.assert_allclose(score, mass.mean(axis=1), atol=gu.F_ABS)


def test_query_tiles_in_several_groups_with_cut_units(df):
    """43 query tiles on 256 workgroup slots run as teams of 15 in 3 groups; with short histories of unequal
    length the spans cut units in every group.  Every row against the oracle."""
    g = torch.Generator().manual_seed(43)
    H, d, Nq, Nc = 4, 64, 256 * 42 + 100, 200
    lens, sinks = [2000, 900, 0, 1300], [64, 0, 0, 1300]
    plan = df.df_attn_plan(Nq, Nc, lens, sinks)
    assert plan["n_groups"] > 1 and plan["takes"] > 0 and plan["consistent"] == 1, plan
    mk = lambda *s: torch.randn(*s, generator=g).to(torch.bfloat16)
    q, kc, vc = mk(Nq, H, d), mk(Nc, H, d), mk(Nc, H, d)
    kh, vh = [mk(n, d) for n in lens], [mk(n, d) for n in lens]
    off = [0]
    for n in lens:
        off.append(off[-1] + n)
    out, score = _direct(df, q, kc, vc, torch.cat(kh), torch.cat(vh), off, sinks, d ** -0.5)
    ref, mass, _ = _oracle_direct(q, kc, vc, kh, vh, sinks, [n - s for n, s in zip(lens, sinks)], d ** -0.5)
    gu.check_out(out, ref, "43 query tiles in 3 groups")
    np.testing.assert_allclose(score, mass.mean(axis=1), atol=gu.F_ABS)
