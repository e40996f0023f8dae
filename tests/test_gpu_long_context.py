"""Shapes of the rows marked "next": a 237-frame window for the neighbour heads (long-context
reallocation, Sec. 4.4) and a 1920x1088 chunk with 8160 tokens per frame (Sec. 4.3).  Outputs and
log-sum-exp on sampled rows against the oracle; the launch is the one a benchmark would time."""
import numpy as np
import pytest

from paper_2601_20499_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def df():
    from paper_2601_20499_amd import binding
    return binding


def check(df, w, n_rows, seed):
    out, score, lse = gu.run_attn(df, w)
    rows = gu.sample_rows(w.Nq, n_rows, seed=seed)
    ref, mass, ref_lse = gu.oracle_rows(w, rows=rows)
    gu.check_out(out[rows], ref, w.name)
    assert np.abs(lse[:, rows] - ref_lse).max() <= gu.LSE_ABS
    np.testing.assert_allclose(score.sum(1), 1.0, atol=1e-5)
    np.testing.assert_allclose(score, mass.mean(axis=1), atol=0.05)   # sampled rows against all rows: loose
    # the same rows on both sides: a launch on the sampled queries alone (all keys) to the score tolerance
    sub = gu.fused_score_on_rows(df, w, rows)
    print(f"{w.name}: fused F on the sampled rows, max err {np.abs(sub - mass.mean(axis=1)).max():.2e}", flush=True)
    np.testing.assert_allclose(sub, mass.mean(axis=1), atol=gu.F_ABS)
    return score


def test_neighbour_heads_with_a_237_frame_window(df):
    w = wl.long_context_layer()
    lens = sorted({w.visible_len(h) for h in range(w.H)})
    assert lens == [1560, 237 * 1560]                   # 369 720 keys of history for a neighbour head
    score = check(df, w, 24, seed=7)
    for h, t in enumerate(w.head_type):
        if t == wl.HEAD_SINK:
            assert score[h, 1] == 0.0
        else:
            assert score[h, 0] == 0.0


def test_1080p_chunk(df):
    w = wl.res1080p()
    assert w.Nq == 24480 and w.Nq % 256 != 0
    check(df, w, 24, seed=8)


def test_forty_heads_per_layer(df):
    """A layer of the 14B-class geometry (40 heads of width 128; the paper gives only the 1600-head
    total): every head type in one call, more heads than any other test, element-wise parity."""
    types = ([wl.HEAD_PACK_DUMMY] * 20 + [wl.HEAD_SINK] * 6 + [wl.HEAD_NEIGHBOR] * 10 + [wl.HEAD_FULL] * 3
             + [wl.HEAD_DUMMY])
    w = wl.small_ragged(77, H=40, d=128, T=90, hist_frames=6, types=types, planted=list(range(20)))
    out, score, lse = gu.run_attn(df, w)
    ref, mass, ref_lse = gu.oracle_rows(w)
    gu.check_out(out, ref, w.name)
    assert np.abs(lse - ref_lse).max() <= gu.LSE_ABS
    np.testing.assert_allclose(score, mass.mean(axis=1), atol=gu.F_ABS)
