"""The paper's full method through the C ABI (Sec. 3.3): scores of every head of a 30-layer stack,
one global Dynamic Head Programming classification with half of the heads dummy (Eq. 6-7), then
attention with sink / neighbour / packed-dummy contexts (Eq. 5, Eq. 8), all against the oracle."""
import numpy as np
import pytest

from oracle import df_oracle as orc
from paper_2601_20499_amd import workloads as wl
from tests import gpu_util as gu
from tests.test_gpu_score import gpu_scores, oracle_scores, TAU

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def df():
    from paper_2601_20499_amd import binding
    return binding


def apply_types(df, w, types):
    """Head types -> visible contexts; dummy heads keep one packing frame (Eq. 8)."""
    for h, t in enumerate(types):
        t = df.DF_HEAD_PACK_DUMMY if t == df.DF_HEAD_DUMMY else int(t)
        w.head_type[h] = t
        w.n_sink[h], w.n_win[h] = df.df_head_context(t, w.T, w.sink_frames, w.hist_frames - w.sink_frames)


def test_global_classification_of_a_30_layer_stack(df):
    """360 heads at a reduced frame size (40 tokens per frame: queries and keys are multiples of no
    tile): scores of all layers to 1e-4, then one sort over all 360 heads."""
    F, R = [], []
    for layer in range(30):
        w = wl.dhp3_layer(layer, T=40)
        F.append(gpu_scores(df, w, q_stride=4))
        R.append(oracle_scores(w, q_stride=4))
    F, R = np.concatenate(F), np.concatenate(R)
    assert np.abs(F - R).max() <= gu.F_ABS, np.abs(F - R).max()
    N = 180
    types, key_gpu = df.df_classify(F.tolist(), N, df.DF_CLASSIFY_DHP)
    o_types, key = orc.classify(R, N, orc.MODE_DHP)
    srt = np.sort(key)
    margin = srt[N] - srt[N - 1]
    types = np.asarray(types)
    assert (types == df.DF_HEAD_DUMMY).sum() == N
    # heads whose key is clear of the dummy boundary and whose two history masses are clear of each
    # other must agree exactly; closer than TAU either result is correct
    clear = (np.abs(key - 0.5 * (srt[N] + srt[N - 1])) >= TAU) & (np.abs(R[:, 0] - R[:, 1]) >= TAU)
    print(f"margin at the dummy boundary {margin:.3e}, {int((~clear).sum())} heads within tau", flush=True)
    assert (types[clear] == o_types[clear]).all()
    if margin >= TAU and clear.all():
        assert types.tolist() == o_types.tolist()
    np.testing.assert_allclose(np.asarray(key_gpu), key, atol=gu.F_ABS)


@pytest.mark.parametrize("layer", [3, 11])
def test_full_size_layer_with_three_head_types(df, layer):
    """Wan-1.3B-shaped layer: scores on the 25 % query sample, Dynamic Head Programming with half of
    the layer's heads dummy, attention with the resulting contexts on sampled rows."""
    w = wl.dhp3_layer(layer)
    F = gpu_scores(df, w)
    R = oracle_scores(w)
    assert np.abs(F - R).max() <= gu.F_ABS, np.abs(F - R).max()
    types, _ = df.df_classify(F.tolist(), 6, df.DF_CLASSIFY_DHP)
    o_types, key = orc.classify(R, 6, orc.MODE_DHP)
    srt = np.sort(key)
    if srt[6] - srt[5] >= TAU and (np.abs(R[:, 0] - R[:, 1]) >= TAU).all():
        assert list(types) == o_types.tolist()
    print(f"layer {layer}: roles {w.roles} -> types {list(types)}", flush=True)
    apply_types(df, w, types)
    assert {df.DF_HEAD_PACK_DUMMY} <= set(w.head_type) and len(set(w.head_type)) >= 2
    out, score, lse = gu.run_attn(df, w)
    ref, mass, ref_lse = gu.oracle_rows(w)                      # every row: the fused score is a mean over all of them
    gu.check_out(out, ref, w.name)
    assert np.abs(lse - ref_lse).max() <= gu.LSE_ABS
    # fused scores are under each head's own visibility: a sink head has no neighbour mass and
    # the other way round
    for h, t in enumerate(w.head_type):
        if t == df.DF_HEAD_SINK:
            assert score[h, 1] == 0.0
        if t in (df.DF_HEAD_NEIGHBOR, df.DF_HEAD_PACK_DUMMY):
            assert score[h, 0] == 0.0
    np.testing.assert_allclose(score.sum(1), 1.0, atol=1e-5)
    print(f"layer {layer}: fused F max err {np.abs(score - mass.mean(axis=1)).max():.2e}", flush=True)
    np.testing.assert_allclose(score, mass.mean(axis=1), atol=gu.F_ABS)
