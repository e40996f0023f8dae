"""The paper's full method on a seeded 30-layer stack (Sec. 3.3, Eq. 5-8): sink / neighbour /
dummy heads, half of the 360 heads dummy, one global classification.  CPU only: pins the oracle's
classification and the stand-in workload against what the paper's equations fix."""
import numpy as np

from oracle import df_oracle as orc
from paper_2601_20499_amd import workloads as wl
from tests import gpu_util as gu

LAYERS, N_DUMMY = 30, 180


def stack_scores(T=24, d=128):
    F, roles = [], []
    for layer in range(LAYERS):
        w = wl.dhp3_layer(layer, T=T, d=d)
        _, mass, _ = gu.oracle_rows(w)
        F.append(mass.mean(axis=1))
        roles += w.roles
    return np.concatenate(F), roles


def test_roles_show_in_the_frame_attention_scores():
    F, roles = stack_scores()
    assert F.shape == (360, 3)
    np.testing.assert_allclose(F.sum(1), 1.0, atol=1e-12)           # the three regions partition the keys (Eq. 3)
    by = lambda r: F[[i for i, x in enumerate(roles) if x == r]]
    assert by("current")[:, 2].min() > 0.5 and by("current")[:, 2].mean() > 0.75
    assert by("sink")[:, 0].min() > 0.3 and by("sink")[:, 0].mean() > 0.55
    assert (by("sink")[:, 0] > by("sink")[:, 1]).all()
    # un-planted Gaussian heads spread over the keys: mass ~ share of keys (1, 5, 3 frames of 9)
    nb = by("neighbor")
    assert abs(nb[:, 0].mean() - 1 / 9) < 0.03 and nb[:, 1].mean() > 0.4


def test_global_dhp_classification_is_optimal_and_follows_the_roles():
    F, roles = stack_scores()
    types, key = orc.classify(F, N_DUMMY, orc.MODE_DHP)
    assert (types == orc.HEAD_DUMMY).sum() == N_DUMMY
    np.testing.assert_array_equal(key, np.maximum(F[:, 0], F[:, 1]))
    # value of the greedy assignment = closed form of App. A
    dummy = types == orc.HEAD_DUMMY
    v_star = np.maximum(F[:, 0], F[:, 1])[~dummy].sum() + F[:, 2].sum()
    assert abs(orc.dhp_value(F, types) - v_star) < 1e-12
    # exchange argument: no swap of one dummy with one non-dummy head (re-typed at its best) gains
    best = np.maximum(F[:, 0], F[:, 1])
    assert best[dummy].max() <= best[~dummy].min() + 1e-15
    # non-dummy heads take the larger of their two history masses
    for h in np.flatnonzero(~dummy):
        assert types[h] == (orc.HEAD_SINK if F[h, 0] >= F[h, 1] else orc.HEAD_NEIGHBOR)
    # planted roles: strong current-leaning heads end up dummy, sink-planted non-dummy heads are sink heads
    cur = np.array([r == "current" for r in roles])
    assert dummy[cur].mean() > 0.95
    snk = np.array([r == "sink" for r in roles])
    assert (types[snk & ~dummy] == orc.HEAD_SINK).all()
    nbr = np.array([r == "neighbor" for r in roles])
    assert (types[nbr & ~dummy] == orc.HEAD_NEIGHBOR).all()


def test_cache_kept_by_the_full_method():
    """Half of the heads keep one packing frame, the others 1 sink or L-1 neighbour frames
    (Eq. 5, Eq. 8): cached frames per head over the 6-frame baseline window, for a given split."""
    frames = [1] * 3 + [5] * 3 + [1] * 6          # 3 sink heads, 3 neighbour heads, 6 packed dummy heads
    assert abs(orc.cache_kept_fraction(frames, 6) - (3 * 1 + 3 * 5 + 6 * 1) / (12 * 6)) < 1e-12
    # and the token counts the head types resolve to
    T = 1560
    assert orc.head_context_tokens(orc.HEAD_SINK, T, 1, 5) == (T, 0)
    assert orc.head_context_tokens(orc.HEAD_NEIGHBOR, T, 1, 5) == (0, 5 * T)
    assert orc.head_context_tokens(orc.HEAD_PACK_DUMMY, T, 1, 5) == (0, T)
