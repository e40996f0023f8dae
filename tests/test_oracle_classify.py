"""Pins for the oracle's head classification (Observation 1; Eq. 6-7, greedy rule, App. A)."""
import itertools

import numpy as np
import pytest

from oracle import df_oracle as orc


def _random_F(rng, n):
    F = rng.random((n, 3)) + 0.01
    return F / F.sum(1, keepdims=True)


@pytest.mark.parametrize("n,N", [(1, 0), (1, 1), (4, 2), (6, 3), (7, 2), (7, 7), (8, 4)])
def test_greedy_reaches_the_exhaustive_optimum(n, N):
    """Every assignment in {sink, neighbour, dummy}^n with exactly N dummies is enumerated;
    the greedy rule must reach the maximum of Eq. 6, and that maximum must equal the closed
    form V* = sum_{h not dummy} max(F_h0, F_h1) + sum_h F_h2 of the optimality proof."""
    rng = np.random.default_rng(100 + 10 * n + N)
    for _ in range(5):
        F = _random_F(rng, n)
        best = -1.0
        for assign in itertools.product((orc.HEAD_SINK, orc.HEAD_NEIGHBOR, orc.HEAD_DUMMY), repeat=n):
            if sum(c == orc.HEAD_DUMMY for c in assign) != N:
                continue
            val = 0.0
            for h, c in enumerate(assign):     # Eq. 7 retyped
                val += F[h, 2] + (F[h, 0] if c == orc.HEAD_SINK else F[h, 1] if c == orc.HEAD_NEIGHBOR else 0.0)
            best = max(best, val)
        types, key = orc.classify(F, N, orc.MODE_DHP)
        assert (types == orc.HEAD_DUMMY).sum() == N
        got = orc.dhp_value(F, types)
        assert got == pytest.approx(best, abs=1e-12)
        closed = sum(max(F[h, 0], F[h, 1]) for h in range(n) if types[h] != orc.HEAD_DUMMY) + F[:, 2].sum()
        assert got == pytest.approx(closed, abs=1e-12)


def test_greedy_rule_by_hand():
    # l = max(F0, F1): heads 0..4 -> .5, .1, .45, .3, .3 ; N=2 smallest: head 1 (.1) and head 3 (.3, lower index wins the tie with head 4)
    F = np.array([[0.5, 0.2, 0.3],
                  [0.1, 0.05, 0.85],
                  [0.2, 0.45, 0.35],
                  [0.3, 0.3, 0.4],
                  [0.1, 0.3, 0.6]])
    types, key = orc.classify(F, 2, orc.MODE_DHP)
    assert types.tolist() == [orc.HEAD_SINK, orc.HEAD_DUMMY, orc.HEAD_NEIGHBOR, orc.HEAD_DUMMY, orc.HEAD_NEIGHBOR]
    np.testing.assert_allclose(key, [0.5, 0.1, 0.45, 0.3, 0.3])
    # F_h0 == F_h1 on a kept head -> sink (">=" in the rule)
    types, _ = orc.classify(F, 1, orc.MODE_DHP)
    assert types[3] == orc.HEAD_SINK


def test_two_class_is_top_n_alpha_current():
    rng = np.random.default_rng(5)
    for n, N in [(12, 3), (12, 6), (360, 90)]:
        F = _random_F(rng, n)
        types, key = orc.classify(F, N, orc.MODE_TWO_CLASS)
        top = set(np.argsort(-F[:, 2], kind="stable")[:N].tolist())
        assert set(np.flatnonzero(types == orc.HEAD_DUMMY).tolist()) == top
        assert set(np.unique(types).tolist()) <= {orc.HEAD_FULL, orc.HEAD_DUMMY}
        np.testing.assert_allclose(key, 1.0 - F[:, 2], atol=1e-15)


def test_degenerate_counts_and_errors():
    F = _random_F(np.random.default_rng(6), 5)
    assert (orc.classify(F, 0, orc.MODE_DHP)[0] != orc.HEAD_DUMMY).all()
    assert (orc.classify(F, 5, orc.MODE_DHP)[0] == orc.HEAD_DUMMY).all()
    with pytest.raises(ValueError):
        orc.classify(F, 6, orc.MODE_DHP)
    with pytest.raises(ValueError):
        orc.dhp_value(F, [orc.HEAD_FULL] * 5)
