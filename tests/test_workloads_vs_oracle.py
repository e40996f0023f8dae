"""The input generator's bookkeeping against the oracle and the library (CPU only).

paper_2601_20499_amd/workloads.py draws tensors and also states, per head type, how many sink and
window tokens a head sees and which history rows that selects; both the oracle's arguments and
the packed history the GPU receives come from it.  These tests tie that bookkeeping to the
oracle's own statement of Eq. 2 / 5 / 8 and of the sliding window (Sec. 3.1), and to the
library's df_head_context, so that a mistake in the generator cannot hide from parity."""
import numpy as np
import pytest
import torch

from oracle import df_oracle as orc
from paper_2601_20499_amd import workloads as wl

GEOMETRIES = [(1560, 1, 5), (3600, 1, 11), (64, 1, 2), (37, 1, 4), (1, 1, 2), (97, 2, 3), (50, 0, 6), (8160, 1, 236)]


@pytest.fixture(scope="module")
def b():
    from paper_2601_20499_amd import binding
    return binding


@pytest.mark.parametrize("T,S,W", GEOMETRIES)
def test_context_table_generator_oracle_library(b, T, S, W):
    for t in (wl.HEAD_FULL, wl.HEAD_SINK, wl.HEAD_NEIGHBOR, wl.HEAD_DUMMY, wl.HEAD_PACK_DUMMY):
        ref = orc.head_context_tokens(t, T, S, W)
        assert wl._context(t, T, S, W) == ref, (t, T, S, W)
        assert tuple(b.df_head_context(t, T, S, W)) == ref, (t, T, S, W)
    assert (wl.HEAD_FULL, wl.HEAD_SINK, wl.HEAD_NEIGHBOR, wl.HEAD_DUMMY, wl.HEAD_PACK_DUMMY) == \
           (orc.HEAD_FULL, orc.HEAD_SINK, orc.HEAD_NEIGHBOR, orc.HEAD_DUMMY, orc.HEAD_PACK_DUMMY) == \
           (b.DF_HEAD_FULL, b.DF_HEAD_SINK, b.DF_HEAD_NEIGHBOR, b.DF_HEAD_DUMMY, b.DF_HEAD_PACK_DUMMY)


def _token_id_workload(H, d, T, chunk_frames, hist_frames, types, sink_frames=1):
    """A workload whose history rows carry their own (row, head) identity instead of random values."""
    w = wl._typed("ids", H, d, T, chunk_frames, hist_frames, types, seed=0, sink_frames=sink_frames)
    ids = torch.arange(w.Nh * H, dtype=torch.float32).reshape(w.Nh, H, 1).expand(w.Nh, H, d).contiguous()
    w.k_hist, w.v_hist = ids.clone(), -ids.clone()
    w.q = torch.zeros(w.Nq, H, d)
    return w


@pytest.mark.parametrize("T,chunk,hist,sink", [(5, 3, 7, 1), (3, 2, 1, 1), (4, 1, 0, 1), (7, 3, 4, 2), (2, 2, 9, 0), (6, 1, 2, 3)])
def test_packed_history_rows_are_the_oracles_visible_set(T, chunk, hist, sink):
    types = [wl.HEAD_FULL, wl.HEAD_SINK, wl.HEAD_NEIGHBOR, wl.HEAD_DUMMY, wl.HEAD_PACK_DUMMY]
    w = _token_id_workload(len(types), 2, T, chunk, hist, types, sink_frames=sink)
    kp, vp, off, sl = wl.packed_history(w)
    assert off[0] == 0 and len(off) == w.H + 1 and len(sl) == w.H
    for h, t in enumerate(types):
        n_sink, n_win = orc.head_context_tokens(t, T, w.sink_frames, w.hist_frames - w.sink_frames)
        assert (w.n_sink[h], w.n_win[h]) == (n_sink, n_win)
        s_idx, w_idx = orc.visible_history(w.Nh, n_sink, n_win)
        want = np.concatenate([s_idx, w_idx])
        assert wl.visible_history_rows(w, h).tolist() == want.tolist()
        assert w.visible_len(h) == len(want) == off[h + 1] - off[h]
        assert sl[h] == len(s_idx)
        got = kp[off[h]:off[h + 1], 0].long().tolist()
        assert got == [int(r) * w.H + h for r in want]                       # the right rows of the right head
        assert (vp[off[h]:off[h + 1], 0].long() == -kp[off[h]:off[h + 1], 0].long()).all()


def test_named_workloads_use_the_oracles_contexts():
    """Every named workload's per-head (n_sink, n_win) is the oracle's value for its head type
    (config 5 and the long-context layers override the window on purpose: checked separately)."""
    for w in (wl._typed("c2", 12, 128, 1560, 3, 6, [wl.HEAD_DUMMY if h in (2, 5, 9) else wl.HEAD_FULL for h in range(12)], 1),
              wl._typed("c4", 12, 128, 3600, 3, 12, [wl.HEAD_DUMMY if h in (0, 6, 7) else wl.HEAD_FULL for h in range(12)], 3),
              wl._typed("c3", 12, 128, 1560, 3, 21, [wl.HEAD_FULL] * 12, 2)):
        for h, t in enumerate(w.head_type):
            assert (w.n_sink[h], w.n_win[h]) == orc.head_context_tokens(t, w.T, w.sink_frames, w.hist_frames - w.sink_frames)
    full2 = sum(orc.head_context_tokens(orc.HEAD_FULL, 1560, 1, 5)) + 3 * 1560
    assert full2 == 14040
    assert sum(orc.head_context_tokens(orc.HEAD_FULL, 1560, 1, 20)) == 32760
    assert sum(orc.head_context_tokens(orc.HEAD_FULL, 3600, 1, 11)) == 43200
