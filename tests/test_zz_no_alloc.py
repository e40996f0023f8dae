"""df_attn_fwd_static (the entry point that allocates nothing) against df_attn_fwd, through the C ABI:
same kernels on the library's static device scratch instead of a caller workspace, so outputs, LSE and
scores must agree bit for bit; two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared scratch is seen not to matter."""
import pytest
import torch

from paper_2601_20499_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def df():
    from paper_2601_20499_amd import binding
    return binding


def _both(df, w):
    d = gu.dev()
    kp, vp, off, sl = wl.packed_history(w)
    q, kc, vc, kp, vp = (t.to(d) for t in (w.q, w.k_cur, w.v_cur, kp, vp))
    res = []
    for static in (False, True):
        out = torch.full_like(q, float("nan"))
        lse = torch.full((w.H, w.Nq), float("nan"), dtype=torch.float32, device=d)
        score = torch.full((w.H, 3), float("nan"), dtype=torch.float32, device=d)
        if static:
            df.df_attn_fwd_static(q, kc, vc, kp, vp, off, sl, out, w.scale, lse_out=lse, score_out=score)
        else:
            ws = torch.empty(df.df_attn_workspace_bytes(w.H, w.d, w.Nq), dtype=torch.uint8, device=d).fill_(0x5A)
            df.df_attn_fwd(q, kc, vc, kp, vp, off, sl, out, w.scale, lse_out=lse, score_out=score, workspace=ws)
        torch.cuda.synchronize()
        res.append((out, lse, score))
    for a, b in zip(*res):
        assert torch.isfinite(a.float()).all()
        assert torch.equal(a, b)


def test_static_scratch_matches_workspace_call_twice_in_a_row(df):
    # first a launch whose heads are cut by many span boundaries (partial results fill the scratch) ...
    _both(df, wl.small_ragged(91, H=5, d=128, T=400, hist_frames=6,
                              types=[wl.HEAD_FULL, wl.HEAD_DUMMY, wl.HEAD_NEIGHBOR, wl.HEAD_SINK, wl.HEAD_PACK_DUMMY], planted=[1]))
    # ... then a smaller one, other head dim, on the same scratch
    _both(df, wl.small_ragged(92, H=3, d=64, T=70, hist_frames=3, types=[wl.HEAD_FULL, wl.HEAD_SINK, wl.HEAD_DUMMY]))


def test_static_scratch_rejects_what_does_not_fit(df):
    d = gu.dev()
    H, Nq = 64, 261761                  # one query more than the static scratch holds at 64 heads, d = 128
    assert df.df_attn_workspace_bytes(H, 128, Nq - 1) <= df.DF_STATIC_SCRATCH_BYTES
    assert df.df_attn_workspace_bytes(H, 128, Nq) > df.DF_STATIC_SCRATCH_BYTES
    q = torch.empty(1, H, 128, dtype=torch.bfloat16, device=d)           # never read: the size check comes first
    a = df.df_attn_args()
    a.q = a.k_cur = a.v_cur = a.out = q.data_ptr()
    a.H, a.d, a.Nq, a.Nc, a.softmax_scale = H, 128, Nq, 1, 1.0
    assert df.lib.df_attn_fwd_static(a, None) == df.DF_ERR_WORKSPACE
