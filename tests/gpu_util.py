"""Helpers of the GPU parity tests: run a workload through the C ABI and through the oracle."""
import numpy as np
import torch

from oracle import df_oracle as orc
from paper_2601_20499_amd import workloads as wl

# Tolerances of the parity bar: bf16 outputs against the fp64 oracle on identical bf16 inputs.
MAX_ABS = 2e-2
MEAN_ABS = 2e-3
REL_L2 = 1e-2      # extra guard: i.i.d. values average out, so the absolute bar alone is loose
F_ABS = 1e-4
# log-sum-exp: m*scale (fp32, |m*scale| up to a few tens: 2^-24 relative) + ln of an fp32 sum of up to 4e5
# hardware exp2 values (1 ulp each, summed in tile order) through the hardware log2: a few 1e-6 (measured
# 1.9e-6 at the Wan-shaped size over all rows); the bar leaves a factor of fifty
LSE_ABS = 1e-4


def dev():
    return torch.device("cuda:0")


def run_attn(df, w, want_score=True, want_lse=True, layout="thd"):
    """Launch df_attn_fwd on workload w.  layout 'thd' = [tok, head, d]; 'htd' = head-major storage
    viewed as [tok, head, d] (exercises the stride arguments)."""
    d = dev()
    kp, vp, off, sl = wl.packed_history(w)

    def put(t):
        t = t.to(torch.bfloat16)
        if layout == "htd":
            return t.permute(1, 0, 2).contiguous().to(d).permute(1, 0, 2)
        return t.contiguous().to(d)

    q, kc, vc = put(w.q), put(w.k_cur), put(w.v_cur)
    out = torch.full_like(q, float("nan"))
    score = torch.full((w.H, 3), float("nan"), dtype=torch.float32, device=d) if want_score else None
    n_q = w.q.shape[0]           # normally w.Nq; a caller may have replaced w.q by a subset of its rows
    lse = torch.full((w.H, n_q), float("nan"), dtype=torch.float32, device=d) if want_lse else None
    ws = torch.empty(df.df_attn_workspace_bytes(w.H, w.d, n_q), dtype=torch.uint8, device=d)
    df.df_attn_fwd(q, kc, vc, kp.to(torch.bfloat16).to(d), vp.to(torch.bfloat16).to(d), off, sl, out, w.scale,
                   lse_out=lse, score_out=score, workspace=ws)
    torch.cuda.synchronize()
    return (out.float().cpu().double().numpy(),
            None if score is None else score.cpu().double().numpy(),
            None if lse is None else lse.cpu().double().numpy())


def oracle_rows(w, rows=None):
    """Oracle on the same bf16-rounded inputs, optionally on a subset of query rows."""
    b = lambda t: t.to(torch.bfloat16).double().numpy()
    kh = [b(w.k_hist[:, h]) for h in range(w.H)]
    vh = [b(w.v_hist[:, h]) for h in range(w.H)]
    return orc.layer_attention(b(w.q), kh, vh, b(w.k_cur), b(w.v_cur), w.n_sink, w.n_win, w.scale, rows=rows)


def check_out(got, ref, what=""):
    err = np.abs(got - ref)
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    msg = f"{what}: max|err|={err.max():.3e} mean|err|={err.mean():.3e} relL2={rel:.3e}"
    print(msg, flush=True)
    assert np.isfinite(got).all(), msg
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS and rel <= REL_L2, msg
    return err.max(), err.mean(), rel


def sample_rows(Nq, n, seed, tile=256):
    """Seeded row sample that always contains the first and last rows and the ragged tail tile."""
    g = np.random.default_rng(seed)
    tail0 = (Nq - 1) // tile * tile
    fixed = {0, 1, Nq - 1, Nq - 2, tail0, max(tail0 - 1, 0), min(127, Nq - 1), min(128, Nq - 1)}
    extra = g.choice(Nq, size=max(0, n - len(fixed)), replace=False).tolist()
    return np.array(sorted(fixed | set(extra)))


def fused_score_on_rows(df, w, rows):
    """df_attn_fwd launched on the queries `rows` only (all keys): the fused frame attention score is then
    the mean over exactly the rows the oracle was run on, so it can be held to the score tolerance at
    sizes where the oracle cannot cover every query."""
    import copy
    sub = copy.copy(w)
    sub.q = w.q[torch.as_tensor(rows)].contiguous()
    _, score, _ = run_attn(df, sub, want_lse=False)
    return score
