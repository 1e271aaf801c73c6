"""Helpers for the GPU parity tests: device upload and a thin runner over the C-ABI binding."""
import math

import numpy as np
import torch

import sp_synth
from paper_2404_06910_amd import binding as B

TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}
SP_DT = {"f32": B.SP_F32, "bf16": B.SP_BF16}


def dev(x, dtype="f32"):
    """numpy array (already rounded to dtype) -> CUDA tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x))
    if t.dtype in (torch.float32, torch.float64):
        t = t.to(TORCH_DT[dtype])
    return t.cuda()


def make_plan(ctx, st, Hq, Hkv, d, dtype, tok_pos=None, slopes=None, seg_cached=None):
    return B.Plan(ctx, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, st.seg_path, st.n_tokens,
                  Hq, Hkv, d, SP_DT[dtype], tok_pos=tok_pos, alibi_slopes=slopes, seg_cached=seg_cached)


def run_prefill(ctx, st, q, k, v, dtype, scale=None, tok_pos=None, slopes=None, plan=None):
    """q/k/v: numpy fp32 (rounded).  Returns (O as fp32 numpy, plan)."""
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    plan = plan or make_plan(ctx, st, Hq, Hkv, d, dtype, tok_pos, slopes)
    Q, K, V = dev(q, dtype), dev(k, dtype), dev(v, dtype)
    O = torch.full_like(Q, float("nan"))
    ctx.sp_forkjoin_prefill(plan, Q, K, V, O, scale or 1.0 / math.sqrt(d))
    torch.cuda.synchronize()
    return O.float().cpu().numpy(), plan


def covered_tokens(st):
    m = np.zeros(st.n_tokens, bool)
    for s in range(st.n_segments):
        m[st.seg_tok_start[s]:st.seg_tok_start[s] + st.seg_tok_len[s]] = True
    return m


def attn_tol(dtype):
    """(max-abs, mean-abs) bounds against the fp64 oracle."""
    return (2e-2, 2e-3) if dtype == "bf16" else (1e-4, 1e-4)


def check_attn(got, ref, dtype, what=""):
    mask = ~np.isnan(ref)
    assert mask.any()
    assert not np.isnan(got[mask]).any(), "NaN in output " + what
    err = np.abs(got[mask].astype(np.float64) - ref[mask])
    mx, mean = attn_tol(dtype)
    assert err.max() <= mx, "%s max-abs %.3e > %.1e" % (what, err.max(), mx)
    assert err.mean() <= mean, "%s mean-abs %.3e > %.1e" % (what, err.mean(), mean)
    return err.max(), err.mean()
