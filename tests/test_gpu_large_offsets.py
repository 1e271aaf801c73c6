"""Addresses beyond 4 GB: the packed tensors hold more than 2^32 bytes and the prompts under test sit
at their far end, so every byte offset in the kernels has to be formed in 64 bits (prefill, decode)."""
import math

import numpy as np
import pytest
import torch

import sp_synth
from oracle import sp_oracle as orc
from paper_2404_06910_amd import binding as B

from gpu_util import attn_tol, check_attn

pytestmark = pytest.mark.gpu


def test_prompts_behind_the_4GB_mark():
    print("case: large offsets", flush=True)
    Hq = Hkv = 32
    d = 128
    P, Lq = 40, 9
    lens = [[70, 33, 101]]
    base = sp_synth.forkjoin_segtable(P, lens, Lq)
    n_used = base.n_tokens
    T = (1 << 19) + 4096 + n_used                 # > 2^32 / (32 * 128 * 2) tokens per tensor
    shift = T - n_used
    assert shift * Hkv * d * 2 > (1 << 32)
    rng = np.random.default_rng(9)
    f = lambda h: sp_synth.round_to_dtype(rng.standard_normal((n_used, h, d), dtype=np.float32), "bf16")
    q, k, v = f(Hq), f(Hkv), f(Hkv)
    Q = torch.empty((T, Hq, d), dtype=torch.bfloat16, device="cuda")
    K = torch.empty((T, Hkv, d), dtype=torch.bfloat16, device="cuda")
    V = torch.empty((T, Hkv, d), dtype=torch.bfloat16, device="cuda")
    O = torch.empty((T, Hq, d), dtype=torch.bfloat16, device="cuda")
    for t, a in ((Q, q), (K, k), (V, v)):
        t[shift:] = torch.from_numpy(a).to(torch.bfloat16).cuda()
    O[shift:] = float("nan")
    ctx = B.Context(0)
    starts = (np.asarray(base.seg_tok_start) + shift).astype(np.int32)
    plan = B.Plan(ctx, base.prompt_seg_off, starts, base.seg_tok_len, base.seg_parent, base.seg_path, T, Hq, Hkv, d,
                  B.SP_BF16)
    scale = 1 / math.sqrt(d)
    ctx.sp_forkjoin_prefill(plan, Q, K, V, O, scale)
    torch.cuda.synchronize()
    got = O[shift:].float().cpu().numpy()
    heads = [0, 17, 31]
    ref = orc.forkjoin_prefill(q, k, v, base.prompt_seg_off, base.seg_tok_start, base.seg_tok_len, base.seg_parent, scale,
                               heads=heads)
    check_attn(got, ref, "bf16", "prefill behind 4 GB")

    # decode over the same far-away cache
    kept = torch.tensor([[2, 0]], dtype=torch.int32, device="cuda")
    dq = sp_synth.round_to_dtype(rng.standard_normal((1, Hq, d), dtype=np.float32), "bf16")
    dk = sp_synth.round_to_dtype(rng.standard_normal((1, Hkv, d), dtype=np.float32), "bf16")
    dv = sp_synth.round_to_dtype(rng.standard_normal((1, Hkv, d), dtype=np.float32), "bf16")
    Kr = torch.zeros((1, 2, Hkv, d), dtype=torch.bfloat16, device="cuda"); Vr = torch.zeros_like(Kr)
    o = torch.empty((1, Hq, d), dtype=torch.bfloat16, device="cuda")
    tb = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    ctx.sp_pruned_decode(plan, kept, 2, K, V, Kr, Vr, 2, tb(dq), tb(dk), tb(dv), o, scale)
    torch.cuda.synchronize()
    idx = orc.joined_cache_index(base.prompt_seg_off, base.seg_tok_start, base.seg_tok_len, base.seg_path, 0, [2, 0])
    r = orc.pruned_decode_step(dq[0], dk[0], dv[0], k, v, idx, dk[:0, 0], dv[:0, 0], scale)
    err = np.abs(o[0].float().cpu().numpy() - r)
    mx, mean = attn_tol("bf16")
    assert err.max() <= mx and err.mean() <= mean
    ctx.close()
