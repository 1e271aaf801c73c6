"""Two table-only variants of the path, through the C ABI against the oracle:

* the superposition factor (App. "Superposition Factor Ablation"): adjacent documents are merged,
  round(m / gamma) per path, sweeping from the fully superposed prompt (gamma = m) to the classical
  one (gamma = 1, a single path that is plain causal attention);
* the join of the kept paths for a multi-token postamble (Alg. 3, the tokens after the pruned
  paths): one prefill launch over a re-linked chain of cached segments equals the same tokens fed
  one by one through the decode step.
"""
import math

import numpy as np
import pytest
import torch

import sp_synth
from oracle import sp_oracle as orc
from paper_2404_06910_amd import binding as B

from gpu_util import attn_tol, check_attn, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = B.Context(0)
    yield c
    c.close()


def _factor_table(P, doc_len, Lq, gamma):
    """Preamble -> per path a chain of round(m/gamma) adjacent documents -> the path's query copy."""
    m = len(doc_len)
    per = int(np.floor(m / gamma + 0.5))
    start, length, parent, path = [0], [P], [-1], [-1]
    tok = P
    n_paths = 0
    for first in range(0, m, per):
        tail = 0
        for dd in range(first, min(first + per, m)):
            start.append(tok); length.append(int(doc_len[dd])); parent.append(tail); path.append(n_paths)
            tail = len(start) - 1; tok += int(doc_len[dd])
        start.append(tok); length.append(Lq); parent.append(tail); path.append(n_paths); tok += Lq
        n_paths += 1
    i32 = lambda a: np.asarray(a, np.int32)
    return dict(prompt_seg_off=i32([0, len(start)]), seg_tok_start=i32(start), seg_tok_len=i32(length),
                seg_parent=i32(parent), seg_path=i32(path), n_tokens=tok, n_paths=n_paths)


@pytest.mark.parametrize("gamma", [12, 4, 2.4, 1])
def test_superposition_factor_tables(ctx, gamma):
    print("case: superposition factor", gamma, flush=True)
    rng = np.random.default_rng(int(gamma * 10))
    P, Lq, Hq, Hkv, d = 21, 7, 4, 2, 128
    doc_len = rng.integers(10, 50, 12)
    t = _factor_table(P, doc_len, Lq, gamma)
    assert t["n_paths"] == math.ceil(12 / int(np.floor(12 / gamma + 0.5)))
    T = t["n_tokens"]
    f = lambda *s: sp_synth.round_to_dtype(rng.standard_normal(s, dtype=np.float32), "bf16")
    q, k, v = f(T, Hq, d), f(T, Hkv, d), f(T, Hkv, d)
    plan = B.Plan(ctx, t["prompt_seg_off"], t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], t["seg_path"], T,
                  Hq, Hkv, d, B.SP_BF16)
    Q, K, V = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16")
    O = torch.full_like(Q, float("nan"))
    scale = 1 / math.sqrt(d)
    ctx.sp_forkjoin_prefill(plan, Q, K, V, O, scale)
    torch.cuda.synchronize()
    got = O.float().cpu().numpy()
    ref = orc.forkjoin_prefill(q, k, v, t["prompt_seg_off"], t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], scale)
    check_attn(got, ref, "bf16", "gamma %s" % gamma)
    if gamma == 1:
        # the classical prompt: one sequence, plain causal attention (library routine as a second opinion)
        assert t["n_paths"] == 1
        G = Hq // Hkv
        qq = torch.from_numpy(q).permute(1, 0, 2)[None]
        kk = torch.from_numpy(k).repeat_interleave(G, dim=1).permute(1, 0, 2)[None]
        vv = torch.from_numpy(v).repeat_interleave(G, dim=1).permute(1, 0, 2)[None]
        sd = torch.nn.functional.scaled_dot_product_attention(qq.double(), kk.double(), vv.double(), is_causal=True,
                                                              scale=scale)[0].permute(1, 0, 2).numpy()
        check_attn(got, sd, "bf16", "classical prompt")
    # fewer, longer paths see more: visible pairs grow monotonically as gamma falls (pinned per table)
    toks, M = orc.dag_mask(t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], range(len(t["seg_parent"])))
    assert plan.visible_pairs() == int(M.sum())


def test_postamble_join_prefill_equals_decode_steps(ctx):
    print("case: postamble join", flush=True)
    rng = np.random.default_rng(77)
    P, Lq, Hq, Hkv, d, n_post = 30, 11, 8, 2, 128, 6
    lens = [[40, 75, 33, 58]]
    st = sp_synth.forkjoin_segtable(P, lens, Lq)
    T = st.n_tokens
    f = lambda *s: sp_synth.round_to_dtype(rng.standard_normal(s, dtype=np.float32), "bf16")
    q, k, v = f(T, Hq, d), f(T, Hkv, d), f(T, Hkv, d)
    pq, pk, pv = f(n_post, 1, Hq, d), f(n_post, 1, Hkv, d), f(n_post, 1, Hkv, d)   # postamble tokens
    kept_paths = [2, 0]
    scale = 1 / math.sqrt(d)
    mx, mean = attn_tol("bf16")

    # (a) token by token through the decode step
    plan = B.Plan(ctx, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, st.seg_path, T, Hq, Hkv, d,
                  B.SP_BF16)
    K, V = dev(k, "bf16"), dev(v, "bf16")
    kept = dev(np.asarray([kept_paths], np.int32))
    Kr = torch.zeros((1, n_post, Hkv, d), dtype=torch.bfloat16, device="cuda"); Vr = torch.zeros_like(Kr)
    dec = []
    for s in range(n_post):
        o = torch.empty((1, Hq, d), dtype=torch.bfloat16, device="cuda")
        ctx.sp_pruned_decode(plan, kept, 2, K, V, Kr, Vr, n_post, dev(pq[s], "bf16"), dev(pk[s], "bf16"),
                             dev(pv[s], "bf16"), o, scale, resp_len_add=s)
        torch.cuda.synchronize()
        dec.append(o[0].float().cpu().numpy())
    dec = np.stack(dec)
    idx = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, 0, kept_paths)
    for s in range(n_post):
        r = orc.pruned_decode_step(pq[s, 0], pk[s, 0], pv[s, 0], k, v, idx, pk[:s, 0], pv[:s, 0], scale)
        err = np.abs(dec[s] - r)
        assert err.max() <= mx and err.mean() <= mean, "decode step %d" % s

    # (b) one prefill launch: the kept paths re-linked into a chain of cached segments, the postamble
    # as the only computed segment behind it
    seg = lambda name, slot: int(getattr(st, name)[slot])
    chain = [int(st.preamble_seg[0])]
    for p in kept_paths:
        chain += [seg("doc_seg", p), seg("query_seg", p)]
    start = [int(st.seg_tok_start[s]) for s in chain] + [T]
    length = [int(st.seg_tok_len[s]) for s in chain] + [n_post]
    parent = [-1] + list(range(len(chain) - 1)) + [len(chain) - 1]
    path = [-1] * len(chain) + [0]
    cached = [1] * len(chain) + [0]
    i32 = lambda a: np.asarray(a, np.int32)
    q2 = np.concatenate([q, pq[:, 0]]); k2 = np.concatenate([k, pk[:, 0]]); v2 = np.concatenate([v, pv[:, 0]])
    plan2 = B.Plan(ctx, i32([0, len(start)]), i32(start), i32(length), i32(parent), i32(path), T + n_post, Hq, Hkv, d,
                   B.SP_BF16, seg_cached=np.asarray(cached, np.uint8))
    Q2, K2, V2 = dev(q2, "bf16"), dev(k2, "bf16"), dev(v2, "bf16")
    O2 = torch.full_like(Q2, float("nan"))
    ctx.sp_forkjoin_prefill(plan2, Q2, K2, V2, O2, scale)
    torch.cuda.synchronize()
    got = O2.float().cpu().numpy()
    assert np.isnan(got[:T]).all()
    join = got[T:]
    assert np.abs(join - dec).max() <= mx            # the two routes agree (both within tolerance of the oracle)
    ref = orc.forkjoin_prefill(q2, k2, v2, i32([0, len(start)]), i32(start), i32(length), i32(parent), scale)
    ref[:T] = np.nan
    check_attn(got, ref, "bf16", "join prefill")
