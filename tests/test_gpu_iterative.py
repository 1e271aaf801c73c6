"""Iterative superposition (Sec. 4.1.2 MuSiQue setup; App. B, iterative-superposition figure) driven
through the C ABI: t rounds of superpose -> score -> prune, the kept documents joining a running
prefix behind which the remaining documents are superposed again, then generation from the chain.

The token pool is fixed (preamble, m documents, one query copy per document); each round only
changes the segment table: prefix segments are flagged cached (their K/V exist already), so the
launch computes the remaining documents and their query copies.  Every round's attention output,
scores and kept set are compared with the oracle run on the same tables."""
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


def _round_table(P, doc_rng, qry_rng, chain, remaining, first_round):
    """One prompt: preamble -> chain of kept documents -> {remaining doc -> its query copy}."""
    start = [0]; length = [P]; parent = [-1]; path = [-1]; cached = [0 if first_round else 1]
    tail = 0
    for dch in chain:
        start.append(doc_rng[dch][0]); length.append(doc_rng[dch][1]); parent.append(tail); path.append(-1); cached.append(1)
        tail = len(start) - 1
    for j, dr in enumerate(remaining):
        start.append(doc_rng[dr][0]); length.append(doc_rng[dr][1]); parent.append(tail); path.append(j); cached.append(0)
        start.append(qry_rng[dr][0]); length.append(qry_rng[dr][1]); parent.append(len(start) - 2); path.append(j); cached.append(0)
    i32 = lambda a: np.asarray(a, np.int32)
    return dict(prompt_seg_off=i32([0, len(start)]), seg_tok_start=i32(start), seg_tok_len=i32(length),
                seg_parent=i32(parent), seg_path=i32(path), seg_cached=np.asarray(cached, np.uint8))


@pytest.mark.parametrize("t_rounds,k", [(2, 4), (4, 1), (1, 4)])
def test_iterative_superposition_rounds(ctx, t_rounds, k):
    print("case: iterative superposition t=%d k=%d" % (t_rounds, k), flush=True)
    rng = np.random.default_rng(1000 + 10 * t_rounds + k)
    m, P, Lq, Hq, Hkv, d, vocab = 12, 40, 9, 4, 2, 128, 512
    doc_len = rng.integers(20, 90, m)
    # pool layout: preamble, then document i followed by its query copy
    doc_rng, qry_rng, tok = [], [], P
    for i in range(m):
        doc_rng.append((tok, int(doc_len[i]))); tok += int(doc_len[i])
        qry_rng.append((tok, Lq)); tok += Lq
    T = tok
    f = lambda *s: sp_synth.round_to_dtype(rng.standard_normal(s, dtype=np.float32), "bf16")
    q, kk, v = f(T, Hq, d), f(T, Hkv, d), f(T, Hkv, d)
    Q, K, V = dev(q, "bf16"), dev(kk, "bf16"), dev(v, "bf16")
    scale = 1 / math.sqrt(d)
    target_q = rng.integers(0, vocab, Lq).astype(np.int32)          # same query tokens on every path

    chain, remaining = [], list(range(m))
    for it in range(t_rounds):
        tb = _round_table(P, doc_rng, qry_rng, chain, remaining, it == 0)
        n_paths = len(remaining)
        plan = B.Plan(ctx, tb["prompt_seg_off"], tb["seg_tok_start"], tb["seg_tok_len"], tb["seg_parent"], tb["seg_path"],
                      T, Hq, Hkv, d, B.SP_BF16, seg_cached=tb["seg_cached"])
        O = torch.full_like(Q, float("nan"))
        ctx.sp_forkjoin_prefill(plan, Q, K, V, O, scale)
        # the round's logits stand in for the model head on the query rows (one row per query token and path)
        logits = sp_synth.round_to_dtype((3.0 * rng.standard_normal((n_paths * Lq, vocab))).astype(np.float32), "bf16")
        row_path = np.repeat(np.arange(n_paths, dtype=np.int32), Lq)
        target = np.tile(target_q, n_paths)
        score = torch.empty(n_paths, device="cuda")
        kept = torch.empty((1, k), dtype=torch.int32, device="cuda")
        ctx.sp_path_saliency(dev(logits, "bf16"), dev(target), dev(row_path), n_paths, score)
        ctx.sp_prune_topk(score, plan.path_offsets_device(), 1, n_paths, k, kept)
        torch.cuda.synchronize()

        ref = orc.forkjoin_prefill(q, kk, v, tb["prompt_seg_off"], tb["seg_tok_start"], tb["seg_tok_len"], tb["seg_parent"], scale)
        for s in np.nonzero(tb["seg_cached"])[0]:
            ref[tb["seg_tok_start"][s]:tb["seg_tok_start"][s] + tb["seg_tok_len"][s]] = np.nan
        got = O.float().cpu().numpy()
        check_attn(got, ref, "bf16", "round %d" % it)
        assert np.isnan(got[np.isnan(ref).all(axis=(1, 2))]).all()          # prefix rows and pruned documents untouched
        ref_score = orc.path_saliency(logits, target, row_path, n_paths)
        np.testing.assert_allclose(score.cpu().numpy(), ref_score, rtol=1e-3)
        ref_kept = orc.prune_topk(ref_score, np.array([0, n_paths]), k)
        srt = np.sort(ref_score)[::-1]
        assert srt[k - 1] - srt[k] > 1e-3 * abs(srt[k])                     # kept set decided beyond the tolerance
        assert np.array_equal(kept.cpu().numpy(), ref_kept)
        chosen = [remaining[j] for j in ref_kept[0]]
        chain += chosen
        remaining = [r for r in remaining if r not in chosen]
    assert len(chain) == t_rounds * k

    # generation: preamble -> chain of t*k documents -> query; the query rows are recomputed against
    # the final prefix, then two response tokens attend to the joined cache
    qr = (T, Lq)                                                            # a fresh query slot at the pool's end
    T2 = T + Lq
    q2, k2, v2 = (np.concatenate([a, f(Lq, a.shape[1], d)]) for a in (q, kk, v))
    tb = _round_table(P, doc_rng, qry_rng, chain, [], False)
    i32 = lambda a: np.asarray(a, np.int32)
    tb["seg_tok_start"] = np.append(tb["seg_tok_start"], qr[0]).astype(np.int32)
    tb["seg_tok_len"] = np.append(tb["seg_tok_len"], Lq).astype(np.int32)
    tb["seg_parent"] = np.append(tb["seg_parent"], len(chain)).astype(np.int32)
    tb["seg_path"] = np.append(tb["seg_path"], 0).astype(np.int32)
    tb["seg_cached"] = np.append(tb["seg_cached"], 0).astype(np.uint8)
    tb["prompt_seg_off"] = i32([0, len(tb["seg_parent"])])
    plan = B.Plan(ctx, tb["prompt_seg_off"], tb["seg_tok_start"], tb["seg_tok_len"], tb["seg_parent"], tb["seg_path"],
                  T2, Hq, Hkv, d, B.SP_BF16, seg_cached=tb["seg_cached"])
    Q2, K2, V2 = dev(q2, "bf16"), dev(k2, "bf16"), dev(v2, "bf16")
    O2 = torch.full_like(Q2, float("nan"))
    ctx.sp_forkjoin_prefill(plan, Q2, K2, V2, O2, scale)
    torch.cuda.synchronize()
    ref = orc.forkjoin_prefill(q2, k2, v2, tb["prompt_seg_off"], tb["seg_tok_start"], tb["seg_tok_len"], tb["seg_parent"], scale)
    ref[:T] = np.nan
    check_attn(O2.float().cpu().numpy(), ref, "bf16", "final query rows")
    assert plan.visible_pairs() == Lq * (P + int(sum(doc_len[c] for c in chain))) + Lq * (Lq + 1) // 2

    steps = 2
    kept = dev(np.zeros((1, 1), np.int32))
    Kr = torch.zeros((1, steps, Hkv, d), dtype=torch.bfloat16, device="cuda"); Vr = torch.zeros_like(Kr)
    dq, dk, dv = f(steps, 1, Hq, d), f(steps, 1, Hkv, d), f(steps, 1, Hkv, d)
    idx = orc.joined_cache_index(tb["prompt_seg_off"], tb["seg_tok_start"], tb["seg_tok_len"], tb["seg_path"], 0, [0])
    assert len(idx) == P + int(sum(doc_len[c] for c in chain)) + Lq
    mx, mean = attn_tol("bf16")
    for s in range(steps):
        o = torch.empty((1, Hq, d), dtype=torch.bfloat16, device="cuda")
        ctx.sp_pruned_decode(plan, kept, 1, K2, V2, Kr, Vr, steps, dev(dq[s], "bf16"), dev(dk[s], "bf16"),
                             dev(dv[s], "bf16"), o, scale, resp_len_add=s)
        torch.cuda.synchronize()
        r = orc.pruned_decode_step(dq[s, 0], dk[s, 0], dv[s, 0], k2, v2, idx, dk[:s, 0], dv[:s, 0], scale)
        err = np.abs(o[0].float().cpu().numpy() - r)
        assert err.max() <= mx and err.mean() <= mean, "decode step %d" % s
