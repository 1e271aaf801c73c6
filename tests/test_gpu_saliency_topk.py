"""GPU parity of sp_path_saliency and sp_prune_topk against the CPU oracle."""
import numpy as np
import pytest
import torch

import sp_synth
from oracle import sp_oracle as orc
from paper_2404_06910_amd import binding as B

from gpu_util import dev

pytestmark = pytest.mark.gpu
REL = 1e-3          # saliency tolerance (relative), as stated for the workloads


@pytest.fixture(scope="module")
def ctx():
    c = B.Context(0)
    yield c
    c.close()


def _saliency(ctx, logits_t, target, row_path, n_slots, prior=None, mode=B.SALIENCY_SUM):
    score = torch.full((n_slots,), float("nan"), device="cuda")
    ctx.sp_path_saliency(logits_t, dev(target), dev(row_path), n_slots, score,
                         prior=None if prior is None else dev(prior), mode=mode)
    torch.cuda.synchronize()
    return score.cpu().numpy()


def _close(got, ref):
    np.testing.assert_allclose(got, ref, rtol=REL, atol=1e-5)


def test_config1_saliency_and_chained_topk(ctx):
    inp = sp_synth.make_inputs(sp_synth.WORKLOADS["c1_tiny_f32"], with_decode=False)
    n = inp.st.n_slots
    got = _saliency(ctx, dev(inp.logits), inp.target, inp.row_path, n)
    ref = orc.path_saliency(inp.logits, inp.target, inp.row_path, n)
    _close(got, ref)
    kept = torch.full((1, 1), -7, dtype=torch.int32, device="cuda")
    ctx.sp_prune_topk(dev(got), dev(inp.st.path_off), 1, 4, 1, kept)
    assert kept.cpu().numpy().tolist() == orc.prune_topk(got, inp.st.path_off, 1).tolist()
    assert kept.cpu().numpy().tolist() == orc.prune_topk(ref, inp.st.path_off, 1).tolist()


@pytest.mark.parametrize("dtype,vocab", [("bf16", 50432), ("bf16", 1003), ("f32", 4099), ("f32", 8), ("bf16", 5),
                                          ("bf16", 8192 + 8)])
def test_saliency_modes_skips_prior_tails(ctx, dtype, vocab):
    print("case:", dtype, vocab, flush=True)
    rng = np.random.default_rng(vocab)
    R, n = 53, 7
    x = sp_synth.round_to_dtype(rng.standard_normal((R, vocab), dtype=np.float32) * 3, dtype)
    x[5, :] = -np.inf; x[5, 2] = 1.0                       # a row with a single possible token
    x[6, 1::2] = -np.inf                                   # zero-probability entries
    tgt = rng.integers(0, vocab, size=R).astype(np.int32)
    tgt[5] = 2; tgt[6] = 0; tgt[[0, 9, 30]] = -1
    rp = rng.integers(0, n - 1, size=R).astype(np.int32)   # slot n-1 has no rows
    prior = rng.standard_normal(n).astype(np.float32)
    # row stride larger than vocab (padded to a 16-byte multiple)
    pad = (-vocab) % 8 + 8
    full = torch.zeros((R, vocab + pad), dtype=torch.float32)
    full[:, :vocab] = torch.from_numpy(x)
    full[:, vocab:] = 1e4                                  # must never be read as logits
    lt = dev(full.numpy(), dtype)[:, :vocab]
    for mode, mname in ((B.SALIENCY_SUM, "sum"), (B.SALIENCY_MEAN, "mean")):
        got = _saliency(ctx, lt, tgt, rp, n, prior=prior, mode=mode)
        ref = orc.path_saliency(x, tgt, rp, n, prior=prior, mode=mname)
        _close(got, ref)
    got = _saliency(ctx, lt, tgt, rp, n)
    assert got[n - 1] == 0.0
    again = _saliency(ctx, lt, tgt, rp, n)
    assert np.array_equal(got, again)                      # deterministic reduction order


def test_saliency_closed_forms(ctx):
    V = 50432
    x = torch.full((4, V), 1.75, dtype=torch.bfloat16, device="cuda")
    got = _saliency(ctx, x, np.array([0, 1, 2, V - 1], np.int32), np.zeros(4, np.int32), 1)
    np.testing.assert_allclose(got[0], -4 * np.log(V), rtol=1e-5)
    y = torch.zeros((2, V), dtype=torch.float32, device="cuda"); y[0, 7] = 200.0; y[1, 9] = 200.0
    got = _saliency(ctx, y, np.array([7, 9], np.int32), np.zeros(2, np.int32), 1)
    assert abs(got[0]) < 1e-6


@pytest.mark.parametrize("name", ["c2_mha7b_bf16", "c3_ragged_bf16", "c4_gqa_bf16"])
def test_full_size_saliency_every_slot(ctx, name):
    """Full logit matrix generated on the device (seeded); the oracle scores EVERY path slot (rows are
    copied back a few hundred at a time).  Two launches on the same input give bit-identical scores
    (integer accumulation: no dependence on the order in which rows finish)."""
    wl = sp_synth.WORKLOADS[name]
    print("case:", name, flush=True)
    n_slots = wl.n_prompts * wl.n_paths
    R = n_slots * wl.query_len
    g = torch.Generator(device="cuda"); g.manual_seed(wl.seed)
    logits = torch.empty((R, wl.vocab), dtype=torch.bfloat16, device="cuda")
    step = 512
    for r in range(0, R, step):
        logits[r:r + step] = (torch.randn((min(step, R - r), wl.vocab), generator=g, device="cuda") * wl.logit_std)
    rng = np.random.default_rng(wl.seed)
    target = np.concatenate([np.tile(rng.integers(0, wl.vocab, size=wl.query_len), wl.n_paths)
                             for _ in range(wl.n_prompts)]).astype(np.int32)
    row_path = np.repeat(np.arange(n_slots), wl.query_len).astype(np.int32)
    got = _saliency(ctx, logits, target, row_path, n_slots)
    assert np.isfinite(got).all()
    again = _saliency(ctx, logits, target, row_path, n_slots)
    assert np.array_equal(got, again)
    per = 16                                                # slots per copy
    for s0 in range(0, n_slots, per):
        s1 = min(n_slots, s0 + per)
        rows = slice(s0 * wl.query_len, s1 * wl.query_len)
        x = logits[rows].float().cpu().numpy()
        ref = orc.path_saliency(x, target[rows], row_path[rows] - s0, s1 - s0)
        np.testing.assert_allclose(got[s0:s1], ref, rtol=REL)
    # chained top-k on the device scores equals the oracle's top-k of the same scores
    off = np.arange(0, n_slots + 1, wl.n_paths).astype(np.int32)
    kept = torch.empty((wl.n_prompts, wl.top_k), dtype=torch.int32, device="cuda")
    ctx.sp_prune_topk(dev(got), dev(off), wl.n_prompts, wl.n_paths, wl.top_k, kept)
    assert np.array_equal(kept.cpu().numpy(), orc.prune_topk(got, off, wl.top_k))


def test_saliency_scattered_rows_many_slots_and_nonfinite(ctx):
    """Rows of a path scattered over the matrix (the fused reduction does not assume runs), more slots
    than rows, a slot whose rows hold -inf and NaN log-likelihoods, MEAN counts, repeatability."""
    rng = np.random.default_rng(21)
    R, n, vocab = 700, 900, 2048
    x = sp_synth.round_to_dtype(rng.standard_normal((R, vocab), dtype=np.float32) * 3, "f32")
    tgt = rng.integers(0, vocab, size=R).astype(np.int32)
    rp = rng.integers(0, n, size=R).astype(np.int32)
    rp[:40] = 7                                             # one crowded slot
    x[3, tgt[3]] = -np.inf                                  # lp = -inf in slot 7
    x[50, :] = np.nan; rp[50] = 11                          # lp = NaN in slot 11
    tgt[[5, 6]] = -1
    X = dev(x, "f32")
    for mode, name in ((B.SALIENCY_SUM, "sum"), (B.SALIENCY_MEAN, "mean")):
        got = _saliency(ctx, X, tgt, rp, n, mode=mode)
        with np.errstate(invalid="ignore", divide="ignore"):
            ref = orc.path_saliency(x, tgt, rp, n, mode=name)
        assert np.isneginf(got[7]) and np.isneginf(ref[7]) and np.isnan(got[11]) and np.isnan(ref[11])
        ok = np.isfinite(ref)
        np.testing.assert_allclose(got[ok], ref[ok], rtol=REL, atol=1e-5)
        assert np.array_equal(got, _saliency(ctx, X, tgt, rp, n, mode=mode), equal_nan=True)


def test_saliency_more_slots_than_the_initial_workspace(ctx):
    """A call that needs more workspace than a new context holds grows it once (this size also takes the
    many-workgroup reduction with accumulators in global memory); results before and after agree with the
    oracle, and a small call afterwards (single-workgroup reduction) as well."""
    rng = np.random.default_rng(4)
    R, n, vocab = 64, 40000, 512
    x = sp_synth.round_to_dtype(rng.standard_normal((R, vocab), dtype=np.float32), "bf16")
    tgt = rng.integers(0, vocab, size=R).astype(np.int32)
    rp = rng.integers(0, n, size=R).astype(np.int32)
    got = _saliency(ctx, dev(x, "bf16"), tgt, rp, n)
    _close(got, orc.path_saliency(x, tgt, rp, n))
    got = _saliency(ctx, dev(x, "bf16"), tgt, rp % 100, 100)
    _close(got, orc.path_saliency(x, tgt, rp % 100, 100))


# ----------------------------------------------------------------------------- top-k

def _topk(ctx, score, off, k, n_max=None):
    off = np.asarray(off, np.int32)
    B_ = len(off) - 1
    kept = torch.full((B_, k), -99, dtype=torch.int32, device="cuda")
    n_max = n_max or int(np.diff(off).max())
    ctx.sp_prune_topk(dev(np.asarray(score, np.float32)), dev(off), B_, n_max, k, kept)
    torch.cuda.synchronize()
    return kept.cpu().numpy()


def test_topk_random_ragged_prompts(ctx):
    rng = np.random.default_rng(0)
    sizes = [1, 4, 20, 64, 7, 300, 1000]
    off = np.concatenate([[0], np.cumsum(sizes)])
    sc = rng.standard_normal(off[-1]).astype(np.float32)
    for k in (1, 2, 4):
        got = _topk(ctx, sc, off, k)
        for b, n in enumerate(sizes):
            kk = min(k, n)
            ref = orc.prune_topk(sc[off[b]:off[b + 1]], [0, n], kk)[0]
            assert got[b, :kk].tolist() == ref.tolist()
            assert np.all(got[b, kk:] == -1)


def test_topk_prompt_larger_than_the_stated_bound_is_not_truncated(ctx):
    rng = np.random.default_rng(8)
    sizes = [300, 5, 64]
    off = np.concatenate([[0], np.cumsum(sizes)])
    sc = rng.standard_normal(off[-1]).astype(np.float32)
    got = _topk(ctx, sc, off, 4, n_max=64)                  # the first prompt has 300 paths
    assert np.array_equal(got, orc.prune_topk(sc, off, 4))


def test_topk_ties_zero_signs_inf_nan_full_ranking(ctx):
    s = np.array([1.0, 3.0, 3.0, -0.0, 0.0, 3.0, 1.0, -np.inf, np.nan, -np.inf, np.nan], np.float32)
    n = len(s)
    got = _topk(ctx, s, [0, n], n)
    assert got[0].tolist() == orc.prune_topk(s, [0, n], n)[0].tolist() == [1, 2, 5, 0, 6, 3, 4, 7, 9, 8, 10]
    eq = np.zeros(64, np.float32)
    assert _topk(ctx, eq, [0, 64], 4)[0].tolist() == [0, 1, 2, 3]
    rng = np.random.default_rng(2)
    q = rng.integers(0, 4, size=(5, 64)).astype(np.float32)          # many exact ties
    off = np.arange(0, 5 * 64 + 1, 64)
    got = _topk(ctx, q.reshape(-1), off, 64)
    assert np.array_equal(got, orc.prune_topk(q.reshape(-1), off, 64))
    # per-prompt additive constant does not change the kept set (App. B.1: C is irrelevant)
    sc = rng.standard_normal(5 * 64).astype(np.float32)
    shifted = (sc.reshape(5, 64) + np.array([[4.0], [-2.0], [0.5], [8.0], [-16.0]], np.float32)).reshape(-1)
    assert np.array_equal(_topk(ctx, sc, off, 4), _topk(ctx, shifted, off, 4))


def test_argument_errors(ctx):
    s = torch.zeros(4, device="cuda"); off = dev(np.array([0, 4], np.int32))
    kept = torch.zeros((1, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(B.SpError) as e:
        ctx.sp_prune_topk(s, off, 1, 4, 0, kept)
    assert e.value.status == -1
    with pytest.raises(B.SpError) as e:
        ctx.sp_prune_topk(s, off, 1, 5000, 1, kept)
    assert e.value.status == -3
    x = torch.zeros((2, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.SpError) as e:
        ctx.sp_path_saliency(x, dev(np.zeros(2, np.int32)), dev(np.zeros(2, np.int32)), 0, s)
    assert e.value.status == -1
