"""Pins for the saliency and top-k oracles (CPU only)."""
import itertools
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import sp_oracle as orc


def test_uniform_logits_give_minus_log_vocab():
    V = 37
    x = np.full((5, V), 1.75)
    lp = orc.token_log_likelihood(x, np.array([0, 5, 36, 7, 1]))
    np.testing.assert_allclose(lp, -math.log(V), rtol=1e-14)


def test_matches_library_log_softmax_and_logsumexp():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((23, 101)) * 3
    tgt = rng.integers(0, 101, size=23)
    lp = orc.token_log_likelihood(x, tgt)
    ref_t = torch.log_softmax(torch.from_numpy(x), dim=-1).gather(1, torch.from_numpy(tgt)[:, None])[:, 0].numpy()
    ref_s = x[np.arange(23), tgt] - scipy.special.logsumexp(x, axis=1)
    np.testing.assert_allclose(lp, ref_t, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lp, ref_s, rtol=1e-12, atol=1e-13)


def test_row_shift_invariance_dominant_logit_and_minus_inf():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, 50))
    tgt = rng.integers(0, 50, size=6)
    a = orc.token_log_likelihood(x, tgt)
    b = orc.token_log_likelihood(x + rng.standard_normal((6, 1)) * 100, tgt)
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-11)
    y = x.copy(); y[np.arange(6), tgt] += 200.0
    assert np.all(np.abs(orc.token_log_likelihood(y, tgt)) < 1e-60)
    z = x.copy(); z[:, 3] = -np.inf                     # a vocabulary entry with zero probability
    tz = np.where(tgt == 3, 4, tgt)
    ref = z[np.arange(6), tz] - scipy.special.logsumexp(z, axis=1)
    np.testing.assert_allclose(orc.token_log_likelihood(z, tz), ref, rtol=1e-12)


def test_path_reduction_sum_mean_prior_and_skipped_rows():
    rng = np.random.default_rng(2)
    R, V, n = 40, 29, 5
    x = rng.standard_normal((R, V)) * 2
    tgt = rng.integers(0, V, size=R); tgt[[3, 17, 18]] = -1            # not scored
    rp = rng.integers(0, n - 1, size=R)                                # slot n-1 stays empty
    prior = rng.standard_normal(n)
    ref_lp = torch.log_softmax(torch.from_numpy(x), dim=-1).numpy()
    s_ref = np.zeros(n); c_ref = np.zeros(n)
    for r in range(R):
        if tgt[r] >= 0:
            s_ref[rp[r]] += ref_lp[r, tgt[r]]; c_ref[rp[r]] += 1
    s = orc.path_saliency(x, tgt, rp, n, mode="sum")
    m = orc.path_saliency(x, tgt, rp, n, mode="mean")
    np.testing.assert_allclose(s, s_ref, rtol=1e-12)
    np.testing.assert_allclose(m * c_ref, s_ref, rtol=1e-12)             # MEAN * count == SUM
    assert s[n - 1] == 0.0 and m[n - 1] == 0.0
    np.testing.assert_allclose(orc.path_saliency(x, tgt, rp, n, prior=prior), s_ref + prior, rtol=1e-12)


def test_shifted_cross_entropy_form():
    # App. B.1 footnote: the language-model cross-entropy drops the first token and the last
    # logit row.  With targets[r] = tokens[r+1] for r < L-1 and -1 on the last row, SUM
    # saliency equals minus the summed token-level cross-entropy of the library routine.
    rng = np.random.default_rng(3)
    L, V = 9, 31
    logits = rng.standard_normal((L, V)); toks = rng.integers(0, V, size=L)
    tgt = np.concatenate([toks[1:], [-1]])
    s = orc.path_saliency(logits, tgt, np.zeros(L, int), 1, mode="sum")[0]
    ce = torch.nn.functional.cross_entropy(torch.from_numpy(logits[:-1]), torch.from_numpy(toks[1:]), reduction="sum")
    np.testing.assert_allclose(s, -float(ce), rtol=1e-12)
    m = orc.path_saliency(logits, tgt, np.zeros(L, int), 1, mode="mean")[0]
    ce_m = torch.nn.functional.cross_entropy(torch.from_numpy(logits[:-1]), torch.from_numpy(toks[1:]))
    np.testing.assert_allclose(m, -float(ce_m), rtol=1e-12)


# ---------------------------------------------------------------- top-k

def _brute_topk(s, k):
    """Exhaustive: the ordered k-tuple that is lexicographically best under
    (score descending, index ascending), found by repeated selection."""
    left = list(range(len(s)))
    out = []
    for _ in range(k):
        best = left[0]
        for i in left[1:]:
            if s[i] > s[best]:
                best = i
        out.append(best); left.remove(best)
    return out


def test_topk_brute_force_and_library_stable_sort():
    rng = np.random.default_rng(4)
    for n in (1, 2, 5, 20, 64):
        s = rng.standard_normal(n)
        for k in sorted({1, min(2, n), min(4, n), n}):
            got = orc.prune_topk(s, [0, n], k)[0].tolist()
            assert got == _brute_topk(s, k)
            assert got == np.argsort(-s, kind="stable")[:k].tolist()


def test_topk_ties_signed_zero_full_ranking_and_shift():
    s = np.array([1.0, 3.0, 3.0, -0.0, 0.0, 3.0, 1.0])
    assert orc.prune_topk(s, [0, 7], 7)[0].tolist() == [1, 2, 5, 0, 6, 3, 4]
    assert orc.prune_topk(s, [0, 7], 2)[0].tolist() == [1, 2]
    rng = np.random.default_rng(5)
    sc = rng.standard_normal(12 + 7)
    off = [0, 12, 19]
    a = orc.prune_topk(sc, off, 3)
    shifted = sc.copy(); shifted[:12] += 5.0; shifted[12:] -= 11.0     # per-prompt constant C
    assert np.array_equal(a, orc.prune_topk(shifted, off, 3))
    for b in range(2):
        assert a[b].tolist() == _brute_topk(sc[off[b]:off[b + 1]], 3)


def test_topk_exhaustive_small_with_ties():
    vals = [0.0, 1.0, 1.0, 2.0]
    for perm in set(itertools.permutations(vals)):
        s = np.array(perm)
        for k in (1, 2, 3, 4):
            assert orc.prune_topk(s, [0, 4], k)[0].tolist() == _brute_topk(s, k)


def test_topk_minus_inf_and_nan_order():
    s = np.array([-np.inf, np.nan, 2.0, -np.inf, np.nan, 1.0])
    assert orc.prune_topk(s, [0, 6], 6)[0].tolist() == [2, 5, 0, 3, 1, 4]
