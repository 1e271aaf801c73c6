"""sp_path_saliency_static (the entry point that allocates nothing) against sp_path_saliency, through
the C ABI: two calls in a row, the second with a smaller input, bit for bit; and against the oracle."""
import numpy as np
import pytest
import torch

import sp_synth
from oracle import sp_oracle as orc
from paper_2404_06910_amd import binding as B

from gpu_util import dev

pytestmark = pytest.mark.gpu


def _case(rng, R, n, vocab, dtype):
    x = sp_synth.round_to_dtype(rng.standard_normal((R, vocab), dtype=np.float32) * 3, dtype)
    tgt = rng.integers(0, vocab, size=R).astype(np.int32)
    tgt[rng.integers(0, R, size=max(1, R // 10))] = -1            # some rows are not scored
    rp = rng.integers(0, n, size=R).astype(np.int32)
    prior = rng.standard_normal(n).astype(np.float32)
    return x, tgt, rp, prior


def test_static_scratch_entry_point_matches_the_allocating_one():
    ctx = B.Context(0)
    rng = np.random.default_rng(77)
    # second call smaller in rows, slots and vocabulary: accumulators left by the first must be clean
    for (R, n, vocab, dtype, mode) in [(301, 37, 4104, "bf16", B.SALIENCY_SUM), (64, 5, 1000, "bf16", B.SALIENCY_MEAN),
                                       (200, 64, 520, "f32", B.SALIENCY_SUM)]:
        print("case:", R, n, vocab, dtype, mode, flush=True)
        x, tgt, rp, prior = _case(rng, R, n, vocab, dtype)
        X, T, P, PR = dev(x, dtype), dev(tgt), dev(rp), dev(prior)
        a = torch.full((n,), float("nan"), device="cuda")
        b = torch.full((n,), float("nan"), device="cuda")
        ctx.sp_path_saliency(X, T, P, n, a, prior=PR, mode=mode)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]              # device-wide: sees any hipMalloc, not only torch's
        ctx.sp_path_saliency_static(X, T, P, n, b, prior=PR, mode=mode)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before
        got_a, got_b = a.cpu().numpy(), b.cpu().numpy()
        assert np.array_equal(got_a, got_b), (got_a, got_b)
        ref = orc.path_saliency(x, tgt, rp, n, prior=prior, mode="mean" if mode == B.SALIENCY_MEAN else "sum")
        np.testing.assert_allclose(got_b, ref, rtol=1e-3, atol=1e-5)
    # many slots and rows scattered over them: per-lane atomics into the static array's accumulators
    R, n, vocab = 96, 5000, 520
    x, tgt, rp, prior = _case(rng, R, n, vocab, "f32")
    X, T, P = dev(x, "f32"), dev(tgt), dev(rp)
    for _ in range(2):                                          # twice: the accumulators must come back to zero
        b = torch.full((n,), float("nan"), device="cuda")
        ctx.sp_path_saliency_static(X, T, P, n, b)
        torch.cuda.synchronize()
        np.testing.assert_allclose(b.cpu().numpy(), orc.path_saliency(x, tgt, rp, n), rtol=1e-3, atol=1e-5)
    # beyond the static maximum: a clear error, nothing launched
    n_big = 16384 + 1
    with pytest.raises(B.SpError) as e:
        ctx.sp_path_saliency_static(X, T, P, n_big, torch.empty(n_big, device="cuda"))
    assert e.value.status == -3 and "static scratch" in str(e.value)
    ctx.close()
