"""Host-decided error paths of sp_forkjoin_prefill / sp_pruned_decode through the C ABI (nothing is
launched: every check happens before any kernel), and sp_plan_update / plan recycling with parity after
every change of table."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

import sp_synth
from oracle import sp_oracle as orc
from paper_2404_06910_amd import binding as B

from gpu_util import check_attn, dev, make_plan

pytestmark = pytest.mark.gpu

INVALID, BAD_TABLE, UNSUPPORTED = -1, -2, -3


@pytest.fixture(scope="module")
def ctx():
    c = B.Context(0)
    yield c
    c.close()


def _expect(ctx, status, fn, *args):
    st = fn(*args)
    assert st == status, (st, status)
    msg = B.lib().sp_last_error(ctx._h)
    assert msg and len(msg) > 8, msg


def test_prefill_argument_errors(ctx):
    st = sp_synth.forkjoin_segtable(8, [[16, 9]], 4)
    Hq, Hkv, d = 4, 2, 128
    plan = make_plan(ctx, st, Hq, Hkv, d, "bf16")
    Q = torch.zeros((st.n_tokens, Hq, d), dtype=torch.bfloat16, device="cuda")
    K = torch.zeros((st.n_tokens, Hkv, d), dtype=torch.bfloat16, device="cuda")
    V = torch.zeros_like(K); O = torch.zeros_like(Q)
    L = B.lib()
    q, k, v, o = Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr()
    qts, qhs, kts, khs = Hq * d, d, Hkv * d, d
    call = lambda *a: L.sp_forkjoin_prefill(ctx._h, plan._h, *a)
    ok = (q, k, v, o, qts, qhs, kts, khs, 0.1)
    assert call(*ok) == 0
    _expect(ctx, INVALID, call, None, k, v, o, qts, qhs, kts, khs, 0.1)            # NULL tensor
    _expect(ctx, INVALID, call, q, k, v, q, qts, qhs, kts, khs, 0.1)               # O aliases Q
    _expect(ctx, INVALID, call, q, k, v, k, qts, qhs, kts, khs, 0.1)               # O aliases K
    _expect(ctx, UNSUPPORTED, call, q + 2, k, v, o, qts, qhs, kts, khs, 0.1)       # base not 16-byte aligned
    _expect(ctx, UNSUPPORTED, call, q, k, v, o, qts + 4, qhs, kts, khs, 0.1)       # stride not a multiple of 16 B
    _expect(ctx, INVALID, call, q, k, v, o, qts, d - 8, kts, khs, 0.1)             # head stride < head_dim
    _expect(ctx, INVALID, call, q, k, v, o, d, 2 * d, kts, khs, 0.1)               # Q not token-major
    _expect(ctx, UNSUPPORTED, call, q, k, v, o, 1 << 26, qhs, kts, khs, 0.1)       # token stride too large
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        _expect(ctx, INVALID, call, q, k, v, o, qts, qhs, kts, khs, bad)           # softmax scale
    other = B.Context(0)
    st_ = L.sp_forkjoin_prefill(other._h, plan._h, *ok)                            # plan of another context
    assert st_ == INVALID and b"context" in L.sp_last_error(other._h)
    host_only = B.Plan(None, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, st.seg_path,
                       st.n_tokens, Hq, Hkv, d, B.SP_BF16)
    assert L.sp_forkjoin_prefill(ctx._h, host_only._h, *ok) == INVALID             # host-only plan cannot launch
    other.close()
    torch.cuda.synchronize()


def test_decode_argument_errors(ctx):
    st = sp_synth.forkjoin_segtable(8, [[16, 9, 12]], 4)
    H, d = 2, 64
    pos = sp_synth.classical_positions(st)
    plan = make_plan(ctx, st, H, H, d, "bf16")
    plan_b = make_plan(ctx, st, H, H, d, "bf16", tok_pos=pos, slopes=sp_synth.geometric_slopes(H))
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    K, V = z(st.n_tokens, H, d), z(st.n_tokens, H, d)
    Kr, Vr = z(1, 4, H, d), z(1, 4, H, d)
    qn, kn, vn, o = z(1, H, d), z(1, H, d), z(1, H, d), z(1, H, d)
    kept = dev(np.array([[0, 2]], np.int32))
    L = B.lib()

    def call(plan_, kept_=kept.data_ptr(), k=2, Kp=K.data_ptr(), kts=H * d, khs=d, cap=4, add=0, pos_resp=None,
             new_pos=None, scale=0.125, q=qn.data_ptr()):
        return L.sp_pruned_decode(ctx._h, plan_._h, kept_, k, Kp, V.data_ptr(), kts, khs, Kr.data_ptr(), Vr.data_ptr(),
                                  pos_resp, cap, None, add, new_pos, q, kn.data_ptr(), vn.data_ptr(), o.data_ptr(), scale)

    assert call(plan) == 0
    _expect(ctx, INVALID, lambda: call(plan, k=-1))
    _expect(ctx, INVALID, lambda: call(plan, kept_=None))
    _expect(ctx, INVALID, lambda: call(plan, cap=0))
    _expect(ctx, INVALID, lambda: call(plan, add=-1))
    _expect(ctx, INVALID, lambda: call(plan, Kp=None))
    _expect(ctx, INVALID, lambda: call(plan, scale=float("nan")))
    _expect(ctx, UNSUPPORTED, lambda: call(plan, kts=H * d + 4))
    _expect(ctx, UNSUPPORTED, lambda: call(plan, khs=d - 8))
    _expect(ctx, UNSUPPORTED, lambda: call(plan, q=qn.data_ptr() + 2))
    _expect(ctx, INVALID, lambda: call(plan_b))                                     # slopes without positions
    pr = torch.zeros((1, 4), device="cuda"); npos = torch.zeros(1, device="cuda")
    assert call(plan_b, pos_resp=pr.data_ptr(), new_pos=npos.data_ptr()) == 0
    # a joined cache of more than 120 disjoint ranges: 61 kept paths whose two segments are not adjacent
    n = 61
    st2 = sp_synth.forkjoin_segtable(4, [[2] * n], 2, "grouped")
    plan2 = make_plan(ctx, st2, H, H, d, "bf16")
    K2 = z(st2.n_tokens, H, d)
    kept2 = dev(np.arange(n, dtype=np.int32)[None])
    st_ = L.sp_pruned_decode(ctx._h, plan2._h, kept2.data_ptr(), n, K2.data_ptr(), K2.data_ptr(), H * d, d, Kr.data_ptr(),
                             Vr.data_ptr(), None, 4, None, 0, None, qn.data_ptr(), kn.data_ptr(), vn.data_ptr(),
                             o.data_ptr(), 0.125)
    assert st_ == UNSUPPORTED and b"ranges" in L.sp_last_error(ctx._h)
    torch.cuda.synchronize()


def _prefill_and_check(ctx, plan, st, rng, Hq, Hkv, d, what):
    f = lambda *s: sp_synth.round_to_dtype(rng.standard_normal(s, dtype=np.float32), "bf16")
    q, k, v = f(st.n_tokens, Hq, d), f(st.n_tokens, Hkv, d), f(st.n_tokens, Hkv, d)
    Q, K, V = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16")
    O = torch.full_like(Q, float("nan"))
    ctx.sp_forkjoin_prefill(plan, Q, K, V, O, 1 / math.sqrt(d))
    torch.cuda.synchronize()
    ref = orc.forkjoin_prefill(q, k, v, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent,
                               1 / math.sqrt(d))
    check_attn(O.float().cpu().numpy(), ref, "bf16", what)


def test_plan_update_across_three_tables_and_recycled_blocks(ctx):
    """One plan object rebuilt in place for three different tables (a larger one, then a smaller one) with
    parity after each, the update enqueued right behind the launch that still reads the old tables; then
    plans created and destroyed in a loop (their device blocks are recycled) with parity each time."""
    rng = np.random.default_rng(12)
    Hq, Hkv, d = 4, 2, 128
    tables = [sp_synth.forkjoin_segtable(16, [[40, 33]], 8),
              sp_synth.forkjoin_segtable(50, [[70, 129, 64], [64, 31]], 7, "grouped"),
              sp_synth.forkjoin_segtable(3, [[20]], 5)]
    plan = make_plan(ctx, tables[0], Hq, Hkv, d, "bf16")
    _prefill_and_check(ctx, plan, tables[0], rng, Hq, Hkv, d, "table 0")
    for i in (1, 2, 0):
        t = tables[i]
        plan.update(t.prompt_seg_off, t.seg_tok_start, t.seg_tok_len, t.seg_parent, t.seg_path, t.n_tokens)
        _prefill_and_check(ctx, plan, t, rng, Hq, Hkv, d, "updated to table %d" % i)
    plan.close()
    for rep in range(6):
        t = tables[rep % 3]
        p = make_plan(ctx, t, Hq, Hkv, d, "bf16")
        _prefill_and_check(ctx, p, t, rng, Hq, Hkv, d, "recycled %d" % rep)
        p.close()


def test_context_may_be_destroyed_before_its_plans():
    c = B.Context(0)
    st = sp_synth.forkjoin_segtable(8, [[16, 9]], 4)
    p = make_plan(c, st, 2, 2, 64, "bf16")
    c.close()
    p.close()                                               # must not touch freed memory
