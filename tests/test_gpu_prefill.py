"""GPU parity of sp_forkjoin_prefill against the CPU oracle (through the C ABI)."""
import math
import zlib

import numpy as np
import pytest
import torch

import sp_synth
from oracle import sp_oracle as orc
from paper_2404_06910_amd import binding as B

from fullsize_oracle import oracle_by_segment as _oracle_by_segment
from gpu_util import check_attn, covered_tokens, dev, make_plan, run_prefill

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = B.Context(0)
    yield c
    c.close()


def _oracle(st, q, k, v, scale, **kw):
    return orc.forkjoin_prefill(q, k, v, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, scale, **kw)


def _rand(rng, T, Hq, Hkv, d, dtype):
    f = lambda *s: sp_synth.round_to_dtype(rng.standard_normal(s, dtype=np.float32), dtype)
    return f(T, Hq, d), f(T, Hkv, d), f(T, Hkv, d)


def test_config1_tiny_fp32_all_elements(ctx):
    print("case: c1_tiny_f32", flush=True)
    inp = sp_synth.make_inputs(sp_synth.WORKLOADS["c1_tiny_f32"], with_logits=False, with_decode=False)
    got, _ = run_prefill(ctx, inp.st, inp.q, inp.k, inp.v, "f32")
    ref = _oracle(inp.st, inp.q, inp.k, inp.v, 1 / 8.0)
    check_attn(got, ref, "f32", "c1")
    # with linear distance bias on classical positions
    slopes = sp_synth.geometric_slopes(4)
    got, _ = run_prefill(ctx, inp.st, inp.q, inp.k, inp.v, "f32", tok_pos=inp.tok_pos, slopes=slopes)
    ref = _oracle(inp.st, inp.q, inp.k, inp.v, 1 / 8.0, tok_pos=inp.tok_pos, alibi_slopes=slopes)
    check_attn(got, ref, "f32", "c1+bias")


SMALL = [
    # (dtype, Hq, Hkv, d, P, doc_lens per prompt, Lq, packing, bias)
    ("bf16", 2, 2, 128, 16, [[32, 32]], 8, "interleaved", False),
    ("bf16", 4, 4, 128, 64, [[128, 100, 1, 33], [5, 200]], 24, "interleaved", False),     # ragged, path of length 1
    ("bf16", 8, 2, 128, 37, [[65, 31, 96]], 1, "interleaved", True),                      # GQA 4, Lq = 1, bias
    ("bf16", 4, 2, 64, 50, [[70, 129], [64]], 7, "grouped", False),                       # GQA 2, d = 64, grouped
    ("bf16", 8, 1, 64, 3, [[40, 41, 42]], 9, "grouped", True),                            # GQA 8
    ("bf16", 3, 3, 128, 130, [[300]], 31, "interleaved", False),                          # one doc = causal, 461 rows
    ("bf16", 6, 2, 128, 20, [[45, 77]], 5, "interleaved", False),                         # GQA 3 (odd group)
    ("bf16", 4, 4, 128, 40, [[100, 64, 77], [33, 128]], 24, "interleaved", True),         # ungrouped heads, bias
    ("bf16", 4, 2, 128, 64, [[128, 31], [200]], 9, "grouped", True),                      # GQA 2, bias
    ("bf16", 8, 8, 64, 16, [[32, 17]], 8, "interleaved", True),                           # one head group per XCD slice
    ("bf16", 16, 16, 128, 600, [[40, 33]], 8, "interleaved", False),                      # sliced; long preamble: head chunks of 1
    ("bf16", 4, 4, 128, 1100, [[20, 31]], 4, "grouped", False),                           # unsliced; head chunks of 1
    ("f32", 4, 2, 128, 33, [[47, 20], [64, 3, 9]], 6, "grouped", True),
    ("f32", 2, 2, 64, 1, [[1]], 1, "interleaved", False),                                 # degenerate: 3 tokens
]


@pytest.mark.parametrize("case", SMALL, ids=lambda c: "%s-h%d/%d-d%d-P%d-%s%s" % (c[0], c[1], c[2], c[3], c[4], c[7][:3], "-b" if c[8] else ""))
def test_small_shapes_all_elements(ctx, case):
    dtype, Hq, Hkv, d, P, lens, Lq, packing, bias = case
    print("case:", case, flush=True)
    rng = np.random.default_rng(zlib.crc32(str(case).encode()))
    st = sp_synth.forkjoin_segtable(P, lens, Lq, packing)
    q, k, v = _rand(rng, st.n_tokens, Hq, Hkv, d, dtype)
    pos = slopes = None
    if bias:
        # equilibrium positions from the oracle (ragged documents -> real-valued positions)
        pos = np.zeros(st.n_tokens, np.float32)
        for b, ll in enumerate(lens):
            a, dd, qq = orc.equilibrium_positions(P, ll, Lq)
            s0 = st.seg_tok_start[st.preamble_seg[b]]; pos[s0:s0 + P] = a
            for i in range(len(ll)):
                slot = st.path_off[b] + i
                s0 = st.seg_tok_start[st.doc_seg[slot]]; pos[s0:s0 + ll[i]] = dd[i]
                s0 = st.seg_tok_start[st.query_seg[slot]]; pos[s0:s0 + Lq] = qq
        slopes = sp_synth.geometric_slopes(Hq)
    got, plan = run_prefill(ctx, st, q, k, v, dtype, tok_pos=pos, slopes=slopes)
    ref = _oracle(st, q, k, v, 1 / math.sqrt(d), tok_pos=pos, alibi_slopes=slopes)
    check_attn(got, ref, dtype, str(case))
    # bitwise determinism (no float atomics, fixed reduction order)
    again, _ = run_prefill(ctx, st, q, k, v, dtype, tok_pos=pos, slopes=slopes, plan=plan)
    assert np.array_equal(got, again, equal_nan=True)


def test_general_tree_with_gaps_and_untouched_rows(ctx):
    # deeper chains, several shared segments, scrambled packing with uncovered tokens
    from test_host_plan import _random_table
    for seed in (11, 12):
        rng = np.random.default_rng(seed)
        t = _random_table(rng, 3, scramble=True)
        T = t["n_tokens"]
        q, k, v = _rand(rng, T, 4, 2, 64, "bf16")
        print("case: random tree seed", seed, "tokens", T, flush=True)
        plan = B.Plan(ctx, t["prompt_seg_off"], t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], t["seg_path"], T,
                      4, 2, 64, B.SP_BF16)
        Q, K, V = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16")
        O = torch.full_like(Q, 7.0)
        ctx.sp_forkjoin_prefill(plan, Q, K, V, O, 0.125)
        torch.cuda.synchronize()
        got = O.float().cpu().numpy()
        ref = orc.forkjoin_prefill(q, k, v, t["prompt_seg_off"], t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], 0.125)
        check_attn(got, ref, "bf16", "tree %d" % seed)
        assert np.all(got[np.isnan(ref)] == 7.0)            # uncovered tokens are left untouched


@pytest.mark.parametrize("Hq,Hkv,d,n_chain,bias", [(4, 4, 128, 11, False), (8, 2, 128, 6, True), (2, 2, 64, 12, True),
                                                   (4, 1, 128, 3, False), (2, 2, 128, 40, False)])
def test_deep_chains_of_separate_ranges(ctx, Hq, Hkv, d, n_chain, bias):
    """A leaf behind a chain of documents that lie apart in the token pool (the shape of a late round
    of iterative superposition): its ancestors are n_chain + 1 separate token ranges, of lengths that
    are not multiples of the key-stage size, so stages straddle ranges; more ranges than the kernel
    keeps beside its work items are covered too."""
    rng = np.random.default_rng(100 + n_chain)
    lens = [int(x) for x in rng.integers(9, 70, n_chain)]
    root_len, leaf_len, gap = 21, 83, 5
    # pool: root, then the chain's documents in reverse order with unused tokens between them, then the leaf
    start, tok = {}, root_len + gap
    for i in reversed(range(n_chain)):
        start[i] = tok; tok += lens[i] + gap
    leaf_start = tok; T = tok + leaf_len
    seg_start = [0] + [start[i] for i in range(n_chain)] + [leaf_start]
    seg_len = [root_len] + lens + [leaf_len]
    parent = [-1] + list(range(n_chain)) + [n_chain]
    path = [-1] * (n_chain + 1) + [0]
    i32 = lambda a: np.asarray(a, np.int32)
    off = i32([0, len(seg_start)])
    q, k, v = _rand(rng, T, Hq, Hkv, d, "bf16")
    pos = slopes = None
    if bias:
        pos = rng.uniform(0, 300, T).astype(np.float32); slopes = sp_synth.geometric_slopes(Hq)
    plan = B.Plan(ctx, off, i32(seg_start), i32(seg_len), i32(parent), i32(path), T, Hq, Hkv, d, B.SP_BF16,
                  tok_pos=pos, alibi_slopes=slopes)
    Q, K, V = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16")
    O = torch.full_like(Q, 7.0)
    scale = 1 / math.sqrt(d)
    ctx.sp_forkjoin_prefill(plan, Q, K, V, O, scale)
    torch.cuda.synchronize()
    got = O.float().cpu().numpy()
    ref = orc.forkjoin_prefill(q, k, v, off, i32(seg_start), i32(seg_len), i32(parent), scale, tok_pos=pos,
                               alibi_slopes=slopes)
    check_attn(got, ref, "bf16", "chain of %d" % n_chain)
    assert np.all(got[np.isnan(ref)] == 7.0)                # the gaps are left untouched


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_cached_segments_random_trees(ctx, dtype):
    # Sec. 3.3.1 / Alg. 2: cached segments serve as keys; their output rows are not produced
    from test_host_plan import _random_table
    for seed in (21, 22, 23):
        rng = np.random.default_rng(seed)
        t = _random_table(rng, 3, scramble=seed != 22)
        T = t["n_tokens"]; S = len(t["seg_parent"])
        cached = (rng.random(S) < 0.5).astype(np.uint8)
        q, k, v = _rand(rng, T, 4, 2, 64, dtype)
        print("case: cached random tree seed", seed, dtype, "tokens", T, flush=True)
        plan = B.Plan(ctx, t["prompt_seg_off"], t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], t["seg_path"], T,
                      4, 2, 64, B.SP_BF16 if dtype == "bf16" else B.SP_F32, seg_cached=cached)
        Q, K, V = dev(q, dtype), dev(k, dtype), dev(v, dtype)
        O = torch.full_like(Q, 7.0)
        ctx.sp_forkjoin_prefill(plan, Q, K, V, O, 0.125)
        torch.cuda.synchronize()
        got = O.float().cpu().numpy()
        ref = orc.forkjoin_prefill(q, k, v, t["prompt_seg_off"], t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], 0.125)
        for s in range(S):
            if cached[s]:
                ref[t["seg_tok_start"][s]:t["seg_tok_start"][s] + t["seg_tok_len"][s]] = np.nan
        if not np.isnan(ref).all():
            check_attn(got, ref, dtype, "cached tree %d" % seed)
        assert np.all(got[np.isnan(ref)] == 7.0)            # cached and uncovered rows are left untouched


_SHAPES = [(2, 2, 128), (4, 2, 128), (8, 2, 128), (4, 1, 64), (6, 3, 64), (4, 4, 64), (8, 2, 64), (3, 1, 128)]


@pytest.mark.parametrize("seed", range(10))
def test_random_forests_long_segments(ctx, seed):
    """Random forests with segments of 1..90 tokens scattered over the pool (so ancestors are several
    separate ranges of arbitrary length), random cached flags, every head grouping, with and without
    bias: all computed rows against the oracle, everything else untouched."""
    from test_host_plan import _random_table
    rng = np.random.default_rng(500 + seed)
    t = _random_table(rng, 2 + seed % 2, scramble=seed % 3 != 0)
    S = len(t["seg_parent"])
    # stretch the segments: new lengths, token ranges handed out again in random order with gaps
    lens = rng.integers(1, 91, S).astype(np.int32)
    order = rng.permutation(S) if seed % 3 != 0 else np.arange(S)
    start = np.zeros(S, np.int32); tok = int(rng.integers(0, 5))
    for sgm in order:
        start[sgm] = tok; tok += int(lens[sgm]) + int(rng.integers(0, 4))
    T = tok + 3
    Hq, Hkv, d = _SHAPES[seed % len(_SHAPES)]
    bias = seed % 2 == 1
    cached = (rng.random(S) < 0.3).astype(np.uint8) if seed % 4 >= 2 else None
    q, k, v = _rand(rng, T, Hq, Hkv, d, "bf16")
    pos = slopes = None
    if bias:
        pos = rng.uniform(0, 400, T).astype(np.float32); slopes = sp_synth.geometric_slopes(Hq)
    print("case: forest seed", seed, "tokens", T, "segments", S, (Hq, Hkv, d), "bias", bias, flush=True)
    plan = B.Plan(ctx, t["prompt_seg_off"], start, lens, t["seg_parent"], t["seg_path"], T, Hq, Hkv, d, B.SP_BF16,
                  tok_pos=pos, alibi_slopes=slopes, seg_cached=cached)
    Q, K, V = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16")
    O = torch.full_like(Q, 7.0)
    scale = 1 / math.sqrt(d)
    ctx.sp_forkjoin_prefill(plan, Q, K, V, O, scale)
    torch.cuda.synchronize()
    got = O.float().cpu().numpy()
    ref = orc.forkjoin_prefill(q, k, v, t["prompt_seg_off"], start, lens, t["seg_parent"], scale, tok_pos=pos,
                               alibi_slopes=slopes)
    if cached is not None:
        for sgm in range(S):
            if cached[sgm]:
                ref[start[sgm]:start[sgm] + lens[sgm]] = np.nan
    if not np.isnan(ref).all():
        check_attn(got, ref, "bf16", "forest %d" % seed)
    assert np.all(got[np.isnan(ref)] == 7.0)


@pytest.mark.parametrize("packing", ["interleaved", "grouped"])
def test_split_phase_prefill_equals_one_pass(ctx, packing):
    """Path caching (Sec. 3.3.1): preamble and documents are processed ahead of time, the query
    copies online against the cached K/V. The online pass computes the query rows only and they
    agree with the one-pass result (same oracle)."""
    rng = np.random.default_rng(31)
    lens = [[150, 64, 201], [97, 130]]
    P, Lq, Hq, Hkv, d = 70, 19, 8, 2, 128
    st = sp_synth.forkjoin_segtable(P, lens, Lq, packing)
    q, k, v = _rand(rng, st.n_tokens, Hq, Hkv, d, "bf16")
    print("case: split phase", packing, flush=True)
    is_query = np.zeros(st.n_segments, bool); is_query[np.asarray(st.query_seg)] = True
    ref = _oracle(st, q, k, v, 1 / math.sqrt(d))
    one_pass, _ = run_prefill(ctx, st, q, k, v, "bf16")
    offline = make_plan(ctx, st, Hq, Hkv, d, "bf16", seg_cached=is_query.astype(np.uint8))      # query rows skipped
    online = make_plan(ctx, st, Hq, Hkv, d, "bf16", seg_cached=(~is_query).astype(np.uint8))    # query rows only
    assert offline.visible_pairs() + online.visible_pairs() == make_plan(ctx, st, Hq, Hkv, d, "bf16").visible_pairs()
    Q, K, V = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16")
    O = torch.full_like(Q, float("nan"))
    ctx.sp_forkjoin_prefill(offline, Q, K, V, O, 1 / math.sqrt(d))
    torch.cuda.synchronize()
    qrow = np.zeros(st.n_tokens, bool)
    for s in np.asarray(st.query_seg):
        qrow[st.seg_tok_start[s]:st.seg_tok_start[s] + st.seg_tok_len[s]] = True
    after_offline = O.float().cpu().numpy()
    assert np.isnan(after_offline[qrow]).all() and not np.isnan(after_offline[~qrow]).any()
    ctx.sp_forkjoin_prefill(online, Q, K, V, O, 1 / math.sqrt(d))
    torch.cuda.synchronize()
    got = O.float().cpu().numpy()
    check_attn(got, ref, "bf16", "split phase")
    assert np.array_equal(got[~qrow], after_offline[~qrow])             # the online pass writes query rows only
    assert np.abs(got - one_pass).max() <= 2e-2


def test_independence_of_paths_is_bitwise(ctx):
    rng = np.random.default_rng(5)
    st = sp_synth.forkjoin_segtable(64, [[128, 90, 128]], 24)
    q, k, v = _rand(rng, st.n_tokens, 4, 4, 128, "bf16")
    base, plan = run_prefill(ctx, st, q, k, v, "bf16")
    lo = int(st.seg_tok_start[st.doc_seg[1]]); hi = int(st.seg_tok_start[st.query_seg[1]] + 24)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    k2[lo:hi] = -k2[lo:hi]; v2[lo:hi] = v2[lo:hi] * 2; q2[lo:hi] = 0
    pert, _ = run_prefill(ctx, st, q2, k2, v2, "bf16", plan=plan)
    others = np.ones(st.n_tokens, bool); others[lo:hi] = False
    assert np.array_equal(base[others], pert[others])


@pytest.mark.parametrize("dtype,Hq,Hkv", [("bf16", 4, 4), ("bf16", 8, 2), ("f32", 4, 2)])
def test_head_major_kv_cache_layout(ctx, dtype, Hq, Hkv):
    """K and V stored per head ([n_kv_heads, n_tokens, d], passed as strided [n_tokens, n_kv_heads, d]
    views) give bit for bit what the token-major tensors give, and that matches the oracle."""
    rng = np.random.default_rng(11)
    st = sp_synth.forkjoin_segtable(40, [[100, 64, 77], [33, 128]], 24)
    q, k, v = _rand(rng, st.n_tokens, Hq, Hkv, 128, dtype)
    scale = 1 / math.sqrt(128)
    base, plan = run_prefill(ctx, st, q, k, v, dtype)
    check_attn(base, _oracle(st, q, k, v, scale), dtype, "token-major")
    Q, K, V = dev(q, dtype), dev(k, dtype), dev(v, dtype)
    Kh = K.transpose(0, 1).contiguous().transpose(0, 1)
    Vh = V.transpose(0, 1).contiguous().transpose(0, 1)
    assert Kh.stride(1) > Kh.stride(0) and torch.equal(Kh, K)
    O = torch.full_like(Q, float("nan"))
    ctx.sp_forkjoin_prefill(plan, Q, Kh, Vh, O, scale)
    torch.cuda.synchronize()
    got = O.float().cpu().numpy()
    cov = covered_tokens(st)
    assert np.array_equal(got[cov], base[cov])


FULL = ["c2_mha7b_bf16", "c3_ragged_bf16", "c4_gqa_bf16"]


def _check_every_pair(got, st, q, k, v, scale, name, tok_pos=None, slopes=None):
    """Every (prompt, head) pair, every row, element by element."""
    Hq = q.shape[1]
    worst = 0.0
    for b in range(st.n_prompts):
        toks, ref = _oracle_by_segment(st, q, k, v, scale, b, list(range(Hq)), tok_pos, slopes)
        for h in range(Hq):
            mx, _ = check_attn(got[toks, h], ref[:, h], "bf16", "%s b%d h%d" % (name, b, h))
            worst = max(worst, mx)
        print("  %s prompt %d: all %d heads ok (max-abs so far %.4f)" % (name, b, Hq, worst), flush=True)


@pytest.mark.parametrize("name", FULL)
def test_full_size_every_prompt_head_pair(ctx, name):
    """Full workload shape in the launch configuration the benchmark times: EVERY (prompt, head) pair and
    every token row against the oracle, element by element; two pairs are also evaluated by the oracle's
    dense whole-prompt call."""
    wl = sp_synth.WORKLOADS[name]
    print("case:", name, flush=True)
    inp = sp_synth.make_inputs(wl, with_logits=False, with_decode=False)
    st = inp.st
    got, plan = run_prefill(ctx, st, inp.q, inp.k, inp.v, "bf16")
    assert not np.isnan(got[covered_tokens(st)]).any()
    scale = 1 / math.sqrt(wl.head_dim)
    _check_every_pair(got, st, inp.q, inp.k, inp.v, scale, name)
    rng = np.random.default_rng(1)
    for _ in range(1 if name == "c3_ragged_bf16" else 2):
        b = int(rng.integers(0, wl.n_prompts)); h = int(rng.integers(0, wl.n_q_heads))
        ref = _oracle(st, inp.q, inp.k, inp.v, scale, prompts=[b], heads=[h])
        check_attn(got, ref, "bf16", "%s dense b%d h%d" % (name, b, h))
    # property at full size: constant V rows give that constant back whatever the mask (softmax sums to 1)
    V1 = torch.ones(inp.v.shape, dtype=torch.bfloat16, device="cuda") * 0.5
    Q, K = dev(inp.q, "bf16"), dev(inp.k, "bf16")
    O = torch.empty_like(Q)
    ctx.sp_forkjoin_prefill(plan, Q, K, V1, O, scale)
    torch.cuda.synchronize()
    assert torch.all((O.float() - 0.5).abs() <= 2 ** -8)


def test_full_size_ragged_with_equilibrium_bias_every_pair(ctx):
    """The ragged workload with equilibrium positions (Sec. 3.2.2 Eq. 1, from the oracle) and a linear
    distance penalty per head: the BIAS kernel variant at the size the benchmark times, every pair."""
    wl = sp_synth.WORKLOADS["c3_ragged_bf16"]
    print("case: c3 + bias", flush=True)
    inp = sp_synth.make_inputs(wl, with_logits=False, with_decode=False)
    st = inp.st
    pos = np.zeros(st.n_tokens, np.float32)
    for b in range(st.n_prompts):
        slots = range(int(st.path_off[b]), int(st.path_off[b + 1]))
        lens = [int(st.seg_tok_len[st.doc_seg[s]]) for s in slots]
        a, dd, qq = orc.equilibrium_positions(wl.preamble_len, lens, wl.query_len)
        s0 = st.seg_tok_start[st.preamble_seg[b]]; pos[s0:s0 + wl.preamble_len] = a
        for i, s in enumerate(slots):
            s0 = st.seg_tok_start[st.doc_seg[s]]; pos[s0:s0 + lens[i]] = dd[i]
            s0 = st.seg_tok_start[st.query_seg[s]]; pos[s0:s0 + wl.query_len] = qq
    slopes = sp_synth.geometric_slopes(wl.n_q_heads)
    got, _ = run_prefill(ctx, st, inp.q, inp.k, inp.v, "bf16", tok_pos=pos, slopes=slopes)
    _check_every_pair(got, st, inp.q, inp.k, inp.v, 1 / math.sqrt(wl.head_dim), "c3+bias", pos.astype(np.float64),
                      slopes)
