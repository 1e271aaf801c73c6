"""GPU parity of sp_pruned_decode against the CPU oracle, plus the chained pipeline."""
import math

import numpy as np
import pytest
import torch

import sp_synth
from oracle import sp_oracle as orc
from paper_2404_06910_amd import binding as B

from gpu_util import TORCH_DT, attn_tol, dev, make_plan

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = B.Context(0)
    yield c
    c.close()


class DecodeRun:
    """Drives sp_pruned_decode step by step and keeps what the oracle needs."""

    def __init__(self, ctx, st, k_pre, v_pre, kept, Hq, dtype, cap, tok_pos=None, slopes=None, resp_len0=None):
        self.ctx, self.st, self.dtype, self.cap = ctx, st, dtype, cap
        T, Hkv, d = k_pre.shape
        self.Hq, self.Hkv, self.d = Hq, Hkv, d
        self.plan = make_plan(ctx, st, Hq, Hkv, d, dtype, tok_pos, slopes)
        self.K, self.V = dev(k_pre, dtype), dev(v_pre, dtype)
        Bn = st.n_prompts
        self.kept = dev(np.asarray(kept, np.int32))
        self.k = self.kept.shape[1]
        self.Kr = torch.zeros((Bn, cap, Hkv, d), dtype=TORCH_DT[dtype], device="cuda")
        self.Vr = torch.zeros_like(self.Kr)
        self.bias = slopes is not None
        self.pos_resp = torch.zeros((Bn, cap), device="cuda") if self.bias else None
        self.resp_len = None if resp_len0 is None else dev(np.asarray(resp_len0, np.int32))
        self.scale = 1 / math.sqrt(d)

    def step(self, s, qn, kn, vn, new_pos=None):
        o = torch.full((self.st.n_prompts, self.Hq, self.d), float("nan"), dtype=TORCH_DT[self.dtype], device="cuda")
        self.ctx.sp_pruned_decode(self.plan, self.kept, self.k, self.K, self.V, self.Kr, self.Vr, self.cap,
                                  dev(qn, self.dtype), dev(kn, self.dtype), dev(vn, self.dtype), o, self.scale,
                                  resp_len=self.resp_len, resp_len_add=s, pos_resp=self.pos_resp,
                                  new_pos=None if new_pos is None else dev(np.asarray(new_pos, np.float32)))
        torch.cuda.synchronize()
        return o.float().cpu().numpy()


def _check(got, ref, dtype, what):
    err = np.abs(got.astype(np.float64) - ref)
    mx, mean = attn_tol(dtype)
    assert not np.isnan(got).any(), what
    assert err.max() <= mx and err.mean() <= mean, "%s: max %.3e mean %.3e" % (what, err.max(), err.mean())


def test_config1_four_steps_fp32(ctx):
    wl = sp_synth.WORKLOADS["c1_tiny_f32"]
    inp = sp_synth.make_inputs(wl)
    st = inp.st
    ref_score = orc.path_saliency(inp.logits, inp.target, inp.row_path, st.n_slots)
    kept = orc.prune_topk(ref_score, st.path_off, wl.top_k)
    run = DecodeRun(ctx, st, inp.k, inp.v, kept, wl.n_q_heads, "f32", cap=8)
    idx = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, 0, kept[0])
    assert len(idx) == 16 + 40
    for s in range(wl.decode_steps):
        got = run.step(s, inp.dec_q[s], inp.dec_k[s], inp.dec_v[s])
        ref = orc.pruned_decode_step(inp.dec_q[s, 0], inp.dec_k[s, 0], inp.dec_v[s, 0], inp.k, inp.v, idx,
                                     inp.dec_k[:s, 0], inp.dec_v[:s, 0], 1 / 8.0)
        _check(got[0], ref, "f32", "c1 step %d" % s)
    # the response cache now holds the appended rows
    np.testing.assert_array_equal(run.Kr[0, :4].float().cpu().numpy(), inp.dec_k[:4, 0])
    np.testing.assert_array_equal(run.Vr[0, :4].float().cpu().numpy(), inp.dec_v[:4, 0])


CASES = [
    # dtype, Hq, Hkv, d, P, lens, Lq, packing, k, bias
    ("bf16", 4, 4, 128, 64, [[128, 100, 1, 33], [5, 200, 17, 40]], 24, "interleaved", 2, False),
    ("bf16", 8, 2, 128, 37, [[65, 31, 96]], 1, "grouped", 3, True),
    ("bf16", 8, 1, 64, 3, [[40, 41, 42], [7, 8, 9]], 9, "grouped", 1, True),
    ("bf16", 6, 2, 64, 20, [[45, 77]], 5, "interleaved", 2, False),
    ("f32", 4, 2, 128, 33, [[47, 20, 5], [64, 3, 9]], 6, "grouped", 2, True),
    ("f32", 2, 2, 64, 1, [[1]], 1, "interleaved", 1, False),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "%s-h%d/%d-d%d-k%d%s" % (c[0], c[1], c[2], c[3], c[8], "-b" if c[9] else ""))
def test_decode_small_shapes(ctx, case):
    dtype, Hq, Hkv, d, P, lens, Lq, packing, k, bias = case
    print("case:", case, flush=True)
    rng = np.random.default_rng(len(str(case)) * 7919 + Hq)
    st = sp_synth.forkjoin_segtable(P, lens, Lq, packing)
    f = lambda *s: sp_synth.round_to_dtype(rng.standard_normal(s, dtype=np.float32), dtype)
    kp, vp = f(st.n_tokens, Hkv, d), f(st.n_tokens, Hkv, d)
    Bn = st.n_prompts
    kept = np.stack([rng.permutation(len(lens[b]))[:k] for b in range(Bn)]).astype(np.int32)
    pos = slopes = None
    if bias:
        pos = (sp_synth.classical_positions(st) * 0.75).astype(np.float32)
        slopes = sp_synth.geometric_slopes(Hq)
    steps, cap = 5, 6
    resp0 = np.zeros(Bn, np.int32)
    run = DecodeRun(ctx, st, kp, vp, kept, Hq, dtype, cap, tok_pos=pos, slopes=slopes, resp_len0=resp0)
    dq, dk, dv = f(steps, Bn, Hq, d), f(steps, Bn, Hkv, d), f(steps, Bn, Hkv, d)
    for s in range(steps):
        npos = None
        if bias:
            npos = np.array([pos[orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len,
                                                        st.seg_path, b, kept[b])].max() + 1 + s for b in range(Bn)],
                            np.float32)
        got = run.step(s, dq[s], dk[s], dv[s], new_pos=npos)
        for b in range(Bn):
            idx = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, b, kept[b])
            kw = {}
            if bias:
                kw = dict(pos_new=npos[b], pos_prefill=pos, pos_resp=np.array([npos[b] - s + i for i in range(s)]),
                          alibi_slopes=slopes)
            ref = orc.pruned_decode_step(dq[s, b], dk[s, b], dv[s, b], kp, vp, idx, dk[:s, b], dv[:s, b],
                                         1 / math.sqrt(d), **kw)
            _check(got[b], ref, dtype, "%s step %d prompt %d" % (case, s, b))


def test_ignored_kept_entries_and_k_zero(ctx):
    rng = np.random.default_rng(3)
    st = sp_synth.forkjoin_segtable(8, [[10, 12, 9]], 4)
    f = lambda *s: sp_synth.round_to_dtype(rng.standard_normal(s, dtype=np.float32), "bf16")
    kp, vp = f(st.n_tokens, 2, 64), f(st.n_tokens, 2, 64)
    q, kn, vn = f(1, 2, 64), f(1, 2, 64), f(1, 2, 64)
    a = DecodeRun(ctx, st, kp, vp, [[1, -1]], 2, "bf16", 4).step(0, q, kn, vn)
    b = DecodeRun(ctx, st, kp, vp, [[1]], 2, "bf16", 4).step(0, q, kn, vn)
    assert np.array_equal(a, b)
    idx = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, 0, [])
    run = DecodeRun(ctx, st, kp, vp, np.zeros((1, 0), np.int32), 2, "bf16", 4)
    got = run.step(0, q, kn, vn)
    ref = orc.pruned_decode_step(q[0], kn[0], vn[0], kp, vp, idx, kn[:0], vn[:0], 0.125)
    _check(got[0], ref, "bf16", "k=0")


@pytest.mark.parametrize("bias", [False, True], ids=["plain", "bias"])
def test_config5_full_size_sampled(ctx, bias):
    """64 prompts x 32 heads, 2 of 20 paths kept, 256 steps; the oracle checks 32 (step, prompt) pairs
    spread over the steps (first, last, and a seeded sample in between), all heads; with bias = True the
    cache carries equilibrium positions and every head a linear distance penalty."""
    wl = sp_synth.WORKLOADS["c5_decode_bf16"]
    print("case: c5 bias=%s" % bias, flush=True)
    rng = np.random.default_rng(wl.seed)
    st = sp_synth.forkjoin_segtable(wl.preamble_len, [[wl.doc_len] * wl.n_paths] * wl.n_prompts, wl.query_len)
    Bn, H, d, S = wl.n_prompts, wl.n_kv_heads, wl.head_dim, wl.decode_steps
    g = torch.Generator(device="cuda"); g.manual_seed(wl.seed)
    K = torch.randn((st.n_tokens, H, d), generator=g, device="cuda").to(torch.bfloat16)
    V = torch.randn((st.n_tokens, H, d), generator=g, device="cuda").to(torch.bfloat16)
    dq = torch.randn((S, Bn, H, d), generator=g, device="cuda").to(torch.bfloat16)
    dk = torch.randn((S, Bn, H, d), generator=g, device="cuda").to(torch.bfloat16)
    dv = torch.randn((S, Bn, H, d), generator=g, device="cuda").to(torch.bfloat16)
    kept_np = np.stack([rng.permutation(wl.n_paths)[:wl.top_k] for _ in range(Bn)]).astype(np.int32)
    kept = dev(kept_np)
    pos = slopes = pos_resp = None
    new_pos = [None] * S
    if bias:
        a, dd, qq = orc.equilibrium_positions(wl.preamble_len, [wl.doc_len] * wl.n_paths, wl.query_len)
        pos = np.zeros(st.n_tokens, np.float32)
        for b in range(Bn):
            s0 = st.seg_tok_start[st.preamble_seg[b]]; pos[s0:s0 + wl.preamble_len] = a
            for i in range(wl.n_paths):
                slot = st.path_off[b] + i
                s0 = st.seg_tok_start[st.doc_seg[slot]]; pos[s0:s0 + wl.doc_len] = dd[i]
                s0 = st.seg_tok_start[st.query_seg[slot]]; pos[s0:s0 + wl.query_len] = qq
        slopes = sp_synth.geometric_slopes(H)
        pos_resp = torch.zeros((Bn, S), device="cuda")
        p0 = float(pos.max()) + 1.0
        new_pos = [torch.full((Bn,), p0 + s, device="cuda") for s in range(S)]
    plan = make_plan(ctx, st, H, H, d, "bf16", tok_pos=pos, slopes=slopes)
    Kr = torch.zeros((Bn, S, H, d), dtype=torch.bfloat16, device="cuda"); Vr = torch.zeros_like(Kr)
    outs = torch.empty((S, Bn, H, d), dtype=torch.bfloat16, device="cuda")
    for s in range(S):
        ctx.sp_pruned_decode(plan, kept, wl.top_k, K, V, Kr, Vr, S, dq[s], dk[s], dv[s], outs[s], 1 / math.sqrt(d),
                             resp_len_add=s, pos_resp=pos_resp, new_pos=new_pos[s])
    torch.cuda.synchronize()
    assert torch.equal(Kr, dk.transpose(0, 1)) and torch.equal(Vr, dv.transpose(0, 1))
    assert not torch.isnan(outs.float()).any()
    pairs = [(0, 0), (1, 63), (255, 17), (255, 63)] + [(int(rng.integers(0, S)), int(rng.integers(0, Bn))) for _ in range(28)]
    for s, b in pairs:
        idx = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, b, kept_np[b])
        assert len(idx) == 64 + 2 * 152
        tok = torch.from_numpy(idx).cuda()
        kp = np.zeros((st.n_tokens, H, d), np.float32); vp = np.zeros_like(kp)     # only gathered rows are filled
        kp[idx] = K[tok].float().cpu().numpy(); vp[idx] = V[tok].float().cpu().numpy()
        kw = {}
        if bias:
            kw = dict(pos_prefill=pos, pos_resp=np.array([p0 + i for i in range(s)], np.float64), pos_new=p0 + s,
                      alibi_slopes=slopes)
        ref = orc.pruned_decode_step(dq[s, b].float().cpu().numpy(), dk[s, b].float().cpu().numpy(),
                                     dv[s, b].float().cpu().numpy(), kp, vp, idx, dk[:s, b].float().cpu().numpy(),
                                     dv[:s, b].float().cpu().numpy(), 1 / math.sqrt(d), **kw)
        _check(outs[s, b].float().cpu().numpy(), ref, "bf16", "c5 step %d prompt %d" % (s, b))


def test_chained_pipeline_no_host_sync(ctx):
    """prefill -> saliency -> top-k -> decode with the kept table staying on the device."""
    wl = sp_synth.WORKLOADS["c2_mha7b_bf16"]
    inp = sp_synth.make_inputs(wl, n_prompts=2, decode_steps=2)
    st = inp.st
    Hq, Hkv, d = wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    # small vocabulary slice keeps the oracle quick; the structure is what is tested here
    Vv = 2048
    logits = inp.logits[:, :Vv]; target = inp.target % Vv
    plan = make_plan(ctx, st, Hq, Hkv, d, "bf16")
    Q, K, V = dev(inp.q, "bf16"), dev(inp.k, "bf16"), dev(inp.v, "bf16")
    O = torch.empty_like(Q)
    score = torch.empty(st.n_slots, device="cuda")
    kept = torch.empty((2, wl.top_k), dtype=torch.int32, device="cuda")
    Kr = torch.zeros((2, 4, Hkv, d), dtype=torch.bfloat16, device="cuda"); Vr = torch.zeros_like(Kr)
    o = torch.empty((2, Hq, d), dtype=torch.bfloat16, device="cuda")
    L = dev(np.ascontiguousarray(logits), "bf16")
    scale = 1 / math.sqrt(d)
    ctx.sp_forkjoin_prefill(plan, Q, K, V, O, scale)
    ctx.sp_path_saliency(L, dev(target), dev(inp.row_path), st.n_slots, score)
    ctx.sp_prune_topk(score, plan.path_offsets_device(), 2, wl.n_paths, wl.top_k, kept)
    ctx.sp_pruned_decode(plan, kept, wl.top_k, K, V, Kr, Vr, 4, dev(inp.dec_q[0], "bf16"), dev(inp.dec_k[0], "bf16"),
                         dev(inp.dec_v[0], "bf16"), o, scale)
    torch.cuda.synchronize()
    ref_score = orc.path_saliency(logits, target, inp.row_path, st.n_slots)
    np.testing.assert_allclose(score.cpu().numpy(), ref_score, rtol=1e-3)
    ref_kept = orc.prune_topk(ref_score, st.path_off, wl.top_k)
    # margin between the k-th and (k+1)-th oracle score must exceed the score tolerance for the
    # kept set to be decided; the seed used here satisfies it (asserted, not assumed)
    for b in range(2):
        srt = np.sort(ref_score[st.path_off[b]:st.path_off[b + 1]])[::-1]
        assert srt[wl.top_k - 1] - srt[wl.top_k] > 1e-3 * abs(srt[wl.top_k])
    assert np.array_equal(kept.cpu().numpy(), ref_kept)
    for b in range(2):
        idx = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, b, ref_kept[b])
        ref = orc.pruned_decode_step(inp.dec_q[0, b], inp.dec_k[0, b], inp.dec_v[0, b], inp.k, inp.v, idx,
                                     inp.dec_k[:0, b], inp.dec_v[:0, b], scale)
        _check(o[b].float().cpu().numpy(), ref, "bf16", "chain prompt %d" % b)
