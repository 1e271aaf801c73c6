"""The whole step -- prefill, saliency, top-k, decode -- captured once into a HIP graph and replayed.

The entry points enqueue kernels only (no memsets, no allocation once the saliency workspace
exists), so a caller may capture them.  Every replay is checked against the eager result on the
same buffers, with eager work and synchronisations between the replays and the inputs changed in
between."""
import math

import numpy as np
import pytest
import torch

import sp_synth
from paper_2404_06910_amd import binding as B

from gpu_util import dev, make_plan

pytestmark = pytest.mark.gpu


def test_captured_step_replays_like_eager():
    print("case: graph capture of the chained step", flush=True)
    wl = sp_synth.WORKLOADS["c2_mha7b_bf16"]
    inp = sp_synth.make_inputs(wl, n_prompts=2, decode_steps=2)
    st = inp.st
    Hq, Hkv, d = wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    Vv = 2048
    scale = 1 / math.sqrt(d)
    ctx = B.Context(0)
    plan = make_plan(ctx, st, Hq, Hkv, d, "bf16")
    Q, K, V = dev(inp.q, "bf16"), dev(inp.k, "bf16"), dev(inp.v, "bf16")
    O = torch.zeros_like(Q)
    L = dev(np.ascontiguousarray(inp.logits[:, :Vv]), "bf16")
    target, row_path = dev(inp.target % Vv), dev(inp.row_path)
    score = torch.zeros(st.n_slots, device="cuda")
    kept = torch.zeros((2, wl.top_k), dtype=torch.int32, device="cuda")
    Kr = torch.zeros((2, 4, Hkv, d), dtype=torch.bfloat16, device="cuda"); Vr = torch.zeros_like(Kr)
    dq, dk, dv = dev(inp.dec_q, "bf16"), dev(inp.dec_k, "bf16"), dev(inp.dec_v, "bf16")
    o = torch.zeros((2, 2, Hq, d), dtype=torch.bfloat16, device="cuda")
    path_off = plan.path_offsets_device()

    def step():
        ctx.sp_forkjoin_prefill(plan, Q, K, V, O, scale)
        ctx.sp_path_saliency(L, target, row_path, st.n_slots, score)
        ctx.sp_prune_topk(score, path_off, 2, wl.n_paths, wl.top_k, kept)
        for s in range(2):
            ctx.sp_pruned_decode(plan, kept, wl.top_k, K, V, Kr, Vr, 4, dq[s], dk[s], dv[s], o[s], scale, resp_len_add=s)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (O, score, kept, o, Kr, Vr)]

    step()                                   # eager warm-up: the saliency workspace exists from here on
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ctx.sp_set_stream(torch.cuda.current_stream().cuda_stream)
        step()
    ctx.sp_set_stream(torch.cuda.current_stream().cuda_stream)

    gen = torch.Generator(device="cuda"); gen.manual_seed(3)
    for rep in range(3):
        # new inputs in the same buffers, some unrelated eager work, then eager step vs replay
        Q.copy_(torch.randn(Q.shape, generator=gen, device="cuda").to(torch.bfloat16))
        L.copy_((3 * torch.randn(L.shape, generator=gen, device="cuda")).to(torch.bfloat16))
        _ = (K.float() @ K.float().transpose(1, 2)[:, :, :8]).sum()
        step()
        want = snapshot()
        for t in (O, score, kept, o, Kr, Vr):
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a, b in zip(want, got):
            assert torch.equal(a, b), "replay %d differs from the eager step" % rep
    ctx.close()
