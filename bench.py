#!/usr/bin/env python3
"""Benchmark of the superposition-prompting hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input shaped like
the 7B-class multi-head workload (8 prompts x 20 document paths, 64-token preamble, 128-token
documents, 24-token query copies, vocabulary 50432):

    sp_forkjoin_prefill -> sp_path_saliency -> sp_prune_topk -> 5 x sp_pruned_decode

(5 decode steps: the paper's timing protocol generates a 5-token response, App. C).  Inputs
are resident in HBM before the timed region; two input sets are rotated so that no step finds
its inputs in the 256 MB last-level cache.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-decode-c5]
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import sp_synth  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


def kv_bytes_per_token(n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    """K and V bytes of one token in one layer (the per-layer factor of the paper's cache
    memory model, Sec. 3.3.1)."""
    return 2 * n_kv_heads * head_dim * elem_bytes


def prefill_flops(pairs: int, n_q_heads: int, head_dim: int) -> int:
    """2*d for q.k plus 2*d for p.v per visible (query, key) pair and head."""
    return 4 * head_dim * n_q_heads * pairs


def prefill_bytes(n_tokens: int, n_q_heads: int, n_kv_heads: int, head_dim: int, esz: int) -> int:
    """Compulsory traffic: read Q, K, V once, write O once."""
    return n_tokens * head_dim * esz * (2 * n_q_heads + 2 * n_kv_heads)


def decode_step_bytes(n_keys_total: int, n_kv_heads: int, head_dim: int, esz: int) -> int:
    """K and V rows streamed by one decode step (n_keys_total summed over prompts)."""
    return n_keys_total * kv_bytes_per_token(n_kv_heads, head_dim, esz)


N_WARM, N_TRIALS = 10, 30      # side legs: warm-up launches, timed trials (median of 30, as in App. C)


def _time_launches(torch, launch, n_warm=N_WARM, n_trials=N_TRIALS):
    """Times `launch(i)` with events on the launch stream (torch's current stream, which is the stream the
    binding enqueues on): n_warm untimed calls, then n_trials timed ones.  Returns ms statistics."""
    for i in range(n_warm):
        launch(i)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_trials + 1)]
    ev[0].record()
    for i in range(n_trials):
        launch(i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    t = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(n_trials)])
    return {"median_ms": round(float(np.median(t)), 4), "min_ms": round(float(t.min()), 4),
            "p90_ms": round(float(np.percentile(t, 90)), 4), "mean_ms": round(float(t.mean()), 4),
            "warmup": n_warm, "trials": n_trials}


def _stored_traffic(key):
    """HBM bytes per launch from the committed counter runs (profiles/traffic.json): a STORED figure, not
    measured in this run."""
    try:
        v = json.load(open(os.path.join(ROOT, "profiles", "traffic.json"))).get(key)
    except Exception:
        v = None
    return v


def _prefill_roofline(ms, flops, bytes_, traffic_key):
    """Both roofs of one prefill launch: HBM (the binding one at these shapes) and bf16 MFMA, plus the
    fraction of min(MFMA peak, intensity x HBM peak)."""
    t = ms * 1e-3
    tf, gb = flops / t / 1e12, bytes_ / t / 1e9
    ceil_tf = min(MFMA_BF16_PEAK_TFLOPS, flops / bytes_ * HBM_PEAK_GBS / 1e3)
    return {"tflops": round(tf, 2), "mfma_frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "hbm_GBps": round(gb, 1),
            "hbm_frac": round(gb / HBM_PEAK_GBS, 4), "algorithmic_flops": int(flops), "algorithmic_bytes": int(bytes_),
            "intensity_flop_per_byte": round(flops / bytes_, 1),
            "hbm_ceiling_frac_of_mfma_peak": round(ceil_tf / MFMA_BF16_PEAK_TFLOPS, 4),
            "frac_of_binding_ceiling": round(tf / ceil_tf, 4),
            "traffic": _stored_traffic(traffic_key), "traffic_source": "stored: profiles/traffic.json (rocprofv3 --pmc runs)"}


def _memory_rate_reference(torch, n_bytes=1 << 29):
    """What the memory side of this GPU sustains for plain streaming, measured with library element-wise
    kernels over buffers far larger than the last-level cache: a copy (one read per write) and an
    addcmul (three reads per write, the mix of the prefill: Q, K, V in, O out).  Context for the roofline
    fractions, which are quoted against the 8 TB/s peak; not a target."""
    n = n_bytes // 2
    a, b, c = (torch.ones(n, dtype=torch.bfloat16, device="cuda") for _ in range(3))
    d = torch.empty_like(a)
    t_copy = _time_launches(torch, lambda i: d.copy_(a))
    t_mix = _time_launches(torch, lambda i: torch.addcmul(a, b, c, out=d))
    return {"copy_GBps": round(2 * n_bytes / (t_copy["median_ms"] * 1e-3) / 1e9, 1),
            "three_reads_one_write_GBps": round(4 * n_bytes / (t_mix["median_ms"] * 1e-3) / 1e9, 1),
            "kernels": "torch copy_ and addcmul on bf16", "bytes_per_buffer": n_bytes,
            "warmup": N_WARM, "trials": N_TRIALS}


def _device_inputs(wl, seed, torch):
    """One input set of the workload, generated on the device from a seeded generator."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    st = sp_synth.forkjoin_segtable(wl.preamble_len, sp_synth.draw_doc_lens(wl, np.random.default_rng(seed)),
                                    wl.query_len)
    T = st.n_tokens
    rn = lambda *s: torch.randn(s, generator=g, device="cuda", dtype=torch.float32)
    d = {"st": st}
    d["Q"] = rn(T, wl.n_q_heads, wl.head_dim).to(torch.bfloat16)
    d["K"] = rn(T, wl.n_kv_heads, wl.head_dim).to(torch.bfloat16)
    d["V"] = rn(T, wl.n_kv_heads, wl.head_dim).to(torch.bfloat16)
    d["O"] = torch.empty_like(d["Q"])
    R = st.n_slots * wl.query_len
    logits = torch.empty((R, wl.vocab), dtype=torch.bfloat16, device="cuda")
    for r in range(0, R, 512):
        n = min(512, R - r)
        logits[r:r + n] = rn(n, wl.vocab) * wl.logit_std
    d["logits"] = logits
    rng = np.random.default_rng(seed + 1)
    tgt = np.concatenate([np.tile(rng.integers(0, wl.vocab, size=wl.query_len), wl.n_paths)
                          for _ in range(wl.n_prompts)]).astype(np.int32)
    d["target"] = torch.from_numpy(tgt).cuda()
    d["row_path"] = torch.from_numpy(np.repeat(np.arange(st.n_slots), wl.query_len).astype(np.int32)).cuda()
    d["score"] = torch.empty(st.n_slots, device="cuda")
    d["kept"] = torch.empty((wl.n_prompts, wl.top_k), dtype=torch.int32, device="cuda")
    S = wl.decode_steps
    d["dq"] = rn(S, wl.n_prompts, wl.n_q_heads, wl.head_dim).to(torch.bfloat16)
    d["dk"] = rn(S, wl.n_prompts, wl.n_kv_heads, wl.head_dim).to(torch.bfloat16)
    d["dv"] = rn(S, wl.n_prompts, wl.n_kv_heads, wl.head_dim).to(torch.bfloat16)
    d["Kr"] = torch.zeros((wl.n_prompts, S, wl.n_kv_heads, wl.head_dim), dtype=torch.bfloat16, device="cuda")
    d["Vr"] = torch.zeros_like(d["Kr"])
    d["o"] = torch.empty((wl.n_prompts, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device="cuda")
    return d


def _cpu_baseline(wl, budget_s=12.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: complete
    prefill attention of successive (prompt 0, head h) pairs until the time budget is used."""
    from oracle import sp_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    inp = sp_synth.make_inputs(wl, n_prompts=min(wl.n_prompts, 6), with_logits=False, with_decode=False)
    st = inp.st
    P = wl.preamble_len

    def pairs_of(b):                       # visible pairs per head of prompt b
        n = P * (P + 1) // 2
        for s in range(st.path_off[b], st.path_off[b + 1]):
            L = int(st.seg_tok_len[st.doc_seg[s]] + st.seg_tok_len[st.query_seg[s]])
            n += L * P + L * (L + 1) // 2
        return n

    scale = 1 / math.sqrt(wl.head_dim)
    t0 = time.perf_counter()
    n = 0
    flops = 0
    for b in range(len(st.prompt_seg_off) - 1):
        for h in range(wl.n_q_heads):
            orc.forkjoin_prefill(inp.q, inp.k, inp.v, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len,
                                 st.seg_parent, scale, prompts=[b], heads=[h])
            n += 1
            flops += prefill_flops(pairs_of(b), 1, wl.head_dim)
            if time.perf_counter() - t0 > budget_s:
                break
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": "prefill attention of the first %d (prompt, head) pairs of %s (dense fp64 T x T oracle per "
                      "prompt; rate = algorithmic FLOPs / wall time), %.1f s" % (n, wl.name, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="c2_mha7b_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode-c5", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the leg that replays the whole step from a captured HIP graph")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the prefill and saliency legs on the ragged and the grouped-query workloads")
    ap.add_argument("--no-online-prefill", action="store_true",
                    help="skip the path-cached (query rows only) and iterative-round prefill legs, e.g. so that a "
                         "kernel trace of this run holds full prefill launches only")
    ap.add_argument("--no-memory-reference", action="store_true",
                    help="skip the library element-wise kernels that show what this GPU's memory side sustains")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="short run for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE: a plain elementwise kernel of known "
                         "traffic (calibration), then a few launches of every leg; prints no benchmark line")
    ap.add_argument("--only", default=None, choices=["decode_c5", "c3_ragged_bf16", "c4_gqa_bf16"],
                    help="run one side leg alone (for a kernel trace that holds nothing else); prints its block")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (one process, one MI355X); --gpus %d is not "
              "supported: no collectives or sharding exist in this library" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2404_06910_amd import binding as B

    torch.cuda.set_device(0)
    ctx = B.Context(0)                       # launches on torch's current stream
    if args.only:
        if args.only == "decode_c5":
            print(json.dumps({"decode_c5": _bench_decode_c5(ctx, torch, B)}))
        else:
            print(json.dumps({args.only: _bench_workload_leg(ctx, torch, B, args.only, bias=False)}))
        return
    wl = sp_synth.WORKLOADS[args.workload]
    assert wl.dtype == "bf16"
    sets = [_device_inputs(wl, wl.seed + 17 * i, torch) for i in range(2)]
    st = sets[0]["st"]
    plans = [_make_plan(ctx, B, wl, s["st"]) for s in sets]
    scale = 1 / math.sqrt(wl.head_dim)
    S = wl.decode_steps
    path_off_dev = [p.path_offsets_device() for p in plans]

    def step(i, ev=None):
        d, plan = sets[i % 2], plans[i % 2]
        if ev: ev[0].record()
        ctx.sp_forkjoin_prefill(plan, d["Q"], d["K"], d["V"], d["O"], scale)
        if ev: ev[1].record()
        ctx.sp_path_saliency(d["logits"], d["target"], d["row_path"], d["st"].n_slots, d["score"])
        if ev: ev[2].record()
        ctx.sp_prune_topk(d["score"], path_off_dev[i % 2], wl.n_prompts, wl.n_paths, wl.top_k, d["kept"])
        if ev: ev[3].record()
        for s in range(S):
            ctx.sp_pruned_decode(plan, d["kept"], wl.top_k, d["K"], d["V"], d["Kr"], d["Vr"], S, d["dq"][s],
                                 d["dk"][s], d["dv"][s], d["o"], scale, resp_len_add=s)
        if ev: ev[4].record()

    if args.traffic_probe:
        # calibration: y = x + 1 over 1 GiB of bf16 reads 2^30 bytes and writes 2^30 bytes
        x = torch.zeros(1 << 29, dtype=torch.bfloat16, device="cuda")
        y = torch.empty_like(x)
        for _ in range(3):
            torch.add(x, 1, out=y)
        del x, y
        for i in range(max(args.steps, 2)):
            step(i)
        _bench_online_prefill(ctx, torch, B, wl, sets, scale, n_warm=1, n_trials=3)
        _bench_iterative_round(ctx, torch, B, wl, sets, scale, n_warm=1, n_trials=3)
        torch.cuda.synchronize()
        del sets
        for name in ("c3_ragged_bf16", "c4_gqa_bf16"):
            _bench_workload_leg(ctx, torch, B, name, bias=False, n_warm=1, n_trials=3)
        _bench_decode_c5(ctx, torch, B, steps=8, reps=1)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": True, "calibration_kernel": "torch.add bf16, 2^30 B read + 2^30 B written"}))
        return
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ph = np.array([[ev[j].elapsed_time(ev[j + 1]) for j in range(4)] for ev in events])   # ms
    med, mean, mn, p90 = np.median(ph, axis=0), ph.mean(axis=0), ph.min(axis=0), np.percentile(ph, 90, axis=0)
    names = ["prefill", "saliency", "topk", "decode_%d_steps" % S]
    stat = lambda v: {n: round(float(x), 4) for n, x in zip(names, v)}

    pairs = plans[0].visible_pairs()
    flops = prefill_flops(pairs, wl.n_q_heads, wl.head_dim)
    pbytes = prefill_bytes(st.n_tokens, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, 2)
    t_pre = mean[0] * 1e-3
    tflops = flops / t_pre / 1e12
    sal_bytes = sets[0]["logits"].numel() * 2
    sal_gbs = sal_bytes / (mean[1] * 1e-3) / 1e9
    kept_keys = wl.preamble_len + wl.top_k * (int(st.seg_tok_len[st.doc_seg[0]]) + wl.query_len)
    dec_bytes = sum(decode_step_bytes(wl.n_prompts * (kept_keys + s + 1), wl.n_kv_heads, wl.head_dim, 2) for s in range(S))
    dec_gbs = dec_bytes / (mean[3] * 1e-3) / 1e9

    out = {
        "metric": "forkjoin_prefill_tflops", "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall / args.steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "n_prompts": wl.n_prompts, "n_paths": wl.n_paths, "n_q_heads": wl.n_q_heads,
                   "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "preamble": wl.preamble_len,
                   "doc_len": wl.doc_len, "query_len": wl.query_len, "vocab": wl.vocab, "top_k": wl.top_k,
                   "decode_steps": S, "tokens": st.n_tokens, "input_sets_rotated": 2},
        "phase_ms_mean": stat(mean), "phase_ms_median": stat(med), "phase_ms_min": stat(mn), "phase_ms_p90": stat(p90),
        "plan_create_ms": _plan_create_ms(ctx, B, wl, st),
        # dominant kernel: prefill.  Its arithmetic intensity at this shape (flops/compulsory bytes) is
        # below the machine balance, so HBM is the binding roof; the MFMA view is given next to it.
        "roofline": {"kernel": "prefill_bf16_kernel", "bound": "hbm", "achieved": round(pbytes / t_pre / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(pbytes / t_pre / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": _stored_traffic("prefill_bf16_kernel:" + wl.name),
                     "traffic_source": "stored: profiles/traffic.json (rocprofv3 --pmc runs, not counted in this run)",
                     "algorithmic_bytes": pbytes, "algorithmic_flops": flops,
                     "intensity_flop_per_byte": round(flops / pbytes, 1), "avg_launch_ms": round(mean[0], 4),
                     "median_launch_ms": round(med[0], 4), "min_launch_ms": round(mn[0], 4)},
        "roofline_mfma": {"kernel": "prefill_bf16_kernel", "bound": "mfma", "achieved": round(tflops, 2),
                          "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                          "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                          "hbm_ceiling_frac": round(flops / pbytes * HBM_PEAK_GBS * 1e9 / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)},
        "saliency": {"kernel": "saliency_kernel", "bound": "hbm", "achieved": round(sal_gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(sal_gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes": sal_bytes,
                     "median_ms": round(med[1], 4), "min_ms": round(mn[1], 4), "p90_ms": round(p90[1], 4),
                     "traffic": _stored_traffic("saliency_kernel:" + wl.name),
                     "traffic_source": "stored: profiles/traffic.json"},
        "decode_in_step": {"kernel": "decode_kernel", "bound": "hbm", "achieved": round(dec_gbs, 1),
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(dec_gbs / HBM_PEAK_GBS, 4),
                           "algorithmic_bytes": dec_bytes, "note": "8 prompts only: launch-latency bound"},
    }

    if not args.no_graph:
        # the same step, captured once per input set into a HIP graph and replayed (launch overhead of
        # the eight kernels of a step leaves the host)
        graphs = []
        for j in range(2):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                ctx.sp_set_stream(torch.cuda.current_stream().cuda_stream)
                step(j)
            graphs.append(g)
        ctx.sp_set_stream(torch.cuda.current_stream().cuda_stream)
        for j in range(4):
            graphs[j % 2].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for j in range(args.steps):
            graphs[j % 2].replay()
        torch.cuda.synchronize()
        out["graph_replay"] = {"ms_per_step": round((time.perf_counter() - t0) / args.steps * 1e3, 4),
                               "eager_ms_per_step": out["ms_per_step"]}
        del graphs
    if not args.no_online_prefill:
        out["prefill_online_cached"] = _bench_online_prefill(ctx, torch, B, wl, sets, scale)
        out["prefill_iterative_round"] = _bench_iterative_round(ctx, torch, B, wl, sets, scale)
    del sets, plans
    torch.cuda.empty_cache()
    if not args.no_other_workloads:
        out["other_workloads"] = {
            "c3_ragged_bf16": _bench_workload_leg(ctx, torch, B, "c3_ragged_bf16", bias=False),
            "c3_ragged_bf16+equilibrium_bias": _bench_workload_leg(ctx, torch, B, "c3_ragged_bf16", bias=True,
                                                                   saliency=False),
            "c4_gqa_bf16": _bench_workload_leg(ctx, torch, B, "c4_gqa_bf16", bias=False),
        }
    if not args.no_decode_c5:
        out["decode_c5"] = _bench_decode_c5(ctx, torch, B)
        if not args.no_other_workloads:
            out["decode_c5+equilibrium_bias"] = _bench_decode_c5(ctx, torch, B, steps=64, reps=3, bias=True)
    if not args.no_memory_reference:
        out["memory_rate_reference"] = _memory_rate_reference(torch)
        ref = out["memory_rate_reference"]["three_reads_one_write_GBps"]
        out["roofline"]["frac_of_measured_reference"] = round(out["roofline"]["achieved"] / ref, 4)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(wl)
    print(json.dumps(out))


def _make_plan(ctx, B, wl, st, **kw):
    return B.Plan(ctx, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, st.seg_path, st.n_tokens,
                  wl.n_q_heads, wl.n_kv_heads, wl.head_dim, B.SP_BF16, **kw)


def _plan_create_ms(ctx, B, wl, st, reps=7, **kw):
    """Host time of one sp_plan_create through the binding (validation, work list, one asynchronous
    upload), the per-request cost of a new prompt DAG: median of `reps` create/destroy cycles after two
    warm-up cycles (the device block and the pinned staging buffer are then recycled)."""
    ts = []
    for i in range(reps + 2):
        t0 = time.perf_counter()
        p = _make_plan(ctx, B, wl, st, **kw)
        ts.append(time.perf_counter() - t0)
        p.close()
    return round(float(np.median(ts[2:])) * 1e3, 3)


def _bench_workload_leg(ctx, torch, B, name, bias, saliency=True, n_warm=N_WARM, n_trials=N_TRIALS):
    """Prefill (and saliency) alone on another workload, two input sets rotated; with bias = True the tokens
    carry equilibrium positions (Sec. 3.2.2 Eq. 1, from the library's host helper) and every head a linear
    distance penalty."""
    wl = sp_synth.WORKLOADS[name]
    sets, plans, sts = [], [], []
    pos = slopes = None
    for i in range(2):
        seed = wl.seed + 17 * i
        g = torch.Generator(device="cuda"); g.manual_seed(seed)
        st = sp_synth.forkjoin_segtable(wl.preamble_len, sp_synth.draw_doc_lens(wl, np.random.default_rng(seed)),
                                        wl.query_len)
        rn = lambda h: torch.randn((st.n_tokens, h, wl.head_dim), generator=g, device="cuda").to(torch.bfloat16)
        Q, K, V = rn(wl.n_q_heads), rn(wl.n_kv_heads), rn(wl.n_kv_heads)
        sets.append((Q, K, V, torch.empty_like(Q)))
        if bias:
            pos = B.equilibrium_positions(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent,
                                          st.seg_path, st.n_tokens)
            slopes = sp_synth.geometric_slopes(wl.n_q_heads)
        plans.append(_make_plan(ctx, B, wl, st, tok_pos=pos, alibi_slopes=slopes))
        sts.append(st)
    scale = 1 / math.sqrt(wl.head_dim)
    t = _time_launches(torch, lambda i: ctx.sp_forkjoin_prefill(plans[i % 2], *sets[i % 2], scale), n_warm, n_trials)
    flops = float(np.mean([prefill_flops(p.visible_pairs(), wl.n_q_heads, wl.head_dim) for p in plans]))
    by = float(np.mean([prefill_bytes(s[0].shape[0], wl.n_q_heads, wl.n_kv_heads, wl.head_dim, 2) for s in sets]))
    out = {"prefill": dict(t, kernel="prefill_bf16_kernel", bound="hbm",
                           **_prefill_roofline(t["median_ms"], flops, by, "prefill_bf16_kernel:" + name + ("+bias" if bias else ""))),
           "tokens": int(sets[0][0].shape[0]), "n_prompts": wl.n_prompts,
           "plan_create_ms": _plan_create_ms(ctx, B, wl, sts[1], tok_pos=pos, alibi_slopes=slopes)}   # pos belongs to sts[1]
    del sets, plans
    torch.cuda.empty_cache()
    if saliency:
        out["saliency"] = _bench_saliency(ctx, torch, B, wl, n_warm, n_trials)
    return out


def _bench_saliency(ctx, torch, B, wl, n_warm=N_WARM, n_trials=N_TRIALS):
    """sp_path_saliency alone at the workload's size (rows = prompts x paths x query tokens, its vocabulary),
    two logit matrices rotated (each far larger than the last-level cache when summed)."""
    n_slots = wl.n_prompts * wl.n_paths
    R = n_slots * wl.query_len
    g = torch.Generator(device="cuda"); g.manual_seed(wl.seed + 5)
    mats = []
    for _ in range(2):
        x = torch.empty((R, wl.vocab), dtype=torch.bfloat16, device="cuda")
        for r in range(0, R, 512):
            n = min(512, R - r)
            x[r:r + n] = torch.randn((n, wl.vocab), generator=g, device="cuda") * wl.logit_std
        mats.append(x)
    rng = np.random.default_rng(wl.seed + 6)
    tgt = torch.from_numpy(rng.integers(0, wl.vocab, size=R).astype(np.int32)).cuda()
    rp = torch.from_numpy(np.repeat(np.arange(n_slots), wl.query_len).astype(np.int32)).cuda()
    score = torch.empty(n_slots, device="cuda")
    t = _time_launches(torch, lambda i: ctx.sp_path_saliency(mats[i % 2], tgt, rp, n_slots, score), n_warm, n_trials)
    by = R * wl.vocab * 2
    gbs = by / (t["median_ms"] * 1e-3) / 1e9
    out = dict(t, kernel="saliency_kernel", bound="hbm", achieved=round(gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
               frac=round(gbs / HBM_PEAK_GBS, 4), algorithmic_bytes=by, rows=R, vocab=wl.vocab,
               traffic=_stored_traffic("saliency_kernel:" + wl.name), traffic_source="stored: profiles/traffic.json")
    del mats
    torch.cuda.empty_cache()
    return out


def _bench_online_prefill(ctx, torch, B, wl, sets, scale, n_warm=N_WARM, n_trials=N_TRIALS):
    """Path-cached split (Sec. 3.3.1, Alg. 2): preamble and document K/V are resident from an offline
    pass; the online launch computes the query-copy rows only (keys: the whole path)."""
    plans, cacheds = [], []
    for s in sets:
        t = s["st"]
        cached = np.ones(t.n_segments, np.uint8); cached[np.asarray(t.query_seg)] = 0
        plans.append(_make_plan(ctx, B, wl, t, seg_cached=cached))
        cacheds.append(cached)

    def launch(i):
        d = sets[i % 2]
        ctx.sp_forkjoin_prefill(plans[i % 2], d["Q"], d["K"], d["V"], d["O"], scale)

    tm = _time_launches(torch, launch, n_warm, n_trials)
    ms = tm["median_ms"]
    t = sets[0]["st"]
    q_rows = int(sum(int(t.seg_tok_len[s]) for s in np.asarray(t.query_seg)))
    kvb = t.n_tokens * kv_bytes_per_token(wl.n_kv_heads, wl.head_dim, 2)
    qob = q_rows * 2 * wl.n_q_heads * wl.head_dim * 2
    flops = prefill_flops(plans[0].visible_pairs(), wl.n_q_heads, wl.head_dim)
    gbs = (kvb + qob) / (ms * 1e-3) / 1e9
    return dict(tm, kernel="prefill_bf16_kernel", rows="query copies only", bound="hbm", achieved=round(gbs, 1),
                peak=HBM_PEAK_GBS, unit="GB/s", frac=round(gbs / HBM_PEAK_GBS, 4), algorithmic_bytes=kvb + qob,
                algorithmic_flops=flops, tflops=round(flops / (ms * 1e-3) / 1e12, 2),
                traffic=_stored_traffic("prefill_bf16_kernel:" + wl.name + ":online_cached"),
                traffic_source="stored: profiles/traffic.json",
                plan_create_ms=_plan_create_ms(ctx, B, wl, t, seg_cached=cacheds[0]))


def _iterative_round_table(t, chain):
    """Segment table of a later round of iterative superposition on the token pool of table t: the documents
    kept so far (`chain`) form a cached chain behind the preamble, the others fork behind its tail."""
    start, length, parent, path, cached, off = [], [], [], [], [], [0]
    for b in range(t.n_prompts):
        p0, p1 = int(t.path_off[b]), int(t.path_off[b + 1])
        base = len(start)
        ps = int(t.preamble_seg[b])
        start.append(int(t.seg_tok_start[ps])); length.append(int(t.seg_tok_len[ps])); parent.append(-1)
        path.append(-1); cached.append(1)
        tail = base
        for c in chain:
            ds = int(t.doc_seg[p0 + c])
            start.append(int(t.seg_tok_start[ds])); length.append(int(t.seg_tok_len[ds])); parent.append(tail)
            path.append(-1); cached.append(1)
            tail = len(start) - 1
        j = 0
        for i in range(p1 - p0):
            if i in chain:
                continue
            ds, qs = int(t.doc_seg[p0 + i]), int(t.query_seg[p0 + i])
            start.append(int(t.seg_tok_start[ds])); length.append(int(t.seg_tok_len[ds])); parent.append(tail)
            path.append(j); cached.append(0)
            start.append(int(t.seg_tok_start[qs])); length.append(int(t.seg_tok_len[qs]))
            parent.append(len(start) - 2); path.append(j); cached.append(0)
            j += 1
        off.append(len(start))
    i32 = lambda a: np.asarray(a, np.int32)
    return i32(off), i32(start), i32(length), i32(parent), i32(path), np.asarray(cached, np.uint8)


def _bench_iterative_round(ctx, torch, B, wl, sets, scale, chain=(3, 7, 11, 15), n_warm=N_WARM, n_trials=N_TRIALS):
    """A later round of iterative superposition (Sec. 4.1.2, App. B) on the same token pool: the
    documents kept so far form a cached chain behind the preamble and the remaining documents, each
    with its query copy, are superposed behind the chain's tail.  Their ancestors are several
    separate token ranges (preamble, the chain's documents)."""
    plans, tabs = [], []
    for s in sets:
        t = s["st"]
        off, start, length, parent, path, cached = _iterative_round_table(t, chain)
        plans.append(B.Plan(ctx, off, start, length, parent, path, t.n_tokens, wl.n_q_heads, wl.n_kv_heads,
                            wl.head_dim, B.SP_BF16, seg_cached=cached))
        tabs.append((off, start, length, parent, path, cached, t.n_tokens))

    def launch(i):
        d = sets[i % 2]
        ctx.sp_forkjoin_prefill(plans[i % 2], d["Q"], d["K"], d["V"], d["O"], scale)

    tm = _time_launches(torch, launch, n_warm, n_trials)
    ms = tm["median_ms"]
    flops = prefill_flops(plans[0].visible_pairs(), wl.n_q_heads, wl.head_dim)
    # per-round cost of the new table: the plan object is rebuilt in place (sp_plan_update)
    ts = []
    off, start, length, parent, path, cached, n_tok = tabs[0]
    for i in range(9):
        t0 = time.perf_counter()
        plans[0].update(off, start, length, parent, path, n_tok, seg_cached=cached)
        ts.append(time.perf_counter() - t0)
    torch.cuda.synchronize()
    # compulsory bytes: K and V of every token once (cached chain, preamble and computed rows are all keys),
    # Q read and O written for the rows that are computed
    off, start, length, parent, path, cached, n_tok = tabs[0]
    rows = int(sum(int(l) for l, c in zip(length, cached) if not c))
    by = n_tok * kv_bytes_per_token(wl.n_kv_heads, wl.head_dim, 2) + rows * 2 * wl.n_q_heads * wl.head_dim * 2
    return dict(tm, kernel="prefill_bf16_kernel", rows="documents not yet kept and their query copies",
                chain_documents=len(chain), algorithmic_flops=flops, tflops=round(flops / (ms * 1e-3) / 1e12, 2),
                algorithmic_bytes=by, hbm_frac=round(by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                mfma_frac=round(flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                traffic=_stored_traffic("prefill_bf16_kernel:" + wl.name + ":iterative_round"),
                traffic_source="stored: profiles/traffic.json",
                plan_update_ms=round(float(np.median(ts[2:])) * 1e3, 3))


def _bench_decode_c5(ctx, torch, B, steps=None, reps=7, bias=False):
    """Long pruned decode: 64 prompts, 2 of 20 paths kept, 256 steps over the growing cache.
    With bias = True the cache carries equilibrium positions and every head a distance penalty."""
    wl = sp_synth.WORKLOADS["c5_decode_bf16"]
    st = sp_synth.forkjoin_segtable(wl.preamble_len, [[wl.doc_len] * wl.n_paths] * wl.n_prompts, wl.query_len)
    g = torch.Generator(device="cuda"); g.manual_seed(wl.seed)
    H, d, S, Bn = wl.n_kv_heads, wl.head_dim, (steps or wl.decode_steps), wl.n_prompts
    rn = lambda *s: torch.randn(s, generator=g, device="cuda").to(torch.bfloat16)
    K, V = rn(st.n_tokens, H, d), rn(st.n_tokens, H, d)
    dq, dk, dv = rn(S, Bn, H, d), rn(S, Bn, H, d), rn(S, Bn, H, d)
    rng = np.random.default_rng(wl.seed)
    kept = torch.from_numpy(np.stack([rng.permutation(wl.n_paths)[:wl.top_k] for _ in range(Bn)]).astype(np.int32)).cuda()
    pos = slopes = pos_resp = None
    new_pos = [None] * S
    if bias:
        pos = B.equilibrium_positions(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, st.seg_path,
                                      st.n_tokens)
        slopes = sp_synth.geometric_slopes(H)
        pos_resp = torch.zeros((Bn, S), device="cuda")
        p0 = float(pos.max()) + 1.0
        new_pos = [torch.full((Bn,), p0 + s, device="cuda") for s in range(S)]
    plan = B.Plan(ctx, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, st.seg_path, st.n_tokens,
                  H, H, d, B.SP_BF16, tok_pos=pos, alibi_slopes=slopes)
    Kr = torch.zeros((Bn, S, H, d), dtype=torch.bfloat16, device="cuda"); Vr = torch.zeros_like(Kr)
    o = torch.empty((S, Bn, H, d), dtype=torch.bfloat16, device="cuda")
    scale = 1 / math.sqrt(d)

    def loop():
        for s in range(S):
            ctx.sp_pruned_decode(plan, kept, wl.top_k, K, V, Kr, Vr, S, dq[s], dk[s], dv[s], o[s], scale, resp_len_add=s,
                                 pos_resp=pos_resp, new_pos=new_pos[s])

    loop()
    torch.cuda.synchronize()
    times = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); loop(); e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    ms = float(np.median(times))
    kept_keys = wl.preamble_len + wl.top_k * (wl.doc_len + wl.query_len)
    total = sum(decode_step_bytes(Bn * (kept_keys + s + 1), H, d, 2) for s in range(S))
    gbs = total / (ms * 1e-3) / 1e9
    return {"workload": wl.name, "kernel": "decode_kernel", "bound": "hbm", "achieved": round(gbs, 1),
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes": total,
            "loop_ms_median": round(ms, 3), "loop_ms_min": round(float(np.min(times)), 3),
            "loop_ms_p90": round(float(np.percentile(times, 90)), 3), "loops_timed": reps, "warmup_loops": 1,
            "us_per_step": round(ms * 1e3 / S, 2), "steps": S,
            "traffic": _stored_traffic("decode_kernel:" + wl.name + ("+bias" if bias else "")),
            "traffic_source": "stored: profiles/traffic.json (bytes per step, mean over the steps traced)"}


if __name__ == "__main__":
    main()
