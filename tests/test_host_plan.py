"""CPU-only tests of the C-ABI library: symbols, host planner vs the oracle's explicit mask,
error paths, equilibrium-position helper.  No kernel is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import sp_synth
from oracle import sp_oracle as orc
from paper_2404_06910_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "sp.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(sp_[a-z_0-9]+)\s*\(", hdr)))
    assert {"sp_forkjoin_prefill", "sp_path_saliency", "sp_prune_topk", "sp_pruned_decode", "sp_plan_create",
            "sp_create", "sp_equilibrium_positions"} <= set(names)
    L = ctypes.CDLL(B.lib_path())
    for n in names:
        assert hasattr(L, n), n
    assert b"gfx950" in B.lib().sp_version()


def _random_table(rng, n_prompts, scramble=True):
    """Random forests obeying the table rules: a shared chain/tree, then per-path subtrees; token
    ranges handed out in random order with gaps."""
    seg_off = [0]; parent = []; path = []; lens = []
    for b in range(n_prompts):
        base = len(parent)
        n_shared = int(rng.integers(1, 4))
        for i in range(n_shared):
            parent.append(-1 if i == 0 else base + int(rng.integers(0, i)))
            path.append(-1); lens.append(int(rng.integers(1, 9)))
        n_paths = int(rng.integers(0, 5))
        for p in range(n_paths):
            first = len(parent)
            for j in range(int(rng.integers(1, 4))):
                if j == 0:
                    parent.append(base + int(rng.integers(0, n_shared)))
                else:
                    parent.append(first + int(rng.integers(0, j)))
                path.append(p); lens.append(int(rng.integers(1, 9)))
        seg_off.append(len(parent))
    S = len(parent)
    order = rng.permutation(S) if scramble else np.arange(S)
    start = np.zeros(S, dtype=np.int64); tok = int(rng.integers(0, 3))
    for s in order:
        start[s] = tok
        tok += lens[s] + (int(rng.integers(0, 3)) if scramble else 0)
    return dict(prompt_seg_off=np.array(seg_off, np.int32), seg_tok_start=start.astype(np.int32),
                seg_tok_len=np.array(lens, np.int32), seg_parent=np.array(parent, np.int32),
                seg_path=np.array(path, np.int32), n_tokens=tok + 2)


def _plan(t, Hq=4, Hkv=2, d=64, dtype=B.SP_BF16, **kw):
    return B.Plan(None, t["prompt_seg_off"], t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], t["seg_path"],
                  t["n_tokens"], Hq, Hkv, d, dtype, **kw)


@pytest.mark.parametrize("seed", range(6))
def test_planner_key_lists_match_oracle_mask(seed):
    rng = np.random.default_rng(seed)
    t = _random_table(rng, 3, scramble=seed % 2 == 0)
    p = _plan(t)
    covered = np.zeros(t["n_tokens"], bool)
    pairs = 0
    for b in range(3):
        segs = range(t["prompt_seg_off"][b], t["prompt_seg_off"][b + 1])
        toks, M = orc.dag_mask(t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], segs)
        pairs += int(M.sum())
        for i, tok in enumerate(toks):
            covered[tok] = True
            want = sorted(toks[M[i]].tolist())
            got = p.visible_keys(int(tok)).tolist()
            assert sorted(got) == want, (b, tok)
            assert len(set(got)) == len(got)
            assert got[-1] == tok                      # the token itself comes last
    assert p.visible_pairs() == pairs
    for tok in np.nonzero(~covered)[0]:
        assert len(p.visible_keys(int(tok))) == 0
    # joined cache index lists (Alg. 3) for random kept sets
    off = p.path_offsets()
    for b in range(3):
        n = off[b + 1] - off[b]
        kept = rng.permutation(n)[:min(n, 2)].tolist()
        want = orc.joined_cache_index(t["prompt_seg_off"], t["seg_tok_start"], t["seg_tok_len"], t["seg_path"], b, kept)
        assert p.joined_keys(b, kept).tolist() == want.tolist()
        assert p.joined_keys(b, [-1] + kept).tolist() == want.tolist()      # negative entries are ignored


@pytest.mark.parametrize("seed", range(4))
def test_cached_segments_are_keys_only(seed):
    # Sec. 3.3.1 / Alg. 2: segments whose K/V come from a path cache produce no query rows
    rng = np.random.default_rng(100 + seed)
    t = _random_table(rng, 3, scramble=seed % 2 == 0)
    S = len(t["seg_parent"])
    cached = (rng.random(S) < 0.5).astype(np.uint8)
    p = _plan(t, seg_cached=cached)
    pairs = 0
    for b in range(3):
        segs = list(range(t["prompt_seg_off"][b], t["prompt_seg_off"][b + 1]))
        toks, M = orc.dag_mask(t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], segs)
        live = np.concatenate([np.full(t["seg_tok_len"][s], not cached[s]) for s in segs]) if segs else np.zeros(0, bool)
        pairs += int(M[live].sum())
    assert p.visible_pairs() == pairs
    full = _plan(t)
    assert p.info()["n_row_groups"] == full.info()["n_row_groups"]      # key structure unchanged
    assert p.info()["n_tiles"] <= full.info()["n_tiles"]
    none = _plan(t, seg_cached=np.ones(S, np.uint8))
    assert none.visible_pairs() == 0 and none.info()["n_tiles"] == 0


def test_forkjoin_groups_tiles_and_pairs():
    wl = sp_synth.WORKLOADS["c2_mha7b_bf16"]
    st = sp_synth.forkjoin_segtable(wl.preamble_len, [[wl.doc_len] * wl.n_paths] * 2, wl.query_len)
    p = B.Plan(None, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, st.seg_path, st.n_tokens,
               32, 32, 128, B.SP_BF16)
    info = p.info()
    # interleaved packing: [p; d1; q1] fuse into one run, every other (d_i; q_i) pair into one run
    assert info["n_row_groups"] == 2 * 20 and info["n_path_slots"] == 40 and info["max_ranges"] == 1
    P, L = 64, 152
    per_prompt = P * (P + 1) // 2 + 20 * (L * P + L * (L + 1) // 2)
    assert p.visible_pairs() == 2 * per_prompt == 2 * 429200     # the per-head pair count of this shape
    g = sp_synth.forkjoin_segtable(wl.preamble_len, [[wl.doc_len] * wl.n_paths] * 2, wl.query_len, "grouped")
    pg = B.Plan(None, g.prompt_seg_off, g.seg_tok_start, g.seg_tok_len, g.seg_parent, g.seg_path, g.n_tokens,
                32, 8, 128, B.SP_BF16)
    assert pg.visible_pairs() == 2 * per_prompt


BAD = B.SpError


def _expect(status, fn):
    with pytest.raises(BAD) as e:
        fn()
    assert e.value.status == status, str(e.value)
    assert len(str(e.value)) > 20


def test_error_paths_are_decided_on_the_host():
    rng = np.random.default_rng(0)
    good = _random_table(rng, 2, scramble=False)
    _plan(good)
    def mut(**kw):
        t = {k: (v.copy() if hasattr(v, "copy") else v) for k, v in good.items()}
        for k, f in kw.items():
            t[k] = f(t[k])
        return t
    def seti(i, v):
        def f(a):
            a[i] = v
            return a
        return f
    S = len(good["seg_parent"])
    s1 = int(good["prompt_seg_off"][1])                     # first segment of prompt 1
    _expect(-2, lambda: _plan(mut(seg_parent=seti(s1, 0))))              # parent in another prompt
    _expect(-2, lambda: _plan(mut(seg_parent=seti(0, 0))))               # parent not earlier
    _expect(-2, lambda: _plan(mut(seg_parent=seti(1, S + 5))))
    _expect(-2, lambda: _plan(mut(seg_tok_len=seti(1, 0))))
    _expect(-2, lambda: _plan(mut(seg_tok_start=seti(1, int(good["seg_tok_start"][0])))))   # overlap
    _expect(-2, lambda: _plan(mut(seg_tok_start=seti(S - 1, good["n_tokens"]))))            # out of range
    _expect(-2, lambda: _plan(mut(prompt_seg_off=seti(1, 0))))           # empty prompt
    _expect(-2, lambda: _plan(mut(seg_path=seti(0, -2))))
    _expect(-2, lambda: _plan(mut(seg_path=seti(0, 7))))                 # shared root put on a sparse path id
    _expect(-3, lambda: _plan(good, d=96))
    _expect(-3, lambda: _plan(good, Hq=6, Hkv=4))
    _expect(-1, lambda: _plan(good, Hq=0))
    _expect(-1, lambda: _plan(good, dtype=7))
    T = good["n_tokens"]
    _expect(-1, lambda: _plan(good, alibi_slopes=np.ones(4, np.float32)))                  # slopes without positions
    _expect(-2, lambda: _plan(good, tok_pos=np.full(T, np.nan, np.float32)))
    _expect(-2, lambda: _plan(good, tok_pos=np.zeros(T, np.float32), alibi_slopes=-np.ones(4, np.float32)))
    # a path segment hanging under another path
    t = sp_synth.forkjoin_segtable(3, [[2, 2]], 2)
    par = t.seg_parent.copy(); par[3] = 2                   # doc_2's parent := query_1 (path 0)
    _expect(-2, lambda: B.Plan(None, t.prompt_seg_off, t.seg_tok_start, t.seg_tok_len, par, t.seg_path, t.n_tokens,
                               2, 2, 64, B.SP_F32))


def test_too_many_disjoint_ancestor_ranges_is_unsupported():
    # a 1100-deep chain packed in reverse order: no two ancestors are neighbours in token space
    n = 1100
    start = np.arange(n)[::-1].astype(np.int32) * 2
    t = dict(prompt_seg_off=np.array([0, n], np.int32), seg_tok_start=start, seg_tok_len=np.ones(n, np.int32),
             seg_parent=np.arange(-1, n - 1).astype(np.int32), seg_path=np.full(n, -1, np.int32), n_tokens=2 * n)
    _expect(-3, lambda: _plan(t))
    # the same chain packed forward fuses into one run
    t["seg_tok_start"] = np.arange(n).astype(np.int32)
    assert _plan(t).info()["n_row_groups"] == 1


def test_context_creation_fails_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.SpError) as e:
        B.Context(0, stream=0)
    assert e.value.status == -5


def test_equilibrium_helper_matches_oracle():
    rng = np.random.default_rng(3)
    for lens in ([7, 7, 7], [2, 6], [64, 256, 100, 31], rng.integers(1, 300, size=20).tolist()):
        P, Lq = 5, 4
        st = sp_synth.forkjoin_segtable(P, [lens, lens[::-1]], Lq)
        got = B.equilibrium_positions(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, st.seg_path,
                                      st.n_tokens)
        for b, ll in enumerate([lens, lens[::-1]]):
            pp, pd, pq = orc.equilibrium_positions(P, ll, Lq)
            a = st.seg_tok_start[st.preamble_seg[b]]
            np.testing.assert_array_equal(got[a:a + P], pp.astype(np.float32))
            for i in range(len(ll)):
                slot = st.path_off[b] + i
                a = st.seg_tok_start[st.doc_seg[slot]]
                np.testing.assert_allclose(got[a:a + ll[i]], pd[i], rtol=3e-7)
                a = st.seg_tok_start[st.query_seg[slot]]
                np.testing.assert_allclose(got[a:a + Lq], pq, rtol=3e-7)


def test_kv_bytes_per_token_golden():
    # Sec. 3.3.1: cache bytes per token of a 30-layer, 4096-wide 16-bit model, quoted as 492 KB;
    # the same bytes model (2 * heads * head_dim * element size per layer) prices the decode stream.
    import bench
    with open(os.path.join(ROOT, "tests", "golden", "kv_bytes_per_token.txt")) as f:
        row = [l for l in f if l.strip() and not l.startswith("#")][0].split()
    layers, hidden, esz, expect, quote = (int(x) for x in row)
    got = layers * bench.kv_bytes_per_token(n_kv_heads=32, head_dim=hidden // 32, elem_bytes=esz)
    assert got == expect and round(got / 1000) == quote


def _check_work_list(t, Hq, Hkv, cached=None):
    """The permuted work list covers every computed (token row, query head) exactly once, its key counts
    equal the oracle mask's row sums, and every worker slot owns one contiguous slice."""
    p = _plan(t, Hq=Hq, Hkv=Hkv, d=128, seg_cached=cached)
    items, begin = p.work_items()
    rng_tab = p.key_ranges()
    assert begin[0] == 0 and begin[-1] == len(items) and np.all(np.diff(begin) >= 0)
    G = Hq // Hkv
    hpw = 4 if G % 4 == 0 else 2 if G % 2 == 0 else 1
    seen = np.zeros((t["n_tokens"], Hq), np.int32)
    vis = np.zeros(t["n_tokens"], np.int64)                 # visible keys per token, from the oracle's explicit mask
    for b in range(len(t["prompt_seg_off"]) - 1):
        ids = np.arange(t["prompt_seg_off"][b], t["prompt_seg_off"][b + 1])
        toks, M = orc.dag_mask(t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"], ids)
        vis[toks] = M.sum(axis=1)
    for tok_start, row0, n_rows, anc, r_off, n_rng, heads, r0_start in items:
        h0, kv = heads & 0xffff, heads >> 16
        assert kv == h0 // G and n_rows >= 1 and h0 % hpw == 0
        assert sum(int(rng_tab[r_off + r][1]) for r in range(n_rng)) == anc
        if n_rng:
            assert rng_tab[r_off][0] == r0_start
        for r in range(n_rows):
            tok = tok_start + row0 + r
            assert vis[tok] == anc + row0 + r + 1           # ancestors completely, own run causally
            seen[tok, h0:h0 + hpw] += 1
    live = np.zeros(t["n_tokens"], bool)
    for s in range(len(t["seg_tok_len"])):
        if cached is None or not cached[s]:
            live[t["seg_tok_start"][s]:t["seg_tok_start"][s] + t["seg_tok_len"][s]] = True
    assert np.all(seen[live] == 1) and np.all(seen[~live] == 0)
    p.close()


def test_work_list_covers_every_row_and_head_once():
    rng = np.random.default_rng(11)
    for trial in range(6):
        t = _random_table(rng, int(rng.integers(1, 4)))
        for Hq, Hkv in ((4, 4), (4, 2), (8, 2)):
            _check_work_list(t, Hq, Hkv)
        cached = (rng.random(len(t["seg_tok_len"])) < 0.4).astype(np.uint8)
        _check_work_list(t, 4, 1, cached=cached)
        # head groups that divide by the 8 XCDs (the list is sliced by head groups) and that do not
        for Hq, Hkv in ((8, 8), (16, 16), (32, 8), (12, 12), (24, 3)):
            _check_work_list(t, Hq, Hkv)
    # long shared ancestors: the list goes in chunks of head groups (one at a time here), sliced and unsliced
    for P, Hq, Hkv in ((600, 16, 16), (1100, 4, 4), (1100, 32, 8)):
        st = sp_synth.forkjoin_segtable(P, [[40, 33], [17]], 8)
        t = dict(prompt_seg_off=st.prompt_seg_off, seg_tok_start=st.seg_tok_start, seg_tok_len=st.seg_tok_len,
                 seg_parent=st.seg_parent, seg_path=st.seg_path, n_tokens=st.n_tokens)
        _check_work_list(t, Hq, Hkv)
    for name in ("c2_mha7b_bf16", "c4_gqa_bf16"):
        wl = sp_synth.WORKLOADS[name]
        st = sp_synth.forkjoin_segtable(wl.preamble_len, [[wl.doc_len] * wl.n_paths] * 2, wl.query_len)
        t = dict(prompt_seg_off=st.prompt_seg_off, seg_tok_start=st.seg_tok_start, seg_tok_len=st.seg_tok_len,
                 seg_parent=st.seg_parent, seg_path=st.seg_path, n_tokens=st.n_tokens)
        _check_work_list(t, wl.n_q_heads, wl.n_kv_heads)


def test_work_list_is_balanced_over_the_worker_slots():
    """Load per worker slot (key stages + per-item overhead) stays within a few items of the mean."""
    wl = sp_synth.WORKLOADS["c2_mha7b_bf16"]
    st = sp_synth.forkjoin_segtable(wl.preamble_len, [[wl.doc_len] * wl.n_paths] * wl.n_prompts, wl.query_len)
    p = B.Plan(None, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, st.seg_path, st.n_tokens,
               wl.n_q_heads, wl.n_kv_heads, wl.head_dim, B.SP_BF16)
    items, begin = p.work_items()
    cost = 2 + (items[:, 3] + items[:, 1] + items[:, 2] + 31) // 32
    load = np.add.reduceat(cost, begin[:-1])[np.diff(begin) > 0]
    assert len(load) == len(begin) - 1                      # every slot has work at this size
    assert load.max() <= 1.25 * load.mean() and load.min() >= 0.75 * load.mean()
    p.close()


def test_plan_update_rebuilds_in_place_and_keeps_the_plan_on_error():
    rng = np.random.default_rng(3)
    t1, t2 = _random_table(rng, 2), _random_table(rng, 3)
    p = _plan(t1)
    ref2 = _plan(t2)
    p.update(t2["prompt_seg_off"], t2["seg_tok_start"], t2["seg_tok_len"], t2["seg_parent"], t2["seg_path"], t2["n_tokens"])
    assert p.info() == ref2.info() and p.visible_pairs() == ref2.visible_pairs()
    a, b = p.work_items(), ref2.work_items()
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    bad = dict(t1); bad["seg_parent"] = t1["seg_parent"].copy(); bad["seg_parent"][1] = 1
    with pytest.raises(B.SpError) as e:
        p.update(bad["prompt_seg_off"], bad["seg_tok_start"], bad["seg_tok_len"], bad["seg_parent"], bad["seg_path"], bad["n_tokens"])
    assert e.value.status == -2
    assert p.info() == ref2.info()                          # unchanged after the failed update


def test_equilibrium_helper_equals_the_tree_oracle_on_random_forests():
    """sp_equilibrium_positions applies Eq. 1 to the children of every node; the oracle's tree function
    (pinned by hand-worked fractions) is its reference on forests that are not ForkJoin-shaped: chains of
    shared segments, forks behind chains, several subtrees per path."""
    rng = np.random.default_rng(17)
    for _ in range(25):
        t = _random_table(rng, int(rng.integers(1, 4)))
        got = B.equilibrium_positions(t["prompt_seg_off"], t["seg_tok_start"], t["seg_tok_len"], t["seg_parent"],
                                      t["seg_path"], t["n_tokens"])
        ref = orc.equilibrium_positions_tree(t["seg_parent"], t["seg_tok_len"])
        for s in range(len(ref)):
            a = int(t["seg_tok_start"][s])
            np.testing.assert_allclose(got[a:a + len(ref[s])], ref[s], rtol=1e-6, atol=1e-6)

