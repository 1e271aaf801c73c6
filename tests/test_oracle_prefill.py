"""Pins for the prefill oracle (CPU only).  Each test ties the oracle to something other
than itself: a library causal-attention routine, closed forms, an independently derived
reachability relation, or pure-Python brute force on tiny inputs."""
import math

import numpy as np
import pytest
import torch

import sp_synth
from oracle import sp_oracle as orc


def _rand_qkv(rng, T, Hq, Hkv, d):
    return (rng.standard_normal((T, Hq, d)), rng.standard_normal((T, Hkv, d)), rng.standard_normal((T, Hkv, d)))


def _sdpa_causal(q, k, v, scale, bias=None):
    """Library routine: torch scaled_dot_product_attention on one contiguous sequence.
    q [n, d] etc.; returns [n, d] float64."""
    tq = torch.from_numpy(np.ascontiguousarray(q))[None, None]
    tk = torch.from_numpy(np.ascontiguousarray(k))[None, None]
    tv = torch.from_numpy(np.ascontiguousarray(v))[None, None]
    if bias is None:
        o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    else:
        n = q.shape[0]
        m = torch.full((n, n), float("-inf"), dtype=torch.float64).triu(1) + torch.from_numpy(bias)
        o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=m[None, None], scale=scale)
    return o[0, 0].numpy()


def _run(st, q, k, v, scale, **kw):
    return orc.forkjoin_prefill(q, k, v, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent,
                                scale, **kw)


def test_single_document_is_plain_causal_attention():
    # Sec. 3.2: a classical prompt is the linked-list special case of the DAG.
    rng = np.random.default_rng(1)
    st = sp_synth.forkjoin_segtable(5, [[7]], 3)
    q, k, v = _rand_qkv(rng, st.n_tokens, 2, 2, 8)
    out = _run(st, q, k, v, 0.3)
    for h in range(2):
        ref = _sdpa_causal(q[:, h], k[:, h], v[:, h], 0.3)
        np.testing.assert_allclose(out[:, h], ref, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("packing", ["interleaved", "grouped"])
def test_each_path_equals_causal_attention_on_its_own_concatenation(packing):
    # ForkJoin: rows of path i == causal attention over [preamble; doc_i; query_i].
    rng = np.random.default_rng(2)
    st = sp_synth.forkjoin_segtable(6, [[5, 9, 4], [3, 8]], 4, packing)
    Hq, Hkv, d = 4, 2, 16
    q, k, v = _rand_qkv(rng, st.n_tokens, Hq, Hkv, d)
    scale = 1 / math.sqrt(d)
    out = _run(st, q, k, v, scale)
    assert not np.isnan(out).any()
    for slot in range(st.n_slots):
        b = int(np.searchsorted(st.path_off, slot, side="right") - 1)
        segs = [int(st.preamble_seg[b]), int(st.doc_seg[slot]), int(st.query_seg[slot])]
        toks = np.concatenate([np.arange(st.seg_tok_start[s], st.seg_tok_start[s] + st.seg_tok_len[s]) for s in segs])
        for h in range(Hq):
            g = h // (Hq // Hkv)
            ref = _sdpa_causal(q[toks, h], k[toks, g], v[toks, g], scale)
            np.testing.assert_allclose(out[toks, h], ref, rtol=1e-10, atol=1e-12)


def test_paths_are_independent():
    # Sec. 3.3.2: paths are independent by construction -> bit-identical outputs.
    rng = np.random.default_rng(3)
    st = sp_synth.forkjoin_segtable(4, [[6, 5, 7]], 3)
    q, k, v = _rand_qkv(rng, st.n_tokens, 2, 2, 8)
    base = _run(st, q, k, v, 0.25)
    j = 1
    lo = int(st.seg_tok_start[st.doc_seg[j]]); hi = int(st.seg_tok_start[st.query_seg[j]] + st.seg_tok_len[st.query_seg[j]])
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    k2[lo:hi] += 3.0; v2[lo:hi] -= 2.0; q2[lo:hi] *= -1.0
    pert = _run(st, q2, k2, v2, 0.25)
    others = np.ones(st.n_tokens, bool); others[lo:hi] = False
    assert np.array_equal(base[others], pert[others])
    assert not np.allclose(base[lo:hi], pert[lo:hi])


def _reachability_by_closure(st, segs):
    """Independent derivation of 'there is a path u -> v': boolean transitive closure of the
    segment adjacency matrix by repeated squaring (no parent-pointer walking)."""
    segs = list(segs)
    n = len(segs)
    loc = {s: i for i, s in enumerate(segs)}
    A = np.zeros((n, n), dtype=bool)
    for s in segs:
        p = int(st.seg_parent[s])
        if p >= 0:
            A[loc[p], loc[s]] = True      # edge parent -> child
    R = A.copy()
    for _ in range(n):
        R = R | ((R.astype(np.int64) @ A.astype(np.int64)) > 0)
    return R, loc


def test_onehot_values_reveal_the_attention_distribution_and_visibility():
    # V = one-hot(token) => the output row IS the attention distribution: it sums to 1 and
    # is exactly 0 on tokens with no DAG path to the row's segment (Sec. 3.2).
    rng = np.random.default_rng(4)
    st = sp_synth.forkjoin_segtable(3, [[4, 2, 5]], 2, "grouped")
    T = st.n_tokens
    q = rng.standard_normal((T, 1, 4)); k = rng.standard_normal((T, 1, 4))
    v = np.eye(T)[:, None, :]
    # dag_mask lists tokens in segment order; map back to packed order below
    toks, M = orc.dag_mask(st.seg_tok_start, st.seg_tok_len, st.seg_parent, range(st.n_segments))
    Ploc = orc.masked_attention(q[toks, 0], k[toks, 0], v[toks, 0], M, 0.5)   # rows local, cols packed
    np.testing.assert_allclose(Ploc.sum(axis=1), 1.0, rtol=1e-13)
    P = np.empty_like(Ploc); P[toks] = Ploc
    Mp = np.empty_like(M); Mp[np.ix_(toks, toks)] = M
    M = Mp
    R, loc = _reachability_by_closure(st, range(st.n_segments))
    seg_of = np.empty(T, dtype=int); idx_in = np.empty(T, dtype=int)
    for s in range(st.n_segments):
        a, n = int(st.seg_tok_start[s]), int(st.seg_tok_len[s])
        seg_of[a:a + n] = s; idx_in[a:a + n] = np.arange(n)
    for t in range(T):
        for s in range(T):
            visible = R[loc[seg_of[s]], loc[seg_of[t]]] or (seg_of[s] == seg_of[t] and idx_in[s] <= idx_in[t])
            assert (P[t, s] > 0) == bool(visible), (t, s)
            assert M[t, s] == bool(visible)


def test_equal_keys_give_the_mean_of_visible_values():
    rng = np.random.default_rng(5)
    st = sp_synth.forkjoin_segtable(4, [[3, 6]], 2)
    T = st.n_tokens
    q = rng.standard_normal((T, 1, 8))
    k = np.tile(rng.standard_normal((1, 1, 8)), (T, 1, 1))
    v = rng.standard_normal((T, 1, 8))
    out = _run(st, q, k, v, 0.7)
    toks, M = orc.dag_mask(st.seg_tok_start, st.seg_tok_len, st.seg_parent, range(st.n_segments))
    for t in range(T):
        np.testing.assert_allclose(out[t, 0], v[M[t], 0].mean(axis=0), rtol=1e-12, atol=1e-13)
    # count of visible pairs matches the closed form P(P+1)/2 + sum_i (L_i P + L_i (L_i+1)/2)
    Pn, Ls = 4, [3 + 2, 6 + 2]
    assert int(M.sum()) == Pn * (Pn + 1) // 2 + sum(L * Pn + L * (L + 1) // 2 for L in Ls)


def _brute_force(st, q, k, v, scale, pos=None, slopes=None):
    """Pure-Python triple loop; visibility from explicit ancestor lists built by recursion."""
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    seg_of = {}
    for s in range(st.n_segments):
        for i in range(int(st.seg_tok_len[s])):
            seg_of[int(st.seg_tok_start[s]) + i] = (s, i)

    def ancestors(s):
        p = int(st.seg_parent[s])
        return [] if p < 0 else ancestors(p) + [p]

    out = np.zeros((T, Hq, d))
    for t in range(T):
        s_t, i_t = seg_of[t]
        anc = ancestors(s_t)
        vis = [u for u in range(T) if seg_of[u][0] in anc or (seg_of[u][0] == s_t and seg_of[u][1] <= i_t)]
        for h in range(Hq):
            g = h // (Hq // Hkv)
            sc = []
            for u in vis:
                dot = 0.0
                for c in range(d):
                    dot += q[t, h, c] * k[u, g, c]
                a = scale * dot
                if slopes is not None:
                    a -= slopes[h] * (pos[t] - pos[u])
                sc.append(a)
            mx = max(sc)
            w = [math.exp(a - mx) for a in sc]
            z = sum(w)
            for c in range(d):
                acc = 0.0
                for wi, u in zip(w, vis):
                    acc += wi * v[u, g, c]
                out[t, h, c] = acc / z
    return out


def test_brute_force_tiny():
    rng = np.random.default_rng(6)
    st = sp_synth.forkjoin_segtable(3, [[2, 4], [3]], 2)
    q, k, v = _rand_qkv(rng, st.n_tokens, 2, 1, 4)
    pos = sp_synth.classical_positions(st).astype(np.float64) * 0.75
    slopes = np.array([0.5, 0.125])
    np.testing.assert_allclose(_run(st, q, k, v, 0.5), _brute_force(st, q, k, v, 0.5), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(_run(st, q, k, v, 0.5, tok_pos=pos, alibi_slopes=slopes),
                               _brute_force(st, q, k, v, 0.5, pos, slopes), rtol=1e-11, atol=1e-13)


def test_brute_force_config1_shape():
    wl = sp_synth.WORKLOADS["c1_tiny_f32"]
    inp = sp_synth.make_inputs(wl, with_logits=False, with_decode=False)
    heads = [0, 3]
    out = _run(inp.st, inp.q, inp.k, inp.v, 1 / 8.0, heads=heads)
    ref = _brute_force(inp.st, inp.q[:, heads].astype(np.float64), inp.k[:, heads].astype(np.float64),
                       inp.v[:, heads].astype(np.float64), 1 / 8.0)
    np.testing.assert_allclose(out[:, heads], ref, rtol=1e-10, atol=1e-12)


def test_packing_permutation_only_permutes_outputs():
    rng = np.random.default_rng(7)
    lens = [[5, 3, 6]]
    a = sp_synth.forkjoin_segtable(4, lens, 3, "interleaved")
    b = sp_synth.forkjoin_segtable(4, lens, 3, "grouped")
    qa, ka, va = _rand_qkv(rng, a.n_tokens, 2, 2, 8)
    # token map a -> b, segment by segment (segment ids agree between the two packings)
    perm = np.empty(a.n_tokens, dtype=int)
    for s in range(a.n_segments):
        n = int(a.seg_tok_len[s])
        perm[a.seg_tok_start[s]:a.seg_tok_start[s] + n] = np.arange(b.seg_tok_start[s], b.seg_tok_start[s] + n)
    qb = np.empty_like(qa); kb = np.empty_like(ka); vb = np.empty_like(va)
    qb[perm], kb[perm], vb[perm] = qa, ka, va
    oa = _run(a, qa, ka, va, 0.3)
    ob = _run(b, qb, kb, vb, 0.3)
    np.testing.assert_allclose(ob[perm], oa, rtol=1e-12, atol=1e-14)


def test_bias_properties_and_classical_biased_attention():
    rng = np.random.default_rng(8)
    st = sp_synth.forkjoin_segtable(5, [[6, 6]], 3)            # equal lengths
    Hq = 2
    q, k, v = _rand_qkv(rng, st.n_tokens, Hq, Hq, 8)
    pos = sp_synth.classical_positions(st).astype(np.float64)
    slopes = np.array([0.25, 0.0625])
    base = _run(st, q, k, v, 0.4)
    np.testing.assert_array_equal(_run(st, q, k, v, 0.4, tok_pos=pos, alibi_slopes=np.zeros(Hq)), base)
    o1 = _run(st, q, k, v, 0.4, tok_pos=pos, alibi_slopes=slopes)
    o2 = _run(st, q, k, v, 0.4, tok_pos=pos + 1000.0, alibi_slopes=slopes)
    np.testing.assert_allclose(o1, o2, rtol=1e-9, atol=1e-11)
    assert not np.allclose(o1, base)
    # classical linear-distance bias on each path's own contiguous sequence (library routine)
    for slot in range(st.n_slots):
        segs = [int(st.preamble_seg[0]), int(st.doc_seg[slot]), int(st.query_seg[slot])]
        toks = np.concatenate([np.arange(st.seg_tok_start[s], st.seg_tok_start[s] + st.seg_tok_len[s]) for s in segs])
        n = len(toks)
        dist = np.arange(n)[:, None] - np.arange(n)[None, :]
        for h in range(Hq):
            ref = _sdpa_causal(q[toks, h], k[toks, h], v[toks, h], 0.4, bias=-slopes[h] * dist.astype(np.float64))
            np.testing.assert_allclose(o1[toks, h], ref, rtol=1e-10, atol=1e-12)


def test_deeper_chain_matches_causal_attention():
    # A chain root -> a -> b -> c (iterative superposition builds such prefixes, Sec. 4.1.2)
    # is a linked list, hence one causal sequence.
    rng = np.random.default_rng(9)
    lens = [3, 4, 2, 5]
    start = np.cumsum([0] + lens[:-1]).astype(np.int32)
    parent = np.array([-1, 0, 1, 2], dtype=np.int32)
    T = sum(lens)
    q, k, v = _rand_qkv(rng, T, 1, 1, 8)
    out = orc.forkjoin_prefill(q, k, v, np.array([0, 4]), start, np.array(lens, np.int32), parent, 0.35)
    np.testing.assert_allclose(out[:, 0], _sdpa_causal(q[:, 0], k[:, 0], v[:, 0], 0.35), rtol=1e-11, atol=1e-13)


from fullsize_oracle import oracle_by_segment  # noqa: E402


def test_segment_wise_oracle_equals_dense_oracle():
    """The restricted evaluation used at full size gives what the oracle's dense
    per-prompt evaluation gives, to fp64 rounding, with and without the distance bias."""
    rng = np.random.default_rng(9)
    st = sp_synth.forkjoin_segtable(19, [[40, 7, 33], [12, 50]], 6, "grouped")
    f = lambda *s: sp_synth.round_to_dtype(rng.standard_normal(s, dtype=np.float32), "bf16")
    q, k, v = f(st.n_tokens, 4, 64), f(st.n_tokens, 2, 64), f(st.n_tokens, 2, 64)
    pos = sp_synth.classical_positions(st) * 0.75
    slopes = sp_synth.geometric_slopes(4)
    for kw in ({}, {"tok_pos": pos, "alibi_slopes": slopes}):
        dense = orc.forkjoin_prefill(q, k, v, st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_parent, 0.125, **kw)
        for b in range(2):
            toks, out = oracle_by_segment(st, q, k, v, 0.125, b, [0, 3], kw.get("tok_pos"), kw.get("alibi_slopes"))
            np.testing.assert_allclose(out[:, 0], dense[toks, 0], rtol=0, atol=1e-12)
            np.testing.assert_allclose(out[:, 1], dense[toks, 3], rtol=0, atol=1e-12)
