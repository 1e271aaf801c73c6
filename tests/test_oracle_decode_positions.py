"""Pins for the decode oracle, the joined-cache index and the equilibrium positions (CPU only)."""
import math
from fractions import Fraction
import os

import numpy as np

import sp_synth
from oracle import sp_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _setup(seed=0, lens=((5, 3, 6, 4),), P=4, Lq=3, Hq=4, Hkv=2, d=8):
    rng = np.random.default_rng(seed)
    st = sp_synth.forkjoin_segtable(P, [list(l) for l in lens], Lq)
    q = rng.standard_normal((st.n_tokens, Hq, d)); k = rng.standard_normal((st.n_tokens, Hkv, d))
    v = rng.standard_normal((st.n_tokens, Hkv, d))
    return rng, st, q, k, v


def test_joined_cache_is_preamble_then_kept_doc_query_pairs():
    # Alg. 3: cache = preamble (+) for each kept path (doc (+) query copy).
    _, st, *_ = _setup()
    idx = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, 0, [2, 0])
    exp = []
    for s in (st.preamble_seg[0], st.doc_seg[2], st.query_seg[2], st.doc_seg[0], st.query_seg[0]):
        exp += list(range(st.seg_tok_start[s], st.seg_tok_start[s] + st.seg_tok_len[s]))
    assert idx.tolist() == exp


def test_decode_with_one_kept_path_equals_last_row_of_prefill():
    # k = 1: [preamble; doc_i; query_i; new] is a linked list, so the decode output must be
    # the last row of the prefill oracle run on that 4-segment chain.
    rng, st, q, k, v = _setup(1)
    Hq, d = q.shape[1:]; Hkv = k.shape[1]
    qn = rng.standard_normal((Hq, d)); kn = rng.standard_normal((Hkv, d)); vn = rng.standard_normal((Hkv, d))
    slopes = np.array([0.5, 0.25, 0.125, 0.0625])
    pos = sp_synth.classical_positions(st).astype(np.float64)
    for i in range(st.n_slots):
        idx = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, 0, [i])
        new_pos = pos[idx].max() + 1
        got = orc.pruned_decode_step(qn, kn, vn, k, v, idx, np.zeros((0, Hkv, d)), np.zeros((0, Hkv, d)), 0.3,
                                     pos_new=new_pos, pos_prefill=pos, pos_resp=np.zeros(0), alibi_slopes=slopes)
        # chain table over a re-packed copy [p; d_i; q_i; new]
        n = len(idx)
        qq = np.concatenate([q[idx], qn[None]]); kk = np.concatenate([k[idx], kn[None]]); vv = np.concatenate([v[idx], vn[None]])
        pp = np.concatenate([pos[idx], [new_pos]])
        lens = [st.seg_tok_len[st.preamble_seg[0]], st.seg_tok_len[st.doc_seg[i]], st.seg_tok_len[st.query_seg[i]], 1]
        start = np.cumsum([0] + lens[:-1])
        ref = orc.forkjoin_prefill(qq, kk, vv, [0, 4], start, lens, [-1, 0, 1, 2], 0.3, tok_pos=pp, alibi_slopes=slopes)
        np.testing.assert_allclose(got, ref[n], rtol=1e-11, atol=1e-13)


def test_decode_brute_force_with_response_and_two_kept_paths():
    rng, st, q, k, v = _setup(2)
    Hq, d = q.shape[1:]; Hkv = k.shape[1]
    kept = [3, 1]
    idx = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, 0, kept)
    kr = rng.standard_normal((2, Hkv, d)); vr = rng.standard_normal((2, Hkv, d))
    qn = rng.standard_normal((Hq, d)); kn = rng.standard_normal((Hkv, d)); vn = rng.standard_normal((Hkv, d))
    got = orc.pruned_decode_step(qn, kn, vn, k, v, idx, kr, vr, 0.4)
    keys = [k[t] for t in idx] + [kr[0], kr[1], kn]
    vals = [v[t] for t in idx] + [vr[0], vr[1], vn]
    for h in range(Hq):
        g = h // (Hq // Hkv)
        sc = [0.4 * sum(qn[h, c] * kk[g, c] for c in range(d)) for kk in keys]
        mx = max(sc); w = [math.exp(a - mx) for a in sc]; z = sum(w)
        ref = [sum(wi * vv[g, c] for wi, vv in zip(w, vals)) / z for c in range(d)]
        np.testing.assert_allclose(got[h], ref, rtol=1e-11, atol=1e-13)
    # key order does not matter beyond rounding (Sec. 3.2.3: caches are simply concatenated)
    idx2 = orc.joined_cache_index(st.prompt_seg_off, st.seg_tok_start, st.seg_tok_len, st.seg_path, 0, kept[::-1])
    got2 = orc.pruned_decode_step(qn, kn, vn, k, v, idx2, kr, vr, 0.4)
    np.testing.assert_allclose(got, got2, rtol=1e-12, atol=1e-14)
    assert sorted(idx.tolist()) == sorted(idx2.tolist()) and idx.tolist() != idx2.tolist()


def test_harmonic_span_golden():
    with open(os.path.join(GOLD, "harmonic_span.txt")) as f:
        rows = [l for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) >= 5
    for l in rows:
        lens, frac = l.split(";")
        lens = [int(x) for x in lens.split(",")]
        num, den = frac.strip().split("/")
        np.testing.assert_allclose(orc.harmonic_span(lens), float(Fraction(int(num), int(den))), rtol=1e-14)


def test_equilibrium_positions_properties():
    # equal lengths: step 1, integer positions identical to the classical ones
    pp, pd, pq = orc.equilibrium_positions(5, [7, 7, 7], 3)
    assert pp.tolist() == [0, 1, 2, 3, 4]
    for x in pd:
        assert x.tolist() == list(range(5, 12))
    assert pq.tolist() == [12, 13, 14]
    st = sp_synth.forkjoin_segtable(5, [[7, 7, 7]], 3)
    cl = sp_synth.classical_positions(st)
    for i in range(3):
        a = st.seg_tok_start[st.doc_seg[i]]
        assert cl[a:a + 7].tolist() == pd[i].tolist()
        a = st.seg_tok_start[st.query_seg[i]]
        assert cl[a:a + 3].tolist() == pq.tolist()
    # ragged: all documents start right after the preamble and span the same interval of
    # length S: last position = P + S - S/len, spacing S/len; shorter docs are stretched.
    lens = [2, 6]
    pp, pd, pq = orc.equilibrium_positions(4, lens, 2)
    S = 3.0
    for L, x in zip(lens, pd):
        assert x[0] == 4.0
        np.testing.assert_allclose(np.diff(x), S / L, rtol=1e-14)
        np.testing.assert_allclose(x[-1] + S / L, 4.0 + S, rtol=1e-14)
    assert pq.tolist() == [7.0, 8.0]
    # min(len) <= S <= mean(len)   (harmonic mean bounds)
    rng = np.random.default_rng(0)
    for _ in range(20):
        lens = rng.integers(1, 300, size=rng.integers(1, 30))
        S = orc.harmonic_span(lens)
        assert lens.min() - 1e-9 <= S <= lens.mean() + 1e-9


def test_tree_positions_match_hand_worked_fractions():
    from fractions import Fraction
    path = os.path.join(os.path.dirname(__file__), "golden", "tree_positions.txt")
    n = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parents, lens, expect = [x.strip() for x in line.split(";")]
        parents = [int(x) for x in parents.split(",")]
        lens = [int(x) for x in lens.split(",")]
        got = orc.equilibrium_positions_tree(parents, lens)
        want = [[float(Fraction(x)) for x in seg.split()] for seg in expect.split("|")]
        assert len(got) == len(want)
        for g, w in zip(got, want):
            np.testing.assert_allclose(g, w, rtol=0, atol=1e-12)
        n += 1
    assert n == 3


def test_tree_positions_reduce_to_alg1_on_forkjoin_and_obey_the_span_rule():
    rng = np.random.default_rng(6)
    for _ in range(20):
        P, Lq = int(rng.integers(1, 40)), int(rng.integers(1, 9))
        lens = [int(x) for x in rng.integers(1, 60, size=int(rng.integers(1, 7)))]
        st = sp_synth.forkjoin_segtable(P, [lens], Lq)
        tree = orc.equilibrium_positions_tree(st.seg_parent, st.seg_tok_len)
        pp, pd, pq = orc.equilibrium_positions(P, lens, Lq)
        np.testing.assert_allclose(tree[0], pp, atol=1e-12)
        for i in range(len(lens)):
            np.testing.assert_allclose(tree[st.doc_seg[i]], pd[i], atol=1e-12)
            np.testing.assert_allclose(tree[st.query_seg[i]], pq, atol=1e-12)
    # random forests: siblings start together and cover the same span (the harmonic mean of their
    # lengths); positions increase strictly along every root-to-leaf chain
    for _ in range(20):
        n = int(rng.integers(2, 14))
        parents = [-1] + [int(rng.integers(-1, s)) for s in range(1, n)]
        lens = [int(x) for x in rng.integers(1, 9, size=n)]
        pos = orc.equilibrium_positions_tree(parents, lens)
        for s in range(n):
            sib = [c for c in range(n) if parents[c] == parents[s] and parents[s] >= 0]
            if parents[s] >= 0:
                S = orc.harmonic_span([lens[c] for c in sib])
                step = S / lens[s]
                assert abs((pos[s][-1] + step) - (pos[sib[0]][0] + S)) < 1e-9      # span ends S after the common start
                assert abs(pos[s][0] - pos[sib[0]][0]) < 1e-12
                assert pos[s][0] > pos[parents[s]][-1]                              # strictly after the parent
            assert np.all(np.diff(pos[s]) > 0)

