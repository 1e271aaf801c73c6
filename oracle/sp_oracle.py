"""CPU oracle for the superposition-prompting hot path (TEST INFRASTRUCTURE ONLY).

Plain, slow, dense numpy in fp64.  It is the parity authority for the HIP library and
is never part of the product path: only tests, the smoke check and the benchmark's
CPU-baseline leg may import it.  It shares no code with the HIP path.

What each function follows (all citations are to the superposition-prompting paper):

  dag_mask / forkjoin_prefill   Sec. 3.2: a token sequence attends to another one iff
                                the prompt DAG has a path between them; Sec. 3.2.1: the
                                ForkJoin topology, where each boxed segment is a separate
                                dense causal model call over the caches of its ancestors;
                                App. B.3: the batched model call over per-path caches.
  path_saliency                 Sec. 3.2.3 and App. B.1 (Eq. 2): Bayesian path saliency
                                from language-model log-likelihoods (shifted cross-entropy
                                of the query tokens under each path), optionally length
                                normalised, plus a query-independent per-path prior term.
  prune_topk                    Sec. 3.2.3 / App. B.3 Alg. 3: greedy top-k of the path
                                posterior.
  joined_cache_index /
  pruned_decode_step            Sec. 3.2.3 (kept caches are concatenated and reused as
                                they are) and Alg. 3: cache = preamble + kept (doc+query)
                                pairs + response so far; one new token per step.
  equilibrium_positions         Sec. 3.2.2 Eq. 1, App. B.2 Eq. 3 and Alg. 1.
  equilibrium_positions_tree    the same rule read for any prompt tree (iterative
                                superposition, Sec. 4.1.2, puts forks behind chains of kept
                                documents): Eq. 1 applied to the children of every node.

Pins (tests/test_oracle_*.py): per-path equivalence with textbook causal attention,
single-document reduction to a library causal-attention routine, independence of paths,
closed forms (equal keys -> mean of visible values; one-hot values -> the attention
distribution itself), brute-force loops on tiny inputs, library log-softmax for the
saliency, exhaustive brute force for top-k, gather-vs-concatenate and decode-vs-prefill
consistency, harmonic-mean closed forms for the positions.
What cannot be pinned here: anything that depends on trained weights or on the paper's
datasets (which paths a real model keeps, accuracy) -- parity unpinned for those; they are
not computed by this oracle.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np


# ----------------------------------------------------------------------------------------
# Prompt DAG -> explicit visibility mask                                     (Sec. 3.2)
# ----------------------------------------------------------------------------------------

def prompt_tokens(seg_tok_start, seg_tok_len, seg_ids) -> np.ndarray:
    """Packed token indices of the given segments, in segment order."""
    out = [np.arange(int(seg_tok_start[s]), int(seg_tok_start[s]) + int(seg_tok_len[s])) for s in seg_ids]
    return np.concatenate(out) if out else np.zeros(0, dtype=np.int64)


def dag_mask(seg_tok_start, seg_tok_len, seg_parent, seg_ids) -> tuple:
    """Explicit boolean mask M[t, s] over the tokens of the segments `seg_ids` (one prompt).

    M[t, s] is True iff token s belongs to a strict ancestor segment of token t's segment,
    or both are in the same segment and s is not later than t (each segment is its own
    causal model call on top of its ancestors' caches).
    Returns (token_index_array, M) where M is indexed by position in token_index_array.
    """
    seg_ids = [int(s) for s in seg_ids]
    toks = prompt_tokens(seg_tok_start, seg_tok_len, seg_ids)
    n = toks.shape[0]
    seg_of = np.empty(n, dtype=np.int64)      # segment id of every local token
    idx_in = np.empty(n, dtype=np.int64)      # index of the token inside its segment
    o = 0
    for s in seg_ids:
        L = int(seg_tok_len[s])
        seg_of[o:o + L] = s
        idx_in[o:o + L] = np.arange(L)
        o += L
    # ancestor relation by walking parent pointers
    is_anc = {s: set() for s in seg_ids}
    for s in seg_ids:
        p = int(seg_parent[s])
        while p >= 0:
            is_anc[s].add(p)
            p = int(seg_parent[p])
    M = np.zeros((n, n), dtype=bool)
    for s in seg_ids:
        rows = np.nonzero(seg_of == s)[0]
        for a in is_anc[s]:
            cols = np.nonzero(seg_of == a)[0]
            M[np.ix_(rows, cols)] = True
        # own segment: causal
        own = idx_in[rows]
        M[np.ix_(rows, rows)] = own[None, :] <= own[:, None]
    return toks, M


def _kv_head(h: int, n_q_heads: int, n_kv_heads: int) -> int:
    """Grouped-query head map: consecutive groups of Hq/Hkv query heads share a KV head."""
    return h // (n_q_heads // n_kv_heads)


def masked_attention(q, k, v, M, scale, pos_q=None, pos_k=None, slope=0.0) -> np.ndarray:
    """softmax(scale * q k^T - slope * (pos_q - pos_k)) v restricted to M, all in fp64.
    q [n, d], k [m, d], v [m, d], M [n, m] boolean with at least one True per row."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    a = scale * (q @ k.T)
    if pos_q is not None and slope != 0.0:
        a = a - float(slope) * (np.asarray(pos_q, np.float64)[:, None] - np.asarray(pos_k, np.float64)[None, :])
    a = np.where(M, a, -np.inf)
    a = a - a.max(axis=1, keepdims=True)
    p = np.exp(a)
    p = p / p.sum(axis=1, keepdims=True)
    return p @ v


def forkjoin_prefill(q, k, v, prompt_seg_off, seg_tok_start, seg_tok_len, seg_parent, scale,
                     tok_pos=None, alibi_slopes=None, prompts: Optional[Sequence[int]] = None,
                     heads: Optional[Sequence[int]] = None) -> np.ndarray:
    """Prefill attention over the prompt DAG (Sec. 3.2, App. B.3).

    q [T, Hq, d], k/v [T, Hkv, d] with packed token index T over all prompts.  For every
    prompt the T_b x T_b mask is materialised and dense masked attention is evaluated per
    head.  Returns fp64 [T, Hq, d]; rows of prompts / heads not requested stay NaN.
    """
    q = np.asarray(q); k = np.asarray(k); v = np.asarray(v)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    out = np.full((T, Hq, d), np.nan, dtype=np.float64)
    n_prompts = len(prompt_seg_off) - 1
    for b in (range(n_prompts) if prompts is None else prompts):
        segs = range(int(prompt_seg_off[b]), int(prompt_seg_off[b + 1]))
        toks, M = dag_mask(seg_tok_start, seg_tok_len, seg_parent, segs)
        pos = None if tok_pos is None else np.asarray(tok_pos, np.float64)[toks]
        for h in (range(Hq) if heads is None else heads):
            g = _kv_head(h, Hq, Hkv)
            slope = 0.0 if alibi_slopes is None else float(alibi_slopes[h])
            out[toks, h, :] = masked_attention(q[toks, h, :], k[toks, g, :], v[toks, g, :], M, scale,
                                               pos, pos, slope)
    return out


# ----------------------------------------------------------------------------------------
# Path saliency                                                   (Sec. 3.2.3, App. B.1)
# ----------------------------------------------------------------------------------------

def token_log_likelihood(logits, target) -> np.ndarray:
    """lp[r] = log softmax(logits[r])[target[r]] in fp64; rows with target < 0 give 0."""
    x = np.asarray(logits, dtype=np.float64)
    tgt = np.asarray(target, dtype=np.int64)
    lp = np.zeros(x.shape[0], dtype=np.float64)
    for r in range(x.shape[0]):
        if tgt[r] < 0:
            continue
        row = x[r]
        m = row.max()
        lse = m + np.log(np.exp(row - m).sum())
        lp[r] = row[tgt[r]] - lse
    return lp


def path_saliency(logits, target, row_path, n_slots, prior=None, mode="sum") -> np.ndarray:
    """score[i] = sum (or mean) over the scored rows of path slot i of the token
    log-likelihood, plus prior[i] when given.  Rows with target < 0 are not scored.
    A slot with no scored row gets 0 (+ prior)."""
    lp = token_log_likelihood(logits, target)
    tgt = np.asarray(target, dtype=np.int64)
    rp = np.asarray(row_path, dtype=np.int64)
    score = np.zeros(n_slots, dtype=np.float64)
    count = np.zeros(n_slots, dtype=np.int64)
    for r in range(lp.shape[0]):
        if tgt[r] < 0:
            continue
        score[rp[r]] += lp[r]
        count[rp[r]] += 1
    if mode == "mean":
        score = np.where(count > 0, score / np.maximum(count, 1), 0.0)
    elif mode != "sum":
        raise ValueError(mode)
    if prior is not None:
        score = score + np.asarray(prior, dtype=np.float64)
    return score


# ----------------------------------------------------------------------------------------
# Top-k pruning                                                     (Sec. 3.2.3, Alg. 3)
# ----------------------------------------------------------------------------------------

def prune_topk(score, path_off, k) -> np.ndarray:
    """Per prompt, indices (local to the prompt) of the k largest scores, in descending
    score order; equal scores keep ascending index order; NaN ranks after everything."""
    score = np.asarray(score)
    n_prompts = len(path_off) - 1
    kept = np.zeros((n_prompts, k), dtype=np.int32)
    for b in range(n_prompts):
        s = score[int(path_off[b]):int(path_off[b + 1])].astype(np.float64)
        key = np.where(np.isnan(s), -np.inf, s)
        nan_last = np.isnan(s).astype(np.int64)
        # stable sort: primary = NaN flag ascending, secondary = score descending, then index
        order = sorted(range(len(s)), key=lambda i: (nan_last[i], -key[i], i))
        kept[b] = order[:k]
    return kept


# ----------------------------------------------------------------------------------------
# Joined cache + decode                                              (Sec. 3.2.3, Alg. 3)
# ----------------------------------------------------------------------------------------

def joined_cache_index(prompt_seg_off, seg_tok_start, seg_tok_len, seg_path, b, kept_paths) -> np.ndarray:
    """Packed token indices of the joined cache of prompt b: all shared segments (path -1)
    in segment order, then for every kept path, in the given order, that path's segments
    in segment order (document then query copy in the ForkJoin topology)."""
    segs = list(range(int(prompt_seg_off[b]), int(prompt_seg_off[b + 1])))
    shared = [s for s in segs if int(seg_path[s]) < 0]
    parts = [prompt_tokens(seg_tok_start, seg_tok_len, shared)]
    for p in kept_paths:
        mine = [s for s in segs if int(seg_path[s]) == int(p)]
        parts.append(prompt_tokens(seg_tok_start, seg_tok_len, mine))
    return np.concatenate(parts).astype(np.int64)


def pruned_decode_step(q_new, k_new, v_new, k_prefill, v_prefill, cache_index, k_resp, v_resp, scale,
                       pos_new=None, pos_prefill=None, pos_resp=None, alibi_slopes=None) -> np.ndarray:
    """One decode step for ONE prompt.

    q_new [Hq, d]; k_new/v_new [Hkv, d]; k_prefill/v_prefill [T, Hkv, d] (packed prefill
    cache); cache_index from joined_cache_index; k_resp/v_resp [n_resp, Hkv, d] = response
    tokens generated so far (without the new one).  The cache is physically concatenated
    [prefill[cache_index]; response; new] and the new token attends to all of it.
    Returns fp64 [Hq, d].
    """
    q_new = np.asarray(q_new, np.float64)
    Hq, d = q_new.shape
    Hkv = np.asarray(k_new).shape[0]
    kcat = np.concatenate([np.asarray(k_prefill, np.float64)[cache_index],
                           np.asarray(k_resp, np.float64).reshape(-1, Hkv, d),
                           np.asarray(k_new, np.float64)[None]], axis=0)
    vcat = np.concatenate([np.asarray(v_prefill, np.float64)[cache_index],
                           np.asarray(v_resp, np.float64).reshape(-1, Hkv, d),
                           np.asarray(v_new, np.float64)[None]], axis=0)
    n = kcat.shape[0]
    pos_k = None
    if alibi_slopes is not None:
        pos_k = np.concatenate([np.asarray(pos_prefill, np.float64)[cache_index],
                                np.asarray(pos_resp, np.float64).reshape(-1),
                                np.asarray([pos_new], np.float64)])
    out = np.empty((Hq, d), dtype=np.float64)
    M = np.ones((1, n), dtype=bool)
    for h in range(Hq):
        g = _kv_head(h, Hq, Hkv)
        slope = 0.0 if alibi_slopes is None else float(alibi_slopes[h])
        pq = None if pos_k is None else np.asarray([pos_new], np.float64)
        out[h] = masked_attention(q_new[h][None], kcat[:, g], vcat[:, g], M, scale, pq, pos_k, slope)[0]
    return out


# ----------------------------------------------------------------------------------------
# Equilibrium positions                                   (Sec. 3.2.2 Eq. 1, App. B.2)
# ----------------------------------------------------------------------------------------

def harmonic_span(doc_lens) -> float:
    """S(D) = n / sum_i (1 / |d_i|)  (Eq. 1)."""
    lens = np.asarray(doc_lens, dtype=np.float64)
    return float(len(lens) / np.sum(1.0 / lens))


def arange_positions(start, step, count) -> np.ndarray:
    """<start, start+step, ..., start+(count-1)*step>  (Eq. 3)."""
    return float(start) + float(step) * np.arange(int(count), dtype=np.float64)


def equilibrium_positions(preamble_len, doc_lens, query_len):
    """Alg. 1 plus the query rule of Alg. 3.

    Preamble at 0..P-1.  Document i is spaced with step S/|d_i| starting right after the
    preamble (position max(preamble)+1 = P), so that every document spans [P, P+S).
    All query copies share one position vector: it starts at P + S (one document-span
    after the preamble) with step 1, which for equal-length documents is exactly the
    classical position of the query in [preamble; doc; query].
    Returns (pos_preamble [P], [pos_doc_i], pos_query [Lq]) in fp64.
    """
    P = int(preamble_len)
    pos_p = arange_positions(0, 1, P)
    S = harmonic_span(doc_lens)
    first = (pos_p.max() + 1.0) if P > 0 else 0.0
    pos_d = [arange_positions(first, S / float(L), L) for L in doc_lens]
    pos_q = arange_positions(first + S, 1.0, query_len)
    return pos_p, pos_d, pos_q


def equilibrium_positions_tree(seg_parent, seg_tok_len):
    """Equilibrium positions for a forest of segments (a reading of Sec. 3.2.2 Eq. 1 and App. B.2
    Alg. 1 for prompt trees that are not a single ForkJoin, e.g. the rounds of iterative
    superposition in Sec. 4.1.2).

    Alg. 1 places the documents that fork behind the preamble: they start right after the
    preamble's last position and document i advances by S/|d_i| per token, S the harmonic mean of
    the sibling lengths (Eq. 1), so all siblings cover the same span S.  Read per node of the tree:
    a root segment sits at 0, 1, 2, ...; the children c_1..c_n of a node start where the node's own
    span ends and child i advances by S/|c_i| per token with S = n / sum_i 1/|c_i|; a child's span
    ends S after its start.  A single child has S = |c|, i.e. it simply continues with step 1 --
    which is the query rule of Alg. 3 (the query copy follows its document one span after the
    preamble) and the classical spacing of a chain of kept documents.

    seg_parent[s] is the parent segment of s or -1; parents come before their children.
    Returns a list with one fp64 position array per segment.
    """
    n = len(seg_parent)
    children = [[] for _ in range(n)]
    for s in range(n):
        if int(seg_parent[s]) >= 0:
            children[int(seg_parent[s])].append(s)
    pos = [None] * n
    end = [0.0] * n                                   # where the segment's span ends
    for s in range(n):
        par = int(seg_parent[s])
        L = int(seg_tok_len[s])
        if par < 0:
            pos[s] = arange_positions(0.0, 1.0, L)
            end[s] = float(L)
        else:
            S = harmonic_span([int(seg_tok_len[c]) for c in children[par]])
            pos[s] = arange_positions(end[par], S / float(L), L)
            end[s] = end[par] + S
    return pos

