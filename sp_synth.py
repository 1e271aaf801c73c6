"""Seeded synthetic inputs for the superposition-prompting hot path.

This module only *shapes and draws* inputs: the five workload configurations,
the ForkJoin segment table (preamble -> {doc_i -> query_i}) as plain integer
arrays, and random tensors drawn from one numpy Generator in a fixed order.
It contains none of the method's arithmetic (no attention, no softmax, no
saliency, no equilibrium-position formula) so that the CPU oracle and the HIP
path can both be fed from it without sharing any computation.  The one position
table it can fill is the trivial one of classical prompting (a token's index
inside its own path, `classical_positions`), which is an input convention, not
part of the method; `geometric_slopes` likewise only draws a fixed slope vector.

Workload shapes follow the paper's question-answering setting: 20 documents per
query (Sec. 4.1.1), documents of 64-256 tokens around the reported means of
121-143 tokens (App. E), a short duplicated query per path (Sec. 3.2.1), and
top-k in {1,2,4} (App. A.3).  No dataset item is reproduced; every value is
random.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple, Union

import numpy as np


@dataclass(frozen=True)
class Workload:
    """One named configuration (shapes only)."""
    name: str
    dtype: str                  # "f32" | "bf16"
    n_prompts: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    preamble_len: int
    n_paths: int
    doc_len: Union[int, Tuple[int, int]]   # fixed, or inclusive uniform range
    query_len: int
    vocab: int
    logit_std: float
    top_k: int
    decode_steps: int
    seed: int = 20240406


WORKLOADS: Dict[str, Workload] = {
    # 1: tiny fp32 correctness case
    "c1_tiny_f32": Workload("c1_tiny_f32", "f32", 1, 4, 4, 64, 16, 4, 32, 8, 512, 2.0, 1, 4),
    # 2: 7B-class MHA shape, 20 documents per query
    "c2_mha7b_bf16": Workload("c2_mha7b_bf16", "bf16", 8, 32, 32, 128, 64, 20, 128, 24, 50432, 3.0, 2, 5),
    # 3: heavy retrieval, ragged documents
    "c3_ragged_bf16": Workload("c3_ragged_bf16", "bf16", 4, 32, 32, 128, 64, 64, (64, 256), 32, 50432, 3.0, 4, 5),
    # 4: grouped-query attention, large vocabulary
    "c4_gqa_bf16": Workload("c4_gqa_bf16", "bf16", 16, 32, 8, 128, 96, 20, 160, 24, 128256, 3.0, 2, 5),
    # 5: long pruned decode
    "c5_decode_bf16": Workload("c5_decode_bf16", "bf16", 64, 32, 32, 128, 64, 20, 128, 24, 50432, 3.0, 2, 256),
}


@dataclass
class SegTable:
    """Host-side segment table (all int32 numpy arrays; token indices are packed, global)."""
    n_prompts: int
    n_tokens: int
    prompt_seg_off: np.ndarray   # [n_prompts+1]
    seg_tok_start: np.ndarray    # [n_segments]
    seg_tok_len: np.ndarray      # [n_segments]
    seg_parent: np.ndarray       # [n_segments] global segment id of the parent, -1 = root
    seg_path: np.ndarray         # [n_segments] path id within the prompt, -1 = shared
    # bookkeeping for the harness (not passed to the library):
    path_off: np.ndarray         # [n_prompts+1] CSR of global path slots
    doc_seg: np.ndarray          # [n_slots] segment id of each path's document
    query_seg: np.ndarray        # [n_slots] segment id of each path's query copy
    preamble_seg: np.ndarray     # [n_prompts]

    @property
    def n_segments(self) -> int:
        return int(self.seg_tok_start.shape[0])

    @property
    def n_slots(self) -> int:
        return int(self.path_off[-1])


def forkjoin_segtable(preamble_len: int, doc_lens: Sequence[Sequence[int]], query_len: int,
                      packing: str = "interleaved") -> SegTable:
    """ForkJoin topology for several prompts.

    doc_lens[b][i] is the token count of document i of prompt b.  Every prompt gets one
    preamble segment (root, shared), and per path a document segment (child of the
    preamble) and a query-copy segment (child of that document).

    packing = "interleaved": tokens laid out [p; d_1; q_1; d_2; q_2; ...]
    packing = "grouped":     tokens laid out [p; d_1..d_n; q_1..q_n]
    Segment *ids* are always ordered p, d_1, q_1, d_2, q_2, ... (parents first).
    """
    assert packing in ("interleaved", "grouped")
    starts: List[int] = []
    lens: List[int] = []
    parents: List[int] = []
    paths: List[int] = []
    seg_off = [0]
    path_off = [0]
    doc_seg: List[int] = []
    query_seg: List[int] = []
    pre_seg: List[int] = []
    tok = 0
    for dl in doc_lens:
        n = len(dl)
        base_seg = len(starts)
        pre_seg.append(base_seg)
        starts.append(tok); lens.append(preamble_len); parents.append(-1); paths.append(-1)
        tok += preamble_len
        if packing == "interleaved":
            dstart, qstart = [], []
            for i in range(n):
                dstart.append(tok); tok += int(dl[i])
                qstart.append(tok); tok += query_len
        else:
            dstart, qstart = [], []
            for i in range(n):
                dstart.append(tok); tok += int(dl[i])
            for i in range(n):
                qstart.append(tok); tok += query_len
        for i in range(n):
            d_id = len(starts)
            starts.append(dstart[i]); lens.append(int(dl[i])); parents.append(base_seg); paths.append(i)
            starts.append(qstart[i]); lens.append(query_len); parents.append(d_id); paths.append(i)
            doc_seg.append(d_id); query_seg.append(d_id + 1)
        seg_off.append(len(starts))
        path_off.append(path_off[-1] + n)
    i32 = lambda a: np.asarray(a, dtype=np.int32)
    return SegTable(len(doc_lens), tok, i32(seg_off), i32(starts), i32(lens), i32(parents), i32(paths),
                    i32(path_off), i32(doc_seg), i32(query_seg), i32(pre_seg))


def classical_positions(st: SegTable) -> np.ndarray:
    """Integer position ids: every token sits at its index inside the concatenated
    sequence [preamble; doc_i; query_i] of its own path (distance 1 between neighbours,
    the "classical prompting" spacing of Sec. 3.2.2).  fp32 array [n_tokens]."""
    pos = np.zeros(st.n_tokens, dtype=np.float32)
    depth_end = np.zeros(st.n_segments, dtype=np.int64)   # tokens on the chain up to and incl. segment
    for s in range(st.n_segments):
        par = int(st.seg_parent[s])
        base = 0 if par < 0 else int(depth_end[par])
        a, n = int(st.seg_tok_start[s]), int(st.seg_tok_len[s])
        pos[a:a + n] = base + np.arange(n)
        depth_end[s] = base + n
    return pos


@dataclass
class Inputs:
    wl: Workload
    st: SegTable
    tok_pos: np.ndarray                 # fp32 [n_tokens]
    q: np.ndarray                       # fp32 [n_tokens, Hq, d]   (already rounded to wl.dtype)
    k: np.ndarray                       # fp32 [n_tokens, Hkv, d]
    v: np.ndarray                       # fp32 [n_tokens, Hkv, d]
    logits: Optional[np.ndarray]        # fp32 [R, vocab]          (already rounded to wl.dtype)
    target: Optional[np.ndarray]        # int32 [R]
    row_path: Optional[np.ndarray]      # int32 [R]  global path slot
    dec_q: Optional[np.ndarray]         # fp32 [steps, n_prompts, Hq, d]
    dec_k: Optional[np.ndarray]         # fp32 [steps, n_prompts, Hkv, d]
    dec_v: Optional[np.ndarray]
    extras: dict = field(default_factory=dict)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp32/fp64 array to the storage dtype and return it as fp32
    (bf16 values are exactly representable in fp32)."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        import torch
        return torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16).to(torch.float32).numpy()
    raise ValueError(dtype)


def draw_doc_lens(wl: Workload, rng: np.random.Generator) -> List[List[int]]:
    if isinstance(wl.doc_len, tuple):
        lo, hi = wl.doc_len
        return [[int(x) for x in rng.integers(lo, hi + 1, size=wl.n_paths)] for _ in range(wl.n_prompts)]
    return [[int(wl.doc_len)] * wl.n_paths for _ in range(wl.n_prompts)]


def make_inputs(wl: Workload, *, n_prompts: Optional[int] = None, with_logits: bool = True,
                with_decode: bool = True, decode_steps: Optional[int] = None,
                packing: str = "interleaved", seed: Optional[int] = None) -> Inputs:
    """Draw every tensor of one workload on the host.

    Draw order is fixed: doc lengths, Q, K, V, logits, targets, decode q/k/v.  All float
    tensors are rounded to the workload's storage dtype before being returned (as fp32
    arrays), so the oracle and the device see identical values.
    """
    rng = np.random.default_rng(wl.seed if seed is None else seed)
    B = wl.n_prompts if n_prompts is None else n_prompts
    wl_eff = wl if B == wl.n_prompts else Workload(**{**wl.__dict__, "n_prompts": B})
    doc_lens = draw_doc_lens(wl_eff, rng)
    st = forkjoin_segtable(wl.preamble_len, doc_lens, wl.query_len, packing)
    T = st.n_tokens
    f = lambda *shape: round_to_dtype(rng.standard_normal(shape, dtype=np.float32), wl.dtype)
    q = f(T, wl.n_q_heads, wl.head_dim)
    k = f(T, wl.n_kv_heads, wl.head_dim)
    v = f(T, wl.n_kv_heads, wl.head_dim)
    logits = target = row_path = None
    if with_logits:
        R = st.n_slots * wl.query_len
        logits = round_to_dtype(rng.standard_normal((R, wl.vocab), dtype=np.float32) * np.float32(wl.logit_std),
                                wl.dtype)
        # one set of query target ids per prompt, replicated over that prompt's paths
        # (every query segment is a copy of the same query)
        target = np.empty(R, dtype=np.int32)
        row_path = np.empty(R, dtype=np.int32)
        r = 0
        for b in range(B):
            ids = rng.integers(0, wl.vocab, size=wl.query_len).astype(np.int32)
            for slot in range(int(st.path_off[b]), int(st.path_off[b + 1])):
                target[r:r + wl.query_len] = ids
                row_path[r:r + wl.query_len] = slot
                r += wl.query_len
    dec_q = dec_k = dec_v = None
    if with_decode:
        S = wl.decode_steps if decode_steps is None else decode_steps
        dec_q = f(S, B, wl.n_q_heads, wl.head_dim)
        dec_k = f(S, B, wl.n_kv_heads, wl.head_dim)
        dec_v = f(S, B, wl.n_kv_heads, wl.head_dim)
    return Inputs(wl_eff, st, classical_positions(st), q, k, v, logits, target, row_path, dec_q, dec_k, dec_v)


def geometric_slopes(n_heads: int) -> np.ndarray:
    """A fixed, arbitrary vector of non-negative per-head bias slopes for bias-enabled
    parity runs (a geometric sequence from 1/2 down to 2^-8)."""
    e = np.linspace(1.0, 8.0, n_heads)
    return np.power(2.0, -e).astype(np.float32)
