"""Oracle evaluation that is affordable at the full workload sizes (used by the GPU parity tests)."""
import numpy as np

from oracle import sp_oracle as orc


def oracle_by_segment(st, q, k, v, scale, b, heads, tok_pos=None, slopes=None):
    """The oracle for ALL rows of prompt b and the given heads, affordable at full size: its explicit mask
    of the whole prompt (orc.dag_mask) and its dense attention routine (orc.masked_attention), called once
    per segment on that segment's rows and on the columns the mask marks visible to them.  The columns
    left out are invisible to every row of the segment, i.e. they carry weight exactly 0 in the dense
    evaluation, so this is the dense T x T result and not another algorithm
    (tests/test_oracle_prefill.py::test_segment_wise_oracle_equals_dense_oracle pins that)."""
    segs = range(int(st.prompt_seg_off[b]), int(st.prompt_seg_off[b + 1]))
    toks, M = orc.dag_mask(st.seg_tok_start, st.seg_tok_len, st.seg_parent, segs)
    where = {int(t): i for i, t in enumerate(toks)}
    G = q.shape[1] // k.shape[1]
    out = np.full((len(toks), len(heads), q.shape[2]), np.nan)
    for s in segs:
        rows = np.array([where[int(st.seg_tok_start[s]) + i] for i in range(int(st.seg_tok_len[s]))])
        cols = np.flatnonzero(M[rows].any(axis=0))
        sub = M[np.ix_(rows, cols)]
        tr, tc = toks[rows], toks[cols]
        for j, h in enumerate(heads):
            pq = pk = None
            slope = 0.0
            if slopes is not None:
                pq, pk, slope = tok_pos[tr], tok_pos[tc], float(slopes[h])
            out[rows, j] = orc.masked_attention(q[tr, h], k[tc, h // G], v[tc, h // G], sub, scale, pq, pk, slope)
    return toks, out
