"""Planted mistakes for the oracle, applied to its source text on the CPU only.

Each entry is (name, text in oracle/sp_oracle.py, replacement).  The pins of the oracle
(tests/test_oracle_*.py) are meant to be strong enough that every one of these plausible slips --
a dropped term, a wrong sign or index, a swapped operand, an off-by-one -- makes at least one pin
fail; tests/test_oracle_pins_catch_mistakes.py checks exactly that.
"""

MUTATIONS = [
    ("own segment not causal but strictly causal", "M[np.ix_(rows, rows)] = own[None, :] <= own[:, None]",
     "M[np.ix_(rows, rows)] = own[None, :] < own[:, None]"),
    ("own segment anti-causal", "M[np.ix_(rows, rows)] = own[None, :] <= own[:, None]",
     "M[np.ix_(rows, rows)] = own[None, :] >= own[:, None]"),
    ("only the direct parent is visible", "            is_anc[s].add(p)\n            p = int(seg_parent[p])",
     "            is_anc[s].add(p)\n            p = -1"),
    ("ancestor rows see descendants instead", "            M[np.ix_(rows, cols)] = True", "            M[np.ix_(cols, rows)] = True"),
    ("softmax scale dropped", "    a = scale * (q @ k.T)", "    a = (q @ k.T)"),
    ("values replaced by keys", "    return p @ v", "    return p @ k"),
    ("distance penalty with the wrong sign", "        a = a - float(slope) * (", "        a = a + float(slope) * ("),
    ("query heads mapped to KV heads round-robin", "    return h // (n_q_heads // n_kv_heads)", "    return h % n_kv_heads"),
    ("log-likelihood with the wrong sign", "        lp[r] = row[tgt[r]] - lse", "        lp[r] = lse - row[tgt[r]]"),
    ("log-sum-exp without the maximum added back", "        lse = m + np.log(np.exp(row - m).sum())",
     "        lse = np.log(np.exp(row - m).sum())"),
    ("skipped rows still counted in the mean", "        if tgt[r] < 0:\n            continue\n        score[rp[r]] += lp[r]",
     "        score[rp[r]] += lp[r] if tgt[r] >= 0 else 0.0"),
    ("prior subtracted", "        score = score + np.asarray(prior, dtype=np.float64)",
     "        score = score - np.asarray(prior, dtype=np.float64)"),
    ("lowest scores kept", "key=lambda i: (nan_last[i], -key[i], i))", "key=lambda i: (nan_last[i], key[i], i))"),
    ("ties go to the higher index", "key=lambda i: (nan_last[i], -key[i], i))", "key=lambda i: (nan_last[i], -key[i], -i))"),
    ("NaN ranks first", "key=lambda i: (nan_last[i], -key[i], i))", "key=lambda i: (-nan_last[i], -key[i], i))"),
    ("kept paths joined in index order", "    for p in kept_paths:\n        mine", "    for p in sorted(kept_paths):\n        mine"),
    ("shared segments joined last", "    return np.concatenate(parts).astype(np.int64)",
     "    return np.concatenate(parts[1:] + parts[:1]).astype(np.int64)"),
    ("new token does not attend to itself", "                           np.asarray(v_new, np.float64)[None]], axis=0)\n    n = kcat.shape[0]",
     "                           np.asarray(v_new, np.float64)[None]], axis=0)\n    kcat = kcat[:-1]; vcat = vcat[:-1]\n    n = kcat.shape[0]"),
    ("arithmetic instead of harmonic mean", "    return float(len(lens) / np.sum(1.0 / lens))", "    return float(np.sum(lens) / len(lens))"),
    ("documents start one position late", "    pos_d = [arange_positions(first, S / float(L), L) for L in doc_lens]",
     "    pos_d = [arange_positions(first + 1.0, S / float(L), L) for L in doc_lens]"),
    ("document step not scaled by its length", "    pos_d = [arange_positions(first, S / float(L), L) for L in doc_lens]",
     "    pos_d = [arange_positions(first, 1.0, L) for L in doc_lens]"),
    ("queries start one position early", "    pos_q = arange_positions(first + S, 1.0, query_len)",
     "    pos_q = arange_positions(first + S - 1.0, 1.0, query_len)"),
    ("tree: a child's span ends after its token count instead of the sibling span", "            end[s] = end[par] + S",
     "            end[s] = end[par] + float(L)"),
    ("tree: children start at the parent's last position", "            pos[s] = arange_positions(end[par], S / float(L), L)",
     "            pos[s] = arange_positions(end[par] - 1.0, S / float(L), L)"),
    ("tree: sibling span taken over all segments with any parent", "            S = harmonic_span([int(seg_tok_len[c]) for c in children[par]])",
     "            S = harmonic_span([int(seg_tok_len[c]) for c in range(n) if int(seg_parent[c]) >= 0])"),
]
