"""CPU oracle for two alternative producers of the recompute list Re (arXiv 2511.17560, Experiments,
"Baselines" and "Experimental Settings"): the rule the paper compares against that takes the first and last
tokens of every chunk, and the rule that takes the tokens whose cached values differ most from the true
ones.  Both only replace Eq. 3; steps 4-5 run on their lists unchanged.

TEST INFRASTRUCTURE ONLY, like the other oracle files.

Readings: the deviation of a token is the squared Euclidean distance between its true value vector and its
cached one over all KV heads (the paper says "largest discrepancies between the concatenated values and the
ground-truth values" and fixes no norm; any monotone function of the distance ranks alike); question rows
are not candidates (-inf).  A chunk shorter than n_head + n_tail contributes each of its rows once.

Pinned by tests/test_oracle_selectors.py.
"""
from __future__ import annotations

import numpy as np


def value_deviation_scores(v_true, v_cat, seg_start, ctx_len, dtype=np.float64):
    """scores[t] = sum over heads and coordinates of (v_true[t] - v_cat[t])^2 for context rows, -inf else."""
    a = np.asarray(v_true, dtype=dtype)
    b = np.asarray(v_cat, dtype=dtype)
    dev = ((a - b) ** 2).reshape(a.shape[0], -1).sum(axis=1)
    out = np.full(a.shape[0], -np.inf, dtype=dtype)
    for r in range(len(ctx_len)):
        s, n = int(seg_start[r]), int(ctx_len[r])
        out[s:s + n] = dev[s:s + n]
    return out


def chunk_edge_rows(seg_start, ctx_len, chunk_start, chunk_len, n_head, n_tail):
    """(sel_idx ascending int32, sel_start int32 [R+1]): the first n_head and the last n_tail rows of every
    chunk, per request."""
    chunk_start, chunk_len = np.asarray(chunk_start), np.asarray(chunk_len)
    rows_per_req = []
    for r in range(len(ctx_len)):
        lo, hi = int(seg_start[r]), int(seg_start[r]) + int(ctx_len[r])
        rows = set()
        for s, n in zip(chunk_start, chunk_len):
            s, n = int(s), int(n)
            if not (lo <= s < hi):
                continue
            rows.update(range(s, s + min(n_head, n)))
            rows.update(range(s + max(n - n_tail, 0), s + n))
        rows_per_req.append(np.array(sorted(rows), dtype=np.int32))
    sel_start = np.concatenate([[0], np.cumsum([len(x) for x in rows_per_req])]).astype(np.int32)
    sel_idx = np.concatenate(rows_per_req) if rows_per_req else np.zeros(0, np.int32)
    return sel_idx.astype(np.int32), sel_start
