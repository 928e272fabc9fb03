"""Parity workloads: seeded tensors plus the stale chunk cache the path starts from.

TEST INFRASTRUCTURE ONLY (same rule as a3_oracle.py).  The random draws and the index
layout come from the shared input-generator module; everything that needs the method's
arithmetic (the chunk-local precompute of Eq. 1 and the planting of relevant keys) is
done here with the oracle's own routines.
"""
from __future__ import annotations

import numpy as np

import a3_synth as synth
from . import a3_oracle as ora


def sm_scale_of(w: synth.Workload) -> float:
    return 1.0 / float(np.sqrt(w.shape.head_dim))


def layout_kwargs(w: synth.Workload) -> dict:
    s = w.shape
    return dict(seg_start=w.seg_start, ctx_len=w.ctx_len, q_len=w.q_lens, chunk_start=w.chunk_start,
                chunk_len=w.chunk_len, chunk_delta=w.chunk_delta,
                sel_start=ora.sel_start_from_ratio(w.ctx_len, *w.ratio),       # the oracle's own count (Eq. 3, p = r n)
                positions=w.token_positions(), n_q_heads=s.n_q_heads, n_kv_heads=s.n_kv_heads,
                head_dim=s.head_dim, base=s.rope_base, layout=s.rope_layout,
                sm_scale=sm_scale_of(w), storage=s.dtype)


def plant_relevant_keys(w: synth.Workload, t: synth.Tensors, k_cat: np.ndarray, cosine=0.95, gain=3.0,
                        dtype=np.float64) -> np.ndarray:
    """Overwrite the stale keys of the planted rows so that, after position recovery, each KV
    head's key points along the mean question query of that head's group (cosine ``cosine``)
    with ``gain`` times the median key norm.  Stands in for the high-attention tokens of
    the paper's Fig. 2.  Returns the planted rows."""
    s = w.shape
    rows = w.planted_rows()
    if len(rows) == 0:
        return rows
    pos = w.token_positions()
    req = w.token_requests()
    rng = np.random.Generator(np.random.PCG64(w.seed + 888_000))
    G = s.group
    knorm = float(np.median(np.linalg.norm(np.asarray(k_cat, dtype=np.float64), axis=-1)))
    for r in range(w.n_req):
        q_rows = w.question_rows(r)
        qq, _, _ = ora.selected_qkv_proj(t.x_cur, q_rows, pos[q_rows], t.wq, t.wk, t.wv, s.n_q_heads,
                                         s.n_kv_heads, s.head_dim, s.rope_base, s.rope_layout, s.dtype,
                                         dtype=dtype)
        for row in rows[req[rows] == r]:
            c = int(np.nonzero((w.chunk_start <= row) & (row < w.chunk_start + w.chunk_len))[0][0])
            target = np.zeros((1, s.n_kv_heads, s.head_dim), dtype=np.float64)
            for g in range(s.n_kv_heads):
                m = qq[:, g * G:(g + 1) * G].reshape(-1, s.head_dim).mean(axis=0)
                m_hat = m / np.linalg.norm(m)
                z = rng.standard_normal(s.head_dim)
                z -= (z @ m_hat) * m_hat
                n_hat = z / np.linalg.norm(z)
                target[0, g] = gain * knorm * (cosine * m_hat + np.sqrt(1.0 - cosine ** 2) * n_hat)
            # undo the rotation that position recovery will apply to this chunk
            back = ora.rope_rotate(target, np.array([-int(w.chunk_delta[c])]), s.rope_base, s.rope_layout, dtype)
            k_cat[row] = ora.store(back[0], s.dtype, dtype)
    return rows


def build(w: synth.Workload, stale_equals_current=False, plant=True, dtype=np.float64) -> dict:
    """Everything one layer of the path consumes, as float arrays holding storage-exact values."""
    s = w.shape
    t = synth.draw_tensors(w, stale_equals_current=stale_equals_current)
    k_cat, v_cat = ora.precompute_chunk_cache(t.x_pre, w.token_local_positions(), t.wk, t.wv, s.n_kv_heads,
                                              s.head_dim, s.rope_base, s.rope_layout, s.dtype, dtype)
    planted = plant_relevant_keys(w, t, k_cat, dtype=dtype) if plant else np.zeros(0, np.int32)
    return dict(w=w, t=t, k_cat=k_cat, v_cat=v_cat, planted=planted)


def run_oracle(b: dict, dtype=np.float64, forced_sel_idx=None) -> dict:
    w, t = b["w"], b["t"]
    return ora.fuse_layer(t.x_cur, b["k_cat"], b["v_cat"], t.wq, t.wk, t.wv, dtype=dtype,
                          forced_sel_idx=forced_sel_idx, **layout_kwargs(w))
