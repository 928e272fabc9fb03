"""Pins of the alternative producers of the recompute list (chunk edges, largest value deviation).  No GPU."""
import numpy as np
import torch

from oracle import a3_oracle as ora
from oracle import selectors_oracle as sel


def test_value_deviation_closed_forms_and_library():
    rng = np.random.default_rng(1)
    seg, ctx = np.array([0, 12, 20]), np.array([10, 6])
    v = rng.standard_normal((20, 2, 4))
    assert np.all(sel.value_deviation_scores(v, v, seg, ctx)[[0, 9, 12, 17]] == 0.0)
    c = v.copy()
    c[3] += 0.5                                  # 8 coordinates off by 1/2: 8 * 1/4
    c[14, 1, 2] -= 3.0
    s = sel.value_deviation_scores(v, c, seg, ctx)
    assert abs(s[3] - 2.0) < 1e-15 and abs(s[14] - 9.0) < 1e-15
    assert np.all(np.isneginf(s[[10, 11, 18, 19]])) and np.count_nonzero(s[np.isfinite(s)]) == 2
    w = rng.standard_normal((20, 2, 4))
    s = sel.value_deviation_scores(v, w, seg, ctx)
    want = (torch.from_numpy(v) - torch.from_numpy(w)).pow(2).sum(dim=(1, 2)).numpy()
    rows = np.r_[0:10, 12:18]
    assert np.allclose(s[rows], want[rows], atol=1e-14)
    assert np.allclose(s[rows], np.linalg.norm((v - w).reshape(20, -1), axis=1)[rows] ** 2, atol=1e-13)
    # symmetric, and quadratic in the difference
    assert np.array_equal(s, sel.value_deviation_scores(w, v, seg, ctx))
    assert np.allclose(sel.value_deviation_scores(v, v + 3 * (w - v), seg, ctx)[rows], 9 * s[rows], rtol=1e-12)
    # feeding the unchanged top-p: the rows with the largest deviation, ascending
    picked = ora.topk_select(s, seg, ctx, np.array([0, 3, 5]))
    assert np.array_equal(picked[:3], np.sort(np.argsort(-want[:10])[:3]))
    assert np.array_equal(picked[3:], np.sort(12 + np.argsort(-want[12:18])[:2]))


def test_chunk_edges_against_brute_force():
    seg, ctx = np.array([0, 1100, 1100 + 75]), np.array([1068, 70])
    chunk_start = np.array([0, 512, 1024, 1060, 1100, 1130])
    chunk_len = np.array([512, 512, 36, 8, 30, 40])
    idx, start = sel.chunk_edge_rows(seg, ctx, chunk_start, chunk_len, 20, 20)
    # 512-row chunks give 40 rows each; the 36-row and 8-row chunks are taken whole, once; 30 whole; 40 whole
    assert start.tolist() == [0, 40 + 40 + 36 + 8, 40 + 40 + 36 + 8 + 30 + 40]
    assert np.all(np.diff(idx[start[0]:start[1]]) > 0) and np.all(np.diff(idx[start[1]:start[2]]) > 0)
    want0 = [t for t in range(1068) if any(s <= t < s + n and (t - s < 20 or s + n - t <= 20)
                                           for s, n in zip(chunk_start[:4], chunk_len[:4]))]
    assert idx[:start[1]].tolist() == want0
    assert idx[start[1]:].tolist() == list(range(1100, 1170))
    # asymmetric and empty rules
    idx, start = sel.chunk_edge_rows(seg, ctx, chunk_start, chunk_len, 3, 0)
    assert idx[:12].tolist() == [0, 1, 2, 512, 513, 514, 1024, 1025, 1026, 1060, 1061, 1062]
    idx, start = sel.chunk_edge_rows(seg, ctx, chunk_start, chunk_len, 0, 2)
    assert idx[:8].tolist() == [510, 511, 1022, 1023, 1058, 1059, 1066, 1067]
    idx, start = sel.chunk_edge_rows(seg, ctx, chunk_start, chunk_len, 0, 0)
    assert len(idx) == 0 and start.tolist() == [0, 0, 0]
