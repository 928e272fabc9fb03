"""Pins for the oracle's question-relevance score and top-p selection (Eq. 3) and for the
projection of listed rows (first lines of Eq. 5)."""
import math

import numpy as np
import pytest
import torch

from oracle import a3_oracle as ora
from oracle import workload as wl
import a3_synth as synth


def _rand_problem(seed, ctx_lens=(23, 40), q_lens=(3, 5), Hq=4, Hkv=2, d=8):
    rng = np.random.default_rng(seed)
    seg, row = [0], 0
    for n, q in zip(ctx_lens, q_lens):
        row += n + q
        seg.append(row)
    T = seg[-1]
    k = rng.standard_normal((T, Hkv, d))
    qq = rng.standard_normal((sum(q_lens), Hq, d))
    return qq, k, np.array(seg), np.array(ctx_lens), np.array(q_lens)


def test_scores_two_key_closed_form():
    # one head, one question token, two context keys: logits (ln 3, 0) -> softmax (3/4, 1/4)
    d = 4
    q = np.zeros((1, 1, d)); q[0, 0, 0] = 1.0
    k = np.zeros((3, 1, d)); k[0, 0, 0] = math.log(3.0) * math.sqrt(d)
    s = ora.question_scores(q, k, [0, 3], [2], [1], 1 / math.sqrt(d))
    np.testing.assert_allclose(s[:2], [0.75, 0.25], rtol=1e-14)
    assert s[2] == -np.inf          # the question row is not a candidate


def test_scores_sum_and_uniform_and_permutation():
    qq, k, seg, ctx, ql = _rand_problem(0)
    Hq = qq.shape[1]
    s = ora.question_scores(qq, k, seg, ctx, ql, 0.35)
    for r in range(2):
        rows = slice(seg[r], seg[r] + ctx[r])
        assert np.all(s[rows] >= 0)
        # every softmax row sums to one: total = heads * question tokens
        np.testing.assert_allclose(s[rows].sum(), Hq * ql[r], rtol=1e-12)
    # zero queries: uniform attention
    s0 = ora.question_scores(np.zeros_like(qq), k, seg, ctx, ql, 0.35)
    np.testing.assert_allclose(s0[:ctx[0]], Hq * ql[0] / ctx[0], rtol=1e-13)
    # permuting the context tokens of request 0 permutes its scores and leaves request 1 alone
    perm = np.random.default_rng(1).permutation(ctx[0])
    k2 = k.copy(); k2[:ctx[0]] = k[:ctx[0]][perm]
    s2 = ora.question_scores(qq, k2, seg, ctx, ql, 0.35)
    np.testing.assert_allclose(s2[:ctx[0]], s[:ctx[0]][perm], rtol=1e-12)
    np.testing.assert_allclose(s2[seg[1]:seg[1] + ctx[1]], s[seg[1]:seg[1] + ctx[1]], rtol=0)


def test_scores_against_torch_softmax_library():
    qq, k, seg, ctx, ql = _rand_problem(5, Hq=6, Hkv=2, d=16)
    s = ora.question_scores(qq, k, seg, ctx, ql, 0.25)
    G = 3
    q0 = 0
    for r in range(2):
        K = torch.from_numpy(k[seg[r]:seg[r] + ctx[r]]).repeat_interleave(G, dim=1)   # [N, Hq, d]
        Q = torch.from_numpy(qq[q0:q0 + ql[r]])                                        # [nq, Hq, d]
        p = torch.softmax(torch.einsum("jhd,nhd->hjn", Q, K) * 0.25, dim=-1)
        np.testing.assert_allclose(s[seg[r]:seg[r] + ctx[r]], p.sum(dim=(0, 1)).numpy(), rtol=1e-12)
        q0 += ql[r]


def test_scores_brute_force_python_loops():
    qq, k, seg, ctx, ql = _rand_problem(7, ctx_lens=(9,), q_lens=(2,), Hq=4, Hkv=2, d=4)
    s = ora.question_scores(qq, k, seg, ctx, ql, 0.5)
    want = [0.0] * 9
    for hq in range(4):
        g = hq // 2
        for j in range(2):
            logit = [sum(qq[j, hq, c] * k[i, g, c] for c in range(4)) * 0.5 for i in range(9)]
            z = sum(math.exp(l) for l in logit)
            for i in range(9):
                want[i] += math.exp(logit[i]) / z
    np.testing.assert_allclose(s[:9], want, rtol=1e-12)


def test_scores_gqa_head_mapping_is_contiguous_groups():
    # Hq=4, Hkv=2: query head 1 belongs to KV head 0.  Only query head 1 is non-zero; KV head 0
    # has its aligned key at token 3, KV head 1 at token 5.
    d = 4
    k = np.zeros((8, 2, d)); k[3, 0, 0] = 10.0; k[5, 1, 0] = 10.0
    q = np.zeros((1, 4, d)); q[0, 1, 0] = 10.0
    s = ora.question_scores(q, k, [0, 8], [7], [1], 1.0)
    assert int(np.argmax(s[:7])) == 3


def test_topk_against_library_sorts_and_edges():
    rng = np.random.default_rng(11)
    N = 500
    sc = rng.integers(0, 40, size=N).astype(np.float64) / 8.0       # many exact ties
    seg, ctx = np.array([0, N + 4]), np.array([N])
    full = np.concatenate([sc, np.full(4, -np.inf)])
    for k in (0, 1, 37, 250, N):
        got = ora.topk_select(full, seg, ctx, np.array([0, k]))
        _, order = torch.sort(torch.from_numpy(sc.astype(np.float32)), stable=True, descending=True)
        want = np.sort(order[:k].numpy())
        assert np.array_equal(got, want)
        py = sorted(sorted(range(N), key=lambda i: (-sc[i], i))[:k])
        assert got.tolist() == py
    # all equal: lowest indices win
    assert ora.topk_select(np.ones(10), [0, 10], [10], [0, 4]).tolist() == [0, 1, 2, 3]
    # duplicates straddling the cut: value 2.0 at 1, 4, 6 and k = 3 -> the 5.0 plus the two lowest 2.0
    s = np.array([1.0, 2.0, 5.0, 0.0, 2.0, 1.0, 2.0])
    assert ora.topk_select(s, [0, 7], [7], [0, 3]).tolist() == [1, 2, 4]


def test_topk_decision_is_taken_in_float32_and_offsets_are_packed():
    # two float64 scores that differ below float32 resolution tie -> lowest index
    s = np.array([0.5, 1.0, 1.0 + 1e-12, 0.1, -np.inf, -np.inf, 0.3, 0.9, 0.2, -np.inf])
    seg, ctx, sel = [0, 6, 10], [4, 3], [0, 1, 3]
    got = ora.topk_select(s, seg, ctx, sel)
    assert got.tolist() == [1, 6, 7]


def test_projection_identity_weights_and_library_pin():
    d, H = 8, 2
    h = H * d
    rng = np.random.default_rng(13)
    x = rng.standard_normal((10, h))
    eye = np.eye(h)
    rows = np.array([7, 2, 9])
    pos = np.array([70, 20, 90])
    q, k, v = ora.selected_qkv_proj(x, rows, pos, eye, eye, eye, H, H, d, 1e4, 0, "exact")
    np.testing.assert_array_equal(v, x[rows].reshape(3, H, d))
    np.testing.assert_allclose(q, ora.rope_rotate(x[rows].reshape(3, H, d), pos, 1e4, 0), rtol=0)
    np.testing.assert_allclose(k, q, rtol=0)
    # general weights with bias against torch's matmul: V directly, Q/K by rotating back to position 0
    wq = rng.standard_normal((2 * h, h)); wk = rng.standard_normal((h, h)); wv = rng.standard_normal((h, h))
    bq = rng.standard_normal(2 * h); bk = rng.standard_normal(h); bv = rng.standard_normal(h)
    q, k, v = ora.selected_qkv_proj(x, rows, pos, wq, wk, wv, 2 * H, H, d, 1e4, 1, "exact", bq, bk, bv)
    tx = torch.from_numpy(x[rows])
    want_v = (tx @ torch.from_numpy(wv).T + torch.from_numpy(bv)).numpy().reshape(3, H, d)
    want_q = (tx @ torch.from_numpy(wq).T + torch.from_numpy(bq)).numpy().reshape(3, 2 * H, d)
    np.testing.assert_allclose(v, want_v, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(ora.rope_rotate(q, -pos, 1e4, 1), want_q, rtol=1e-10, atol=1e-10)
    assert q.shape == (3, 2 * H, d) and k.shape == (3, H, d)


@pytest.mark.parametrize("cfg", [1, 2])
def test_invariant_planted_relevant_tokens_are_selected(cfg):
    """Invariant 5: keys aligned with the mean question query collect the highest scores."""
    w = synth.config(cfg)
    b = wl.build(w)
    s = w.shape
    pos = w.token_positions()
    q_rows = w.question_rows()
    qq, _, _ = ora.selected_qkv_proj(b["t"].x_cur, q_rows, pos[q_rows], b["t"].wq, b["t"].wk, b["t"].wv,
                                     s.n_q_heads, s.n_kv_heads, s.head_dim, s.rope_base, s.rope_layout, s.dtype)
    k_re = ora.rope_realign(b["k_cat"], w.chunk_start, w.chunk_len, w.chunk_delta, s.rope_base,
                            s.rope_layout, s.dtype)
    # the planted keys really are aligned with the mean query after position recovery
    G = s.group
    for row in b["planted"]:
        for g in range(s.n_kv_heads):
            m = qq[:, g * G:(g + 1) * G].reshape(-1, s.head_dim).mean(0)
            cosv = (k_re[row, g] @ m) / np.linalg.norm(k_re[row, g]) / np.linalg.norm(m)
            assert cosv >= 0.9
    sc = ora.question_scores(qq, k_re, w.seg_start, w.ctx_len, w.q_lens, wl.sm_scale_of(w))
    sel = ora.topk_select(sc, w.seg_start, w.ctx_len, w.sel_start)
    assert len(sel) == w.total_k == {1: 76, 2: 768}[cfg]
    assert set(b["planted"].tolist()) <= set(sel.tolist())
    # and they rank in the upper half of the selection
    rank = np.argsort(np.argsort(-sc[:w.ctx_len[0]], kind="stable"), kind="stable")
    assert rank[b["planted"]].max() < w.total_k // 2


def test_recompute_count_of_the_five_configurations():
    """Eq. 3, p = r * n with n the request's context length, rounded down: 76 of 512 at 15 %, 768 of 5120 at 15 %,
    1638 of 16384 at 10 %, and floor(0.2 N) / floor(0.15 N_r) for the drawn lengths of configurations 4 and 5
    (checked against exact rational arithmetic written out here, not against the oracle's own expression)."""
    assert ora.recompute_count(512, 15, 100) == 76
    assert ora.recompute_count(5120, 15, 100) == 768
    assert ora.recompute_count(16384, 10, 100) == 1638
    w4, w5 = synth.config(4), synth.config(5)
    n4 = int(w4.ctx_len[0])
    k4 = ora.recompute_count(n4, 20, 100)
    assert 5 * k4 <= n4 < 5 * (k4 + 1)                      # k = floor(N / 5)
    for n in w5.ctx_len:
        k = ora.recompute_count(int(n), 15, 100)
        assert 20 * k <= 3 * int(n) < 20 * (k + 1)          # k = floor(3 N / 20)
    # the running sums the path is handed
    assert np.array_equal(ora.sel_start_from_ratio([512], 15, 100), [0, 76])
    assert np.array_equal(ora.sel_start_from_ratio(w5.ctx_len, 15, 100),
                          np.concatenate([[0], np.cumsum([(3 * int(n)) // 20 for n in w5.ctx_len])]))
    # ends of the range, monotone in both arguments, never more than there are tokens, no float rounding upwards
    assert ora.recompute_count(1000, 0, 100) == 0 and ora.recompute_count(1000, 100, 100) == 1000
    assert ora.recompute_count(0, 15, 100) == 0
    assert ora.recompute_count(100, 29, 100) == 29 and ora.recompute_count(7, 1, 3) == 2
    ks = [ora.recompute_count(n, 15, 100) for n in range(0, 2000)]
    assert all(b - a in (0, 1) for a, b in zip(ks, ks[1:])) and all(k <= n for n, k in enumerate(ks))
    assert [ora.recompute_count(999, r, 100) for r in range(101)] == sorted(ora.recompute_count(999, r, 100) for r in range(101))
