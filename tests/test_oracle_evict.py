"""Pins of the eviction-extension oracle (Method, "Extention") and of the literal normalisation of Eq. 3:
closed forms, library routines (torch softmax / topk / pooling), brute force, invariants.  No GPU."""
import numpy as np
import pytest
import torch

from oracle import a3_oracle as ora
from oracle import evict_oracle as ev


def _rand_case(seed, ctx=(23, 9), nq=(4, 3), Hq=4, Hkv=2, d=8):
    rng = np.random.default_rng(seed)
    seg = np.concatenate([[0], np.cumsum([c + q for c, q in zip(ctx, nq)])])
    T = int(seg[-1])
    k = rng.standard_normal((T, Hkv, d))
    q = rng.standard_normal((sum(nq), Hq, d))
    return q, k, seg, np.array(ctx), np.array(nq)


def test_votes_closed_forms():
    # zero queries: every visible key gets the same weight; question token j sees N + j + 1 keys
    q, k, seg, ctx, nq = _rand_case(1, ctx=(5,), nq=(3,), Hq=2, Hkv=1)
    v = ev.window_votes(np.zeros_like(q), k, seg, ctx, nq, 0.3)
    want = 1 / 6 + 1 / 7 + 1 / 8
    assert np.allclose(v[:, :5], want, atol=1e-15) and np.all(v[:, 5:] == 0)
    # one context key, one question token, logits (a, b): the vote is e^a / (e^a + e^b)
    kk = np.zeros((2, 1, 2)); kk[0, 0] = [1.0, 0.0]; kk[1, 0] = [0.0, 2.0]
    qq = np.array([[[3.0, 0.5]]])
    v = ev.window_votes(qq, kk, np.array([0, 2]), np.array([1]), np.array([1]), 1.0)
    assert abs(v[0, 0] - np.exp(3.0) / (np.exp(3.0) + np.exp(1.0))) < 1e-15
    # the causal variant of Eq. 3 never exceeds the context-normalised score, row by row and in total:
    # its softmax has extra positive terms in the denominator
    q, k, seg, ctx, nq = _rand_case(2)
    lit = ev.question_scores_causal(q, k, seg, ctx, nq, 0.35)
    ctx_only = ora.question_scores(q, k, seg, ctx, nq, 0.35)
    rows = np.concatenate([np.arange(seg[r], seg[r] + ctx[r]) for r in range(2)])
    assert np.all(lit[rows] < ctx_only[rows]) and np.all(np.isneginf(lit[np.setdiff1d(np.arange(seg[-1]), rows)]))
    # with a single question token whose own key has a very low logit the two coincide
    q1, k1, seg1, ctx1, nq1 = _rand_case(3, ctx=(11,), nq=(1,), Hq=2, Hkv=2)
    for g in range(2):
        k1[11, g] = -40.0 * q1[0, g] / np.linalg.norm(q1[0, g])
    lit = ev.question_scores_causal(q1, k1, seg1, ctx1, nq1, 1.0)
    assert np.allclose(lit[:11], ora.question_scores(q1, k1, seg1, ctx1, nq1, 1.0)[:11], rtol=1e-9)


def test_votes_against_torch_causal_attention():
    """The cited strategy written with torch ops: causal softmax of the window queries over the whole
    prompt, summed over the window, prefix columns only."""
    q, k, seg, ctx, nq = _rand_case(4, ctx=(37, 14), nq=(6, 5), Hq=6, Hkv=2, d=16)
    scale = 0.25
    got = ev.window_votes(q, k, seg, ctx, nq, scale)
    q0 = 0
    for r in range(2):
        s, N, n = int(seg[r]), int(ctx[r]), int(nq[r])
        kk = torch.from_numpy(k[s:s + N + n]).repeat_interleave(3, dim=1)          # [L, Hq, d]
        qq = torch.from_numpy(q[q0:q0 + n])
        logits = torch.einsum("jhd,uhd->hju", qq, kk) * scale                       # [Hq, n, L]
        mask = torch.full((n, n), float("-inf")).triu(1)
        logits[:, :, N:] += mask
        att = torch.softmax(logits, dim=-1)
        want = att[:, :, :N].sum(dim=-2).numpy()
        assert np.abs(got[:, s:s + N] - want).max() < 1e-13
        # every window row's weights add up to 1 over what it sees
        assert np.allclose(att.sum(-1).numpy(), 1.0)
        q0 += n
    kv = ev.kv_head_votes(got, 2)
    assert np.allclose(kv[0], got[0] + got[1] + got[2]) and np.allclose(kv[1], got[3:].sum(0))
    assert np.allclose(ev.question_scores_causal(q, k, seg, ctx, nq, scale)[:37], got[:, :37].sum(0))


def test_votes_brute_force():
    q, k, seg, ctx, nq = _rand_case(5, ctx=(4, 3), nq=(2, 2), Hq=2, Hkv=1, d=3)
    got = ev.window_votes(q, k, seg, ctx, nq, 0.7)
    q0 = 0
    for r in range(2):
        s, N, n = int(seg[r]), int(ctx[r]), int(nq[r])
        for hq in range(2):
            col = np.zeros(N)
            for j in range(n):
                ws = [np.exp(0.7 * sum(q[q0 + j, hq, c] * k[s + u, 0, c] for c in range(3))) for u in range(N + j + 1)]
                z = sum(ws)
                for u in range(N):
                    col[u] += ws[u] / z
            assert np.allclose(got[hq, s:s + N], col, atol=1e-14)
        q0 += n


@pytest.mark.parametrize("mode,width", [("max", 3), ("max", 7), ("avg", 5), ("avg", 7), ("max", 1)])
def test_pooling_against_torch(mode, width):
    rng = np.random.default_rng(6)
    seg, ctx = np.array([0, 30, 52]), np.array([25, 19])
    votes = rng.random((3, 52))
    got = ev.pool_votes(votes, seg, ctx, width, mode)
    for r in range(2):
        s, N = int(seg[r]), int(ctx[r])
        x = torch.from_numpy(votes[:, s:s + N])[None]
        if mode == "max":
            want = torch.nn.functional.max_pool1d(x, width, stride=1, padding=width // 2)[0].numpy()
        else:
            want = torch.nn.functional.avg_pool1d(x, width, stride=1, padding=width // 2)[0].numpy()
        assert np.allclose(got[:, s:s + N], want, atol=1e-15)
        assert np.array_equal(got[:, s + N:seg[r + 1]], votes[:, s + N:seg[r + 1]])     # question rows untouched


def test_evict_select_against_torch_topk_and_invariants():
    rng = np.random.default_rng(7)
    ctx, nq, sys_len = np.array([60, 33, 12]), np.array([5, 4, 3]), np.array([7, 0, 4])
    seg = np.concatenate([[0], np.cumsum(ctx + nq)])
    votes = rng.random((3, int(seg[-1]))).astype(np.float32)
    C = 30
    keep, start = ev.evict_select(votes, seg, ctx, nq, sys_len, C)
    budget, n_keep = ev.keep_counts(ctx, nq, sys_len, C)
    assert budget.tolist() == [18, 26, 8] and n_keep.tolist() == [30, 30, 15]       # the third request fits whole
    assert start.tolist() == [0, 30, 60, 75]
    for r in range(3):
        s, N, S, n = int(seg[r]), int(ctx[r]), int(sys_len[r]), int(nq[r])
        for g in range(3):
            got = keep[g, start[r]:start[r + 1]]
            assert np.all(np.diff(got) > 0)
            assert np.array_equal(got[:S], np.arange(s, s + S)) and np.array_equal(got[len(got) - n:], np.arange(s + N, s + N + n))
            top = torch.topk(torch.from_numpy(votes[g, s + S:s + N]), int(budget[r])).indices.numpy() + s + S
            assert np.array_equal(got[S:len(got) - n], np.sort(top))
    # capacity too small for S and Q: nothing else is kept; capacity huge: everything is
    keep0, start0 = ev.evict_select(votes, seg, ctx, nq, sys_len, 3)
    assert (np.diff(start0) == sys_len + nq).all()
    keep_all, start_all = ev.evict_select(votes, seg, ctx, nq, sys_len, 10 ** 6)
    assert np.array_equal(keep_all[1], np.arange(seg[-1]))
    # ties go to the lowest row; the decision is taken in float32
    flat = np.ones((1, 14), dtype=np.float64)
    flat[0, 5] = 1.0 + 1e-12            # equal to its neighbours in float32
    k1, _ = ev.evict_select(flat, np.array([0, 14]), np.array([12]), np.array([2]), np.array([1]), 7)
    assert k1[0].tolist() == [0, 1, 2, 3, 4, 12, 13]


def test_evict_compact_is_a_per_head_gather():
    rng = np.random.default_rng(8)
    k, v = rng.standard_normal((20, 2, 4)), rng.standard_normal((20, 2, 4))
    keep = np.array([[0, 3, 4, 19], [1, 2, 18, 19]], dtype=np.int32)
    ko, vo = ev.evict_compact(k, v, keep)
    assert ko.shape == (4, 2, 4)
    for g in range(2):
        for slot in range(4):
            assert np.array_equal(ko[slot, g], k[keep[g, slot], g]) and np.array_equal(vo[slot, g], v[keep[g, slot], g])


def test_attention_over_the_retained_cache_with_everything_kept_is_unchanged():
    """Keeping every row (capacity >= prompt) must leave a later query's attention output as it was:
    the compacted cache is the cache."""
    q, k, seg, ctx, nq = _rand_case(9, ctx=(17,), nq=(3,), Hq=4, Hkv=2, d=8)
    v = np.random.default_rng(10).standard_normal(k.shape)
    votes = ev.kv_head_votes(ev.window_votes(q, k, seg, ctx, nq, 0.3), 2)
    keep, start = ev.evict_select(votes, seg, ctx, nq, np.array([2]), 100)
    ko, vo = ev.evict_compact(k, v, keep)
    assert np.array_equal(ko, k) and np.array_equal(vo, v)
    # and with a tight capacity the kept context rows are those with the largest votes
    keep, _ = ev.evict_select(votes, seg, ctx, nq, np.array([2]), 9)
    for g in range(2):
        mid = keep[g, 2:-3]
        others = np.setdiff1d(np.arange(2, 17), mid)
        assert votes[g, mid].min() >= votes[g, others].max()
