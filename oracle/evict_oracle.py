"""CPU oracle for the eviction extension of A^3 (arXiv 2511.17560, Method, "Extention") and for the
paper-literal normalisation of Eq. 3.

TEST INFRASTRUCTURE ONLY, like the other oracle files: only tests, the smoke check and the benchmark's
CPU-baseline leg may import it.

What the paper fixes: the system prompt S and the question Q are always retained; with a capacity C, the
C - |S| - |Q| best context tokens are retained per layer and per attention head, ranked the way SnapKV
ranks them; the eviction happens once, after the first token.  SnapKV's ranking, restated: the queries of
an observation window at the end of the prompt (here: the question tokens) attend causally over the whole
prompt; a prefix token's vote is the sum over the window queries of the attention weight it receives; the
votes may be smoothed by a 1-D pooling along the token axis; the top tokens per head are kept.

Readings taken here (listed again in the design notes):
  * the softmax of a window query runs over every key it sees: all context keys of its request and the
    question keys up to itself.  (The same normalisation is the literal reading of Eq. 3's denominator;
    `question_scores_causal` is that variant of the selection score.)
  * votes are formed per query head and added over the query heads that share a KV head, so that the
    retained cache keeps the grouped layout (one index list per KV head);
  * S is the first sys_len[r] context rows of request r; they and the question rows are never candidates;
  * the budget of request r is min(max(C - sys_len[r] - q_len[r], 0), ctx_len[r] - sys_len[r]);
  * pooling (not mentioned by this paper, part of the cited strategy) is optional: width 1 = none; "max"
    pads with -inf, "avg" pads with zeros and always divides by the width; it runs over a request's context
    rows (S included as neighbours), then the candidates are ranked;
  * ties go to the lowest row, retained rows are listed in ascending row order (S, kept context, Q);
  * the ranking decision is taken on the float32 image of the votes, as for the selection of Eq. 3.

Pinned by tests/test_oracle_evict.py.
"""
from __future__ import annotations

import numpy as np


def window_votes(q_question, k, seg_start, ctx_len, q_len, sm_scale, dtype=np.float64):
    """votes[hq, t] for every query head and every packed context row t (0 elsewhere).
    q_question [sum q_len, Hq, d] (requests back to back), k [T, Hkv, d]."""
    q = np.asarray(q_question, dtype=dtype)
    k = np.asarray(k, dtype=dtype)
    T, Hkv, d = k.shape
    Hq = q.shape[1]
    G = Hq // Hkv
    votes = np.zeros((Hq, T), dtype=dtype)
    q0 = 0
    for r in range(len(ctx_len)):
        s, N, nq = int(seg_start[r]), int(ctx_len[r]), int(q_len[r])
        if nq == 0 or N == 0:
            q0 += nq
            continue
        # keys a question token may see: the context and the question up to itself
        visible = np.concatenate([np.ones((nq, N), dtype=bool), np.tril(np.ones((nq, nq), dtype=bool))], axis=1)
        for hq in range(Hq):
            keys = k[s:s + N + nq, hq // G]                       # [N + nq, d]
            logits = (q[q0:q0 + nq, hq] @ keys.T) * dtype(sm_scale)
            logits = np.where(visible, logits, -np.inf)
            e = np.exp(logits - logits.max(axis=1, keepdims=True))
            p = e / e.sum(axis=1, keepdims=True)
            votes[hq, s:s + N] = p[:, :N].sum(axis=0)
        q0 += nq
    return votes


def kv_head_votes(votes_q, n_kv_heads):
    """Sum of the votes over the query heads of each KV head: [Hkv, T]."""
    Hq, T = votes_q.shape
    return votes_q.reshape(n_kv_heads, Hq // n_kv_heads, T).sum(axis=1)


def question_scores_causal(q_question, k, seg_start, ctx_len, q_len, sm_scale, dtype=np.float64):
    """Eq. 3, first line, with the softmax over everything the question token sees (context keys and earlier
    question keys): s[t] for context rows, -inf for question rows."""
    v = window_votes(q_question, k, seg_start, ctx_len, q_len, sm_scale, dtype).sum(axis=0)
    out = np.full(v.shape, -np.inf, dtype=dtype)
    for r in range(len(ctx_len)):
        s, N = int(seg_start[r]), int(ctx_len[r])
        out[s:s + N] = v[s:s + N]
    return out


def pool_votes(votes, seg_start, ctx_len, width, mode="max"):
    """1-D pooling of stride 1 along the context rows of each request, per head.  votes [H, T]."""
    assert width % 2 == 1 and width >= 1
    if width == 1:
        return np.array(votes, copy=True)
    out = np.array(votes, copy=True)
    half = width // 2
    for r in range(len(ctx_len)):
        s, N = int(seg_start[r]), int(ctx_len[r])
        seg = votes[:, s:s + N]
        for i in range(N):
            lo, hi = max(0, i - half), min(N, i + half + 1)
            out[:, s + i] = seg[:, lo:hi].max(axis=1) if mode == "max" else seg[:, lo:hi].sum(axis=1) / width
    return out


def keep_counts(ctx_len, q_len, sys_len, capacity):
    """(budget[r], n_keep[r]) per request."""
    ctx_len, q_len, sys_len = (np.asarray(a, dtype=np.int64) for a in (ctx_len, q_len, sys_len))
    budget = np.minimum(np.maximum(capacity - sys_len - q_len, 0), ctx_len - sys_len)
    return budget, sys_len + budget + q_len


def evict_select(votes_kv, seg_start, ctx_len, q_len, sys_len, capacity):
    """keep_idx [Hkv, sum n_keep]: for each KV head and request, in ascending packed-row order: the
    system-prompt rows, the budget[r] best other context rows (float32 decision, ties to the lowest row),
    the question rows.  Returns (keep_idx int32, keep_start int32 [R+1])."""
    votes32 = np.asarray(votes_kv, dtype=np.float32)
    Hkv = votes32.shape[0]
    budget, n_keep = keep_counts(ctx_len, q_len, sys_len, capacity)
    keep_start = np.concatenate([[0], np.cumsum(n_keep)]).astype(np.int32)
    keep = np.zeros((Hkv, int(keep_start[-1])), dtype=np.int32)
    for r in range(len(ctx_len)):
        s, N, nq, S, b = int(seg_start[r]), int(ctx_len[r]), int(q_len[r]), int(sys_len[r]), int(budget[r])
        cand = np.arange(s + S, s + N)
        for g in range(Hkv):
            v = votes32[g, cand]
            order = np.lexsort((cand, -v.astype(np.float64)))       # by vote descending, then row ascending
            chosen = np.sort(cand[order[:b]])
            keep[g, keep_start[r]:keep_start[r + 1]] = np.concatenate(
                [np.arange(s, s + S), chosen, np.arange(s + N, s + N + nq)])
    return keep, keep_start


def evict_compact(k, v, keep_idx):
    """k_out[slot, g] = k[keep_idx[g, slot], g], same for v: the retained cache, [sum n_keep, Hkv, d]."""
    k, v = np.asarray(k), np.asarray(v)
    Hkv = k.shape[1]
    k_out = np.stack([k[keep_idx[g], g] for g in range(Hkv)], axis=1)
    v_out = np.stack([v[keep_idx[g], g] for g in range(Hkv)], axis=1)
    return k_out, v_out
