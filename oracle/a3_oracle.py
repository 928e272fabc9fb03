"""CPU oracle for the per-layer A^3 KV-cache fusion path (arXiv 2511.17560).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the path
computes, written from the paper's Method section.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product (the HIP library and its Python
binding) never does, and shares no code, table or helper with it.

A^3 is an approximation of a full prefill, so the oracle follows the method's steps in
the paper's order (Eq. 2 position recovery, Eq. 3 scoring and top-p, Eq. 4/5 selective
recompute, cache update and attention), using NumPy primitives (matmul, exp, lexsort) as
steps and nothing else: no blocking, no fusion, no reordering.

Arithmetic: ``dtype`` (float64 by default, float32 on request).  RoPE angles are always
formed and evaluated in float64.  Tensors that the method *stores* (realigned keys,
projected Q/K/V, attention output) are rounded once to the storage type of the
configuration ("f32" or "bf16", round-to-nearest-even) exactly where the path stores them,
because later steps read the stored values.  The top-p decision is taken on the scores
cast to float32, the precision the kernels hold them in.

Readings of the paper this file takes (each is listed again in the design notes):
  * cached keys carry RoPE of their chunk-local position; Eq. 2 is applied as a rotation by
    the chunk's offset, using R(a) R(b) = R(a + b);
  * theta_i = base^(-2i/d) with d the head dimension, i = 0 .. d/2-1 (the printed formula
    uses the hidden size and a garbled index range);
  * softmax scale 1/sqrt(d) with d the head dimension (single-head notation in the paper);
  * Eq. 3 is normalised over the request's context keys, summed over all query heads and
    all question tokens; query head hq reads KV head hq // (Hq/Hkv);
  * p = floor(r * n) with n the request's context length, integer arithmetic; ties go to the
    lowest index; the selection is returned in ascending index order;
  * attention reads the cache after the update of Eq. 5 and is causal by global position;
  * V is never rotated.

Pinned by tests/test_oracle_*.py (closed forms, invariants, library routines, brute force).
Task quality on the paper's benchmark suites: parity unpinned (data and weights absent).
"""
from __future__ import annotations

import numpy as np

ROPE_INTERLEAVED = 0
ROPE_HALF = 1


# ---------------------------------------------------------------------------------------
# storage rounding
# ---------------------------------------------------------------------------------------

def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (round-to-nearest-even on the float32 bit pattern), return float32."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    u = x32.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def store(x: np.ndarray, storage: str, dtype=np.float64) -> np.ndarray:
    """Value a tensor has after being written once in the storage type."""
    if storage == "f32":
        return np.asarray(x, dtype=np.float32).astype(dtype)
    if storage == "bf16":
        return round_bf16(x).astype(dtype)
    if storage == "exact":
        return np.asarray(x, dtype=dtype)
    raise ValueError(storage)


# ---------------------------------------------------------------------------------------
# RoPE (rotation matrix of section "Position Recovery")
# ---------------------------------------------------------------------------------------

def rope_theta(head_dim: int, base: float) -> np.ndarray:
    """theta_i = base^(-2i/d), i = 0 .. d/2 - 1, in float64."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.power(np.float64(base), -2.0 * i / np.float64(head_dim))


def rope_pairs(head_dim: int, layout: int):
    """Index of the first and second coordinate of every rotated pair."""
    half = head_dim // 2
    i = np.arange(half)
    if layout == ROPE_INTERLEAVED:      # block-diagonal 2x2 rotations on adjacent coordinates
        return 2 * i, 2 * i + 1
    if layout == ROPE_HALF:
        return i, i + half
    raise ValueError(layout)


def rope_rotate(x: np.ndarray, m: np.ndarray, base: float, layout: int, dtype=np.float64) -> np.ndarray:
    """R_{Theta,m} x for every row: x is [n, heads, d], m is [n] (rotation amount per row).

    Pair i = (a, b) becomes (x_a cos(m theta_i) - x_b sin(m theta_i),
                             x_a sin(m theta_i) + x_b cos(m theta_i)).
    """
    x = np.asarray(x, dtype=dtype)
    d = x.shape[-1]
    ang = np.asarray(m, dtype=np.float64)[:, None] * rope_theta(d, base)[None, :]   # [n, d/2] float64
    c = np.cos(ang).astype(dtype)[:, None, :]
    s = np.sin(ang).astype(dtype)[:, None, :]
    a, b = rope_pairs(d, layout)
    out = np.empty_like(x)
    out[..., a] = x[..., a] * c - x[..., b] * s
    out[..., b] = x[..., a] * s + x[..., b] * c
    return out


# ---------------------------------------------------------------------------------------
# step 1: position recovery, Eq. 2
# ---------------------------------------------------------------------------------------

def rope_realign(k_cat, chunk_start, chunk_len, chunk_delta, base, layout, storage, dtype=np.float64):
    """K'_cat: every context key, which carries RoPE of its position inside its own chunk,
    is rotated further by the global position of its chunk's first token, so that it carries
    RoPE of its position in the concatenated prompt.  Rows outside every chunk (question rows)
    are returned unchanged."""
    k_cat = np.asarray(k_cat, dtype=dtype)
    out = k_cat.copy()
    for s, L, delta in zip(chunk_start, chunk_len, chunk_delta):
        s, L = int(s), int(L)
        rot = rope_rotate(k_cat[s:s + L], np.full(L, int(delta)), base, layout, dtype)
        out[s:s + L] = store(rot, storage, dtype)
    return out


# ---------------------------------------------------------------------------------------
# steps 2-pre and 4a: Q/K/V of listed rows, first lines of Eq. 5
# ---------------------------------------------------------------------------------------

def selected_qkv_proj(hidden, row_idx, row_pos, wq, wk, wv, n_q_heads, n_kv_heads, head_dim,
                      base, layout, storage, bq=None, bk=None, bv=None, dtype=np.float64):
    """Q = RoPE_p(x Wq^T), K = RoPE_p(x Wk^T), V = x Wv^T for the listed rows; p is the row's
    global position.  Weights are [out, in].  Returns compact [n, heads, d] arrays, each
    rounded once to the storage type."""
    x = np.asarray(hidden, dtype=dtype)[np.asarray(row_idx, dtype=np.int64)]
    n = x.shape[0]

    def lin(w, b, heads):
        y = x @ np.asarray(w, dtype=dtype).T
        if b is not None:
            y = y + np.asarray(b, dtype=dtype)[None, :]
        return y.reshape(n, heads, head_dim)

    q = rope_rotate(lin(wq, bq, n_q_heads), row_pos, base, layout, dtype)
    k = rope_rotate(lin(wk, bk, n_kv_heads), row_pos, base, layout, dtype)
    v = lin(wv, bv, n_kv_heads)
    return store(q, storage, dtype), store(k, storage, dtype), store(v, storage, dtype)


# ---------------------------------------------------------------------------------------
# step 2: question-relevance score, first line of Eq. 3
# ---------------------------------------------------------------------------------------

def question_scores(q_question, k_fused, seg_start, ctx_len, q_len, sm_scale, dtype=np.float64):
    """s(d_i) = sum over query heads and question tokens j of softmax_i(q_j . k'_i * scale),
    the softmax taken over the context keys of the request.  q_question is
    [sum(q_len), Hq, d] in request order, k_fused is the packed [T, Hkv, d] cache.
    Returns [T]; question rows hold -inf (they are not candidates)."""
    q_question = np.asarray(q_question, dtype=dtype)
    k_fused = np.asarray(k_fused, dtype=dtype)
    T = k_fused.shape[0]
    Hq, Hkv = q_question.shape[1], k_fused.shape[1]
    G = Hq // Hkv
    scores = np.full(T, -np.inf, dtype=dtype)
    q0 = 0
    for r in range(len(ctx_len)):
        s, N, nq = int(seg_start[r]), int(ctx_len[r]), int(q_len[r])
        acc = np.zeros(N, dtype=dtype)
        if N > 0:
            for hq in range(Hq):
                K = k_fused[s:s + N, hq // G]                        # [N, d]
                logits = (q_question[q0:q0 + nq, hq] @ K.T) * dtype(sm_scale)   # [nq, N]
                e = np.exp(logits - logits.max(axis=1, keepdims=True))
                acc += (e / e.sum(axis=1, keepdims=True)).sum(axis=0)
        scores[s:s + N] = acc
        q0 += nq
    return scores


# ---------------------------------------------------------------------------------------
# step 3: Re = top_p(s), second line of Eq. 3
# ---------------------------------------------------------------------------------------

def recompute_count(n_ctx: int, ratio_num: int, ratio_den: int) -> int:
    """Eq. 3, p = r * n: the number of context tokens of a request that are recomputed.  n is the request's
    context length (its question tokens are always recomputed and are no candidates), r = ratio_num / ratio_den
    exactly, and p is rounded down."""
    from fractions import Fraction
    import math
    return math.floor(Fraction(int(ratio_num), int(ratio_den)) * int(n_ctx))


def sel_start_from_ratio(ctx_len, ratio_num: int, ratio_den: int) -> np.ndarray:
    """[R+1] offsets of the requests' selections in a packed list: running sum of recompute_count."""
    k = [recompute_count(int(n), ratio_num, ratio_den) for n in ctx_len]
    return np.concatenate([[0], np.cumsum(k)]).astype(np.int32)


def topk_select(scores, seg_start, ctx_len, sel_start):
    """Per request, the packed rows of the k largest context scores (k = sel_start[r+1] -
    sel_start[r]); equal scores go to the lowest index; rows are returned ascending.
    The comparison is made on float32 values."""
    out = np.zeros(int(sel_start[-1]), dtype=np.int32)
    for r in range(len(ctx_len)):
        s, N = int(seg_start[r]), int(ctx_len[r])
        k = int(sel_start[r + 1]) - int(sel_start[r])
        s32 = np.asarray(scores[s:s + N], dtype=np.float32)
        order = np.lexsort((np.arange(N), -s32))          # by score descending, then index ascending
        out[int(sel_start[r]):int(sel_start[r + 1])] = np.sort(order[:k]) + s
    return out


# ---------------------------------------------------------------------------------------
# step 5: cache update, middle lines of Eq. 5
# ---------------------------------------------------------------------------------------

def kv_scatter(k_new, v_new, row_idx, k_fused, v_fused):
    """K'_cat[rows] <- k_new, V_cat[rows] <- v_new; returns updated copies."""
    k_out = np.array(k_fused, copy=True)
    v_out = np.array(v_fused, copy=True)
    idx = np.asarray(row_idx, dtype=np.int64)
    k_out[idx] = k_new
    v_out[idx] = v_new
    return k_out, v_out


# ---------------------------------------------------------------------------------------
# step 4b: attention of the active rows over the fused cache, Eq. 4 and last line of Eq. 5
# ---------------------------------------------------------------------------------------

def fused_attention(q_act, act_idx, k_fused, v_fused, seg_start, sm_scale, storage,
                    dtype=np.float64, row_block=512):
    """O = softmax(q K'^T * scale) V for every active row; a key is visible iff it belongs to
    the same request and its position is <= the row's position (the row itself included).
    q_act is [n_act, Hq, d], act_idx the packed row of each active row.  ``row_block`` only
    bounds the size of the temporary logits array."""
    q_act = np.asarray(q_act, dtype=dtype)
    k_fused = np.asarray(k_fused, dtype=dtype)
    v_fused = np.asarray(v_fused, dtype=dtype)
    act_idx = np.asarray(act_idx, dtype=np.int64)
    n_act, Hq, d = q_act.shape
    G = Hq // k_fused.shape[1]
    seg_start = np.asarray(seg_start, dtype=np.int64)
    req = np.searchsorted(seg_start, act_idx, side="right") - 1
    out = np.zeros((n_act, Hq, d), dtype=dtype)
    for r in np.unique(req):
        members = np.nonzero(req == r)[0]
        base = int(seg_start[r])
        for b0 in range(0, len(members), row_block):
            rows = members[b0:b0 + row_block]
            t = act_idx[rows]                                # packed rows, same request
            hi = int(t.max()) + 1
            visible = np.arange(base, hi)[None, :] <= t[:, None]          # [rows, keys]
            for hq in range(Hq):
                K = k_fused[base:hi, hq // G]
                V = v_fused[base:hi, hq // G]
                logits = (q_act[rows, hq] @ K.T) * dtype(sm_scale)
                logits = np.where(visible, logits, -np.inf)
                e = np.exp(logits - logits.max(axis=1, keepdims=True))
                out[rows, hq] = (e / e.sum(axis=1, keepdims=True)) @ V
    return store(out, storage, dtype)


# ---------------------------------------------------------------------------------------
# reference extras
# ---------------------------------------------------------------------------------------

def full_prefill_layer(hidden, positions, seg_start, wq, wk, wv, n_q_heads, n_kv_heads, head_dim,
                       base, layout, sm_scale, storage, dtype=np.float64):
    """Plain causal prefill of the whole packed prompt at this layer (the "Vanilla" upper
    bound): project every row at its global position, then dense causal attention.
    Returns (out [T,Hq,d], k [T,Hkv,d], v [T,Hkv,d])."""
    T = np.asarray(hidden).shape[0]
    rows = np.arange(T)
    q, k, v = selected_qkv_proj(hidden, rows, positions, wq, wk, wv, n_q_heads, n_kv_heads,
                                head_dim, base, layout, storage, dtype=dtype)
    out = fused_attention(q, rows, k, v, seg_start, sm_scale, storage, dtype)
    return out, k, v


def precompute_chunk_cache(x_pre, local_positions, wk, wv, n_kv_heads, head_dim, base, layout,
                           storage, dtype=np.float64):
    """Eq. 1 restricted to one layer: K and V of every chunk computed on its own, i.e. keys
    carry RoPE of the chunk-local position.  (Synthesises the stale cache the path starts from.)"""
    x = np.asarray(x_pre, dtype=dtype)
    n = x.shape[0]
    k = (x @ np.asarray(wk, dtype=dtype).T).reshape(n, n_kv_heads, head_dim)
    v = (x @ np.asarray(wv, dtype=dtype).T).reshape(n, n_kv_heads, head_dim)
    k = rope_rotate(k, local_positions, base, layout, dtype)
    return store(k, storage, dtype), store(v, storage, dtype)


def fuse_layer(x_cur, k_cat, v_cat, wq, wk, wv, *, seg_start, ctx_len, q_len, chunk_start, chunk_len,
               chunk_delta, sel_start, positions, n_q_heads, n_kv_heads, head_dim, base, layout,
               sm_scale, storage, dtype=np.float64, forced_sel_idx=None):
    """The whole per-layer path in call order.  Returns every intermediate by name."""
    R = len(ctx_len)
    q_rows = np.concatenate([np.arange(int(seg_start[r]) + int(ctx_len[r]), int(seg_start[r + 1]))
                             for r in range(R)]).astype(np.int64)
    proj = dict(n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim, base=base,
                layout=layout, storage=storage, dtype=dtype)
    # question rows are always recomputed; their queries drive the scoring
    qq, kq, vq = selected_qkv_proj(x_cur, q_rows, np.asarray(positions)[q_rows], wq, wk, wv, **proj)
    # step 1
    k_re = rope_realign(k_cat, chunk_start, chunk_len, chunk_delta, base, layout, storage, dtype)
    # step 2
    scores = question_scores(qq, k_re, seg_start, ctx_len, q_len, sm_scale, dtype)
    # step 3
    sel = topk_select(scores, seg_start, ctx_len, sel_start) if forced_sel_idx is None \
        else np.asarray(forced_sel_idx, dtype=np.int32)
    # step 4a
    qs, ks, vs = selected_qkv_proj(x_cur, sel, np.asarray(positions)[sel], wq, wk, wv, **proj)
    # step 5
    k_fused, v_fused = kv_scatter(ks, vs, sel, k_re, np.asarray(v_cat, dtype=dtype))
    k_fused, v_fused = kv_scatter(kq, vq, q_rows, k_fused, v_fused)
    # step 4b: active rows = selected and question rows, ascending packed row
    act = np.concatenate([sel.astype(np.int64), q_rows])
    order = np.argsort(act, kind="stable")
    act_idx = act[order]
    q_act = np.concatenate([qs, qq], axis=0)[order]
    out = fused_attention(q_act, act_idx, k_fused, v_fused, seg_start, sm_scale, storage, dtype)
    return dict(q_question=qq, k_question=kq, v_question=vq, k_realigned=k_re, scores=scores,
                sel_idx=sel, q_sel=qs, k_sel=ks, v_sel=vs, k_fused=k_fused, v_fused=v_fused,
                act_idx=act_idx.astype(np.int32), q_act=q_act, out=out, q_rows=q_rows.astype(np.int32))
