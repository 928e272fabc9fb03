"""CPU oracle for the propagating layer stack of A^3 (arXiv 2511.17560, Method, "Attention Recovery").

TEST INFRASTRUCTURE ONLY, like the per-layer oracle next to it: only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product never does.

What it states
  * H(.) of Eq. 5: the map from the attention output of one layer to the input of the next.  The paper
    describes it in one clause (layer normalisation and the feed-forward network applied to the attention
    output); the models it names (Llama-3, Qwen2.5, Mistral) all use the same pre-norm block, which is the
    reading taken here:
        r1 = r0 + O Wo^T                                  (output projection, residual)
        r2 = r1 + (silu(n1 Wg^T) * (n1 Wu^T)) Wd^T        n1 = RMSNorm(r1; g_post)   (SwiGLU MLP, residual)
        x' = RMSNorm(r2; g_next)                          (input norm of the next block, or the final norm)
    with RMSNorm(x; g) = g * x / sqrt(mean(x^2) + eps).
  * the schedule of the paragraph in front of Eq. 3 and of Eq. 3-5: block 0 runs on the whole input; at
    layer 1 Q, K, V are computed for every token, the question tokens score the context keys, Re is chosen
    once; O_1 is computed for the rows [Re, Q] only; every later layer realigns its cached keys, refreshes
    K and V of the rows [Re, Q] from X_l = H(O_{l-1}) and attends.
  * the plain full prefill of the same stack, and the chunk-wise precompute (Eq. 1) that produces the
    per-layer caches, both as the same block applied to all rows.

Storage rounding follows the per-layer oracle: a tensor the path stores is rounded once where it is
stored ("bf16", "f32", or "exact" for the pins that compare two schedules).

Pinned by tests/test_oracle_stack.py: closed forms of RMSNorm and SiLU, an independent library's decoder
stack on the same weights, brute-force loops, and the two invariants of the schedule (a single chunk at
offset 0, or a recompute ratio of 1, must reproduce the full prefill).
"""
from __future__ import annotations

import numpy as np

from . import a3_oracle as ora


# ---------------------------------------------------------------------------------------
# H(.) of Eq. 5
# ---------------------------------------------------------------------------------------

def rms_norm(x, g, eps, dtype=np.float64):
    x = np.asarray(x, dtype=dtype)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + dtype(eps)) * np.asarray(g, dtype=dtype)


def silu(x):
    return x / (1.0 + np.exp(-x))


def swiglu_mlp(x, w_gate, w_up, w_down, storage, dtype=np.float64):
    """(silu(x Wg^T) * (x Wu^T)) Wd^T; the gated activation is stored (rounded) before the last product."""
    x = np.asarray(x, dtype=dtype)
    gate = x @ np.asarray(w_gate, dtype=dtype).T
    up = x @ np.asarray(w_up, dtype=dtype).T
    act = ora.store(silu(gate) * up, storage, dtype)
    return act @ np.asarray(w_down, dtype=dtype).T, act


def block_tail(attn_out, resid, lw, g_next, eps, storage, dtype=np.float64):
    """H(.) for n rows.  attn_out [n, Hq, d] (or [n, Hq*d]); resid [n, h] is the residual stream in
    front of the attention of this block; lw holds wo [h, Hq*d], g_post [h], w_gate/w_up [f, h],
    w_down [h, f]; g_next [h] is the norm weight that precedes the next consumer.
    Returns dict(resid_mid=r1, normed=n1, act=gated activation, resid=r2, hidden_next=x')."""
    o = np.asarray(attn_out, dtype=dtype).reshape(np.asarray(attn_out).shape[0], -1)
    r1 = ora.store(np.asarray(resid, dtype=dtype) + o @ np.asarray(lw["wo"], dtype=dtype).T, storage, dtype)
    n1 = ora.store(rms_norm(r1, lw["g_post"], eps, dtype), storage, dtype)
    mlp, act = swiglu_mlp(n1, lw["w_gate"], lw["w_up"], lw["w_down"], storage, dtype)
    r2 = ora.store(r1 + mlp, storage, dtype)
    xn = ora.store(rms_norm(r2, g_next, eps, dtype), storage, dtype)
    return dict(resid_mid=r1, normed=n1, act=act, resid=r2, hidden_next=xn)


# ---------------------------------------------------------------------------------------
# plain prefill of a stack, and the chunk-wise precompute of Eq. 1
# ---------------------------------------------------------------------------------------

def _next_norm(layers, g_final, l):
    return layers[l + 1]["g_in"] if l + 1 < len(layers) else g_final


def full_prefill_stack(resid0, positions, seg_start, layers, g_final, shape, storage, dtype=np.float64):
    """Every block on every row.  resid0 [T, h] is the embedding output.  shape: dict(n_q_heads,
    n_kv_heads, head_dim, base, layout, sm_scale, eps).  Returns dict(k=[per layer], v=[per layer],
    resid [T, h], hidden [T, h] (final norm applied), hidden_in=[input of every block])."""
    T = np.asarray(resid0).shape[0]
    rows = np.arange(T)
    r = ora.store(resid0, storage, dtype)
    x = ora.store(rms_norm(r, layers[0]["g_in"], shape["eps"], dtype), storage, dtype)
    ks, vs, xs = [], [], []
    for l, lw in enumerate(layers):
        xs.append(x)
        q, k, v = ora.selected_qkv_proj(x, rows, positions, lw["wq"], lw["wk"], lw["wv"], shape["n_q_heads"],
                                        shape["n_kv_heads"], shape["head_dim"], shape["base"], shape["layout"],
                                        storage, lw.get("bq"), lw.get("bk"), lw.get("bv"), dtype=dtype)
        o = ora.fused_attention(q, rows, k, v, seg_start, shape["sm_scale"], storage, dtype)
        t = block_tail(o, r, lw, _next_norm(layers, g_final, l), shape["eps"], storage, dtype)
        r, x = t["resid"], t["hidden_next"]
        ks.append(k)
        vs.append(v)
    return dict(k=ks, v=vs, resid=r, hidden=x, hidden_in=xs)


def precompute_stack_caches(resid0, chunk_start, chunk_len, layers, g_final, shape, storage, dtype=np.float64):
    """Eq. 1: every chunk is prefilled on its own, at positions 0 .. len-1, and the K and V of every layer
    are kept.  Rows outside the chunks (the question) are left zero.  Returns (k_cat, v_cat) lists."""
    T = np.asarray(resid0).shape[0]
    L = len(layers)
    k_cat = [np.zeros((T, shape["n_kv_heads"], shape["head_dim"]), dtype=dtype) for _ in range(L)]
    v_cat = [np.zeros((T, shape["n_kv_heads"], shape["head_dim"]), dtype=dtype) for _ in range(L)]
    for s, n in zip(np.asarray(chunk_start), np.asarray(chunk_len)):
        s, n = int(s), int(n)
        if n == 0:
            continue
        one = full_prefill_stack(np.asarray(resid0)[s:s + n], np.arange(n), np.array([0, n]), layers, g_final,
                                 shape, storage, dtype)
        for l in range(L):
            k_cat[l][s:s + n] = one["k"][l]
            v_cat[l][s:s + n] = one["v"][l]
    return k_cat, v_cat


# ---------------------------------------------------------------------------------------
# the A^3 schedule over the stack
# ---------------------------------------------------------------------------------------

def fuse_stack(resid0, k_cat, v_cat, layers, g_final, shape, *, seg_start, ctx_len, q_len, chunk_start,
               chunk_len, chunk_delta, sel_start, positions, storage, dtype=np.float64, forced_sel_idx=None):
    """Block 0 on the whole input; selection at layer 1 on the true keys (Eq. 3); rows [Re, Q] only from
    there on (Eq. 4, Eq. 5).  k_cat[l], v_cat[l] are the chunk caches of layer l (used for l >= 2).
    Returns dict(sel_idx, act_idx, scores, resid [n_act, h], hidden [n_act, h], per_layer=[...])."""
    Lr = len(layers)
    assert Lr >= 2
    T = np.asarray(resid0).shape[0]
    all_rows = np.arange(T)
    R = len(ctx_len)
    q_rows = np.concatenate([np.arange(int(seg_start[r]) + int(ctx_len[r]), int(seg_start[r + 1]))
                             for r in range(R)]).astype(np.int64)
    proj = dict(n_q_heads=shape["n_q_heads"], n_kv_heads=shape["n_kv_heads"], head_dim=shape["head_dim"],
                base=shape["base"], layout=shape["layout"], storage=storage, dtype=dtype)
    positions = np.asarray(positions)
    per_layer = []

    # block 0: everything, for every row
    lw = layers[0]
    r = ora.store(resid0, storage, dtype)
    x = ora.store(rms_norm(r, lw["g_in"], shape["eps"], dtype), storage, dtype)
    q, k, v = ora.selected_qkv_proj(x, all_rows, positions, lw["wq"], lw["wk"], lw["wv"],
                                    bq=lw.get("bq"), bk=lw.get("bk"), bv=lw.get("bv"), **proj)
    o = ora.fused_attention(q, all_rows, k, v, seg_start, shape["sm_scale"], storage, dtype)
    t = block_tail(o, r, lw, layers[1]["g_in"], shape["eps"], storage, dtype)
    r, x = t["resid"], t["hidden_next"]
    per_layer.append(dict(k=k, v=v, out=o))

    # layer 1: true Q, K, V of every row; scores of the question over the context keys; Re
    lw = layers[1]
    q, k, v = ora.selected_qkv_proj(x, all_rows, positions, lw["wq"], lw["wk"], lw["wv"],
                                    bq=lw.get("bq"), bk=lw.get("bk"), bv=lw.get("bv"), **proj)
    scores = ora.question_scores(q[q_rows], k, seg_start, ctx_len, q_len, shape["sm_scale"], dtype)
    sel = ora.topk_select(scores, seg_start, ctx_len, sel_start) if forced_sel_idx is None \
        else np.asarray(forced_sel_idx, dtype=np.int32)
    act_idx = np.sort(np.concatenate([sel.astype(np.int64), q_rows]))
    o = ora.fused_attention(q[act_idx], act_idx, k, v, seg_start, shape["sm_scale"], storage, dtype)   # Eq. 4
    t = block_tail(o, r[act_idx], lw, _next_norm(layers, g_final, 1), shape["eps"], storage, dtype)
    r_act, x_act = t["resid"], t["hidden_next"]
    per_layer.append(dict(k=k, v=v, out=o))

    # layers 2 .. L-1: Eq. 2 on the layer's cache, Eq. 5 on the active rows
    for l in range(2, Lr):
        lw = layers[l]
        k_re = ora.rope_realign(k_cat[l], chunk_start, chunk_len, chunk_delta, shape["base"], shape["layout"],
                                storage, dtype)
        # the projection gathers rows of a [T, h] array: place the active rows there
        x_full = np.zeros((T, x_act.shape[1]), dtype=dtype)
        x_full[act_idx] = x_act
        qa, ka, va = ora.selected_qkv_proj(x_full, act_idx, positions[act_idx], lw["wq"], lw["wk"], lw["wv"],
                                           bq=lw.get("bq"), bk=lw.get("bk"), bv=lw.get("bv"), **proj)
        kf, vf = ora.kv_scatter(ka, va, act_idx, k_re, np.asarray(v_cat[l], dtype=dtype))
        o = ora.fused_attention(qa, act_idx, kf, vf, seg_start, shape["sm_scale"], storage, dtype)
        t = block_tail(o, r_act, lw, _next_norm(layers, g_final, l), shape["eps"], storage, dtype)
        r_act, x_act = t["resid"], t["hidden_next"]
        per_layer.append(dict(k=kf, v=vf, out=o))
    return dict(sel_idx=np.asarray(sel, dtype=np.int32), act_idx=act_idx.astype(np.int32), scores=scores,
                resid=r_act, hidden=x_act, per_layer=per_layer)
