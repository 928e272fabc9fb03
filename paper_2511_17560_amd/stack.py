"""The A^3 schedule over a stack of decoder blocks, as a sequence of C-ABI calls (Method, the paragraph in
front of Eq. 3, and Eq. 3-5).  Call sequencing and buffer allocation only; all arithmetic is in liba3.

    block 0        every row: input norm, Q/K/V, causal attention, H(.)
    layer 1        K, V of every row (the true keys of Eq. 3); Q of the question rows -> scores -> top-p (Re);
                   Q of the rows [Re, Q] -> attention (Eq. 4) -> H(.)
    layers >= 2    realign the layer's chunk cache (Eq. 2); Q/K/V of the rows [Re, Q] from X_l = H(O_{l-1}),
                   K/V stored into the cache (Eq. 5); attention; H(.)
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np
import torch

from . import api


def fuse_stack(layout: api.Layout, shape, layers: Sequence[Dict[str, torch.Tensor]], g_final: torch.Tensor,
               resid: torch.Tensor, k_cat: List[torch.Tensor], v_cat: List[torch.Tensor], sel_start: np.ndarray,
               q_rows: np.ndarray, stream=None, keep: bool = False, cache_stream=None) -> dict:
    """``resid`` [T, h] holds the embedding output and is overwritten by the residual stream (all rows after
    block 0, the active rows afterwards).  ``k_cat[l]`` / ``v_cat[l]`` are the chunk caches of layer l >= 2
    (entries 0 and 1 are ignored); ``v_cat[l]`` is updated in place.  Every layer dict holds wq, wk, wv, wo,
    g_in, g_post, w_gate, w_up, w_down and optionally bq, bk, bv.
    With ``cache_stream`` (a loader.ChunkCacheStream) the caches are not resident: layer l's blocks are copied
    from host memory into a ring of device buffers while the layers before it compute, and ``k_cat`` / ``v_cat``
    are ignored; its blocks may be 8-bit (position recovery and dequantisation then run in one kernel).
    Returns dict(sel_idx, act_idx, n_act, scores, resid, hidden): ``hidden`` [T, h] holds the final-normed
    output at the active rows.  With ``keep`` every layer's attention output, caches, residual stream and the
    hidden states handed to the next layer are kept too (``per_layer[l]``: k, v, out, resid, x_next; whole arrays
    for block 0, the active rows afterwards), so that a test can check each layer on the inputs it really had."""
    dev, dt = layout.device, api.torch_dtype(layout.dtype)
    T, h = layout.total_tokens, shape.hidden
    Hq, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    n_layers = len(layers)
    assert n_layers >= 2
    total_k, nq = int(sel_start[-1]), int(len(q_rows))
    n_act = total_k + nq
    eps = float(shape.rms_eps)
    ffn = int(layers[0]["w_gate"].shape[0])
    ws_attn = layout.workspace(T)
    ws_tail = torch.empty(max(api.a3_block_tail_ws_bytes(layout, ffn, T), 256), dtype=torch.uint8, device=dev)
    x = torch.empty((T, h), dtype=dt, device=dev)
    kept = []

    def g_next(l):
        return layers[l + 1]["g_in"] if l + 1 < n_layers else g_final

    def tail(l, out, idx, n):
        lw = layers[l]
        api.a3_block_tail(layout, out, idx, n, lw["wo"], lw["g_post"], lw["w_gate"], lw["w_up"], lw["w_down"],
                          g_next(l), eps, resid, x, ws_tail, stream=stream)

    def bias(lw):
        return dict(bq=lw.get("bq"), bk=lw.get("bk"), bv=lw.get("bv"))

    if cache_stream is not None:
        for l in range(2, min(2 + cache_stream.depth, n_layers)):
            cache_stream.prefetch(l)

    # ---- block 0 on every row ---------------------------------------------------------------------------
    lw = layers[0]
    all_idx = torch.arange(T, dtype=torch.int32, device=dev)
    api.a3_rms_norm(layout, resid, None, T, lw["g_in"], eps, x, stream=stream)
    k_l = torch.empty((T, Hkv, d), dtype=dt, device=dev)
    v_l = torch.empty((T, Hkv, d), dtype=dt, device=dev)
    q_all = torch.empty((T, Hq, d), dtype=dt, device=dev)
    out_all = torch.empty((T, Hq, d), dtype=dt, device=dev)
    api.a3_selected_qkv_proj_scatter(layout, x, None, T, lw["wq"], lw["wk"], lw["wv"], q_out=q_all, k_fused=k_l,
                                     v_fused=v_l, stream=stream, **bias(lw))
    api.a3_fused_attention(layout, q_all, all_idx, T, k_l, v_l, out_all, ws_attn, stream=stream)
    tail(0, out_all, None, T)
    if keep:
        kept.append(dict(k=k_l.clone(), v=v_l.clone(), out=out_all.clone(), resid=resid.clone(), x_next=x.clone()))
    del q_all

    # ---- layer 1: true keys, scores, Re, attention of the rows [Re, Q] --------------------------------------
    lw = layers[1]
    q_rows_d = torch.as_tensor(np.ascontiguousarray(q_rows, dtype=np.int32), device=dev)
    sel_start_d = torch.as_tensor(np.ascontiguousarray(sel_start, dtype=np.int32), device=dev)
    q_question = torch.empty((max(nq, 1), Hq, d), dtype=dt, device=dev)
    scores = torch.empty(T, dtype=torch.float32, device=dev)
    sel_idx = torch.zeros(max(total_k, 1), dtype=torch.int32, device=dev)
    act_idx = torch.zeros(max(n_act, 1), dtype=torch.int32, device=dev)
    q_act = torch.empty((max(n_act, 1), Hq, d), dtype=dt, device=dev)
    out = out_all[:max(n_act, 1)]
    api.a3_selected_qkv_proj_scatter(layout, x, None, T, None, lw["wk"], lw["wv"], k_fused=k_l, v_fused=v_l,
                                     stream=stream, **bias(lw))
    api.a3_selected_qkv_proj(layout, x, q_rows_d, nq, lw["wq"], None, None, bq=lw.get("bq"), q_out=q_question,
                             stream=stream)
    api.a3_question_scores(layout, q_question, k_l, scores, ws_attn, stream=stream)
    # selection, the row list [Re, Q] and the layout of the attention's work in one call.  The rows stay the same
    # from here on: the plan is made once and reused by every layer
    api.a3_topk_select_plan(layout, scores, sel_start_d, total_k, sel_idx, n_act, act_idx, ws_attn, stream=stream)
    api.a3_selected_qkv_proj(layout, x, act_idx, n_act, lw["wq"], None, None, bq=lw.get("bq"), q_out=q_act,
                             stream=stream)
    api.a3_fused_attention_planned(layout, q_act, act_idx, n_act, k_l, v_l, out, ws_attn, stream=stream)
    tail(1, out, act_idx, n_act)
    act_long = act_idx[:n_act].long()
    if keep:
        kept.append(dict(k=k_l.clone(), v=v_l.clone(), out=out[:n_act].clone(), resid=resid[act_long], x_next=x[act_long]))

    # ---- layers 2 ..: Eq. 2, Eq. 5 --------------------------------------------------------------------------
    for l in range(2, n_layers):
        lw = layers[l]
        if cache_stream is not None and cache_stream.q8:
            # 8-bit blocks: both caches are expanded into the layer's own buffers and the ring slot is free again
            api.a3_rope_realign_q8(layout, cache_stream.acquire(l, stream), k_l, v_l, stream=stream)
            v_c = v_l
            cache_stream.release(l, stream)
            cache_stream.prefetch(l + cache_stream.depth)
        else:
            k_c, v_c = (k_cat[l], v_cat[l]) if cache_stream is None else cache_stream.acquire(l, stream)
            api.a3_rope_realign(layout, k_c, k_l, stream=stream)
        api.a3_selected_qkv_proj_scatter(layout, x, act_idx, n_act, lw["wq"], lw["wk"], lw["wv"], q_out=q_act,
                                         k_fused=k_l, v_fused=v_c, stream=stream, **bias(lw))
        api.a3_fused_attention_planned(layout, q_act, act_idx, n_act, k_l, v_c, out, ws_attn, stream=stream)
        if keep:
            kept.append(dict(k=k_l.clone(), v=v_c.clone(), out=out[:n_act].clone()))
        if cache_stream is not None and not cache_stream.q8:
            cache_stream.release(l, stream)
            cache_stream.prefetch(l + cache_stream.depth)
        tail(l, out, act_idx, n_act)
        if keep:
            kept[-1].update(resid=resid[act_long], x_next=x[act_long])
    return dict(sel_idx=sel_idx[:total_k], act_idx=act_idx[:n_act], n_act=n_act, scores=scores, resid=resid, hidden=x,
                per_layer=kept)


def prefill_stack(layout: api.Layout, shape, layers: Sequence[Dict[str, torch.Tensor]], g_final: torch.Tensor,
                  resid: torch.Tensor, stream=None, keep_kv: bool = False) -> dict:
    """Every block on every row: the plain prefill the schedule above is measured against (and, run on one
    chunk alone, the precompute of Eq. 1 that produces a chunk's per-layer K/V).  ``resid`` [T, h] holds the
    embedding output and is overwritten.  Returns dict(resid, hidden, k=[...], v=[...] if keep_kv)."""
    dev, dt = layout.device, api.torch_dtype(layout.dtype)
    T, h = layout.total_tokens, shape.hidden
    Hq, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    n_layers = len(layers)
    eps = float(shape.rms_eps)
    ffn = int(layers[0]["w_gate"].shape[0])
    ws_attn = layout.workspace(T)
    ws_tail = torch.empty(max(api.a3_block_tail_ws_bytes(layout, ffn, T), 256), dtype=torch.uint8, device=dev)
    x = torch.empty((T, h), dtype=dt, device=dev)
    all_idx = torch.arange(T, dtype=torch.int32, device=dev)
    q_all = torch.empty((T, Hq, d), dtype=dt, device=dev)
    out_all = torch.empty((T, Hq, d), dtype=dt, device=dev)
    k_l = torch.empty((T, Hkv, d), dtype=dt, device=dev)
    v_l = torch.empty((T, Hkv, d), dtype=dt, device=dev)
    ks, vs = [], []
    api.a3_rms_norm(layout, resid, None, T, layers[0]["g_in"], eps, x, stream=stream)
    for l, lw in enumerate(layers):
        if keep_kv and l > 0:
            k_l, v_l = torch.empty_like(k_l), torch.empty_like(v_l)
        api.a3_selected_qkv_proj_scatter(layout, x, None, T, lw["wq"], lw["wk"], lw["wv"], bq=lw.get("bq"),
                                         bk=lw.get("bk"), bv=lw.get("bv"), q_out=q_all, k_fused=k_l, v_fused=v_l,
                                         stream=stream)
        api.a3_fused_attention(layout, q_all, all_idx, T, k_l, v_l, out_all, ws_attn, stream=stream)
        g_next = layers[l + 1]["g_in"] if l + 1 < n_layers else g_final
        api.a3_block_tail(layout, out_all, None, T, lw["wo"], lw["g_post"], lw["w_gate"], lw["w_up"], lw["w_down"],
                          g_next, eps, resid, x, ws_tail, stream=stream)
        if keep_kv:
            ks.append(k_l)
            vs.append(v_l)
    return dict(resid=resid, hidden=x, k=ks, v=vs)
