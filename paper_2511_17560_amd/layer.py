"""One pass of the whole per-layer fusion path: the sequence of C-ABI calls of one layer, on
preallocated buffers.  Call sequencing only; all arithmetic happens inside liba3.

    Q of the question rows -> realign keys (Eq. 2) -> scores (Eq. 3) -> top-p (Eq. 3)
    -> project the rows [Re, Q] (Eq. 5) -> update cache (Eq. 5) -> attention (Eq. 4 / Eq. 5)
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from . import api


@dataclass
class LayerBuffers:
    """Everything a layer pass writes, allocated once per batch shape."""
    k_fused: torch.Tensor      # [T, Hkv, d]   realigned + updated keys
    scores: torch.Tensor       # [T] float32
    sel_start: torch.Tensor    # [R+1] int32 (device)
    sel_idx: torch.Tensor      # [total_k] int32 (single request: a view of act_idx)
    act_idx: torch.Tensor      # [n_act] int32
    q_rows: torch.Tensor       # [sum q_len] int32, packed rows of the question tokens
    q_question: torch.Tensor   # [sum q_len, Hq, d]  (single request: a view of q_act)
    q_act: torch.Tensor        # [n_act, Hq, d]
    k_act: torch.Tensor        # [n_act, Hkv, d]
    v_act: torch.Tensor        # [n_act, Hkv, d]
    out: torch.Tensor          # [n_act, Hq, d]
    ws: torch.Tensor
    total_k: int
    n_act: int
    single: bool
    side: object = None        # second stream (default priority) on which the attention plan is made
    ev_rows: object = None     # event: the list of active rows is final
    ev_plan: object = None     # event: the plan is in the workspace


def make_buffers(layout: api.Layout, sel_start: np.ndarray, q_rows: np.ndarray, shape) -> LayerBuffers:
    dev = layout.device
    dt = api.torch_dtype(layout.dtype)
    T = layout.total_tokens
    Hq, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    total_k = int(sel_start[-1])
    nq = int(len(q_rows))
    n_act = total_k + nq
    single = layout.n_req == 1
    act_idx = torch.zeros(max(n_act, 1), dtype=torch.int32, device=dev)
    q_rows_d = torch.as_tensor(np.ascontiguousarray(q_rows, dtype=np.int32), device=dev)
    q_act = torch.empty((max(n_act, 1), Hq, d), dtype=dt, device=dev)
    if single:
        # active order of a single request is [selected | question]: the question part of every
        # active-row buffer can be written by the first projection and never moves
        act_idx[total_k:n_act] = q_rows_d
        sel_idx = act_idx[:total_k]
        q_question = q_act[total_k:n_act]
    else:
        sel_idx = torch.zeros(max(total_k, 1), dtype=torch.int32, device=dev)
        q_question = torch.empty((max(nq, 1), Hq, d), dtype=dt, device=dev)
    return LayerBuffers(
        k_fused=torch.empty((T, Hkv, d), dtype=dt, device=dev),
        scores=torch.empty(T, dtype=torch.float32, device=dev),
        sel_start=torch.as_tensor(np.ascontiguousarray(sel_start, dtype=np.int32), device=dev),
        sel_idx=sel_idx, act_idx=act_idx, q_rows=q_rows_d, q_question=q_question, q_act=q_act,
        k_act=torch.empty((max(n_act, 1), Hkv, d), dtype=dt, device=dev),
        v_act=torch.empty((max(n_act, 1), Hkv, d), dtype=dt, device=dev),
        out=torch.empty((max(n_act, 1), Hq, d), dtype=dt, device=dev),
        ws=layout.workspace(n_act), total_k=total_k, n_act=n_act, single=single,
        side=torch.cuda.Stream(device=dev), ev_rows=torch.cuda.Event(), ev_plan=torch.cuda.Event())


def fuse_layer(layout: api.Layout, b: LayerBuffers, x_cur: torch.Tensor, k_cat: torch.Tensor, v_cache: torch.Tensor,
               wq: torch.Tensor, wk: torch.Tensor, wv: torch.Tensor, stream=None, fused_scatter: bool = True,
               fused_realign: bool = True, overlap_plan: bool = False, fused_plan: bool = True) -> None:
    """Runs steps 1-5 for one layer.  ``k_cat`` is read, ``b.k_fused`` and ``v_cache`` (in place)
    hold the fused cache afterwards, ``b.out`` the attention output of the active rows.

    ``fused_scatter`` (default) lets the projection of the active rows write the fresh K/V straight into the
    caches (a3_selected_qkv_proj_scatter); otherwise the plain sequence a3_selected_qkv_proj ->
    a3_kv_scatter is used.  Both give the same cache, written after the scores were read.
    ``fused_realign`` (default) runs steps 1 and 2 as one call (a3_realign_scores).
    ``fused_plan`` (default) runs the selection, the row list [Re, Q] and the layout of the attention's work as
    one call (a3_topk_select_plan; a single launch for a batch of one request) and attends with
    a3_fused_attention_planned; otherwise a3_topk_select, a3_active_rows and a3_fused_attention.
    ``overlap_plan`` has the attention's work laid out (a3_attention_plan, one small workgroup) on a second
    stream as soon as the active rows are known, beside the projection of the selected rows, and then calls
    a3_fused_attention_planned.  Off by default: on this hardware the two cross-stream waits cost more (about
    20 us) than the 9 us plan kernel they hide."""
    nq = b.n_act - b.total_k
    k = b.total_k
    # Only Q of the question rows is needed before the selection (it scores the context); their K and V come out
    # of the second projection, which covers all active rows: the first call then streams W_q alone, and the few
    # question rows do not add a row tile to the second.
    api.a3_selected_qkv_proj(layout, x_cur, b.q_rows, nq, wq, None, None, q_out=b.q_question, stream=stream)
    if fused_realign:
        api.a3_realign_scores(layout, b.q_question, k_cat, b.k_fused, b.scores, b.ws, stream=stream)
    else:
        api.a3_rope_realign(layout, k_cat, b.k_fused, stream=stream)
        api.a3_question_scores(layout, b.q_question, b.k_fused, b.scores, b.ws, stream=stream)
    rows, n_rows = b.act_idx, b.n_act
    overlap_plan = overlap_plan and b.side is not None and not fused_plan
    if fused_plan:
        api.a3_topk_select_plan(layout, b.scores, b.sel_start, k, b.sel_idx, b.n_act, b.act_idx, b.ws, stream=stream)
    else:
        api.a3_topk_select(layout, b.scores, b.sel_start, k, b.sel_idx, stream=stream)
        if not b.single:       # (a single request: act_idx = [selected | question], filled in place by the top-p)
            api.a3_active_rows(layout, b.sel_idx, b.sel_start, b.n_act, b.act_idx, stream=stream)
    if overlap_plan:
        main = stream if stream is not None else torch.cuda.current_stream()
        b.ev_rows.record(main)
        b.side.wait_event(b.ev_rows)
        api.a3_attention_plan(layout, b.act_idx, b.n_act, b.ws, stream=b.side)
        b.ev_plan.record(b.side)
    if fused_scatter:
        api.a3_selected_qkv_proj_scatter(layout, x_cur, rows, n_rows, wq, wk, wv, q_out=b.q_act, k_fused=b.k_fused,
                                         v_fused=v_cache, stream=stream)
    else:
        api.a3_selected_qkv_proj(layout, x_cur, rows, n_rows, wq, wk, wv, q_out=b.q_act, k_out=b.k_act,
                                 v_out=b.v_act, stream=stream)
        api.a3_kv_scatter(layout, b.k_act, b.v_act, b.act_idx, b.n_act, b.k_fused, v_cache, stream=stream)
    if overlap_plan:
        main.wait_event(b.ev_plan)
    if overlap_plan or fused_plan:
        api.a3_fused_attention_planned(layout, b.q_act, b.act_idx, b.n_act, b.k_fused, v_cache, b.out, b.ws,
                                       stream=stream)
    else:
        api.a3_fused_attention(layout, b.q_act, b.act_idx, b.n_act, b.k_fused, v_cache, b.out, b.ws, stream=stream)
