"""Thin ctypes binding of liba3.so: same entry-point names as include/a3.h, argument
marshalling only.  torch is used for device memory and for the current HIP stream; every
step of the path runs in the library's kernels.  There is no fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liba3.so")

A3_OK, A3_ERR_INVALID_ARG, A3_ERR_UNSUPPORTED, A3_ERR_WORKSPACE, A3_ERR_HIP, A3_ERR_IO = 0, -1, -2, -3, -4, -5
A3_F32, A3_BF16 = 0, 1
A3_ROPE_INTERLEAVED, A3_ROPE_HALF = 0, 1
A3_POOL_MAX, A3_POOL_AVG = 0, 1

EXPORTS = ["a3_workspace_bytes", "a3_layout_prepare", "a3_rope_realign", "a3_question_scores", "a3_question_scores_noalloc", "a3_realign_scores", "a3_topk_select", "a3_topk_select_plan",
           "a3_selected_qkv_proj", "a3_selected_qkv_proj_scatter", "a3_kv_scatter", "a3_fused_attention", "a3_attention_plan", "a3_fused_attention_planned", "a3_fused_attention_planned_events", "a3_active_rows",
           "a3_block_tail_ws_bytes", "a3_block_tail", "a3_rms_norm", "a3_question_scores_causal", "a3_window_votes",
           "a3_evict_ws_bytes", "a3_evict_select", "a3_evict_compact", "a3_value_deviation_scores",
           "a3_select_chunk_edges", "a3_chunk_cache_load", "a3_rope_realign_q8", "a3_q8_row_bytes", "a3_quantize_q8",
           "a3_chunk_cache_load_q8", "a3_chunk_file_read", "a3_set_tuning", "a3_recompute_count", "a3_chunk_edge_sel_start", "a3_strerror", "a3_last_error", "a3_version"]


class A3Error(RuntimeError):
    def __init__(self, status: int, where: str, text: str):
        super().__init__(f"{where}: status {status}: {text}")
        self.status = status


class a3_layout(C.Structure):
    _fields_ = [
        ("dtype", C.c_int), ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int),
        ("hidden", C.c_int), ("rope_layout", C.c_int), ("rope_base", C.c_double), ("sm_scale", C.c_float),
        ("n_req", C.c_int), ("n_chunks", C.c_int), ("total_tokens", C.c_int), ("max_ctx_len", C.c_int),
        ("max_q_len", C.c_int),
        ("seg_start", C.c_void_p), ("ctx_len", C.c_void_p), ("q_len", C.c_void_p),
        ("chunk_start", C.c_void_p), ("chunk_len", C.c_void_p), ("chunk_delta", C.c_void_p),
        ("tok_pos", C.c_void_p), ("tok_req", C.c_void_p), ("tok_chunk", C.c_void_p), ("q_start", C.c_void_p),
        ("rope_chunk_cs", C.c_void_p), ("rope_pos_cs", C.c_void_p),
    ]


class a3_block_weights(C.Structure):
    _fields_ = [("wo", C.c_void_p), ("g_post", C.c_void_p), ("w_gate", C.c_void_p), ("w_up", C.c_void_p),
                ("w_down", C.c_void_p), ("g_next", C.c_void_p), ("ffn", C.c_int), ("eps", C.c_float)]


_lib = None


def lib() -> C.CDLL:
    """Loads liba3.so (built beforehand by ``python -m paper_2511_17560_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_17560_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    P, I, V = C.POINTER(a3_layout), C.c_int, C.c_void_p
    L.a3_workspace_bytes.restype = C.c_size_t
    L.a3_workspace_bytes.argtypes = [P, I]
    L.a3_layout_prepare.argtypes = [P, V]
    L.a3_rope_realign.argtypes = [P, V, V, V]
    L.a3_question_scores.argtypes = [P, V, V, V, V, C.c_size_t, V]
    L.a3_realign_scores.argtypes = [P, V, V, V, V, V, C.c_size_t, V]
    L.a3_question_scores_noalloc.argtypes = [P, V, V, V, V]
    L.a3_question_scores_noalloc.restype = I
    L.a3_topk_select.argtypes = [P, V, V, I, V, V, C.c_size_t, V]
    L.a3_selected_qkv_proj.argtypes = [P, V, V, I, V, V, V, V, V, V, V, V, V, V]
    L.a3_selected_qkv_proj_scatter.argtypes = [P, V, V, I, V, V, V, V, V, V, V, V, V, V]
    L.a3_kv_scatter.argtypes = [P, V, V, V, I, V, V, V]
    L.a3_fused_attention.argtypes = [P, V, V, I, V, V, V, V, C.c_size_t, V]
    L.a3_active_rows.argtypes = [P, V, V, I, V, V]
    L.a3_attention_plan.argtypes = [P, V, I, V, C.c_size_t, V]
    L.a3_fused_attention_planned.argtypes = [P, V, V, I, V, V, V, V, C.c_size_t, V]
    L.a3_fused_attention_planned_events.argtypes = [P, V, V, I, V, V, V, V, C.c_size_t, V, V, V]
    L.a3_fused_attention_planned_events.restype = I
    L.a3_attention_plan.restype = I
    L.a3_fused_attention_planned.restype = I
    L.a3_block_tail_ws_bytes.restype = C.c_size_t
    L.a3_block_tail_ws_bytes.argtypes = [P, I, I]
    L.a3_block_tail.argtypes = [P, V, V, I, C.POINTER(a3_block_weights), V, V, V, C.c_size_t, V]
    L.a3_rms_norm.argtypes = [P, V, V, I, V, C.c_float, V, V]
    L.a3_block_tail.restype = I
    L.a3_question_scores_causal.argtypes = [P, V, V, V, V, C.c_size_t, V]
    L.a3_window_votes.argtypes = [P, V, V, V, V, C.c_size_t, V]
    L.a3_evict_ws_bytes.restype = C.c_size_t
    L.a3_evict_ws_bytes.argtypes = [P]
    L.a3_evict_select.argtypes = [P, V, V, V, I, I, I, V, V, C.c_size_t, V]
    L.a3_evict_compact.argtypes = [P, V, V, V, I, V, V, V]
    L.a3_value_deviation_scores.argtypes = [P, V, V, V, V]
    L.a3_select_chunk_edges.argtypes = [P, I, I, V, I, V, V]
    L.a3_value_deviation_scores.restype = I
    L.a3_chunk_cache_load.argtypes = [P, C.POINTER(C.c_int), C.POINTER(C.c_int), I, C.POINTER(C.c_void_p),
                                      C.POINTER(C.c_void_p), V, V, V]
    L.a3_chunk_cache_load.restype = I
    L.a3_chunk_file_read.argtypes = [I, C.POINTER(C.c_int), C.POINTER(C.c_longlong), C.POINTER(C.c_size_t),
                                     C.POINTER(C.c_void_p), I]
    L.a3_chunk_file_read.restype = I
    L.a3_q8_row_bytes.argtypes = [P]
    L.a3_q8_row_bytes.restype = C.c_size_t
    L.a3_quantize_q8.argtypes = [P, V, V, V, V]
    L.a3_rope_realign_q8.argtypes = [P, V, V, V, V]
    L.a3_chunk_cache_load_q8.argtypes = [P, C.POINTER(C.c_int), C.POINTER(C.c_int), I, C.POINTER(C.c_void_p), V, V]
    for name in ("a3_quantize_q8", "a3_rope_realign_q8", "a3_chunk_cache_load_q8"):
        getattr(L, name).restype = I
    L.a3_select_chunk_edges.restype = I
    for name in ("a3_question_scores_causal", "a3_window_votes", "a3_evict_select", "a3_evict_compact"):
        getattr(L, name).restype = I
    L.a3_rms_norm.restype = I
    for name in ("a3_realign_scores", "a3_selected_qkv_proj_scatter", "a3_active_rows", "a3_layout_prepare", "a3_rope_realign", "a3_question_scores", "a3_topk_select",
                 "a3_selected_qkv_proj", "a3_selected_qkv_proj_scatter", "a3_kv_scatter", "a3_fused_attention"):
        getattr(L, name).restype = I
    L.a3_topk_select_plan.argtypes = [P, V, V, I, V, I, V, V, C.c_size_t, V]
    L.a3_topk_select_plan.restype = I
    L.a3_recompute_count.argtypes = [I, I, I]
    L.a3_recompute_count.restype = I
    L.a3_chunk_edge_sel_start.argtypes = [I, C.POINTER(C.c_int), C.POINTER(C.c_int), I, C.POINTER(C.c_int),
                                          C.POINTER(C.c_int), I, I, C.POINTER(C.c_int)]
    L.a3_chunk_edge_sel_start.restype = I
    L.a3_set_tuning.argtypes = [C.c_char_p, I]
    L.a3_set_tuning.restype = I
    L.a3_strerror.restype = C.c_char_p
    L.a3_strerror.argtypes = [I]
    L.a3_last_error.restype = C.c_char_p
    L.a3_version.restype = I
    _lib = L
    return L


def _check(status: int, where: str):
    if status != A3_OK:
        L = lib()
        raise A3Error(status, where, f"{L.a3_strerror(status).decode()}: {L.a3_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "tensors must be contiguous"
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def torch_dtype(dtype: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


class Layout:
    """Owns the device index arrays and derived tables of one batch and the a3_layout struct
    that points at them."""

    def __init__(self, *, dtype: str, n_q_heads: int, n_kv_heads: int, head_dim: int, hidden: int,
                 rope_base: float, rope_layout: int, seg_start, ctx_len, q_len, chunk_start, chunk_len,
                 chunk_delta, sm_scale: float = 0.0, device="cuda", prepare: bool = True, stream=None):
        dev = torch.device(device)
        i32 = lambda a: torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device=dev)
        self.dtype = dtype
        self.device = dev
        self.seg_start, self.ctx_len, self.q_len = i32(seg_start), i32(ctx_len), i32(q_len)
        self.chunk_start, self.chunk_len, self.chunk_delta = i32(chunk_start), i32(chunk_len), i32(chunk_delta)
        n_req, n_chunks = len(ctx_len), len(chunk_start)
        T = int(np.asarray(seg_start)[-1])
        # what the kernels take for granted about the index arrays (they cannot check device memory): every
        # request is [context | question], the chunks tile the context rows exactly, in ascending order
        seg_h, ctx_h, q_h = (np.asarray(a, dtype=np.int64) for a in (seg_start, ctx_len, q_len))
        if not (len(seg_h) == n_req + 1 and np.array_equal(np.diff(seg_h), ctx_h + q_h) and np.all(ctx_h >= 0)
                and np.all(q_h >= 0)):
            raise ValueError("Layout: seg_start, ctx_len and q_len do not describe [context | question] segments")
        cs_h, cl_h = np.asarray(chunk_start, dtype=np.int64), np.asarray(chunk_len, dtype=np.int64)
        covered = np.zeros(max(T, 1), dtype=np.int32)
        for s0, n in zip(cs_h, cl_h):
            covered[s0:s0 + n] += 1
        want = np.zeros(max(T, 1), dtype=np.int32)
        for r in range(n_req):
            want[seg_h[r]:seg_h[r] + ctx_h[r]] = 1
        if n_chunks and not (np.all(np.diff(cs_h) > 0) and np.array_equal(covered, want)):
            raise ValueError("Layout: the chunks do not tile the context rows exactly")
        max_ctx = int(np.max(ctx_len)) if n_req else 0
        max_q = int(np.max(q_len)) if n_req else 0
        self.total_tokens, self.n_req, self.n_chunks = T, n_req, n_chunks
        self.tok_pos = torch.empty(max(T, 1), dtype=torch.int32, device=dev)
        self.tok_req = torch.empty(max(T, 1), dtype=torch.int32, device=dev)
        self.tok_chunk = torch.empty(max(T, 1), dtype=torch.int32, device=dev)
        self.q_start = torch.empty(n_req + 1, dtype=torch.int32, device=dev)
        self.rope_chunk_cs = torch.empty((max(n_chunks, 1), head_dim // 2, 2), dtype=torch.float32, device=dev)
        self.rope_pos_cs = torch.empty((max(max_ctx + max_q, 1), head_dim // 2, 2), dtype=torch.float32, device=dev)
        s = a3_layout()
        s.dtype = {"f32": A3_F32, "bf16": A3_BF16}[dtype]
        s.n_q_heads, s.n_kv_heads, s.head_dim, s.hidden = n_q_heads, n_kv_heads, head_dim, hidden
        s.rope_layout, s.rope_base, s.sm_scale = rope_layout, rope_base, sm_scale
        s.n_req, s.n_chunks, s.total_tokens, s.max_ctx_len, s.max_q_len = n_req, n_chunks, T, max_ctx, max_q
        s.seg_start, s.ctx_len, s.q_len = self.seg_start.data_ptr(), self.ctx_len.data_ptr(), self.q_len.data_ptr()
        if n_chunks:
            s.chunk_start, s.chunk_len = self.chunk_start.data_ptr(), self.chunk_len.data_ptr()
            s.chunk_delta = self.chunk_delta.data_ptr()
        s.tok_pos, s.tok_req, s.tok_chunk = self.tok_pos.data_ptr(), self.tok_req.data_ptr(), self.tok_chunk.data_ptr()
        s.q_start = self.q_start.data_ptr()
        s.rope_chunk_cs, s.rope_pos_cs = self.rope_chunk_cs.data_ptr(), self.rope_pos_cs.data_ptr()
        self.struct = s
        if prepare:
            a3_layout_prepare(self, stream)

    @classmethod
    def from_workload(cls, w, device="cuda", **kw) -> "Layout":
        s = w.shape
        return cls(dtype=s.dtype, n_q_heads=s.n_q_heads, n_kv_heads=s.n_kv_heads, head_dim=s.head_dim,
                   hidden=s.hidden, rope_base=s.rope_base, rope_layout=s.rope_layout, seg_start=w.seg_start,
                   ctx_len=w.ctx_len, q_len=w.q_lens, chunk_start=w.chunk_start, chunk_len=w.chunk_len,
                   chunk_delta=w.chunk_delta, device=device, **kw)

    @property
    def ref(self):
        return C.byref(self.struct)

    def workspace(self, max_active_rows: int) -> torch.Tensor:
        n = a3_workspace_bytes(self, max_active_rows)
        return torch.empty(max(n, 256), dtype=torch.uint8, device=self.device)


# ---- entry points (same names as the C ABI) -----------------------------------------------------

def a3_version() -> int:
    return lib().a3_version()


def a3_set_tuning(name: str, value: int) -> None:
    _check(lib().a3_set_tuning(name.encode(), int(value)), "a3_set_tuning")


def a3_workspace_bytes(layout: Layout, max_active_rows: int) -> int:
    return int(lib().a3_workspace_bytes(layout.ref, int(max_active_rows)))


def a3_layout_prepare(layout: Layout, stream=None) -> None:
    _check(lib().a3_layout_prepare(layout.ref, _stream(stream)), "a3_layout_prepare")


def a3_rope_realign(layout: Layout, k_cat: torch.Tensor, k_fused: torch.Tensor, stream=None) -> None:
    _check(lib().a3_rope_realign(layout.ref, _ptr(k_cat), _ptr(k_fused), _stream(stream)), "a3_rope_realign")


def a3_question_scores(layout: Layout, q_question: torch.Tensor, k_fused: torch.Tensor, scores: torch.Tensor,
                       ws: torch.Tensor, stream=None) -> None:
    _check(lib().a3_question_scores(layout.ref, _ptr(q_question), _ptr(k_fused), _ptr(scores), _ptr(ws),
                                    ws.numel() if ws is not None else 0, _stream(stream)), "a3_question_scores")


def a3_question_scores_noalloc(layout: Layout, q_question: torch.Tensor, k_fused: torch.Tensor, scores: torch.Tensor,
                               stream=None) -> None:
    _check(lib().a3_question_scores_noalloc(layout.ref, _ptr(q_question), _ptr(k_fused), _ptr(scores),
                                            _stream(stream)), "a3_question_scores_noalloc")


def a3_realign_scores(layout: Layout, q_question: torch.Tensor, k_cat: torch.Tensor, k_fused: torch.Tensor,
                      scores: torch.Tensor, ws: torch.Tensor, stream=None) -> None:
    _check(lib().a3_realign_scores(layout.ref, _ptr(q_question), _ptr(k_cat), _ptr(k_fused), _ptr(scores), _ptr(ws),
                                   ws.numel() if ws is not None else 0, _stream(stream)), "a3_realign_scores")


def a3_topk_select(layout: Layout, scores: torch.Tensor, sel_start: torch.Tensor, total_k: int,
                   sel_idx: torch.Tensor, ws: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(lib().a3_topk_select(layout.ref, _ptr(scores), _ptr(sel_start), int(total_k), _ptr(sel_idx), _ptr(ws),
                                ws.numel() if ws is not None else 0, _stream(stream)), "a3_topk_select")


def a3_topk_select_plan(layout: Layout, scores: torch.Tensor, sel_start: torch.Tensor, total_k: int,
                        sel_idx: torch.Tensor, n_act: int, act_idx: torch.Tensor, ws: torch.Tensor, stream=None) -> None:
    _check(lib().a3_topk_select_plan(layout.ref, _ptr(scores), _ptr(sel_start), int(total_k), _ptr(sel_idx), int(n_act),
                                     _ptr(act_idx), _ptr(ws), ws.numel() if ws is not None else 0, _stream(stream)),
           "a3_topk_select_plan")


def a3_selected_qkv_proj(layout: Layout, hidden: torch.Tensor, row_idx: Optional[torch.Tensor], n_rows: int,
                         wq, wk, wv, bq=None, bk=None, bv=None, q_out=None, k_out=None, v_out=None,
                         stream=None) -> None:
    _check(lib().a3_selected_qkv_proj(layout.ref, _ptr(hidden), _ptr(row_idx), int(n_rows), _ptr(wq), _ptr(wk),
                                      _ptr(wv), _ptr(bq), _ptr(bk), _ptr(bv), _ptr(q_out), _ptr(k_out), _ptr(v_out),
                                      _stream(stream)), "a3_selected_qkv_proj")


def a3_selected_qkv_proj_scatter(layout: Layout, hidden: torch.Tensor, row_idx: Optional[torch.Tensor], n_rows: int,
                                 wq, wk, wv, bq=None, bk=None, bv=None, q_out=None, k_fused=None, v_fused=None,
                                 stream=None) -> None:
    _check(lib().a3_selected_qkv_proj_scatter(layout.ref, _ptr(hidden), _ptr(row_idx), int(n_rows), _ptr(wq),
                                              _ptr(wk), _ptr(wv), _ptr(bq), _ptr(bk), _ptr(bv), _ptr(q_out),
                                              _ptr(k_fused), _ptr(v_fused), _stream(stream)),
           "a3_selected_qkv_proj_scatter")


def a3_kv_scatter(layout: Layout, k_new: torch.Tensor, v_new: torch.Tensor, row_idx: torch.Tensor, n_rows: int,
                  k_fused: torch.Tensor, v_fused: torch.Tensor, stream=None) -> None:
    _check(lib().a3_kv_scatter(layout.ref, _ptr(k_new), _ptr(v_new), _ptr(row_idx), int(n_rows), _ptr(k_fused),
                               _ptr(v_fused), _stream(stream)), "a3_kv_scatter")


def a3_fused_attention(layout: Layout, q_act: torch.Tensor, act_idx: torch.Tensor, n_act: int, k_fused: torch.Tensor,
                       v_fused: torch.Tensor, out: torch.Tensor, ws: torch.Tensor, stream=None) -> None:
    _check(lib().a3_fused_attention(layout.ref, _ptr(q_act), _ptr(act_idx), int(n_act), _ptr(k_fused), _ptr(v_fused),
                                    _ptr(out), _ptr(ws), ws.numel() if ws is not None else 0, _stream(stream)),
           "a3_fused_attention")


def a3_active_rows(layout: Layout, sel_idx: Optional[torch.Tensor], sel_start: torch.Tensor, n_act: int,
                   act_idx: torch.Tensor, stream=None) -> None:
    _check(lib().a3_active_rows(layout.ref, _ptr(sel_idx), _ptr(sel_start), int(n_act), _ptr(act_idx),
                                _stream(stream)), "a3_active_rows")


def a3_block_tail_ws_bytes(layout: Layout, ffn: int, n_rows: int) -> int:
    return int(lib().a3_block_tail_ws_bytes(layout.ref, int(ffn), int(n_rows)))


def a3_block_tail(layout: Layout, attn_out: torch.Tensor, act_idx: Optional[torch.Tensor], n_act: int, wo, g_post,
                  w_gate, w_up, w_down, g_next, eps: float, resid: torch.Tensor, hidden_next: torch.Tensor,
                  ws: torch.Tensor, stream=None) -> None:
    w = a3_block_weights(_ptr(wo), _ptr(g_post), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(g_next),
                         int(w_gate.shape[0]), float(eps))
    _check(lib().a3_block_tail(layout.ref, _ptr(attn_out), _ptr(act_idx), int(n_act), C.byref(w), _ptr(resid),
                               _ptr(hidden_next), _ptr(ws), ws.numel() if ws is not None else 0, _stream(stream)),
           "a3_block_tail")


def a3_rms_norm(layout: Layout, x: torch.Tensor, row_idx: Optional[torch.Tensor], n_rows: int, g: torch.Tensor,
                eps: float, out: torch.Tensor, stream=None) -> None:
    _check(lib().a3_rms_norm(layout.ref, _ptr(x), _ptr(row_idx), int(n_rows), _ptr(g), float(eps), _ptr(out),
                             _stream(stream)), "a3_rms_norm")


def a3_question_scores_causal(layout: Layout, q_question: torch.Tensor, k_fused: torch.Tensor, scores: torch.Tensor,
                              ws: torch.Tensor, stream=None) -> None:
    _check(lib().a3_question_scores_causal(layout.ref, _ptr(q_question), _ptr(k_fused), _ptr(scores), _ptr(ws),
                                           ws.numel() if ws is not None else 0, _stream(stream)),
           "a3_question_scores_causal")


def a3_window_votes(layout: Layout, q_question: torch.Tensor, k_fused: torch.Tensor, votes: torch.Tensor,
                    ws: torch.Tensor, stream=None) -> None:
    _check(lib().a3_window_votes(layout.ref, _ptr(q_question), _ptr(k_fused), _ptr(votes), _ptr(ws),
                                 ws.numel() if ws is not None else 0, _stream(stream)), "a3_window_votes")


def a3_evict_ws_bytes(layout: Layout) -> int:
    return int(lib().a3_evict_ws_bytes(layout.ref))


def a3_evict_select(layout: Layout, votes: torch.Tensor, sys_len: torch.Tensor, keep_start: torch.Tensor,
                    total_keep: int, keep_idx: torch.Tensor, pool_width: int = 1, pool_mode: int = A3_POOL_MAX,
                    ws: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(lib().a3_evict_select(layout.ref, _ptr(votes), _ptr(sys_len), _ptr(keep_start), int(total_keep),
                                 int(pool_width), int(pool_mode), _ptr(keep_idx), _ptr(ws),
                                 ws.numel() if ws is not None else 0, _stream(stream)), "a3_evict_select")


def a3_evict_compact(layout: Layout, k_fused: torch.Tensor, v_fused: torch.Tensor, keep_idx: torch.Tensor,
                     total_keep: int, k_out: torch.Tensor, v_out: torch.Tensor, stream=None) -> None:
    _check(lib().a3_evict_compact(layout.ref, _ptr(k_fused), _ptr(v_fused), _ptr(keep_idx), int(total_keep),
                                  _ptr(k_out), _ptr(v_out), _stream(stream)), "a3_evict_compact")


def a3_value_deviation_scores(layout: Layout, v_true: torch.Tensor, v_cat: torch.Tensor, scores: torch.Tensor,
                              stream=None) -> None:
    _check(lib().a3_value_deviation_scores(layout.ref, _ptr(v_true), _ptr(v_cat), _ptr(scores), _stream(stream)),
           "a3_value_deviation_scores")


def a3_recompute_count(n_ctx: int, ratio_num: int, ratio_den: int) -> int:
    k = int(lib().a3_recompute_count(int(n_ctx), int(ratio_num), int(ratio_den)))
    if k < 0:
        raise A3Error(A3_ERR_INVALID_ARG, "a3_recompute_count", lib().a3_last_error().decode())
    return k


def a3_chunk_edge_sel_start(seg_start, ctx_len, chunk_start, chunk_len, n_head: int, n_tail: int) -> np.ndarray:
    """sel_start [R+1] for a3_select_chunk_edges, from host arrays."""
    i32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
    seg, ctx, cs, cl = i32(seg_start), i32(ctx_len), i32(chunk_start), i32(chunk_len)
    out = np.zeros(len(ctx) + 1, dtype=np.int32)
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int))
    _check(lib().a3_chunk_edge_sel_start(len(ctx), p(seg), p(ctx), len(cs), p(cs), p(cl), int(n_head), int(n_tail), p(out)),
           "a3_chunk_edge_sel_start")
    return out


def a3_select_chunk_edges(layout: Layout, n_head: int, n_tail: int, sel_start: torch.Tensor, total_k: int,
                          sel_idx: torch.Tensor, stream=None) -> None:
    _check(lib().a3_select_chunk_edges(layout.ref, int(n_head), int(n_tail), _ptr(sel_start), int(total_k),
                                       _ptr(sel_idx), _stream(stream)), "a3_select_chunk_edges")


def a3_chunk_cache_load(layout: Layout, chunk_start, chunk_len, host_k, host_v, k_cat: torch.Tensor,
                        v_cat: torch.Tensor, stream=None) -> None:
    """host_k / host_v: one CPU tensor per chunk ([chunk_len, Hkv, d], pinned for asynchronous copies); the
    caller keeps them alive until the stream has passed the copies."""
    n = len(chunk_start)
    starts = (C.c_int * n)(*[int(x) for x in chunk_start])
    lens = (C.c_int * n)(*[int(x) for x in chunk_len])
    for t in list(host_k) + list(host_v):
        assert t is None or (t.device.type == "cpu" and t.is_contiguous())
    pk = (C.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in host_k])
    pv = (C.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in host_v])
    _check(lib().a3_chunk_cache_load(layout.ref, starts, lens, n, pk, pv, _ptr(k_cat), _ptr(v_cat), _stream(stream)),
           "a3_chunk_cache_load")


def a3_attention_plan(layout: Layout, act_idx: torch.Tensor, n_act: int, ws: torch.Tensor, stream=None) -> None:
    _check(lib().a3_attention_plan(layout.ref, _ptr(act_idx), int(n_act), _ptr(ws), ws.numel() if ws is not None else 0,
                                   _stream(stream)), "a3_attention_plan")


def a3_fused_attention_planned(layout: Layout, q_act: torch.Tensor, act_idx: torch.Tensor, n_act: int,
                               k_fused: torch.Tensor, v_fused: torch.Tensor, out: torch.Tensor, ws: torch.Tensor,
                               stream=None) -> None:
    _check(lib().a3_fused_attention_planned(layout.ref, _ptr(q_act), _ptr(act_idx), int(n_act), _ptr(k_fused),
                                            _ptr(v_fused), _ptr(out), _ptr(ws), ws.numel() if ws is not None else 0,
                                            _stream(stream)), "a3_fused_attention_planned")


def a3_fused_attention_planned_events(layout: Layout, q_act: torch.Tensor, act_idx: torch.Tensor, n_act: int,
                                      k_fused: torch.Tensor, v_fused: torch.Tensor, out: torch.Tensor, ws: torch.Tensor,
                                      ev_main_begin: Optional[int], ev_main_end: Optional[int], stream=None) -> None:
    """ev_main_begin / ev_main_end: raw hipEvent_t handles (integers) or None."""
    _check(lib().a3_fused_attention_planned_events(layout.ref, _ptr(q_act), _ptr(act_idx), int(n_act), _ptr(k_fused),
                                                   _ptr(v_fused), _ptr(out), _ptr(ws),
                                                   ws.numel() if ws is not None else 0, _stream(stream), ev_main_begin,
                                                   ev_main_end), "a3_fused_attention_planned_events")


def a3_q8_row_bytes(layout: Layout) -> int:
    return int(lib().a3_q8_row_bytes(layout.ref))


def a3_quantize_q8(layout: Layout, k: torch.Tensor, v: torch.Tensor, cache_q8: torch.Tensor, stream=None) -> None:
    _check(lib().a3_quantize_q8(layout.ref, _ptr(k), _ptr(v), _ptr(cache_q8), _stream(stream)), "a3_quantize_q8")


def a3_rope_realign_q8(layout: Layout, cache_q8: torch.Tensor, k_fused: Optional[torch.Tensor],
                       v_fused: Optional[torch.Tensor], stream=None) -> None:
    _check(lib().a3_rope_realign_q8(layout.ref, _ptr(cache_q8), _ptr(k_fused), _ptr(v_fused), _stream(stream)),
           "a3_rope_realign_q8")


def a3_chunk_cache_load_q8(layout: Layout, chunk_start, chunk_len, host_q8, cache_q8: torch.Tensor, stream=None) -> None:
    n = len(chunk_start)
    starts = (C.c_int * n)(*[int(x) for x in chunk_start])
    lens = (C.c_int * n)(*[int(x) for x in chunk_len])
    for t in host_q8:
        assert t is None or (t.device.type == "cpu" and t.is_contiguous())
    blocks = (C.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in host_q8])
    _check(lib().a3_chunk_cache_load_q8(layout.ref, starts, lens, n, blocks, _ptr(cache_q8), _stream(stream)),
           "a3_chunk_cache_load_q8")


def a3_chunk_file_read(fds, file_offset, n_bytes, host_dst, n_threads: int = 4) -> None:
    """Blocking: block c = n_bytes[c] bytes at file_offset[c] of descriptor fds[c] into the CPU tensor host_dst[c]
    (the GIL is released meanwhile, so a Python thread can run it beside the launches)."""
    n = len(fds)
    for t, b in zip(host_dst, n_bytes):
        assert t is None or (t.device.type == "cpu" and t.is_contiguous() and t.numel() * t.element_size() >= b)
    _check(lib().a3_chunk_file_read(n, (C.c_int * n)(*[int(f) for f in fds]),
                                    (C.c_longlong * n)(*[int(o) for o in file_offset]),
                                    (C.c_size_t * n)(*[int(b) for b in n_bytes]),
                                    (C.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in host_dst]),
                                    int(n_threads)), "a3_chunk_file_read")
