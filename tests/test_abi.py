"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes workspaces, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2511_17560_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "a3.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(a3_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = api.lib()
    names = _declared_symbols()
    assert len(names) >= 11
    for n in names:
        assert hasattr(L, n), n
    assert sorted(api.EXPORTS) == names
    assert L.a3_version() >= 100


def _host_layout(**over):
    s = api.a3_layout()
    s.dtype, s.n_q_heads, s.n_kv_heads, s.head_dim, s.hidden = api.A3_BF16, 32, 8, 128, 4096
    s.rope_layout, s.rope_base, s.sm_scale = 0, 5e5, 0.0
    s.n_req, s.n_chunks, s.total_tokens, s.max_ctx_len, s.max_q_len = 1, 32, 16448, 16384, 64
    fake = 0x1000     # never dereferenced on the host: argument checks only look at NULL-ness
    for f in ("seg_start", "ctx_len", "q_len", "chunk_start", "chunk_len", "chunk_delta", "tok_pos", "tok_req",
              "tok_chunk", "q_start", "rope_chunk_cs", "rope_pos_cs"):
        setattr(s, f, fake)
    for k, v in over.items():
        setattr(s, k, v)
    return s


def test_workspace_bytes_is_host_only_and_monotone():
    L = api.lib()
    s = _host_layout()
    a = L.a3_workspace_bytes(C.byref(s), 1702)
    b = L.a3_workspace_bytes(C.byref(s), 16448)
    assert 0 < a <= b
    assert L.a3_workspace_bytes(C.byref(_host_layout(head_dim=96)), 10) == 0
    assert L.a3_workspace_bytes(None, 10) == 0


@pytest.mark.parametrize("over,status", [
    (dict(dtype=7), api.A3_ERR_INVALID_ARG),
    (dict(n_q_heads=30), api.A3_ERR_INVALID_ARG),          # not a multiple of n_kv_heads
    (dict(head_dim=96), api.A3_ERR_UNSUPPORTED),
    (dict(hidden=100), api.A3_ERR_UNSUPPORTED),
    (dict(rope_base=0.5), api.A3_ERR_INVALID_ARG),
    (dict(seg_start=None), api.A3_ERR_INVALID_ARG),
    (dict(tok_pos=None), api.A3_ERR_INVALID_ARG),
    (dict(total_tokens=10), api.A3_ERR_INVALID_ARG),       # max lengths exceed T
])
def test_bad_layouts_are_rejected_before_launch(over, status):
    L = api.lib()
    s = _host_layout(**over)
    assert L.a3_rope_realign(C.byref(s), 0x1000, 0x1000, None) == status
    assert L.a3_last_error() != b""
    assert L.a3_strerror(status) not in (b"", b"ok")


def test_bad_arguments_are_rejected_before_launch():
    L = api.lib()
    s = _host_layout()
    p = C.byref(s)
    assert L.a3_rope_realign(p, None, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_rope_realign(p, 0x1004, 0x1000, None) == api.A3_ERR_INVALID_ARG       # misaligned
    assert L.a3_question_scores(p, 0x1000, 0x1000, 0x1000, None, 0, None) == api.A3_ERR_WORKSPACE
    assert L.a3_question_scores(p, 0x1000, 0x1000, 0x1000, 0x1000, 16, None) == api.A3_ERR_WORKSPACE
    assert L.a3_topk_select(p, 0x1000, 0x1000, -1, 0x1000, None, 0, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_topk_select(p, 0x1000, 0x1000, 10 ** 6, 0x1000, None, 0, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_topk_select(p, 0x1000, 0x1000, 0, None, None, 0, None) == api.A3_OK     # nothing to do
    assert L.a3_selected_qkv_proj(p, 0x1000, None, -3, *([0x1000] * 3), *([None] * 3), *([0x1000] * 3), None) \
        == api.A3_ERR_INVALID_ARG
    assert L.a3_selected_qkv_proj(p, 0x1000, None, 5, None, None, None, *([None] * 3), 0x1000, None, None, None) \
        == api.A3_ERR_INVALID_ARG                                                          # output without weight
    assert L.a3_selected_qkv_proj(p, 0x1000, None, 0, *([0x1000] * 3), *([None] * 3), *([0x1000] * 3), None) == api.A3_OK
    assert L.a3_kv_scatter(p, 0x1000, 0x1000, None, 4, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_kv_scatter(p, None, None, None, 0, None, None, None) == api.A3_OK
    assert L.a3_fused_attention(p, 0x1000, 0x1000, 10, 0x1000, 0x1000, 0x1000, None, 0, None) == api.A3_ERR_WORKSPACE
    assert L.a3_fused_attention(p, 0x1000, 0x1000, 10 ** 6, 0x1000, 0x1000, 0x1000, None, 0, None) \
        == api.A3_ERR_INVALID_ARG
    assert L.a3_fused_attention(p, None, None, 0, None, None, None, None, 0, None) == api.A3_OK
    assert L.a3_active_rows(p, None, None, 5, None, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_attention_plan(p, None, 10, 0x1000, 1 << 40, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_attention_plan(p, 0x1000, 10, None, 0, None) == api.A3_ERR_WORKSPACE
    assert L.a3_attention_plan(p, 0x1000, 0, None, 0, None) == api.A3_OK
    assert L.a3_fused_attention_planned(p, None, 0x1000, 10, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 40, None) \
        == api.A3_ERR_INVALID_ARG
    assert L.a3_fused_attention_planned(p, 0x1000, 0x1000, 10, 0x1000, 0x1000, 0x1000, None, 0, None) \
        == api.A3_ERR_WORKSPACE
    # the single-launch variants check what their plain counterparts check
    assert L.a3_realign_scores(p, 0x1000, None, 0x1000, 0x1000, 0x1000, 1 << 40, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_realign_scores(p, 0x1000, 0x1008, 0x1000, 0x1000, 0x1000, 1 << 40, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_realign_scores(p, 0x1000, 0x1000, None, 0x1000, 0x1000, 1 << 40, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_realign_scores(p, 0x1000, 0x1000, 0x1000, 0x1000, None, 0, None) == api.A3_ERR_WORKSPACE
    assert L.a3_realign_scores(p, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 16, None) == api.A3_ERR_WORKSPACE
    assert L.a3_selected_qkv_proj_scatter(p, 0x1000, None, -3, *([0x1000] * 3), *([None] * 3), *([0x1000] * 3), None) \
        == api.A3_ERR_INVALID_ARG
    assert L.a3_selected_qkv_proj_scatter(p, 0x1000, None, 5, None, None, None, *([None] * 3), 0x1000, None, None,
                                          None) == api.A3_ERR_INVALID_ARG
    assert L.a3_selected_qkv_proj_scatter(p, 0x1000, None, 0, *([0x1000] * 3), *([None] * 3), *([0x1000] * 3), None) \
        == api.A3_OK
    # layer-stack entry points
    bw = api.a3_block_weights(*([0x1000] * 6), 14336, 1e-5)
    wp = C.byref(bw)
    need = L.a3_block_tail_ws_bytes(p, 14336, 1702)
    assert need >= 1702 * (4096 + 14336) * 2 and L.a3_block_tail_ws_bytes(p, 0, 10) == 0
    assert L.a3_block_tail_ws_bytes(None, 14336, 10) == 0
    assert L.a3_block_tail(p, 0x1000, None, 0, wp, 0x1000, 0x1000, None, 0, None) == api.A3_OK        # nothing to do
    assert L.a3_block_tail(p, 0x1000, None, -1, wp, 0x1000, 0x1000, 0x1000, need, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_block_tail(p, 0x1000, None, 10, None, 0x1000, 0x1000, 0x1000, need, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_block_tail(p, None, None, 10, wp, 0x1000, 0x1000, 0x1000, need, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_block_tail(p, 0x1000, None, 1702, wp, 0x1000, 0x1000, None, 0, None) == api.A3_ERR_WORKSPACE
    assert L.a3_block_tail(p, 0x1000, None, 1702, wp, 0x1000, 0x1000, 0x1000, need - 1, None) == api.A3_ERR_WORKSPACE
    no_gate = api.a3_block_weights(0x1000, 0x1000, None, 0x1000, 0x1000, 0x1000, 14336, 1e-5)
    assert L.a3_block_tail(p, 0x1000, None, 10, C.byref(no_gate), 0x1000, 0x1000, 0x1000, need, None) \
        == api.A3_ERR_INVALID_ARG
    odd_ffn = api.a3_block_weights(*([0x1000] * 6), 1000, 1e-5)
    assert L.a3_block_tail(p, 0x1000, None, 10, C.byref(odd_ffn), 0x1000, 0x1000, 0x1000, need, None) \
        == api.A3_ERR_UNSUPPORTED
    neg_eps = api.a3_block_weights(*([0x1000] * 6), 14336, -1.0)
    assert L.a3_block_tail(p, 0x1000, None, 10, C.byref(neg_eps), 0x1000, 0x1000, 0x1000, need, None) \
        == api.A3_ERR_INVALID_ARG
    assert L.a3_rms_norm(p, 0x1000, None, 0, 0x1000, 1e-5, 0x1000, None) == api.A3_OK
    assert L.a3_rms_norm(p, None, None, 5, 0x1000, 1e-5, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_rms_norm(p, 0x1000, None, 5, 0x1000, -1.0, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_rms_norm(p, 0x1004, None, 5, 0x1000, 1e-5, 0x1000, None) == api.A3_ERR_INVALID_ARG
    # selection-score variant and eviction extension
    assert L.a3_question_scores_causal(p, 0x1000, 0x1000, None, 0x1000, 1 << 40, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_question_scores_causal(p, 0x1000, 0x1000, 0x1000, None, 0, None) == api.A3_ERR_WORKSPACE
    assert L.a3_window_votes(p, 0x1000, 0x1000, None, 0x1000, 1 << 40, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_window_votes(p, 0x1000, 0x1000, 0x1000, 0x1000, 16, None) == api.A3_ERR_WORKSPACE
    assert L.a3_evict_ws_bytes(p) >= 8 * 16448 * 4 and L.a3_evict_ws_bytes(None) == 0
    ev = lambda *a: L.a3_evict_select(p, *a)
    assert ev(0x1000, 0x1000, 0x1000, 0, 1, 0, None, None, 0, None) == api.A3_OK                      # nothing kept
    assert ev(None, 0x1000, 0x1000, 1024, 1, 0, 0x1000, None, 0, None) == api.A3_ERR_INVALID_ARG
    assert ev(0x1000, 0x1000, 0x1000, -1, 1, 0, 0x1000, None, 0, None) == api.A3_ERR_INVALID_ARG
    assert ev(0x1000, 0x1000, 0x1000, 10 ** 6, 1, 0, 0x1000, None, 0, None) == api.A3_ERR_INVALID_ARG
    assert ev(0x1000, 0x1000, 0x1000, 1024, 4, 0, 0x1000, None, 0, None) == api.A3_ERR_INVALID_ARG     # even width
    assert ev(0x1000, 0x1000, 0x1000, 1024, 65, 0, 0x1000, None, 0, None) == api.A3_ERR_INVALID_ARG
    assert ev(0x1000, 0x1000, 0x1000, 1024, 7, 5, 0x1000, None, 0, None) == api.A3_ERR_INVALID_ARG     # pooling mode
    assert ev(0x1000, 0x1000, 0x1000, 1024, 7, 0, 0x1000, None, 0, None) == api.A3_ERR_WORKSPACE       # pooling needs ws
    assert ev(0x1000, 0x1000, 0x1000, 1024, 1, 0, None, None, 0, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_evict_compact(p, 0x1000, 0x1000, 0x1000, 0, 0x1000, 0x1000, None) == api.A3_OK
    assert L.a3_evict_compact(p, 0x1000, None, 0x1000, 8, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_evict_compact(p, 0x1000, 0x1008, 0x1000, 8, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    # alternative producers of the recompute list
    assert L.a3_value_deviation_scores(p, None, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_value_deviation_scores(p, 0x1000, 0x1004, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_select_chunk_edges(p, -1, 20, 0x1000, 100, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_select_chunk_edges(p, 20, 20, 0x1000, 10 ** 6, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_select_chunk_edges(p, 20, 20, None, 100, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_select_chunk_edges(p, 20, 20, 0x1000, 0, None, None) == api.A3_OK
    # chunk-cache staging: every argument is checked before a copy is enqueued
    starts, lens = (C.c_int * 2)(0, 512), (C.c_int * 2)(512, 512)
    blocks = (C.c_void_p * 2)(0x1000, 0x1000)
    load = lambda *a: L.a3_chunk_cache_load(p, *a)
    assert load(starts, lens, 0, blocks, blocks, 0x1000, 0x1000, None) == api.A3_OK
    assert load(starts, lens, -1, blocks, blocks, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert load(starts, lens, 2, blocks, blocks, None, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert load(None, lens, 2, blocks, blocks, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    past = (C.c_int * 2)(0, 16448 - 100)
    assert load(past, lens, 2, blocks, blocks, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG       # runs past the last row
    holes = (C.c_void_p * 2)(0x1000, None)
    assert load(starts, lens, 2, holes, blocks, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    # 8-bit caches
    assert L.a3_q8_row_bytes(p) == 8 * (2 * 128 + 8) and L.a3_q8_row_bytes(None) == 0
    assert L.a3_rope_realign_q8(p, None, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_rope_realign_q8(p, 0x1000, None, None, None) == api.A3_ERR_INVALID_ARG              # nothing to write
    assert L.a3_rope_realign_q8(p, 0x1008, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_rope_realign_q8(None, 0x1000, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_quantize_q8(p, 0x1000, 0x1000, None, None) == api.A3_ERR_INVALID_ARG
    assert L.a3_quantize_q8(p, 0x1000, 0x1004, 0x1000, None) == api.A3_ERR_INVALID_ARG
    load8 = lambda *a: L.a3_chunk_cache_load_q8(p, *a)
    assert load8(starts, lens, 0, blocks, 0x1000, None) == api.A3_OK
    assert load8(starts, lens, 2, None, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert load8(starts, lens, 2, blocks, None, None) == api.A3_ERR_INVALID_ARG
    assert load8(past, lens, 2, blocks, 0x1000, None) == api.A3_ERR_INVALID_ARG
    assert load8(starts, lens, 2, holes, 0x1000, None) == api.A3_ERR_INVALID_ARG
    f32_d64 = _host_layout(dtype=api.A3_F32, head_dim=64)
    assert L.a3_rope_realign(C.byref(f32_d64), None, None, None) == api.A3_ERR_INVALID_ARG
    bf16_d64 = _host_layout(head_dim=64)
    assert L.a3_rope_realign(C.byref(bf16_d64), 0x1000, 0x1000, None) == api.A3_ERR_UNSUPPORTED


def test_block_weights_struct_matches_header_order():
    text = open(os.path.join(ROOT, "include", "a3.h")).read()
    body = text[text.index("typedef struct a3_block_weights {"):text.index("} a3_block_weights;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b\*?\s*([a-z_]+)\s*;", body)
    assert fields == [f[0] for f in api.a3_block_weights._fields_]


def test_struct_layout_matches_header_order():
    text = open(os.path.join(ROOT, "include", "a3.h")).read()
    body = text[text.index("typedef struct a3_layout {"):text.index("} a3_layout;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b\*?\s*([a-z_]+)\s*;", body)
    assert fields == [f[0] for f in api.a3_layout._fields_]


def test_set_tuning_knows_its_names():
    L = api.lib()
    for name in (b"attn_wgs", b"attn_item_cost", b"proj_ntw", b"proj_k64", b"gemm_tb", b"gemm_k64"):
        assert L.a3_set_tuning(name, 3) == api.A3_OK
        assert L.a3_set_tuning(name, -1) == api.A3_OK
    assert L.a3_set_tuning(b"no_such_value", 1) == api.A3_ERR_INVALID_ARG
    assert L.a3_set_tuning(None, 1) == api.A3_ERR_INVALID_ARG


def test_recompute_count_and_chunk_edge_counts_on_the_host():
    L = api.lib()
    assert L.a3_recompute_count(512, 15, 100) == 76 and L.a3_recompute_count(16384, 10, 100) == 1638
    assert L.a3_recompute_count(100, 0, 100) == 0 and L.a3_recompute_count(100, 100, 100) == 100
    assert L.a3_recompute_count(-1, 15, 100) == -1 and L.a3_recompute_count(10, 3, 2) == -1
    assert L.a3_recompute_count(10, 1, 0) == -1
    # two requests: chunks of 100, 30 | 50 rows; 20 + 20 edge rows per chunk, a shorter chunk counts once
    got = api.a3_chunk_edge_sel_start([0, 140, 200], [130, 50], [0, 100, 140], [100, 30, 50], 20, 20)
    assert got.tolist() == [0, 70, 110]
