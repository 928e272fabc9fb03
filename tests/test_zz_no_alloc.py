"""a3_question_scores_noalloc (the entry point for callers that cannot allocate): called through the C ABI
twice in a row, the second time on a smaller batch, each time against a3_question_scores on the same inputs
(bit for bit: same kernels, only the scratch memory differs) and against the CPU oracle (1e-4 of the largest
score per request, the bar of the scoring step).  The scratch array keeps the first call's contents, so the
second call also shows that nothing stale is read.  A batch beyond the array's size is refused on the host."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import workload as wl
import a3_synth as synth
from paper_2511_17560_amd import api
from gpu_util import max_abs_rel, to_dev

SHAPE = synth.ModelShape("noalloc-bf16", "bf16", 256, 8, 2, 128, 500000.0)


def _scores_both_ways(w):
    b = wl.build(w)
    res = wl.run_oracle(b)
    lay = api.Layout.from_workload(w)
    dt = w.shape.dtype
    qq = to_dev(res["q_question"], dt)
    k_re = to_dev(res["k_realigned"], dt)
    with_ws = torch.zeros(w.total_tokens, dtype=torch.float32, device="cuda")
    api.a3_question_scores(lay, qq, k_re, with_ws, lay.workspace(w.total_k + w.total_q))
    no_alloc = torch.full((w.total_tokens,), 7.0, dtype=torch.float32, device="cuda")
    # straight through the C ABI: raw pointers, no workspace argument
    st = api.lib().a3_question_scores_noalloc(lay.ref, qq.data_ptr(), k_re.data_ptr(), no_alloc.data_ptr(),
                                              torch.cuda.current_stream().cuda_stream)
    assert st == api.A3_OK, api.lib().a3_last_error()
    torch.cuda.synchronize()
    return w, res, with_ws, no_alloc


@pytest.mark.gpu
def test_noalloc_scores_twice_second_call_smaller():
    big = synth.custom(SHAPE, [[700, 300, 513], [257, 64, 90]], [33, 12], ratio=(15, 100), n_planted=2, seed=71)
    small = synth.custom(SHAPE, [[100, 37, 65]], [19], ratio=(15, 100), seed=72)
    for w in (big, small):
        w, res, with_ws, no_alloc = _scores_both_ways(w)
        assert torch.equal(with_ws, no_alloc)
        got = no_alloc.cpu().numpy().astype(np.float64)
        for r in range(w.n_req):
            rows = w.ctx_rows(r)
            assert max_abs_rel(got[rows], res["scores"][rows]) <= 1e-4
            assert abs(got[rows].sum() - w.shape.n_q_heads * w.q_lens[r]) <= 1e-3 * w.shape.n_q_heads * w.q_lens[r]
        assert np.all(np.isneginf(got[w.question_rows()]))


@pytest.mark.gpu
def test_noalloc_scores_fp32_path():
    w = synth.custom(synth.TINY, [[128, 70, 130]], [9], ratio=(15, 100), seed=73)
    w, res, with_ws, no_alloc = _scores_both_ways(w)
    assert torch.equal(with_ws, no_alloc)
    got = no_alloc.cpu().numpy().astype(np.float64)
    rows = w.ctx_rows(0)
    assert max_abs_rel(got[rows], res["scores"][rows]) <= 1e-4


def test_noalloc_refuses_a_batch_beyond_the_scratch_array():
    """Host-side check only (nothing is launched, no GPU needed): 64 requests of 32K context and 128 question tokens."""
    L = api.lib()
    s = api.a3_layout()
    s.dtype, s.n_q_heads, s.n_kv_heads, s.head_dim, s.hidden = api.A3_BF16, 32, 8, 128, 4096
    s.rope_layout, s.rope_base, s.sm_scale = 0, 5e5, 0.0
    s.n_req, s.n_chunks, s.total_tokens, s.max_ctx_len, s.max_q_len = 64, 64, 64 * 32896, 32768, 128
    for f in ("seg_start", "ctx_len", "q_len", "chunk_start", "chunk_len", "chunk_delta", "tok_pos", "tok_req",
              "tok_chunk", "q_start", "rope_chunk_cs", "rope_pos_cs"):
        setattr(s, f, 0x1000)     # never dereferenced on the host
    assert L.a3_question_scores_noalloc(C.byref(s), 0x1000, 0x1000, 0x1000, None) == api.A3_ERR_WORKSPACE
    assert b"scratch" in L.a3_last_error()
    assert L.a3_question_scores_noalloc(C.byref(s), None, 0x1000, 0x1000, None) == api.A3_ERR_INVALID_ARG
