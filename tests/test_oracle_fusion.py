"""Pins for the oracle's selective recompute, cache update and attention (Eq. 4 / Eq. 5)
and for the chained layer: the invariants the method fixes at recompute ratios 0 and 1,
a library attention routine, and brute force on tiny inputs."""
import math

import numpy as np
import pytest
import torch

from oracle import a3_oracle as ora
from oracle import workload as wl
import a3_synth as synth

SMALL = synth.ModelShape("small", "f32", 48, 4, 2, 8, 1e4)


def _small(ratio, chunks=((20, 13, 17), (9, 30)), q=(4, 6), seed=3, layout=0, **kw):
    shape = synth.ModelShape("small", "f32", 48, 4, 2, 8, 1e4, layout)
    w = synth.custom(shape, chunks, q, ratio=ratio, seed=seed)
    return w, wl.build(w, plant=False, **kw)


def _prefill(w, b, storage=None):
    s, t = w.shape, b["t"]
    return ora.full_prefill_layer(t.x_cur, w.token_positions(), w.seg_start, t.wq, t.wk, t.wv, s.n_q_heads,
                                  s.n_kv_heads, s.head_dim, s.rope_base, s.rope_layout, wl.sm_scale_of(w),
                                  storage or s.dtype)


def test_full_prefill_against_torch_sdpa():
    w, b = _small((15, 100), chunks=((20, 13, 17),), q=(4,))
    out, k, v = _prefill(w, b, "exact")
    s, t = w.shape, b["t"]
    rows = np.arange(w.total_tokens)
    q, _, _ = ora.selected_qkv_proj(t.x_cur, rows, w.token_positions(), t.wq, t.wk, t.wv, s.n_q_heads,
                                    s.n_kv_heads, s.head_dim, s.rope_base, s.rope_layout, "exact")
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]                                     # [1, Hq, T, d]
    tk = torch.from_numpy(k).repeat_interleave(s.group, dim=1).permute(1, 0, 2)[None]
    tv = torch.from_numpy(v).repeat_interleave(s.group, dim=1).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)  # scale = 1/sqrt(d)
    np.testing.assert_allclose(out, ref[0].permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_attention_brute_force_python_loops():
    """Invariant 4: dense masked softmax written out with scalar loops, two requests, a sparse
    set of active rows."""
    rng = np.random.default_rng(5)
    Hq, Hkv, d = 4, 2, 4
    seg = np.array([0, 7, 12])
    T = 12
    k = rng.standard_normal((T, Hkv, d)); v = rng.standard_normal((T, Hkv, d))
    act = np.array([0, 3, 6, 8, 11])
    q = rng.standard_normal((len(act), Hq, d))
    got = ora.fused_attention(q, act, k, v, seg, 0.5, "exact")
    for a, t in enumerate(act):
        base = 0 if t < 7 else 7
        for hq in range(Hq):
            g = hq // 2
            lg = [sum(q[a, hq, c] * k[i, g, c] for c in range(d)) * 0.5 for i in range(base, t + 1)]
            z = sum(math.exp(x) for x in lg)
            want = [sum(math.exp(lg[i - base]) / z * v[i, g, c] for i in range(base, t + 1)) for c in range(d)]
            np.testing.assert_allclose(got[a, hq], want, rtol=1e-12, atol=1e-14)


def test_attention_special_cases():
    rng = np.random.default_rng(6)
    seg = np.array([0, 5, 9])
    k = rng.standard_normal((9, 1, 4)); v = rng.standard_normal((9, 1, 4))
    q = rng.standard_normal((3, 2, 4))
    out = ora.fused_attention(q, [0, 5, 8], k, v, seg, 1.0, "exact")
    # first row of a request sees only itself
    np.testing.assert_allclose(out[0, 0], v[0, 0], rtol=1e-15)
    np.testing.assert_allclose(out[1, 1], v[5, 0], rtol=1e-15)
    # zero query: plain mean of the visible values of its own request
    out0 = ora.fused_attention(np.zeros((1, 2, 4)), [8], k, v, seg, 1.0, "exact")
    np.testing.assert_allclose(out0[0, 0], v[5:9, 0].mean(0), rtol=1e-14)


@pytest.mark.parametrize("layout", [0, 1])
def test_invariant_full_ratio_reproduces_full_prefill(layout):
    """Invariant 2: recomputing every context token is a plain causal prefill."""
    w, b = _small((100, 100), layout=layout)
    res = wl.run_oracle(b)
    out, k, v = _prefill(w, b)
    assert len(res["sel_idx"]) == w.total_ctx
    assert np.array_equal(res["act_idx"], np.arange(w.total_tokens))
    assert np.array_equal(res["k_fused"], k) and np.array_equal(res["v_fused"], v)
    assert np.array_equal(res["out"], out)


def test_invariant_zero_ratio_is_position_recovered_concatenation():
    """Invariant 3: nothing selected -> context rows of the fused cache are the realigned stale
    cache bit for bit, and only the question rows attend."""
    w, b = _small((0, 100))
    s = w.shape
    res = wl.run_oracle(b)
    assert len(res["sel_idx"]) == 0
    k_re = ora.rope_realign(b["k_cat"], w.chunk_start, w.chunk_len, w.chunk_delta, s.rope_base, s.rope_layout, s.dtype)
    for r in range(w.n_req):
        rows = w.ctx_rows(r)
        assert np.array_equal(res["k_fused"][rows], k_re[rows])
        assert np.array_equal(res["v_fused"][rows], b["v_cat"][rows])
    assert np.array_equal(res["act_idx"], w.question_rows())
    # the question rows' output: attention over [realigned stale ctx | fresh question K/V]
    qrows = w.question_rows()
    qq, kq, vq = ora.selected_qkv_proj(b["t"].x_cur, qrows, w.token_positions()[qrows], b["t"].wq, b["t"].wk,
                                       b["t"].wv, s.n_q_heads, s.n_kv_heads, s.head_dim, s.rope_base,
                                       s.rope_layout, s.dtype)
    kk = k_re.copy(); kk[qrows] = kq
    vv = np.array(b["v_cat"]); vv[qrows] = vq
    want = ora.fused_attention(qq, qrows, kk, vv, w.seg_start, wl.sm_scale_of(w), s.dtype)
    assert np.array_equal(res["out"], want)


@pytest.mark.parametrize("ratio", [(15, 100), (50, 100)])
def test_invariant_lossless_cache_needs_no_fix(ratio):
    """If the stale hidden states equal the true ones and a chunk sits at offset 0 its cache is
    lossless; with equal hidden states everywhere the fused result equals full prefill on the
    active rows at any ratio (up to the one extra rounding of the realigned keys)."""
    w, b = _small(ratio, stale_equals_current=True)
    res = wl.run_oracle(b)
    out, k, v = _prefill(w, b)
    assert np.abs(res["k_fused"] - k).max() / np.abs(k).max() < 1e-6
    assert np.array_equal(res["v_fused"], v)
    assert np.abs(res["out"] - out[res["act_idx"]]).max() / np.abs(out).max() < 1e-5


def test_fusion_differs_from_prefill_when_cache_is_stale_and_updates_selected_rows():
    w, b = _small((15, 100))
    res = wl.run_oracle(b)
    out, k, v = _prefill(w, b)
    sel = res["sel_idx"]
    assert len(sel) == w.total_k == (50 * 15) // 100 + (39 * 15) // 100
    # selected and question rows of the cache are the true K/V; the rest stay stale
    upd = np.concatenate([sel, w.question_rows()])
    assert np.array_equal(res["k_fused"][upd], k[upd]) and np.array_equal(res["v_fused"][upd], v[upd])
    stale = np.setdiff1d(np.arange(w.total_tokens), upd)
    assert np.abs(res["v_fused"][stale] - v[stale]).max() > 1e-2
    assert np.abs(res["out"] - out[res["act_idx"]]).max() > 1e-3


def test_requests_are_independent():
    w, b = _small((25, 100))
    res = wl.run_oracle(b)
    # request 1 alone, same tensors
    rows1 = np.arange(w.seg_start[1], w.seg_start[2])
    shape = w.shape
    w1 = synth.custom(shape, [w.chunk_lens[1]], [w.q_lens[1]], ratio=(25, 100))
    t = b["t"]
    t1 = synth.Tensors(t.x_pre[rows1], t.x_cur[rows1], t.wq, t.wk, t.wv)
    b1 = dict(w=w1, t=t1, k_cat=b["k_cat"][rows1], v_cat=b["v_cat"][rows1])
    res1 = wl.run_oracle(b1)
    off = int(w.seg_start[1])
    in1 = res["act_idx"] >= off
    assert np.array_equal(res["act_idx"][in1] - off, res1["act_idx"])
    np.testing.assert_allclose(res["out"][in1], res1["out"], rtol=0, atol=0)
    np.testing.assert_allclose(res["scores"][rows1], res1["scores"], rtol=0, atol=0)


def test_attention_reads_updated_rows_of_other_selected_tokens():
    # scatter-then-attend: changing the fresh K/V of an earlier selected row changes a later row's output
    w, b = _small((30, 100), chunks=((16, 16),), q=(2,))
    res = wl.run_oracle(b)
    first = int(res["sel_idx"][0])
    k2 = res["k_fused"].copy(); k2[first] += 1.0
    out2 = ora.fused_attention(res["q_act"], res["act_idx"], k2, res["v_fused"], w.seg_start, wl.sm_scale_of(w), "f32")
    later = res["act_idx"] > first
    assert np.abs(out2[later] - res["out"][later]).max() > 1e-4


def test_float32_mode_agrees_with_float64_mode():
    w = synth.config(1)
    b = wl.build(w)
    r64 = wl.run_oracle(b)
    r32 = wl.run_oracle(b, dtype=np.float32)
    assert np.array_equal(r64["sel_idx"], r32["sel_idx"])
    assert np.abs(r64["out"] - r32["out"]).max() / np.abs(r64["out"]).max() < 1e-5
    assert np.abs(r64["scores"][:512] - r32["scores"][:512]).max() / r64["scores"][:512].max() < 1e-5
