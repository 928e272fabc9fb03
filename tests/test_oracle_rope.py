"""Pins for the oracle's RoPE and position recovery (Eq. 2, rotation matrix of section
"Position Recovery").  None of these re-derive the oracle's formula: they are closed-form
outcomes, invariants of rotations, and special cases."""
import math
import os

import numpy as np
import pytest

from oracle import a3_oracle as ora
from oracle import workload as wl
import a3_synth as synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_theta_closed_form_values():
    # theta_i = base^(-2i/d): d=8, base=10^4 gives exact decades
    np.testing.assert_allclose(ora.rope_theta(8, 1e4), [1.0, 0.1, 0.01, 0.001], rtol=1e-15)
    np.testing.assert_allclose(ora.rope_theta(4, 1e4), [1.0, 0.01], rtol=1e-15)
    th = ora.rope_theta(128, 5e5)
    assert th[0] == 1.0 and th.shape == (64,)
    # geometric progression with ratio base^(-2/d)
    np.testing.assert_allclose(th[1:] / th[:-1], 5e5 ** (-2 / 128), rtol=1e-13)


def test_quarter_and_half_turn_exact_outcomes():
    # base chosen so that theta_1 = pi/2 for d=4: position 1 turns pair 1 by 90 degrees,
    # position 2 by 180 degrees.  The rotation matrix maps (a, b) -> (-b, a) and (-a, -b).
    base = (2.0 / math.pi) ** 2
    x = np.array([[[0.0, 0.0, 3.0, 5.0]]])
    y1 = ora.rope_rotate(x, np.array([1]), base, ora.ROPE_INTERLEAVED)
    np.testing.assert_allclose(y1[0, 0, 2:], [-5.0, 3.0], atol=1e-15)
    y2 = ora.rope_rotate(x, np.array([2]), base, ora.ROPE_INTERLEAVED)
    np.testing.assert_allclose(y2[0, 0, 2:], [-3.0, -5.0], atol=1e-15)
    # half layout: pair 1 is coordinates (1, 3)
    xh = np.array([[[0.0, 3.0, 0.0, 5.0]]])
    yh = ora.rope_rotate(xh, np.array([1]), base, ora.ROPE_HALF)
    np.testing.assert_allclose(yh[0, 0], [0.0, -5.0, 0.0, 3.0], atol=1e-15)


def test_golden_unit_vector_rotation():
    """Worked example stored as text: e_0 and e_2 of a d=4 head at position 100, base 10^4.
    Pair 0 turns by 100 rad, pair 1 by 1 rad; the first column of each 2x2 block of the
    rotation matrix is (cos, sin)."""
    rows = [l.split() for l in open(os.path.join(GOLD, "rope_unit_vectors.txt")) if l.strip() and l[0] != "#"]
    for layout_name, src, m, *vals in rows:
        layout = ora.ROPE_INTERLEAVED if layout_name == "interleaved" else ora.ROPE_HALF
        x = np.zeros((1, 1, 4))
        x[0, 0, int(src)] = 1.0
        y = ora.rope_rotate(x, np.array([int(m)]), 1e4, layout)
        np.testing.assert_allclose(y[0, 0], [float(v) for v in vals], atol=1e-14)


@pytest.mark.parametrize("layout", [ora.ROPE_INTERLEAVED, ora.ROPE_HALF])
def test_rotation_invariants(layout):
    rng = np.random.default_rng(1)
    d = 64
    q = rng.standard_normal((5, 3, d))
    k = rng.standard_normal((5, 3, d))
    m = np.array([0, 7, 513, 16000, 32767])
    n = np.array([3, 1000, 12, 15999, 4])
    rq = ora.rope_rotate(q, m, 5e5, layout)
    rk = ora.rope_rotate(k, n, 5e5, layout)
    # rotations preserve the norm of every pair, hence of the vector
    np.testing.assert_allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    # relative-position property: <R_m q, R_n k> depends on m - n only
    lhs = (rq * rk).sum(-1)
    rhs = (ora.rope_rotate(q, m - n, 5e5, layout) * k).sum(-1)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-9, atol=1e-9)
    # position 0 is the identity, bit for bit
    assert np.array_equal(ora.rope_rotate(q, np.zeros(5, int), 5e5, layout), q)
    # R(-m) undoes R(m)
    back = ora.rope_rotate(rq, -m, 5e5, layout)
    np.testing.assert_allclose(back, q, atol=1e-12)


def test_half_layout_is_interleaved_under_the_pair_permutation():
    rng = np.random.default_rng(2)
    d = 16
    x = rng.standard_normal((4, 2, d))
    m = np.array([1, 5, 100, 4097])
    perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])   # interleaved coords -> half coords
    y_int = ora.rope_rotate(x, m, 1e4, ora.ROPE_INTERLEAVED)
    y_half = ora.rope_rotate(x[..., perm], m, 1e4, ora.ROPE_HALF)
    np.testing.assert_allclose(y_half, y_int[..., perm], atol=1e-14)


@pytest.mark.parametrize("layout", [ora.ROPE_INTERLEAVED, ora.ROPE_HALF])
@pytest.mark.parametrize("storage,tol", [("exact", 1e-12), ("f32", 1e-5)])
def test_invariant_realigned_keys_equal_direct_rope_at_global_positions(layout, storage, tol):
    """Invariant 1: rotating chunk-local keys by the chunk offset gives RoPE at the global
    position, because R(a) R(b) = R(a+b)."""
    shape = synth.ModelShape("t", "f32", 64, 4, 2, 32, 5e5, layout)
    w = synth.custom(shape, [[100, 37, 64], [50, 50]], [8, 5])
    rng = np.random.default_rng(3)
    raw = rng.standard_normal((w.total_tokens, 2, 32))            # keys before any rotation
    k_local = ora.store(ora.rope_rotate(raw, w.token_local_positions(), 5e5, layout), storage)
    k_direct = ora.rope_rotate(raw, w.token_positions(), 5e5, layout)
    k_re = ora.rope_realign(k_local, w.chunk_start, w.chunk_len, w.chunk_delta, 5e5, layout, storage)
    for r in range(w.n_req):
        rows = w.ctx_rows(r)
        err = np.abs(k_re[rows] - k_direct[rows]).max() / np.abs(k_direct[rows]).max()
        assert err <= tol
    # first chunk of each request has offset 0: untouched bit for bit
    assert np.array_equal(k_re[:100], k_local[:100])
    # question rows are not context: returned unchanged
    qrows = w.question_rows()
    assert np.array_equal(k_re[qrows], k_local[qrows])


def test_realign_uses_chunk_offset_not_token_position():
    # one-hot keys: every token of a chunk is rotated by the same angle
    shape = synth.ModelShape("t", "f32", 8, 1, 1, 4, (2.0 / math.pi) ** 2)
    w = synth.custom(shape, [[3, 2]], [1])
    k = np.zeros((w.total_tokens, 1, 4))
    k[:, 0, 2] = 1.0
    out = ora.rope_realign(k, w.chunk_start, w.chunk_len, w.chunk_delta, shape.rope_base, 0, "exact")
    # chunk 1 starts at position 3: pair 1 turns by 3 * pi/2  ->  (1,0) -> (0,-1)
    np.testing.assert_allclose(out[3:5, 0, 2:], [[0.0, -1.0]] * 2, atol=1e-14)
    np.testing.assert_allclose(out[0:3, 0, 2:], [[1.0, 0.0]] * 3, atol=0)


def test_bf16_rounding_matches_library():
    import torch
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(100000) * np.exp(rng.uniform(-20, 20, 100000))).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]     # exact ties: round to even
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ora.round_bf16(x), ref)


def test_precompute_cache_then_realign_equals_projection_at_global_position():
    w = synth.config(1)
    b = wl.build(w, plant=False)
    s = w.shape
    k_re = ora.rope_realign(b["k_cat"], w.chunk_start, w.chunk_len, w.chunk_delta, s.rope_base,
                            s.rope_layout, "f32")
    rows = w.ctx_rows(0)
    _, k_true, _ = ora.selected_qkv_proj(b["t"].x_pre, rows, w.token_positions()[rows], b["t"].wq, b["t"].wk,
                                         b["t"].wv, s.n_q_heads, s.n_kv_heads, s.head_dim, s.rope_base,
                                         s.rope_layout, "f32")
    assert np.abs(k_re[rows] - k_true).max() / np.abs(k_true).max() <= 1e-5
