"""Pins of the 8-bit chunk-cache oracle: closed forms, the error bound of the format, library rounding.  No GPU."""
import numpy as np
import torch

from oracle import a3_oracle as ora
from oracle import q8_oracle as q8


def test_quantize_closed_forms():
    x = np.zeros((3, 2, 4))
    x[0, 0] = [127.0, -63.5, 1.0, 0.0]          # scale 1: 63.5 rounds to the even 64
    x[0, 1] = [0.5, 1.5, 2.5, -254.0]           # scale 2: 0.25 -> 0, 0.75 -> 1, 1.25 -> 1, -127
    x[1, 0] = [1e-3, -1e-3, 5e-4, 0.0]
    q, s = q8.quantize_q8(x)
    assert s[0, 0] == 1.0 and q[0, 0].tolist() == [127, -64, 1, 0]
    assert s[0, 1] == 2.0 and q[0, 1].tolist() == [0, 1, 1, -127]
    assert q[1, 0, :2].tolist() == [127, -127] and abs(s[1, 0] - 1e-3 / 127) < 1e-10
    assert np.all(s[2] == 0) and np.all(q[2] == 0) and np.all(q8.dequantize_q8(q, s)[2] == 0)   # rows of zeros
    assert q.dtype == np.int8 and s.dtype == np.float32


def test_error_bound_and_idempotence():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((200, 4, 64)) * rng.uniform(0.01, 30, size=(200, 4, 1))
    q, s = q8.quantize_q8(x)
    xh = q8.dequantize_q8(q, s)
    # half a step, plus what rounding the scale to float32 moves the grid (|q| <= 127 steps of 2^-24 relative)
    bound = 0.5 * s[..., None].astype(np.float64) * (1 + 1e-6) + 127 * np.abs(s[..., None]) * 2.0 ** -23
    assert np.all(np.abs(xh - x) <= bound)
    assert np.abs(q).max() == 127 and np.all(np.abs(q).max(axis=-1) == 127)          # every row uses the full range
    q2, s2 = q8.quantize_q8(xh)                                                       # codes of a dequantised row
    assert np.array_equal(q2, q) and np.allclose(s2, s, rtol=1e-6)
    # against torch's rounding (round half to even) and clamp
    tq = torch.clamp(torch.round(torch.from_numpy(x) / torch.from_numpy(s.astype(np.float64))[..., None]), -127, 127)
    assert np.array_equal(tq.numpy().astype(np.int8), q)
    # sign symmetry and scale equivariance by powers of two
    qn, sn = q8.quantize_q8(-x)
    assert np.array_equal(qn, -q) and np.array_equal(sn, s)
    q4, s4 = q8.quantize_q8(4.0 * x)
    assert np.array_equal(q4, q) and np.array_equal(s4, 4.0 * s)


def test_dequantised_caches_feed_the_unchanged_path():
    rng = np.random.default_rng(2)
    T, H, d = 40, 2, 16
    k = rng.standard_normal((T, H, d))
    q, s = q8.quantize_q8(k)
    cs, cl, cd = np.array([0, 10, 25]), np.array([10, 15, 12]), np.array([0, 10, 25])
    got = q8.rope_realign_q8(q, s, cs, cl, cd, 1e4, ora.ROPE_HALF, "bf16")
    want = ora.rope_realign(q8.dequantize_q8(q, s), cs, cl, cd, 1e4, ora.ROPE_HALF, "bf16")
    assert np.array_equal(got[10:37], want[10:37])                                   # the turned rows
    assert np.array_equal(got[:10], ora.round_bf16(q8.dequantize_q8(q, s)[:10]).astype(np.float64))   # offset 0: no turn
    assert np.array_equal(got[37:], ora.round_bf16(q8.dequantize_q8(q, s)[37:]).astype(np.float64))   # question rows
    v = q8.dequant_values(q, s, "bf16")
    assert np.array_equal(v, ora.round_bf16(q.astype(np.float64) * s.astype(np.float64)[..., None]).astype(np.float64))
    # the rotation keeps norms, so the realigned keys are as far from the true ones as the codes were
    exact = ora.rope_realign(k, cs, cl, cd, 1e4, ora.ROPE_HALF, "exact")
    err_in = np.linalg.norm(q8.dequantize_q8(q, s) - k, axis=-1)
    err_out = np.linalg.norm(ora.rope_realign(q8.dequantize_q8(q, s), cs, cl, cd, 1e4, ora.ROPE_HALF, "exact") - exact, axis=-1)
    assert np.allclose(err_in, err_out, atol=1e-12)
