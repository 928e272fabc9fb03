"""GPU parity of the 8-bit chunk-cache path (quantisation, dequantisation, position recovery of Eq. 2 on the dequantised keys,
staging of the 8-bit host blocks) against the CPU oracle.

Tolerances: the codes and scales are the oracle's own (the quantisation is done once, offline, by the oracle);
the kernel multiplies code * scale in float32 and rounds once to the storage type.  Values: the product of an
8-bit integer and a float32 is exact in float64 and its float32 rounding lies within 2^-24, so a bf16 result
differs from the oracle's only where the float32 rounding crosses a bf16 rounding boundary: at most 1 bf16 ulp
on < 0.1 % of the elements; float32 storage is bit-exact against the float32 rounding of the oracle.  Keys: the
bar of the unquantised position recovery (1e-5 of the row maximum in float32, one bf16 rounding on < 2 % of the
elements in bf16).
"""
import numpy as np
import pytest
import torch

from oracle import a3_oracle as ora
from oracle import q8_oracle as q8
from paper_2511_17560_amd import api
from gpu_util import max_abs_rel, to_host
from test_gpu_parity import ctx_of

pytestmark = pytest.mark.gpu

NAMES = ["cfg1", "ragged-bf16", "batched-bf16-half", "g7-bf16", "batched-f32-d128", "cfg2"]


def pack_records(kq, ks, vq, vs):
    """The device format, written out: per packed row [K codes | V codes | K scales | V scales] as bytes."""
    T = kq.shape[0]
    return np.concatenate([kq.reshape(T, -1).view(np.uint8), vq.reshape(T, -1).view(np.uint8),
                           np.ascontiguousarray(ks, dtype="<f4").view(np.uint8).reshape(T, -1),
                           np.ascontiguousarray(vs, dtype="<f4").view(np.uint8).reshape(T, -1)], axis=1)


def _quantised(name):
    c = ctx_of(name)
    w, b = c["w"], c["b"]
    kq, ks = q8.quantize_q8(b["k_cat"])
    vq, vs = q8.quantize_q8(b["v_cat"])
    assert pack_records(kq, ks, vq, vs).shape[1] == api.a3_q8_row_bytes(c["lay"])
    return c, w, kq, ks, vq, vs


@pytest.mark.parametrize("name", NAMES)
def test_dequant_and_realign_q8(name):
    c, w, kq, ks, vq, vs = _quantised(name)
    s, lay = w.shape, c["lay"]
    dt = api.torch_dtype(s.dtype)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    rec = dev(pack_records(kq, ks, vq, vs))
    # values
    v_out = torch.zeros((w.total_tokens, s.n_kv_heads, s.head_dim), dtype=dt, device="cuda")
    k_out = torch.zeros_like(v_out)
    api.a3_rope_realign_q8(lay, rec, k_out, v_out)
    only_v, only_k = torch.zeros_like(v_out), torch.zeros_like(v_out)
    api.a3_rope_realign_q8(lay, rec, None, only_v)
    api.a3_rope_realign_q8(lay, rec, only_k, None)
    torch.cuda.synchronize()
    assert torch.equal(only_v, v_out) and torch.equal(only_k, k_out)
    got, want = to_host(v_out), q8.dequant_values(vq, vs, s.dtype)
    if s.dtype == "f32":
        assert np.array_equal(got, want.astype(np.float32).astype(np.float64))
    else:
        assert max_abs_rel(got, want) <= 2.0 ** -8 and np.mean(got != want) < 1e-3
    # keys: dequantise, turn by the chunk offset, round once
    got = to_host(k_out)
    want = q8.rope_realign_q8(kq, ks, w.chunk_start, w.chunk_len, w.chunk_delta, s.rope_base, s.rope_layout, s.dtype)
    for r in range(w.n_req):
        rows = w.ctx_rows(r)
        err = max_abs_rel(got[rows], want[rows])
        if s.dtype == "f32":
            assert err <= 1e-5, err
        else:
            assert err <= 2.0 ** -7, err
            assert np.mean(got[rows] != want[rows]) < 0.02
    # question rows and chunks at offset 0 are the dequantised keys
    plain = q8.dequant_values(kq, ks, s.dtype)
    rows = list(w.question_rows())
    for ci in np.nonzero(w.chunk_delta == 0)[0]:
        rows += list(range(w.chunk_start[ci], w.chunk_start[ci] + w.chunk_len[ci]))
    if rows:
        assert max_abs_rel(got[rows], plain[rows]) <= (1e-6 if s.dtype == "f32" else 2.0 ** -8)
    # and the quantisation error itself stays within half a code step of the unquantised realigned keys
    exact = c["res"]["k_realigned"]
    ctx = np.concatenate([w.ctx_rows(r) for r in range(w.n_req)])
    step = ks.astype(np.float64)[ctx][..., None]
    # a rotation of a pair moves the error between its two coordinates: bound by the pair's error norm
    assert np.all(np.abs(got[ctx] - exact[ctx]) <= 0.5 * np.sqrt(2.0) * step * 1.001 + np.abs(exact[ctx]) * 2.0 ** -7 + 1e-12)


@pytest.mark.parametrize("name", NAMES)
def test_quantize_q8(name):
    """Codes and scales bit for bit (the integer decision is taken in float64 on both sides), on the caches, on
    rows of zeros and on values that sit exactly on a rounding tie."""
    c, w, kq, ks, vq, vs = _quantised(name)
    s, lay = w.shape, c["lay"]
    x = np.array(c["b"]["v_cat"], dtype=np.float64, copy=True)
    x[3] = 0.0                                              # zero rows: scale 0, codes 0
    x[5, 0, :] = 0.0
    x[5, 0, 0], x[5, 0, 1], x[5, 0, 2], x[5, 0, 3] = 127.0, 62.5, -63.5, 0.5      # scale 1: exact ties, half to even
    wq, wscale = q8.quantize_q8(x)
    assert wq[5, 0, :4].tolist() == [127, 62, -64, 0] and wscale[5, 0] == 1.0 and wscale[3].max() == 0
    y = np.array(c["b"]["k_cat"], dtype=np.float64, copy=True)
    yq, yscale = q8.quantize_q8(y)
    td = lambda a: torch.from_numpy(a.astype(np.float32)).to(api.torch_dtype(s.dtype)).cuda()
    rec = torch.full((w.total_tokens, api.a3_q8_row_bytes(lay)), 99, dtype=torch.uint8, device="cuda")
    api.a3_quantize_q8(lay, td(y), td(x), rec)
    torch.cuda.synchronize()
    assert np.array_equal(rec.cpu().numpy(), pack_records(yq, yscale, wq, wscale))


@pytest.mark.parametrize("name", ["ragged-bf16", "batched-f32-d128"])
def test_chunk_cache_load_q8(name):
    """Host blocks per chunk (pinned) -> packed device rows; rows outside every chunk are left as they were."""
    c, w, kq, ks, vq, vs = _quantised(name)
    s, lay = w.shape, c["lay"]
    rec = pack_records(kq, ks, vq, vs)
    blocks = [torch.from_numpy(np.ascontiguousarray(rec[cs:cs + cl])).pin_memory() if cl > 0 else None
              for cs, cl in zip(w.chunk_start, w.chunk_len)]
    T = w.total_tokens
    d_rec = torch.full((T, rec.shape[1]), 7, dtype=torch.uint8, device="cuda")
    api.a3_chunk_cache_load_q8(lay, w.chunk_start, w.chunk_len, blocks, d_rec)
    torch.cuda.synchronize()
    inside = np.zeros(T, dtype=bool)
    for cs, cl in zip(w.chunk_start, w.chunk_len):
        inside[cs:cs + cl] = True
    got = d_rec.cpu().numpy()
    assert np.array_equal(got[inside], rec[inside]) and np.all(got[~inside] == 7)
    with pytest.raises(api.A3Error):
        api.a3_chunk_cache_load_q8(lay, [T - 3], [10], [blocks[0]], d_rec)          # runs past the last row


def test_attention_on_the_q8_caches_16k():
    """Config 3 at full size: 8-bit caches -> a3_rope_realign_q8 -> the unchanged attention; the
    output of sampled active rows against the oracle's attention over the oracle's dequantised caches."""
    c = ctx_of("cfg3-layer0")
    w, b, res, lay = c["w"], c["b"], c["res"], c["lay"]
    s = w.shape
    dt = api.torch_dtype(s.dtype)
    kq, ks = q8.quantize_q8(b["k_cat"])
    vq, vs = q8.quantize_q8(b["v_cat"])
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    k_f = torch.zeros((w.total_tokens, s.n_kv_heads, s.head_dim), dtype=dt, device="cuda")
    v_f = torch.zeros_like(k_f)
    api.a3_rope_realign_q8(lay, dev(pack_records(kq, ks, vq, vs)), k_f, v_f)
    act = res["act_idx"]
    n_act = len(act)
    q_sel = torch.from_numpy(np.ascontiguousarray(res["q_act"], dtype=np.float32)).to(dt).cuda()
    out = torch.zeros((n_act, s.n_q_heads, s.head_dim), dtype=dt, device="cuda")
    act_d = torch.as_tensor(np.ascontiguousarray(act, dtype=np.int32), device="cuda")
    api.a3_fused_attention(lay, q_sel, act_d, n_act, k_f, v_f, out, lay.workspace(n_act))
    torch.cuda.synchronize()
    k_want = q8.rope_realign_q8(kq, ks, w.chunk_start, w.chunk_len, w.chunk_delta, s.rope_base, s.rope_layout, s.dtype)
    v_want = q8.dequant_values(vq, vs, s.dtype)
    sample = np.unique(np.concatenate([[0, 1, n_act - 1], np.random.default_rng(3).integers(0, n_act, 12)]))
    want = ora.fused_attention(res["q_act"][sample], act[sample], k_want, v_want, w.seg_start, 1.0 / np.sqrt(s.head_dim),
                               s.dtype)
    got = to_host(out)[sample]
    assert max_abs_rel(got, want) <= 2e-2


@pytest.mark.parametrize("case", ["batched-f32", "batched-bf16"])
def test_streamed_stack_on_q8_blocks(case):
    """The schedule over 6 blocks with the caches of layers 2.. streamed as 8-bit host blocks (quantised by the
    oracle) against the same schedule on resident caches that hold the oracle's dequantised values.  The
    selection happens on layer 1's true keys and must be identical; the two differ afterwards only in where the
    keys are rounded (once after the turn, against once before and once after it), so the hidden states of the
    active rows agree to a few storage roundings: 1e-4 in float32, 2e-2 in bf16."""
    import a3_synth as synth
    from paper_2511_17560_amd import loader, stack
    from gpu_util import to_dev
    from test_gpu_stack import STACK_CASES
    shape, chunk_lens, q_lens, ratio, _ = STACK_CASES[case]
    n_layers, dt = 6, shape.dtype
    w = synth.custom(shape, chunk_lens, q_lens, ratio=ratio, seed=80)
    sw = synth.draw_stack_weights(w, n_layers)
    for lw in sw["layers"]:
        for k in ("wq", "wk"):
            lw[k] = synth.round_to_storage(lw[k] * np.float32(5.0), dt)
    lay = api.Layout.from_workload(w)
    rng = np.random.default_rng(4)
    T = w.total_tokens
    ctx_mask = np.zeros(T, dtype=bool)
    for r in range(w.n_req):
        ctx_mask[w.ctx_rows(r)] = True
    host = [None, None]
    res_k, res_v = [None, None], [None, None]
    for _ in range(n_layers - 2):
        per = []
        for res in (res_k, res_v):
            x = rng.standard_normal((T, shape.n_kv_heads, shape.head_dim)) * rng.uniform(0.2, 3.0, size=(T, shape.n_kv_heads, 1))
            codes, scale = q8.quantize_q8(x)
            per += [codes, scale]
            res.append(to_dev(np.where(ctx_mask[:, None, None], q8.dequant_values(codes, scale, dt), 0.0), dt))
        rec = pack_records(*per)
        host.append([torch.from_numpy(np.ascontiguousarray(rec[s0:s0 + n])).pin_memory()
                     for s0, n in zip(w.chunk_start, w.chunk_len)])
    dev_layers = [{k: to_dev(v, dt) for k, v in lw.items()} for lw in sw["layers"]]
    g_final = to_dev(sw["g_final"], dt)
    a = stack.fuse_stack(lay, shape, dev_layers, g_final, to_dev(sw["resid0"], dt), res_k, res_v, w.sel_start,
                         w.question_rows())
    cs = loader.ChunkCacheStream(lay, shape, w.chunk_start, w.chunk_len, host, None, depth=2)
    b = stack.fuse_stack(lay, shape, dev_layers, g_final, to_dev(sw["resid0"], dt), None, None, w.sel_start,
                         w.question_rows(), cache_stream=cs)
    torch.cuda.synchronize()
    assert torch.equal(a["act_idx"], b["act_idx"])
    rows = a["act_idx"].long()
    tol = 1e-4 if dt == "f32" else 2e-2
    assert max_abs_rel(to_host(b["hidden"][rows]), to_host(a["hidden"][rows])) <= tol
    assert max_abs_rel(to_host(b["resid"][rows]), to_host(a["resid"][rows])) <= tol
    assert not torch.equal(a["hidden"][rows], torch.zeros_like(a["hidden"][rows]))
    # the same records read from files (one per chunk, layer after layer) by the loader's worker thread: bit for bit
    # what the host blocks gave, with two and with three buffers in the ring
    import os
    import tempfile
    with tempfile.TemporaryDirectory() as tmp:
        paths = []
        for ci in range(len(w.chunk_start)):
            paths.append(os.path.join(tmp, f"chunk{ci}.q8"))
            with open(paths[-1], "wb") as f:
                for l in range(2, n_layers):
                    f.write(host[l][ci].numpy().tobytes())
        for depth in (2, 3):
            fs = loader.ChunkFileStream(lay, shape, w.chunk_start, w.chunk_len, paths, n_layers, depth=depth, io_threads=3)
            try:
                c = stack.fuse_stack(lay, shape, dev_layers, g_final, to_dev(sw["resid0"], dt), None, None, w.sel_start,
                                     w.question_rows(), cache_stream=fs)
                torch.cuda.synchronize()
            finally:
                fs.close()
            assert torch.equal(c["act_idx"], b["act_idx"])
            assert torch.equal(c["hidden"][rows], b["hidden"][rows]) and torch.equal(c["resid"][rows], b["resid"][rows])


def test_chunk_file_stream_reports_a_short_file(tmp_path):
    """A chunk file that ends inside the requested layer: the read fails in the worker thread and the error
    reaches the caller of acquire(); nothing is copied for that layer and close() still works."""
    from paper_2511_17560_amd import loader
    c = ctx_of("ragged-bf16")
    w, lay = c["w"], c["lay"]
    row = api.a3_q8_row_bytes(lay)
    paths = []
    for ci, n in enumerate(w.chunk_len):
        p = tmp_path / f"c{ci}.q8"
        layers_in_file = 1 if ci == 1 else 2                   # chunk 1 holds one layer only
        p.write_bytes(bytes([ci + 1]) * (int(n) * row * layers_in_file))
        paths.append(str(p))
    fs = loader.ChunkFileStream(lay, w.shape, w.chunk_start, w.chunk_len, paths, n_layers=4, first_layer=2, depth=2)
    try:
        fs.prefetch(2)
        rec = fs.acquire(2)
        torch.cuda.synchronize()
        got = rec.cpu().numpy()
        for ci, (s0, n) in enumerate(zip(w.chunk_start, w.chunk_len)):
            assert np.all(got[s0:s0 + n] == ci + 1)
        fs.release(2)
        fs.prefetch(3)
        with pytest.raises(api.A3Error) as e:
            fs.acquire(3)
        assert e.value.status == api.A3_ERR_IO and "block 1" in str(e.value)
    finally:
        fs.close()
