"""Pins of the stack oracle (H(.) of Eq. 5 and the layer schedule around Eq. 3-5): closed forms, an
independent library's decoder stack on the same weights, brute-force loops, and the invariants of the
schedule.  No GPU."""
import numpy as np
import pytest

from oracle import a3_oracle as ora
from oracle import stack_oracle as st
import a3_synth as synth

F64 = np.float64


# ---------------------------------------------------------------------------------------
# closed forms
# ---------------------------------------------------------------------------------------

def test_rms_norm_closed_forms():
    g = np.array([1.0, 2.0, -3.0, 0.5])
    c, eps = 3.0, 1e-3
    out = st.rms_norm(np.full((2, 4), c), g, eps)
    assert np.allclose(out, g * c / np.sqrt(c * c + eps), rtol=0, atol=1e-15)
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 64))
    y = st.rms_norm(x, np.ones(64), 0.0)
    assert np.allclose(np.mean(y * y, axis=-1), 1.0, atol=1e-13)          # unit mean square
    assert np.allclose(st.rms_norm(7.5 * x, np.ones(64), 0.0), y, atol=1e-13)   # scale invariant at eps = 0
    # a one-hot row of length n has mean square 1/n: the hot entry becomes sqrt(n)
    e = np.zeros((1, 16)); e[0, 3] = -2.0
    assert np.allclose(st.rms_norm(e, np.ones(16), 0.0)[0, 3], -4.0)
    # eps matters: mean square 1, eps 3 -> halved
    assert np.allclose(st.rms_norm(np.ones((1, 8)), np.ones(8), 3.0), 0.5)


def test_silu_closed_forms_and_library():
    from scipy.special import expit
    x = np.linspace(-20, 20, 401)
    assert st.silu(np.array([0.0]))[0] == 0.0
    assert np.allclose(st.silu(x) - st.silu(-x), x, atol=1e-13)            # x (sigma(x) + sigma(-x)) = x
    assert np.allclose(st.silu(x), x * expit(x), atol=1e-14)
    h = 1e-6
    assert abs((st.silu(np.array([h])) - st.silu(np.array([-h])))[0] / (2 * h) - 0.5) < 1e-9   # slope 1/2 at 0
    assert abs(st.silu(np.array([1.0]))[0] - 1.0 / (1.0 + np.exp(-1.0))) < 1e-15


def test_swiglu_mlp_against_loops():
    rng = np.random.default_rng(2)
    n, h, f = 3, 5, 7
    x, wg, wu, wd = rng.standard_normal((n, h)), rng.standard_normal((f, h)), rng.standard_normal((f, h)), \
        rng.standard_normal((h, f))
    got, act = st.swiglu_mlp(x, wg, wu, wd, "exact")
    for i in range(n):
        a = np.zeros(f)
        for j in range(f):
            gate = sum(x[i, k] * wg[j, k] for k in range(h))
            up = sum(x[i, k] * wu[j, k] for k in range(h))
            a[j] = gate / (1.0 + np.exp(-gate)) * up
        assert np.allclose(act[i], a, atol=1e-13)
        for o in range(h):
            assert abs(got[i, o] - sum(a[j] * wd[o, j] for j in range(f))) < 1e-12


def _tail_weights(rng, h, f, hq_d):
    return dict(wo=rng.standard_normal((h, hq_d)) * 0.1, g_post=1 + 0.1 * rng.standard_normal(h),
                w_gate=rng.standard_normal((f, h)) * 0.1, w_up=rng.standard_normal((f, h)) * 0.1,
                w_down=rng.standard_normal((h, f)) * 0.1)


def test_block_tail_special_cases():
    rng = np.random.default_rng(3)
    n, h, f, hq, d = 4, 16, 24, 2, 8
    lw = _tail_weights(rng, h, f, hq * d)
    o, r0, g_next = rng.standard_normal((n, hq, d)), rng.standard_normal((n, h)), 1 + 0.1 * rng.standard_normal(h)
    full = st.block_tail(o, r0, lw, g_next, 1e-5, "exact")
    # no output projection and no down projection: the residual stream passes through
    z = dict(lw, wo=np.zeros_like(lw["wo"]), w_down=np.zeros_like(lw["w_down"]))
    t = st.block_tail(o, r0, z, g_next, 1e-5, "exact")
    assert np.array_equal(t["resid"], r0) and np.allclose(t["hidden_next"], st.rms_norm(r0, g_next, 1e-5))
    # a zero gate closes the MLP (silu(0) = 0): only the attention branch is added
    z = dict(lw, w_gate=np.zeros_like(lw["w_gate"]))
    t = st.block_tail(o, r0, z, g_next, 1e-5, "exact")
    assert np.allclose(t["resid"], r0 + o.reshape(n, -1) @ lw["wo"].T, atol=1e-14)
    assert np.allclose(t["resid"], full["resid_mid"], atol=1e-14)
    # rows are independent
    one = st.block_tail(o[2:3], r0[2:3], lw, g_next, 1e-5, "exact")
    assert np.allclose(one["resid"], full["resid"][2:3], atol=1e-14)
    # the MLP branch is linear in w_down; the attention branch is linear in attn_out
    t2 = st.block_tail(o, r0, dict(lw, w_down=2 * lw["w_down"]), g_next, 1e-5, "exact")
    assert np.allclose(t2["resid"] - full["resid_mid"], 2 * (full["resid"] - full["resid_mid"]), atol=1e-13)
    # storage rounding happens: bf16 results are bf16 numbers
    tb = st.block_tail(o, r0, lw, g_next, 1e-5, "bf16")
    for key in ("resid_mid", "normed", "act", "resid", "hidden_next"):
        assert np.array_equal(ora.round_bf16(tb[key]).astype(F64), tb[key]), key


# ---------------------------------------------------------------------------------------
# an independent library's decoder stack on the same weights
# ---------------------------------------------------------------------------------------

def _hf_stack(kind):
    torch = pytest.importorskip("torch")
    tf = pytest.importorskip("transformers")
    common = dict(vocab_size=32, hidden_size=64, intermediate_size=160, num_hidden_layers=3,
                  num_attention_heads=4, num_key_value_heads=2, rms_norm_eps=1e-5, rope_theta=10000.0,
                  max_position_embeddings=256, attn_implementation="eager")
    torch.manual_seed(11)
    if kind == "llama":
        model = tf.LlamaModel(tf.LlamaConfig(head_dim=16, attention_bias=False, **common))
    else:
        model = tf.Qwen2Model(tf.Qwen2Config(**common))          # q/k/v projections carry a bias
    model = model.double().eval()
    with torch.no_grad():
        for name, p in model.named_parameters():                  # norms start at 1 and biases at 0: move them
            if "layernorm" in name or name == "norm.weight":
                p.add_(0.2 * torch.randn_like(p))
            if name.endswith("proj.bias"):
                p.add_(0.3 * torch.randn_like(p))
    sd = {k: v.detach().numpy().astype(F64) for k, v in model.state_dict().items()}
    layers = []
    for l in range(3):
        a, m = f"layers.{l}.self_attn.", f"layers.{l}.mlp."
        lw = dict(wq=sd[a + "q_proj.weight"], wk=sd[a + "k_proj.weight"], wv=sd[a + "v_proj.weight"],
                  wo=sd[a + "o_proj.weight"], g_in=sd[f"layers.{l}.input_layernorm.weight"],
                  g_post=sd[f"layers.{l}.post_attention_layernorm.weight"], w_gate=sd[m + "gate_proj.weight"],
                  w_up=sd[m + "up_proj.weight"], w_down=sd[m + "down_proj.weight"])
        if kind != "llama":
            lw.update(bq=sd[a + "q_proj.bias"], bk=sd[a + "k_proj.bias"], bv=sd[a + "v_proj.bias"])
        layers.append(lw)
    shape = dict(n_q_heads=4, n_kv_heads=2, head_dim=16, base=10000.0, layout=ora.ROPE_HALF,
                 sm_scale=1.0 / np.sqrt(16.0), eps=1e-5)
    return model, layers, sd["norm.weight"], shape


@pytest.mark.parametrize("kind", ["llama", "qwen2"])
def test_full_prefill_stack_against_library_decoder(kind):
    """The whole chain (input norm, projections with bias, half-layout RoPE, grouped causal attention,
    output projection, residuals, post norm, gated MLP, final norm) against the library's model in
    float64 on the same weights.  The library forms its rotary angles and (cos, sin) in float32 whatever
    the model's type, which shows as ~1e-7 relative differences: the bar is 5e-6, four orders of magnitude
    below what a wrong term, sign or index produces."""
    import torch
    tol = 5e-6
    model, layers, g_final, shape = _hf_stack(kind)
    T = 37
    x = torch.randn(1, T, 64, dtype=torch.float64, generator=torch.Generator().manual_seed(5))
    with torch.no_grad():
        ref = model(inputs_embeds=x, output_hidden_states=True)
    got = st.full_prefill_stack(x[0].numpy(), np.arange(T), np.array([0, T]), layers, g_final, shape, "exact")
    assert np.abs(got["hidden"] - ref.last_hidden_state[0].numpy()).max() < tol
    # the library reports the residual stream in front of every block
    one = st.full_prefill_stack(x[0].numpy(), np.arange(T), np.array([0, T]), layers[:1], g_final, shape, "exact")
    assert np.abs(one["resid"] - ref.hidden_states[1][0].numpy()).max() < tol
    # two packed requests = two separate runs of the library
    T2 = 21
    y = torch.randn(1, T2, 64, dtype=torch.float64, generator=torch.Generator().manual_seed(6))
    with torch.no_grad():
        ref2 = model(inputs_embeds=y)
    packed = st.full_prefill_stack(np.concatenate([x[0].numpy(), y[0].numpy()]),
                                   np.concatenate([np.arange(T), np.arange(T2)]), np.array([0, T, T + T2]),
                                   layers, g_final, shape, "exact")
    assert np.abs(packed["hidden"][:T] - ref.last_hidden_state[0].numpy()).max() < tol
    assert np.abs(packed["hidden"][T:] - ref2.last_hidden_state[0].numpy()).max() < tol


# ---------------------------------------------------------------------------------------
# invariants of the schedule
# ---------------------------------------------------------------------------------------

def _small_stack(chunk_lens, q_lens, ratio, n_layers=4, seed=3):
    shape = synth.ModelShape("pin", "f32", 64, 4, 2, 16, 10000.0, synth.ROPE_HALF, ffn=96)
    w = synth.custom(shape, chunk_lens, q_lens, ratio=ratio, seed=seed)
    sw = synth.draw_stack_weights(w, n_layers)
    sh = dict(n_q_heads=4, n_kv_heads=2, head_dim=16, base=10000.0, layout=synth.ROPE_HALF,
              sm_scale=1.0 / np.sqrt(16.0), eps=shape.rms_eps)
    layers = [{k: v.astype(F64) * (6.0 if k.startswith("w") else 1.0) for k, v in lw.items()} for lw in sw["layers"]]
    idx = dict(seg_start=w.seg_start, ctx_len=w.ctx_len, q_len=w.q_lens, chunk_start=w.chunk_start,
               chunk_len=w.chunk_len, chunk_delta=w.chunk_delta, sel_start=w.sel_start, positions=w.token_positions())
    return w, sw["resid0"].astype(F64), layers, sw["g_final"].astype(F64), sh, idx


def test_single_chunk_at_offset_zero_reproduces_full_prefill():
    """One chunk per request, starting at position 0: its precomputed K/V are the true ones (causal
    attention never looks at the question), so whatever rows are chosen, the question rows must come out
    as in the full prefill."""
    w, r0, layers, g_final, sh, idx = _small_stack([[40], [25]], [6, 4], (30, 100))
    full = st.full_prefill_stack(r0, idx["positions"], w.seg_start, layers, g_final, sh, "exact")
    k_cat, v_cat = st.precompute_stack_caches(r0, w.chunk_start, w.chunk_len, layers, g_final, sh, "exact")
    got = st.fuse_stack(r0, k_cat, v_cat, layers, g_final, sh, storage="exact", **idx)
    assert len(got["sel_idx"]) == 12 + 7
    assert np.abs(got["hidden"] - full["hidden"][got["act_idx"]]).max() < 1e-11
    assert np.abs(got["resid"] - full["resid"][got["act_idx"]]).max() < 1e-11


def test_ratio_one_reproduces_full_prefill_and_lower_ratio_does_not():
    w, r0, layers, g_final, sh, idx = _small_stack([[16, 9, 20], [12, 14]], [5, 3], (1, 1))
    full = st.full_prefill_stack(r0, idx["positions"], w.seg_start, layers, g_final, sh, "exact")
    k_cat, v_cat = st.precompute_stack_caches(r0, w.chunk_start, w.chunk_len, layers, g_final, sh, "exact")
    got = st.fuse_stack(r0, k_cat, v_cat, layers, g_final, sh, storage="exact", **idx)
    assert np.array_equal(got["act_idx"], np.arange(w.total_tokens))
    assert np.abs(got["hidden"] - full["hidden"]).max() < 1e-11
    for l in range(4):
        assert np.abs(got["per_layer"][l]["k"] - full["k"][l]).max() < 1e-11
    # the caches of later chunks are stale (their tokens never saw the earlier chunks): at a lower ratio
    # the result must differ, and layers 0 and 1 must still be exact (they use no cache)
    w2, r0, layers, g_final, sh, idx2 = _small_stack([[16, 9, 20], [12, 14]], [5, 3], (20, 100))
    low = st.fuse_stack(r0, k_cat, v_cat, layers, g_final, sh, storage="exact", **idx2)
    a = low["act_idx"]
    assert len(a) < w.total_tokens
    assert np.abs(low["per_layer"][1]["out"] - got["per_layer"][1]["out"][a]).max() < 1e-11
    assert np.abs(low["hidden"] - full["hidden"][a]).max() > 1e-4
    # the scores of Eq. 3 at layer 1 use the true keys: every request's scores add up to Hq * nq
    for r in range(w.n_req):
        s0, n = int(w.seg_start[r]), int(w.ctx_len[r])
        assert abs(low["scores"][s0:s0 + n].sum() - 4 * int(w.q_lens[r])) < 1e-9


def test_precompute_keeps_chunk_local_positions():
    """Eq. 1: a chunk's cached keys are those of a prompt that holds the chunk alone."""
    w, r0, layers, g_final, sh, idx = _small_stack([[10, 13]], [4], (1, 2), n_layers=2)
    k_cat, v_cat = st.precompute_stack_caches(r0, w.chunk_start, w.chunk_len, layers, g_final, sh, "exact")
    alone = st.full_prefill_stack(r0[10:23], np.arange(13), np.array([0, 13]), layers, g_final, sh, "exact")
    assert np.array_equal(k_cat[1][10:23], alone["k"][1]) and np.array_equal(v_cat[1][10:23], alone["v"][1])
    assert not np.any(k_cat[1][23:])                                       # question rows: nothing cached
    # first chunk: identical to the prefix of the full prompt (offset 0)
    full = st.full_prefill_stack(r0, idx["positions"], w.seg_start, layers, g_final, sh, "exact")
    assert np.abs(k_cat[1][:10] - full["k"][1][:10]).max() < 1e-12
    assert np.abs(k_cat[1][10:23] - full["k"][1][10:23]).max() > 1e-3
