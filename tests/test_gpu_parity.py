"""GPU parity: every C-ABI entry point against the CPU oracle, element by element, on the
same seeded inputs ("teacher forced": each function gets the oracle's inputs for its
stage), then the chained layer.  Sizes span several tiles and ragged tails.

Tolerances (max |a-b| / max |b| per tensor):
  realigned keys   fp32 1e-5; bf16 one rounding of the stored value (checked as <= 2^-7 with
                   at most 2% of elements differing at all)
  scores           1e-4 of the request's largest score; and, over the rows without a planted key (whose huge
                   scores would hide everything else), 2e-5 both of their largest score and element by element
  selected rows    bit-exact on the oracle's float32 scores
  projections, fused K/V, attention output   fp32 1e-5, bf16 2e-2
Element by element (|a-b| / max(|b|, 1e-3 max |b|)): projections 1e-2 in bf16 (the one rounding of the stored
value, 2^-8 .. 2^-7 of the element) and 1e-3 in fp32 (accumulation order over `hidden` products); attention output
|a-b| <= 2^-8 |b| + 2^-8 max |V| (the stored rounding of the output plus the bf16 rounding of the softmax weights
in front of the PV product, each 2^-9, with a factor of two in hand).
"""
import numpy as np
import pytest
import torch

from oracle import a3_oracle as ora
from oracle import workload as wl
import a3_synth as synth
from paper_2511_17560_amd import api, layer
from gpu_util import idev, max_abs_rel, max_elem_rel, to_dev, to_host

pytestmark = pytest.mark.gpu

SMALL_BF16 = synth.ModelShape("small-bf16", "bf16", 256, 8, 2, 128, 500000.0)
SMALL_BF16_HALF = synth.ModelShape("small-bf16-half", "bf16", 256, 8, 2, 128, 500000.0, synth.ROPE_HALF)
SMALL_G7 = synth.ModelShape("small-g7", "bf16", 192, 7, 1, 128, 1000000.0)
SMALL_F32_D128 = synth.ModelShape("small-f32-d128", "f32", 96, 4, 2, 128, 10000.0, synth.ROPE_HALF)


RANDOM_SHAPES = [SMALL_BF16, SMALL_BF16_HALF, SMALL_G7, SMALL_F32_D128,
                 synth.ModelShape("small-g8", "bf16", 128, 8, 1, 128, 10000.0),
                 synth.ModelShape("small-g1", "bf16", 128, 2, 2, 128, 10000.0, synth.ROPE_HALF),
                 synth.ModelShape("small-g2", "bf16", 192, 8, 4, 128, 500000.0)]


def _random_workload(seed):
    """A seeded draw over what the fixed cases hold constant: the model shape (G = 1, 2, 4, 7, 8), 1-6 requests of 1-5
    chunks, chunk and question lengths from one token up to a few hundred (now and then a couple of thousand), and
    the ratio, the degenerate 0 and 1 included."""
    rng = np.random.default_rng(seed)
    shape = RANDOM_SHAPES[rng.integers(len(RANDOM_SHAPES))]
    long_chunks = rng.random() < 0.3
    chunk_lens, q_lens = [], []
    for _ in range(int(rng.integers(1, 7))):
        hi = 2000 if long_chunks else 300
        chunk_lens.append([int(rng.integers(1, hi)) if rng.random() < 0.8 else int(rng.integers(1, 4))
                           for _ in range(int(rng.integers(1, 6)))])
        q_lens.append(int(rng.integers(1, 150)) if rng.random() < 0.8 else int(rng.integers(1, 4)))
    num = int(rng.choice([0, 1, 5, 10, 15, 25, 50, 99, 100]))
    return synth.custom(shape, chunk_lens, q_lens, ratio=(num, 100), seed=seed, name=f"random-{seed}")


def _workload(name):
    if name == "cfg1":
        return synth.config(1)
    if name == "cfg1-half":
        return synth.config(1, rope_layout=synth.ROPE_HALF)
    if name == "cfg2":
        return synth.config(2)
    if name == "ragged-bf16":
        return synth.custom(SMALL_BF16, [[100, 37, 300, 65]], [19], ratio=(15, 100), n_planted=3, seed=41)
    if name == "batched-bf16-half":
        return synth.custom(SMALL_BF16_HALF, [[130, 70], [33], [257, 64, 90]], [5, 33, 12], ratio=(20, 100), seed=42)
    if name == "g7-bf16":
        return synth.custom(SMALL_G7, [[200, 150, 93]], [9], ratio=(25, 100), seed=43)
    if name == "manyq-bf16":     # more than 256 (question token, head) rows per KV head: two row chunks in the scoring step
        return synth.custom(SMALL_BF16, [[300, 129, 260]], [90], ratio=(10, 100), n_planted=2, seed=48)
    if name == "manyq-g7-bf16":  # the same with 7 query heads per KV head, two requests, one of them with a single row chunk
        return synth.custom(SMALL_G7, [[140, 200], [90]], [40, 11], ratio=(20, 100), seed=49)
    if name == "longq-bf16":     # a question far longer than the context: 19 row chunks in the scoring step, and more row tiles
        # in the attention plan than the selection kernel's LDS (sized by the context) can hold next to each other
        return synth.custom(SMALL_BF16, [[20, 12]], [1200], ratio=(25, 100), seed=50)
    if name == "ratio0-bf16":    # nothing recomputed but the question (the concatenation with recovered positions)
        return synth.custom(SMALL_BF16, [[120, 3, 211], [64]], [21, 2], ratio=(0, 100), seed=51)
    if name == "ratio100-g7":    # everything recomputed (the full prefill), with one-token and two-token chunks
        return synth.custom(SMALL_G7, [[183, 1, 112, 2], [93]], [5, 40], ratio=(100, 100), seed=52)
    if name.startswith("random-"):
        return _random_workload(int(name[len("random-"):]))
    if name == "cfg3-layer0":    # the 16K benchmark configuration, first and last of its 32 independent layers
        return synth.config(3, layer=0)
    if name in ("cfg3-layer1", "cfg3-layer15", "cfg3-layer31"):
        return synth.config(3, layer=int(name[len("cfg3-layer"):]))
    if name == "cfg4":
        return synth.config(4)
    if name == "cfg5":
        return synth.config(5)
    if name == "long-bf16":      # visible keys beyond 1.5 x 4096: tiles are cut into key segments and merged
        return synth.custom(SMALL_BF16, [[3000, 2500, 2100]], [40], ratio=(10, 100), n_planted=4, seed=45)
    if name == "k64-bf16":       # reduction dimension of one 64-element slab, and of two
        return synth.custom(synth.ModelShape("k64", "bf16", 64, 2, 1, 128, 10000.0), [[300, 211]], [13], ratio=(40, 100), seed=46)
    if name == "k128-bf16":
        return synth.custom(synth.ModelShape("k128", "bf16", 128, 4, 2, 128, 10000.0, synth.ROPE_HALF), [[150, 260]], [7],
                            ratio=(50, 100), seed=47)
    if name == "batched-f32-d128":
        return synth.custom(SMALL_F32_D128, [[40, 77], [129]], [7, 3], ratio=(30, 100), seed=44)
    raise KeyError(name)


NAMES = ["cfg1", "cfg1-half", "ragged-bf16", "batched-bf16-half", "g7-bf16", "batched-f32-d128", "cfg2", "long-bf16",
         "manyq-bf16", "manyq-g7-bf16", "longq-bf16", "ratio0-bf16", "ratio100-g7"]
# full-size configurations: one oracle layer each takes tens of seconds, so each is built once and runs
# the chained test and the teacher-forced tests of the three kernels whose behaviour depends on scale
BIG_NAMES = ["cfg3-layer0", "cfg3-layer1", "cfg3-layer15", "cfg3-layer31", "cfg4", "cfg5"]
_cache = {}


def ctx_of(name):
    if name in BIG_NAMES and name not in _cache:       # keep one full-size context at a time
        for k in [k for k in _cache if k in BIG_NAMES]:
            del _cache[k]
    if name not in _cache:
        w = _workload(name)
        b = wl.build(w)
        res = wl.run_oracle(b)
        lay = api.Layout.from_workload(w)
        _cache[name] = dict(w=w, b=b, res=res, lay=lay)
    return _cache[name]


def tol(w):
    return 1e-5 if w.shape.dtype == "f32" else 2e-2


@pytest.mark.parametrize("name", NAMES)
def test_layout_tables(name):
    c = ctx_of(name)
    w, lay = c["w"], c["lay"]
    torch.cuda.synchronize()
    assert np.array_equal(lay.tok_pos.cpu().numpy(), w.token_positions())
    assert np.array_equal(lay.tok_req.cpu().numpy(), w.token_requests())
    chunk = np.full(w.total_tokens, -1, np.int32)
    for ci in range(w.n_chunks):
        chunk[w.chunk_start[ci]:w.chunk_start[ci] + w.chunk_len[ci]] = ci
    assert np.array_equal(lay.tok_chunk.cpu().numpy(), chunk)
    assert np.array_equal(lay.q_start.cpu().numpy(), np.concatenate([[0], np.cumsum(w.q_lens)]))
    # RoPE tables against the oracle's float64 angles
    th = ora.rope_theta(w.shape.head_dim, w.shape.rope_base)
    pos = np.arange(lay.rope_pos_cs.shape[0])[:, None] * th[None, :]
    got = lay.rope_pos_cs.cpu().numpy().astype(np.float64)
    assert np.abs(got[..., 0] - np.cos(pos)).max() < 1e-7 and np.abs(got[..., 1] - np.sin(pos)).max() < 1e-7
    ang = w.chunk_delta[:, None] * th[None, :]
    gotc = lay.rope_chunk_cs.cpu().numpy().astype(np.float64)
    assert np.abs(gotc[..., 0] - np.cos(ang)).max() < 1e-7 and np.abs(gotc[..., 1] - np.sin(ang)).max() < 1e-7


@pytest.mark.parametrize("inplace", [False, True])
@pytest.mark.parametrize("name", NAMES)
def test_rope_realign(name, inplace):
    c = ctx_of(name)
    w, b, res, lay = c["w"], c["b"], c["res"], c["lay"]
    k_cat = to_dev(b["k_cat"], w.shape.dtype)
    k_out = k_cat if inplace else torch.zeros_like(k_cat)
    api.a3_rope_realign(lay, k_cat, k_out)
    got = to_host(k_out)
    want = res["k_realigned"]
    for r in range(w.n_req):
        rows = w.ctx_rows(r)
        err = max_abs_rel(got[rows], want[rows])
        if w.shape.dtype == "f32":
            assert err <= 1e-5, err
        else:
            assert err <= 2.0 ** -7, err
            assert np.mean(got[rows] != want[rows]) < 0.02
    # chunks at offset 0 are returned bit for bit
    for ci in np.nonzero(w.chunk_delta == 0)[0]:
        s, L = w.chunk_start[ci], w.chunk_len[ci]
        assert np.array_equal(got[s:s + L], np.asarray(b["k_cat"][s:s + L], dtype=np.float64))
    if inplace:      # question rows untouched
        q = w.question_rows()
        assert np.array_equal(got[q], np.asarray(b["k_cat"][q], dtype=np.float64))


@pytest.mark.parametrize("name", NAMES)
def test_selected_qkv_proj(name):
    c = ctx_of(name)
    w, b, res, lay = c["w"], c["b"], c["res"], c["lay"]
    s, t = w.shape, b["t"]
    dt = s.dtype
    x = to_dev(t.x_cur, dt)
    wq, wk, wv = to_dev(t.wq, dt), to_dev(t.wk, dt), to_dev(t.wv, dt)
    for rows_np, wantq, wantk, wantv in ((res["sel_idx"], res["q_sel"], res["k_sel"], res["v_sel"]),
                                         (res["q_rows"], res["q_question"], res["k_question"], res["v_question"])):
        n = len(rows_np)
        q = torch.zeros((n, s.n_q_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
        k = torch.zeros((n, s.n_kv_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
        v = torch.zeros_like(k)
        api.a3_selected_qkv_proj(lay, x, idev(rows_np), n, wq, wk, wv, q_out=q, k_out=k, v_out=v)
        assert max_abs_rel(to_host(q), wantq) <= tol(w)
        assert max_abs_rel(to_host(k), wantk) <= tol(w)
        assert max_abs_rel(to_host(v), wantv) <= tol(w)
        etol = 1e-3 if dt == "f32" else 1e-2
        assert max_elem_rel(to_host(q), wantq) <= etol and max_elem_rel(to_host(k), wantk) <= etol
        assert max_elem_rel(to_host(v), wantv) <= etol
    # Q of the question rows alone (what the layer pass asks for first; few heads: the few-row kernel then runs
    # with 32 rows per workgroup), and K and V alone
    rows_np = res["q_rows"]
    n = len(rows_np)
    q = torch.zeros((n, s.n_q_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
    api.a3_selected_qkv_proj(lay, x, idev(rows_np), n, wq, None, None, q_out=q)
    assert max_abs_rel(to_host(q), res["q_question"]) <= tol(w)
    k = torch.zeros((n, s.n_kv_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
    v = torch.zeros_like(k)
    api.a3_selected_qkv_proj(lay, x, idev(rows_np), n, None, wk, wv, k_out=k, v_out=v)
    assert max_abs_rel(to_host(k), res["k_question"]) <= tol(w)
    assert max_abs_rel(to_host(v), res["v_question"]) <= tol(w)
    # NULL row list = rows 0..n-1, only K requested, with a bias
    n = min(w.total_tokens, 150)
    bk_np = synth.round_to_storage(np.random.default_rng(9).standard_normal(s.n_kv_heads * s.head_dim), dt)
    k = torch.zeros((n, s.n_kv_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
    api.a3_selected_qkv_proj(lay, x, None, n, wq, wk, wv, bk=to_dev(bk_np, dt), k_out=k)
    _, want, _ = ora.selected_qkv_proj(t.x_cur, np.arange(n), w.token_positions()[:n], t.wq, t.wk, t.wv, s.n_q_heads,
                                       s.n_kv_heads, s.head_dim, s.rope_base, s.rope_layout, dt, bk=bk_np)
    assert max_abs_rel(to_host(k), want) <= tol(w)


@pytest.mark.parametrize("k64", ["1", "0"])
@pytest.mark.parametrize("ntw", ["2", "3", "4"])
@pytest.mark.parametrize("name", ["g7-bf16", "batched-bf16-half", "cfg2", "k64-bf16", "k128-bf16"])
def test_selected_qkv_proj_every_tile_width(name, ntw, k64, tuning):
    """The large-tile GEMM kernel in each of its three workgroup shapes (the library normally
    picks one by row count; few rows go to the weight-streaming kernel instead), with the main loop on
    128-byte row pieces (the default for the two larger shapes) and on 64-byte pieces."""
    tuning("proj_ntw", ntw)
    tuning("proj_k64", k64)
    c = ctx_of(name)
    w, b, res, lay = c["w"], c["b"], c["res"], c["lay"]
    s, t = w.shape, b["t"]
    dt = s.dtype
    rows_np = res["act_idx"]
    n = len(rows_np)
    q = torch.zeros((n, s.n_q_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
    k = torch.zeros((n, s.n_kv_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
    v = torch.zeros_like(k)
    api.a3_selected_qkv_proj(lay, to_dev(t.x_cur, dt), idev(rows_np), n, to_dev(t.wq, dt), to_dev(t.wk, dt),
                             to_dev(t.wv, dt), q_out=q, k_out=k, v_out=v)
    assert max_abs_rel(to_host(q), res["q_act"]) <= tol(w)
    assert max_abs_rel(to_host(k), res["k_fused"][rows_np]) <= tol(w)
    assert max_abs_rel(to_host(v), res["v_fused"][rows_np]) <= tol(w)


@pytest.mark.parametrize("name", NAMES)
def test_question_scores(name):
    c = ctx_of(name)
    w, res, lay = c["w"], c["res"], c["lay"]
    dt = w.shape.dtype
    qq = to_dev(res["q_question"], dt)
    k_re = to_dev(res["k_realigned"], dt)
    scores = torch.zeros(w.total_tokens, dtype=torch.float32, device="cuda")
    ws = lay.workspace(w.total_k + w.total_q)
    api.a3_question_scores(lay, qq, k_re, scores, ws)
    got = scores.cpu().numpy().astype(np.float64)
    want = res["scores"]
    for r in range(w.n_req):
        rows = w.ctx_rows(r)
        assert max_abs_rel(got[rows], want[rows]) <= 1e-4
        plain = np.setdiff1d(rows, c["b"]["planted"])        # without the planted keys' scores, which dwarf the rest
        assert max_abs_rel(got[plain], want[plain]) <= 2e-5 and max_elem_rel(got[plain], want[plain]) <= 2e-5
        # every softmax row sums to one
        assert abs(got[rows].sum() - w.shape.n_q_heads * w.q_lens[r]) <= 1e-3 * w.shape.n_q_heads * w.q_lens[r]
    assert np.all(np.isneginf(got[w.question_rows()]))


@pytest.mark.parametrize("inplace", [False, True])
@pytest.mark.parametrize("name", NAMES)
def test_realign_scores_single_call(name, inplace):
    """a3_realign_scores = a3_rope_realign then a3_question_scores: the realigned cache must equal the one
    a3_rope_realign writes bit for bit, the scores meet the same bar as test_question_scores."""
    c = ctx_of(name)
    w, b, res, lay = c["w"], c["b"], c["res"], c["lay"]
    dt = w.shape.dtype
    qq = to_dev(res["q_question"], dt)
    k_cat = to_dev(b["k_cat"], dt)
    k_two = torch.zeros_like(k_cat)
    api.a3_rope_realign(lay, k_cat, k_two)
    k_one = k_cat.clone() if inplace else torch.zeros_like(k_cat)
    scores = torch.zeros(w.total_tokens, dtype=torch.float32, device="cuda")
    ws = lay.workspace(w.total_k + w.total_q)
    api.a3_realign_scores(lay, qq, k_one if inplace else k_cat, k_one, scores, ws)
    ctx = np.concatenate([w.ctx_rows(r) for r in range(w.n_req)])
    assert np.array_equal(to_host(k_one)[ctx], to_host(k_two)[ctx])
    q = w.question_rows()
    assert np.array_equal(to_host(k_one)[q], np.asarray(b["k_cat"][q], dtype=np.float64) if inplace else np.zeros_like(to_host(k_one)[q]))
    got = scores.cpu().numpy().astype(np.float64)
    # the oracle scored its own realigned keys; ours differ from those by at most one rounding
    for r in range(w.n_req):
        rows = w.ctx_rows(r)
        assert max_abs_rel(got[rows], res["scores"][rows]) <= (1e-4 if dt == "f32" else 2e-2)
        assert abs(got[rows].sum() - w.shape.n_q_heads * w.q_lens[r]) <= 1e-3 * w.shape.n_q_heads * w.q_lens[r]
    # and exactly what the two separate calls give
    scores2 = torch.zeros_like(scores)
    api.a3_question_scores(lay, qq, k_two, scores2, ws)
    assert torch.equal(scores, scores2)
    assert np.all(np.isneginf(got[q]))


@pytest.mark.parametrize("name", NAMES)
def test_topk_select_bit_exact_on_oracle_scores(name):
    c = ctx_of(name)
    w, res, lay = c["w"], c["res"], c["lay"]
    s32 = np.asarray(res["scores"], dtype=np.float32)
    scores = torch.from_numpy(s32).cuda()
    sel = torch.full((max(w.total_k, 1),), -1, dtype=torch.int32, device="cuda")
    api.a3_topk_select(lay, scores, idev(w.sel_start), w.total_k, sel)
    assert np.array_equal(sel.cpu().numpy()[:w.total_k], res["sel_idx"])


@pytest.mark.parametrize("name", NAMES)
def test_kv_scatter_and_active_rows(name):
    c = ctx_of(name)
    w, res, lay = c["w"], c["res"], c["lay"]
    dt = w.shape.dtype
    act = res["act_idx"]
    # active rows helper
    got_act = torch.full((len(act),), -1, dtype=torch.int32, device="cuda")
    api.a3_active_rows(lay, idev(res["sel_idx"]) if w.total_k else None, idev(w.sel_start), len(act), got_act)
    assert np.array_equal(got_act.cpu().numpy(), act)
    # scatter the oracle's fresh K/V of the active rows into the realigned cache
    kf = to_dev(res["k_realigned"], dt)
    vf = to_dev(c["b"]["v_cat"], dt)
    api.a3_kv_scatter(lay, to_dev(res["k_fused"][act], dt), to_dev(res["v_fused"][act], dt), idev(act), len(act), kf, vf)
    assert np.array_equal(to_host(kf), res["k_fused"])
    assert np.array_equal(to_host(vf), res["v_fused"])


@pytest.mark.parametrize("name", NAMES)
def test_fused_attention(name):
    c = ctx_of(name)
    w, res, lay = c["w"], c["res"], c["lay"]
    s = w.shape
    dt = s.dtype
    act = res["act_idx"]
    out = torch.zeros((len(act), s.n_q_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
    ws = lay.workspace(len(act))
    api.a3_fused_attention(lay, to_dev(res["q_act"], dt), idev(act), len(act), to_dev(res["k_fused"], dt),
                           to_dev(res["v_fused"], dt), out, ws)
    got = to_host(out)
    assert max_abs_rel(got, res["out"]) <= tol(w)
    ulp = 2.0 ** -8 if dt == "bf16" else 1e-5
    assert np.all(np.abs(got - res["out"]) <= ulp * np.abs(res["out"]) + ulp * np.abs(res["v_fused"]).max())


@pytest.mark.parametrize("wgs,item_cost", [("1", None), ("3", None), ("37", None), ("300", None), ("37", "0"),
                                           ("5", "64"), ("300", "1"), ("32", "30")])
@pytest.mark.parametrize("name", ["ragged-bf16", "batched-bf16-half", "g7-bf16", "cfg2", "long-bf16"])
def test_fused_attention_with_other_share_counts(name, wgs, item_cost, tuning):
    """The work of all tiles (key steps plus a start-up cost per tile) is cut into one equal share per
    workgroup of a KV head.  Other numbers of workgroups and other start-up costs move the cuts: none at
    all (1), a few long shares, many short ones (tiles cut into several items, items that start or end
    exactly on a tile boundary, cuts that fall into a tile's start-up units, rows that see nothing of a
    later item, ordered merge of the partial results)."""
    tuning("attn_wgs", wgs)
    if item_cost is not None:
        tuning("attn_item_cost", item_cost)
    c = ctx_of(name)
    w, res, lay = c["w"], c["res"], c["lay"]
    s = w.shape
    act = res["act_idx"]
    out = torch.zeros((len(act), s.n_q_heads, s.head_dim), dtype=torch.bfloat16, device="cuda")
    ws = lay.workspace(len(act))
    api.a3_fused_attention(lay, to_dev(res["q_act"], "bf16"), idev(act), len(act), to_dev(res["k_fused"], "bf16"),
                           to_dev(res["v_fused"], "bf16"), out, ws)
    assert max_abs_rel(to_host(out), res["out"]) <= tol(w)


@pytest.mark.parametrize("name", NAMES)
def test_topk_select_plan_equals_the_three_calls(name):
    """a3_topk_select_plan = a3_topk_select, a3_active_rows, a3_attention_plan: the same selection, the same row
    list, and an attention that gives the same output bit for bit with either plan.  In a batch of one request
    (one launch) the selection may be written straight into the head of the row list."""
    c = ctx_of(name)
    w, res, lay = c["w"], c["res"], c["lay"]
    s = w.shape
    dt = s.dtype
    scores = torch.from_numpy(np.asarray(res["scores"], dtype=np.float32)).cuda()
    n_act = w.total_k + w.total_q
    k = w.total_k
    sel_start = idev(w.sel_start)
    q, kf, vf = to_dev(res["q_act"], dt), to_dev(res["k_fused"], dt), to_dev(res["v_fused"], dt)
    # the three calls
    sel3 = torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
    act3 = torch.full((n_act,), -1, dtype=torch.int32, device="cuda")
    ws3 = lay.workspace(n_act)
    api.a3_topk_select(lay, scores, sel_start, k, sel3)
    api.a3_active_rows(lay, sel3, sel_start, n_act, act3)
    api.a3_attention_plan(lay, act3, n_act, ws3)
    out3 = torch.zeros((n_act, s.n_q_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
    api.a3_fused_attention_planned(lay, q, act3, n_act, kf, vf, out3, ws3)
    assert np.array_equal(act3.cpu().numpy(), res["act_idx"])
    variants = [False] + ([True] if w.n_req == 1 else [])
    for in_place in variants:
        act1 = torch.full((n_act,), -1, dtype=torch.int32, device="cuda")
        sel1 = act1 if in_place else torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
        ws1 = lay.workspace(n_act)
        ws1.fill_(0xAB)
        api.a3_topk_select_plan(lay, scores, sel_start, k, sel1, n_act, act1, ws1)
        out1 = torch.zeros_like(out3)
        api.a3_fused_attention_planned(lay, q, act1, n_act, kf, vf, out1, ws1)
        torch.cuda.synchronize()
        assert torch.equal(act1, act3)
        assert torch.equal(sel1[:k], sel3[:k])
        assert torch.equal(out1, out3)
    assert max_abs_rel(to_host(out3), res["out"]) <= tol(w)


@pytest.mark.parametrize("name", ["cfg1", "ragged-bf16", "batched-bf16-half", "cfg2"])
def test_chained_layer_separate_select_rows_plan(name):
    """Same as test_chained_layer with a3_topk_select, a3_active_rows and a3_fused_attention instead of
    a3_topk_select_plan and a3_fused_attention_planned."""
    test_chained_layer(name, fused_plan=False)


@pytest.mark.parametrize("name", ["cfg1", "ragged-bf16", "batched-bf16-half", "cfg2"])
def test_chained_layer_plain_six_call_sequence(name):
    """Same as test_chained_layer, through the six plain calls: a3_rope_realign and a3_question_scores
    instead of a3_realign_scores, a3_selected_qkv_proj + a3_kv_scatter instead of the projection that
    writes into the caches."""
    test_chained_layer(name, fused_scatter=False, fused_realign=False, fused_plan=False)


@pytest.mark.parametrize("name", NAMES)
def test_chained_layer(name, fused_scatter=True, fused_realign=True, fused_plan=True):
    """All steps on the GPU's own intermediates.  The selected set must equal the oracle's up to
    near-ties: a row in the symmetric difference must score within 1e-3 (relative) of the
    oracle's k-th score.  Planted rows must be selected.  Downstream tensors are compared on the
    rows both sides selected."""
    c = ctx_of(name)
    w, b, res, lay = c["w"], c["b"], c["res"], c["lay"]
    s, t = w.shape, b["t"]
    dt = s.dtype
    bufs = layer.make_buffers(lay, w.sel_start, w.question_rows(), s)
    x = to_dev(t.x_cur, dt)
    k_cat, v_cache = to_dev(b["k_cat"], dt), to_dev(b["v_cat"], dt)
    wq, wk, wv = to_dev(t.wq, dt), to_dev(t.wk, dt), to_dev(t.wv, dt)
    layer.fuse_layer(lay, bufs, x, k_cat, v_cache, wq, wk, wv, fused_scatter=fused_scatter, fused_realign=fused_realign,
                     fused_plan=fused_plan)
    torch.cuda.synchronize()
    got_act = bufs.act_idx.cpu().numpy()[:bufs.n_act]
    want_act = res["act_idx"]
    got_set, want_set = set(got_act.tolist()), set(want_act.tolist())
    flips = got_set ^ want_set
    for r in range(w.n_req):
        k_r = int(w.sel_start[r + 1] - w.sel_start[r])
        if k_r == 0:
            continue
        rows = w.ctx_rows(r)
        kth = np.sort(res["scores"][rows])[::-1][k_r - 1]
        for row in flips:
            if rows[0] <= row <= rows[-1]:
                assert abs(res["scores"][row] - kth) <= 1e-3 * abs(kth), (row, res["scores"][row], kth)
    assert len(flips) <= max(2, len(want_act) // 50)
    assert set(b["planted"].tolist()) <= got_set
    assert np.all(np.diff(got_act) > 0)
    common_g = np.nonzero(np.isin(got_act, want_act))[0]
    common_w = np.nonzero(np.isin(want_act, got_act))[0]
    out = to_host(bufs.out)[:bufs.n_act]
    assert max_abs_rel(out[common_g], res["out"][common_w]) <= tol(w)
    rows = got_act[common_g]
    assert max_abs_rel(to_host(bufs.k_fused)[rows], res["k_fused"][rows]) <= tol(w)
    assert max_abs_rel(to_host(v_cache)[rows], res["v_fused"][rows]) <= tol(w)
    # rows nobody selected keep the realigned stale keys / stale values
    stale = np.setdiff1d(np.arange(w.total_tokens), np.union1d(got_act, want_act))
    assert max_abs_rel(to_host(bufs.k_fused)[stale], res["k_fused"][stale]) <= (1e-5 if dt == "f32" else 2.0 ** -7)
    assert np.array_equal(to_host(v_cache)[stale], res["v_fused"][stale])


@pytest.mark.parametrize("seed", range(7000, 7024))
def test_random_workloads(seed):
    """Every step against the oracle, the merged calls against the separate ones, and the chained layer in both call
    sequences, on seeded random batches."""
    name = f"random-{seed}"
    try:
        for check in (test_layout_tables, test_question_scores, test_topk_select_bit_exact_on_oracle_scores,
                      test_selected_qkv_proj, test_kv_scatter_and_active_rows, test_fused_attention,
                      test_topk_select_plan_equals_the_three_calls, test_attention_in_two_calls, test_chained_layer,
                      test_chained_layer_plain_six_call_sequence):
            check(name)
        test_rope_realign(name, True)
        test_realign_scores_single_call(name, False)
    finally:
        _cache.pop(name, None)


@pytest.mark.parametrize("case", ["ties", "all-equal", "k-zero-and-full", "long-global-path", "negatives", "vector-tail-4k",
                                  "vector-tail-16k", "dups-at-cut"])
def test_topk_select_edge_cases(case):
    """Top-p on hand-made score arrays, bit-exact against the oracle: heavy ties across the cut,
    all-equal scores (lowest rows win), k = 0 and k = N per request, a request longer than the
    register-resident limit (global re-read path), scores of both signs with +-0, lengths that end
    inside a lane's vector load, and otherwise distinct scores whose k-th largest value occurs several
    times (the few candidates left after two radix rounds are ranked by one wave: some of the equal ones
    are taken, in row order, the others are not)."""
    rng = np.random.default_rng(99)
    shape = synth.ModelShape("topk", "f32", 32, 1, 1, 64, 1e4)
    if case == "long-global-path":
        w = synth.custom(shape, [[20000, 20001], [777]], [3, 2], ratio=(10, 100))
    elif case == "vector-tail-4k":       # 16-byte aligned runs of 4 scores per lane, the last one cut short
        w = synth.custom(shape, [[4001]], [3], ratio=(10, 100))
    elif case == "vector-tail-16k":      # runs of 16, the last lane with scores holds 11
        w = synth.custom(shape, [[8000, 8379]], [2], ratio=(10, 100))
    elif case == "k-zero-and-full":
        w = synth.custom(shape, [[300], [1025, 40], [64]], [2, 2, 2], ratio=(100, 100))
    else:
        w = synth.custom(shape, [[1500, 900], [3000]], [4, 1], ratio=(15, 100))
    T = w.total_tokens
    if case == "all-equal":
        sc = np.full(T, 0.25, np.float32)
    elif case == "ties":
        sc = (rng.integers(0, 12, size=T) / 16.0).astype(np.float32)
    elif case == "negatives":
        sc = rng.standard_normal(T).astype(np.float32)
        sc[::7] = 0.0
        sc[3::11] = -0.0
    else:
        sc = rng.random(T).astype(np.float32) * np.exp(rng.uniform(-8, 3, T)).astype(np.float32)
    if case == "dups-at-cut":
        for r in range(w.n_req):
            rows = w.ctx_rows(r)
            k_r = int(w.sel_start[r + 1] - w.sel_start[r])
            order = rows[np.argsort(-sc[rows], kind="stable")]
            kth = sc[order[k_r - 1]]
            lower = order[k_r + 5:]                          # rows that would not be selected
            sc[np.sort(rng.choice(lower, size=6, replace=False))] = kth          # 7 equal values, one is wanted
            sc[order[k_r - 2]] = kth                                             # and the one above the cut too: 8, two wanted
    sc[w.question_rows()] = -np.inf
    sel_start = w.sel_start.copy()
    if case == "k-zero-and-full":
        sel_start = np.array([0, 0, 0 + w.ctx_len[1], w.ctx_len[1] + 1], np.int32)   # k = 0, N, 1
    want = ora.topk_select(sc, w.seg_start, w.ctx_len, sel_start)
    lay = api.Layout.from_workload(w)
    total_k = int(sel_start[-1])
    sel = torch.full((max(total_k, 1),), -1, dtype=torch.int32, device="cuda")
    api.a3_topk_select(lay, torch.from_numpy(sc).cuda(), idev(sel_start), total_k, sel)
    assert np.array_equal(sel.cpu().numpy()[:total_k], want)


@pytest.mark.parametrize("name", BIG_NAMES)
def test_full_size_config(name):
    """Configurations 3 (two of its 32 layers), 4 and 5 at full size, in the launch configuration the
    benchmark uses: scores, top-p and attention on the oracle's inputs, then the chained layer."""
    test_question_scores(name)
    test_topk_select_bit_exact_on_oracle_scores(name)
    test_fused_attention(name)
    test_chained_layer(name)
    _cache.pop(name, None)


def test_layer_at_128k_context():
    """One layer on 131072 context tokens (256 chunks of 512) and a 64-token question in the Llama-3-8B shape, r = 5 %:
    eight times the benchmark's context, a gigabyte of hidden states, 2048 key tiles per row of the attention, the
    selection's path for inputs that do not fit its LDS.  The inputs are drawn on the device; the oracle then gets
    what each step read on the GPU: the realigned cache for all of Eq. 3 (every score is compared), the GPU's scores
    for the selection (bit-exact), and sampled rows for Eq. 2, Eq. 5 and Eq. 4."""
    shape = synth.ModelShape("llama-3-8b", "bf16", 4096, 32, 8, 128, 500000.0)
    dt, n_ctx, nq = "bf16", 131072, 64
    w = synth.custom(shape, [[512] * (n_ctx // 512)], [nq], ratio=(5, 100), seed=93)
    T, h, Hq, Hkv, d = w.total_tokens, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    g = torch.Generator(device="cuda")
    g.manual_seed(93)
    draw = lambda *sz, std: (torch.randn(sz, generator=g, device="cuda", dtype=torch.float32) * std).to(torch.bfloat16)
    x = draw(T, h, std=1.0)
    k_cat, v_cache = draw(T, Hkv, d, std=0.02 * h ** 0.5), draw(T, Hkv, d, std=0.02 * h ** 0.5)
    # wider query/key weights than 0.02, so that the scores are not all alike and the ranking means something
    wq, wk, wv = draw(Hq * d, h, std=0.04), draw(Hkv * d, h, std=0.04), draw(Hkv * d, h, std=0.02)
    v_stale = v_cache.clone()
    lay = api.Layout.from_workload(w)
    bufs = layer.make_buffers(lay, w.sel_start, w.question_rows(), shape)
    layer.fuse_layer(lay, bufs, x, k_cat, v_cache, wq, wk, wv)
    torch.cuda.synchronize()
    n_act, total_k = bufs.n_act, int(w.sel_start[-1])
    assert total_k == 6553 and n_act == total_k + nq
    act = bufs.act_idx.cpu().numpy()[:n_act].astype(np.int64)
    q_rows = np.asarray(w.question_rows(), dtype=np.int64)
    assert np.all(np.diff(act) > 0) and np.array_equal(act[total_k:], q_rows)
    rng = np.random.default_rng(94)
    pos = np.asarray(w.token_positions())
    proj = dict(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, base=shape.rope_base, layout=shape.rope_layout, storage=dt)
    scale = 1.0 / np.sqrt(d)
    host = lambda t, rows: to_host(t[torch.as_tensor(rows, device="cuda")])
    wq_h, wk_h, wv_h = to_host(wq), to_host(wk), to_host(wv)
    k_fused = to_host(bufs.k_fused)

    # Eq. 2: the cache the scores were taken on is the realign kernel's output bit for bit (checked at small sizes
    # for every element); here on the rows nobody recomputed, and against the oracle on sampled rows, chunk edges
    # among them (rotation by the chunk's offset, one rounding)
    k_re = torch.empty_like(k_cat)
    api.a3_rope_realign(lay, k_cat, k_re)
    torch.cuda.synchronize()
    rest = np.setdiff1d(np.arange(T), act)
    rest_d = torch.as_tensor(rest, device="cuda")
    assert torch.equal(bufs.k_fused[rest_d], k_re[rest_d]) and torch.equal(v_cache[rest_d], v_stale[rest_d])
    rows = np.unique(np.concatenate([[0, 1, 511, 512, 513, 130559, 130560, n_ctx - 1], rng.choice(n_ctx, size=56, replace=False)]))
    want = ora.store(ora.rope_rotate(host(k_cat, rows), (rows // 512) * 512, shape.rope_base, shape.rope_layout), dt)
    assert max_abs_rel(host(k_re, rows), want) <= 2.0 ** -7

    # Eq. 3, first line: every score, on that cache
    k_scored = to_host(k_re)
    del k_re
    # (with the Q the layer pass scored with: its first call, repeated here; the question rows of q_act hold the
    # second projection's Q by now, which may differ from it in a last bit)
    q_scored = torch.empty((nq, Hq, d), dtype=torch.bfloat16, device="cuda")
    api.a3_selected_qkv_proj(lay, x, bufs.q_rows, nq, wq, None, None, q_out=q_scored)
    torch.cuda.synchronize()
    qq, _, _ = ora.selected_qkv_proj(host(x, q_rows), np.arange(nq), pos[q_rows], wq_h, wk_h, wv_h, **proj)
    assert max_abs_rel(to_host(q_scored), qq) <= 2e-2 and max_abs_rel(to_host(bufs.q_act)[total_k:], qq) <= 2e-2
    want_scores = ora.question_scores(to_host(q_scored), k_scored, w.seg_start, w.ctx_len, w.q_lens, scale)
    got_scores = to_host(bufs.scores)
    assert max_abs_rel(got_scores[:n_ctx], want_scores[:n_ctx]) <= 1e-4
    assert max_elem_rel(got_scores[:n_ctx], want_scores[:n_ctx]) <= 1e-3
    assert abs(got_scores[:n_ctx].sum() - Hq * nq) <= 1e-3 * Hq * nq and np.all(np.isneginf(got_scores[n_ctx:]))

    # Eq. 3, second line: exactly the 6553 best of the GPU's own scores, ties to the lower row
    want_sel = ora.topk_select(got_scores.astype(np.float32), w.seg_start, w.ctx_len, w.sel_start)
    assert np.array_equal(act[:total_k], want_sel)
    overlap = len(set(want_sel.tolist()) & set(ora.topk_select(want_scores, w.seg_start, w.ctx_len, w.sel_start).tolist()))
    assert overlap >= 0.98 * total_k

    # Eq. 5 on sampled active rows (the first and last selected row and the question's ends among them)
    pick = np.unique(np.concatenate([[0, 1, total_k - 1, total_k, n_act - 1], rng.choice(n_act, size=19, replace=False)]))
    q, k, v = ora.selected_qkv_proj(host(x, act[pick]), np.arange(len(pick)), pos[act[pick]], wq_h, wk_h, wv_h, **proj)
    assert max_abs_rel(to_host(bufs.q_act)[pick], q) <= 2e-2
    assert max_abs_rel(k_fused[act[pick]], k) <= 2e-2 and max_abs_rel(host(v_cache, act[pick]), v) <= 2e-2
    # Eq. 4 for those rows over up to 131136 keys each, on the caches the GPU attended
    o = ora.fused_attention(to_host(bufs.q_act)[pick], act[pick], k_fused, to_host(v_cache), w.seg_start, scale, dt)
    got_o = to_host(bufs.out)[pick]
    assert max_abs_rel(got_o, o) <= 2e-2
    vmax = float(torch.abs(v_cache.float()).max())
    assert np.all(np.abs(got_o - o) <= 2.0 ** -8 * np.abs(o) + 2.0 ** -8 * vmax)


def test_planned_attention_leaves_out_alone_when_the_plan_was_made_with_another_tuning(tuning):
    """The number of workgroups per head decides where the plan's tables lie in the workspace.  A planned call
    that finds a plan made with another value must not read those tables: it leaves `out` as it was."""
    c = ctx_of("ragged-bf16")
    w, res, lay = c["w"], c["res"], c["lay"]
    dt = w.shape.dtype
    act = res["act_idx"]
    q, k, v, idx = to_dev(res["q_act"], dt), to_dev(res["k_fused"], dt), to_dev(res["v_fused"], dt), idev(act)
    out = torch.full((len(act), w.shape.n_q_heads, w.shape.head_dim), 3.0, dtype=api.torch_dtype(dt), device="cuda")
    ws = lay.workspace(len(act))
    api.a3_attention_plan(lay, idx, len(act), ws)
    tuning("attn_wgs", 5)
    api.a3_fused_attention_planned(lay, q, idx, len(act), k, v, out, ws)
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())
    tuning("attn_wgs", -1)
    api.a3_fused_attention_planned(lay, q, idx, len(act), k, v, out, ws)
    torch.cuda.synchronize()
    assert max_abs_rel(to_host(out), res["out"]) <= tol(w)


@pytest.mark.parametrize("name", ["ragged-bf16", "batched-bf16-half", "cfg2", "cfg1"])
def test_attention_in_two_calls(name):
    """a3_attention_plan (on a second stream, ordered by events) + a3_fused_attention_planned give what
    a3_fused_attention gives, bit for bit; and the layer pass with and without that overlap agrees (the overlap
    is off by default: the cross-stream waits cost more than the plan kernel they hide)."""
    c = ctx_of(name)
    w, res, lay = c["w"], c["res"], c["lay"]
    s = w.shape
    dt = s.dtype
    act = res["act_idx"]
    q, k, v, idx = to_dev(res["q_act"], dt), to_dev(res["k_fused"], dt), to_dev(res["v_fused"], dt), idev(act)
    one = torch.zeros((len(act), s.n_q_heads, s.head_dim), dtype=api.torch_dtype(dt), device="cuda")
    two = torch.zeros_like(one)
    ws = lay.workspace(len(act))
    api.a3_fused_attention(lay, q, idx, len(act), k, v, one, ws)
    torch.cuda.synchronize()
    ws.zero_()
    side = torch.cuda.Stream()
    ready, planned = torch.cuda.Event(), torch.cuda.Event()
    ready.record()
    side.wait_event(ready)
    api.a3_attention_plan(lay, idx, len(act), ws, stream=side)
    planned.record(side)
    torch.cuda.current_stream().wait_event(planned)
    api.a3_fused_attention_planned(lay, q, idx, len(act), k, v, two, ws)
    torch.cuda.synchronize()
    assert torch.equal(one, two)
    b, t = c["b"], c["b"]["t"]
    outs = []
    for overlap in (False, True, True):
        bufs = layer.make_buffers(lay, w.sel_start, w.question_rows(), s)
        v_cache = to_dev(b["v_cat"], dt)
        layer.fuse_layer(lay, bufs, to_dev(t.x_cur, dt), to_dev(b["k_cat"], dt), v_cache, to_dev(t.wq, dt),
                         to_dev(t.wk, dt), to_dev(t.wv, dt), overlap_plan=overlap)
        torch.cuda.synchronize()
        outs.append((bufs.out[:bufs.n_act].clone(), bufs.act_idx[:bufs.n_act].clone()))
    for o, a in outs[1:]:
        assert torch.equal(a, outs[0][1]) and torch.equal(o, outs[0][0])
