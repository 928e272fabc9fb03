"""GPU parity of the selection-score variant with the literal denominator of Eq. 3 and of the eviction
extension (window votes, per-head retention, compaction) against the CPU oracle, teacher forced on the
oracle's per-layer results.

Tolerances: scores and votes 1e-4 (max |a-b| / max |b|); retained row lists and compacted caches bit-exact
(the ranking is taken on the same float32 votes on both sides; pooling is done in float32 on both sides).
"""
import numpy as np
import pytest
import torch

from oracle import a3_oracle as ora
from oracle import evict_oracle as ev
import a3_synth as synth
from paper_2511_17560_amd import api
from gpu_util import idev, max_abs_rel, to_dev, to_host
from test_gpu_parity import ctx_of

pytestmark = pytest.mark.gpu

NAMES = ["cfg1", "ragged-bf16", "batched-bf16-half", "g7-bf16", "batched-f32-d128", "cfg2", "manyq-bf16",
         "manyq-g7-bf16"]


def _inputs(name):
    c = ctx_of(name)
    w, res, lay = c["w"], c["res"], c["lay"]
    kw = dict(seg_start=w.seg_start, ctx_len=w.ctx_len, q_len=w.q_lens)
    scale = 1.0 / np.sqrt(w.shape.head_dim)
    return c, w, res, lay, kw, scale


@pytest.mark.parametrize("name", NAMES)
def test_question_scores_causal(name):
    c, w, res, lay, kw, scale = _inputs(name)
    dt = w.shape.dtype
    want = ev.question_scores_causal(res["q_question"], res["k_fused"], sm_scale=scale, **kw)
    scores = torch.zeros(w.total_tokens, dtype=torch.float32, device="cuda")
    api.a3_question_scores_causal(lay, to_dev(res["q_question"], dt), to_dev(res["k_fused"], dt), scores,
                                  lay.workspace(w.total_k + w.total_q))
    torch.cuda.synchronize()
    got = to_host(scores)
    ctx = np.concatenate([w.ctx_rows(r) for r in range(w.n_req)])
    assert max_abs_rel(got[ctx], want[ctx]) <= 1e-4
    assert np.all(np.isneginf(got[w.question_rows()]))
    # it is a different score from the context-normalised one on the same keys, and never larger
    plain = ora.question_scores(res["q_question"], res["k_fused"], w.seg_start, w.ctx_len, w.q_lens, scale)
    assert np.all(got[ctx] <= plain[ctx] * (1 + 1e-4) + 1e-6)
    assert np.abs(got[ctx] - plain[ctx]).max() > 1e-3 * np.abs(plain[ctx]).max()


@pytest.mark.parametrize("name", NAMES)
def test_window_votes_select_compact(name):
    c, w, res, lay, kw, scale = _inputs(name)
    s = w.shape
    dt = s.dtype
    votes_q = ev.window_votes(res["q_question"], res["k_fused"], sm_scale=scale, **kw)
    want = ev.kv_head_votes(votes_q, s.n_kv_heads)
    votes = torch.zeros((s.n_kv_heads, w.total_tokens), dtype=torch.float32, device="cuda")
    k_dev, v_dev = to_dev(res["k_fused"], dt), to_dev(res["v_fused"], dt)
    api.a3_window_votes(lay, to_dev(res["q_question"], dt), k_dev, votes, lay.workspace(0))
    torch.cuda.synchronize()
    ctx = np.concatenate([w.ctx_rows(r) for r in range(w.n_req)])
    got = to_host(votes)
    assert max_abs_rel(got[:, ctx], want[:, ctx]) <= 1e-4
    # each head's votes are a share of the per-layer score with the literal denominator
    lit = ev.question_scores_causal(res["q_question"], res["k_fused"], sm_scale=scale, **kw)
    assert max_abs_rel(got[:, ctx].sum(0), lit[ctx]) <= 1e-4

    # retention, teacher forced on the oracle's votes (float32), three capacities and the pooling modes
    votes32 = want.astype(np.float32)
    rng = np.random.default_rng(5)
    sys_len = np.array([min(int(rng.integers(0, 40)), int(n)) for n in w.ctx_len], dtype=np.int32)
    for capacity, width, mode in [(int(w.ctx_len.max()) // 3, 1, "max"), (64, 7, "max"), (int(w.ctx_len.min()) // 2 + 50, 5, "avg"),
                                  (10 ** 6, 1, "max"), (1, 3, "max")]:
        ranked = ev.pool_votes(votes32, w.seg_start, w.ctx_len, width, mode)
        assert ranked.dtype == np.float32
        keep_want, keep_start = ev.evict_select(ranked, w.seg_start, w.ctx_len, w.q_lens, sys_len, capacity)
        total_keep = int(keep_start[-1])
        keep = torch.full((s.n_kv_heads, max(total_keep, 1)), -1, dtype=torch.int32, device="cuda")
        ws = torch.empty(api.a3_evict_ws_bytes(lay), dtype=torch.uint8, device="cuda")
        api.a3_evict_select(lay, torch.from_numpy(votes32).cuda(), idev(sys_len), idev(keep_start), total_keep, keep,
                            pool_width=width, pool_mode=api.A3_POOL_MAX if mode == "max" else api.A3_POOL_AVG, ws=ws)
        torch.cuda.synchronize()
        assert np.array_equal(keep.cpu().numpy()[:, :total_keep], keep_want), (capacity, width, mode)
        # the eviction itself
        k_out = torch.zeros((max(total_keep, 1), s.n_kv_heads, s.head_dim), dtype=k_dev.dtype, device="cuda")
        v_out = torch.zeros_like(k_out)
        api.a3_evict_compact(lay, k_dev, v_dev, keep, total_keep, k_out, v_out)
        torch.cuda.synchronize()
        kw_, vw_ = ev.evict_compact(res["k_fused"], res["v_fused"], keep_want)
        assert np.array_equal(to_host(k_out)[:total_keep], kw_) and np.array_equal(to_host(v_out)[:total_keep], vw_)


def test_evict_on_the_gpus_own_votes_16k():
    """Config 3 at full size, chained on the GPU: votes -> retention at C = 1024 (the paper's setting) ->
    compaction.  Checked by properties that hold at any size: per head the list is ascending, starts with the
    system prompt, ends with the question, holds C rows, and no evicted row has a larger vote than a kept
    one; the compacted cache holds the listed rows."""
    c, w, res, lay, kw, scale = _inputs("cfg3-layer0")
    s = w.shape
    dt = s.dtype
    k_dev, v_dev = to_dev(res["k_fused"], dt), to_dev(res["v_fused"], dt)
    votes = torch.zeros((s.n_kv_heads, w.total_tokens), dtype=torch.float32, device="cuda")
    api.a3_window_votes(lay, to_dev(res["q_question"], dt), k_dev, votes, lay.workspace(0))
    C, S, N, nq = 1024, 37, int(w.ctx_len[0]), int(w.q_lens[0])
    keep_start = np.array([0, C], dtype=np.int32)
    keep = torch.full((s.n_kv_heads, C), -1, dtype=torch.int32, device="cuda")
    api.a3_evict_select(lay, votes, idev([S]), idev(keep_start), C, keep)
    k_out = torch.zeros((C, s.n_kv_heads, s.head_dim), dtype=k_dev.dtype, device="cuda")
    v_out = torch.zeros_like(k_out)
    api.a3_evict_compact(lay, k_dev, v_dev, keep, C, k_out, v_out)
    torch.cuda.synchronize()
    kp, vt = keep.cpu().numpy(), votes.cpu().numpy()
    for g in range(s.n_kv_heads):
        assert np.all(np.diff(kp[g]) > 0)
        assert np.array_equal(kp[g, :S], np.arange(S)) and np.array_equal(kp[g, C - nq:], np.arange(N, N + nq))
        mid = kp[g, S:C - nq]
        others = np.setdiff1d(np.arange(S, N), mid)
        assert vt[g, mid].min() >= vt[g, others].max()
        assert torch.equal(k_out[:, g], k_dev[keep[g].long(), g]) and torch.equal(v_out[:, g], v_dev[keep[g].long(), g])
    # and the votes themselves against the oracle, all 8 x 16384 of them
    want = ev.kv_head_votes(ev.window_votes(res["q_question"], res["k_fused"], sm_scale=scale, **kw), s.n_kv_heads)
    assert max_abs_rel(vt[:, :N], want[:, :N]) <= 1e-4


# ---------------------------------------------------------------------------------------
# alternative producers of the recompute list
# ---------------------------------------------------------------------------------------
from oracle import selectors_oracle as sel_ora   # noqa: E402


@pytest.mark.parametrize("name", NAMES)
def test_value_deviation_scores_and_selection(name):
    """|V_true - V_cat|^2 per context row (1e-5), then the unchanged top-p on the GPU's own scores: checked by
    the property that defines it (no unselected row scores higher than a selected one, count and order)."""
    c, w, res, lay, kw, scale = _inputs(name)
    s, t, b = w.shape, c["b"]["t"], c["b"]
    dt = s.dtype
    rows = np.arange(w.total_tokens)
    _, _, v_true = ora.selected_qkv_proj(t.x_cur, rows, w.token_positions(), t.wq, t.wk, t.wv, s.n_q_heads, s.n_kv_heads,
                                         s.head_dim, s.rope_base, s.rope_layout, dt)
    want = sel_ora.value_deviation_scores(v_true, b["v_cat"], w.seg_start, w.ctx_len)
    scores = torch.zeros(w.total_tokens, dtype=torch.float32, device="cuda")
    api.a3_value_deviation_scores(lay, to_dev(v_true, dt), to_dev(b["v_cat"], dt), scores)
    sel = torch.full((max(w.total_k, 1),), -1, dtype=torch.int32, device="cuda")
    api.a3_topk_select(lay, scores, idev(w.sel_start), w.total_k, sel)
    torch.cuda.synchronize()
    got = to_host(scores)
    ctx = np.concatenate([w.ctx_rows(r) for r in range(w.n_req)])
    assert max_abs_rel(got[ctx], want[ctx]) <= 1e-5
    assert np.all(np.isneginf(got[w.question_rows()]))
    picked = sel.cpu().numpy()[:w.total_k]
    for r in range(w.n_req):
        mine = picked[w.sel_start[r]:w.sel_start[r + 1]]
        assert np.all(np.diff(mine) > 0) and np.all(np.isin(mine, w.ctx_rows(r)))
        rest = np.setdiff1d(w.ctx_rows(r), mine)
        if len(mine) and len(rest):
            assert got[mine].min() >= got[rest].max()
    # and it is the oracle's list wherever the oracle's ranking is not a near-tie
    want_sel = ora.topk_select(want, w.seg_start, w.ctx_len, w.sel_start)
    flips = set(picked.tolist()) ^ set(want_sel.tolist())
    assert len(flips) <= max(2, w.total_k // 50)


@pytest.mark.parametrize("name", NAMES)
@pytest.mark.parametrize("n_head,n_tail", [(20, 20), (3, 0), (0, 5), (600, 600), (0, 0)])
def test_select_chunk_edges(name, n_head, n_tail):
    c, w, res, lay, kw, scale = _inputs(name)
    want_idx, want_start = sel_ora.chunk_edge_rows(w.seg_start, w.ctx_len, w.chunk_start, w.chunk_len, n_head, n_tail)
    start = api.a3_chunk_edge_sel_start(w.seg_start, w.ctx_len, w.chunk_start, w.chunk_len, n_head, n_tail)
    assert np.array_equal(start, want_start)
    total = int(start[-1])
    out = torch.full((max(total, 1),), -1, dtype=torch.int32, device="cuda")
    api.a3_select_chunk_edges(lay, n_head, n_tail, idev(start), total, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy()[:total], want_idx)
