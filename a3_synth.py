"""Seeded synthetic workloads for the A^3 KV-cache fusion path.

A module of its own, owned neither by the HIP library's package nor by the CPU oracle: both are fed from it.
It only draws random numbers and lays out index arrays.  It holds none of
the method's arithmetic (no RoPE, no projection, no softmax, no selection, not even the number of recomputed
tokens p = r * n of Eq. 3: whoever uses a workload says how that is counted, see ``use_recompute_count``): the
stale per-chunk K/V cache and the planted relevant tokens are produced by whoever
calls it (the tests do that with the CPU oracle, the benchmark draws the cache
directly with a matched standard deviation).

The shapes follow the paper's experimental setting (section "Experimental Settings":
512-token chunks, recompute ratio 0.15, Llama3-8B / Qwen2.5-7B sized layers) and the
input structure X = (S, D_1..D_k, Q) of section "Background": every request is a run
of context chunks followed by its question tokens, packed back to back:

    packed rows:  [ req0 ctx chunks | req0 question | req1 ctx chunks | req1 question | ... ]

All generators are NumPy PCG64 streams seeded with ``1000 * cfg + layer``.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Tuple

import numpy as np

_count_fn = None


def use_recompute_count(fn) -> None:
    """``fn(n_ctx, ratio_num, ratio_den) -> int``: how many context tokens of a request are recomputed (Eq. 3,
    p = r * n).  The library's binding and the oracle each bring their own; ``Workload.sel_start`` calls it."""
    global _count_fn
    _count_fn = fn


ROPE_INTERLEAVED = 0   # pairs (2i, 2i+1): the rotation matrix printed in "Position Recovery"
ROPE_HALF = 1          # pairs (i, i+d/2): the layout common runtimes use for Llama/Qwen checkpoints


@dataclass(frozen=True)
class ModelShape:
    name: str
    dtype: str            # "f32" or "bf16": storage type of every tensor on the path
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_base: float
    rope_layout: int = ROPE_INTERLEAVED
    ffn: int = 0                      # width of the gated MLP (only the layer stack uses it)
    rms_eps: float = 1e-5

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


TINY = ModelShape("tiny", "f32", 512, 8, 8, 64, 10000.0, ffn=1024)
LLAMA3_8B = ModelShape("llama3-8b", "bf16", 4096, 32, 8, 128, 500000.0, ffn=14336)
QWEN25_7B = ModelShape("qwen2.5-7b", "bf16", 3584, 28, 4, 128, 1000000.0, ffn=18944, rms_eps=1e-6)


@dataclass
class Workload:
    """Index structure of one batch of requests (no tensors)."""
    shape: ModelShape
    chunk_lens: List[np.ndarray]      # per request: int array of chunk lengths
    q_lens: np.ndarray                # [R]
    ratio: Tuple[int, int]            # recompute ratio as (numerator, denominator)
    n_planted: int = 0
    seed: int = 0
    name: str = ""
    # derived (filled by __post_init__)
    seg_start: np.ndarray = field(init=False)
    ctx_len: np.ndarray = field(init=False)
    chunk_start: np.ndarray = field(init=False)
    chunk_len: np.ndarray = field(init=False)
    chunk_delta: np.ndarray = field(init=False)
    chunk_req: np.ndarray = field(init=False)
    _sel_start: object = field(init=False, default=None, repr=False)

    def __post_init__(self):
        R = len(self.chunk_lens)
        self.q_lens = np.asarray(self.q_lens, dtype=np.int32)
        assert self.q_lens.shape == (R,)
        seg_start = np.zeros(R + 1, dtype=np.int32)
        ctx_len = np.zeros(R, dtype=np.int32)
        cs, cl, cd, cr = [], [], [], []
        row = 0
        for r in range(R):
            lens = np.asarray(self.chunk_lens[r], dtype=np.int32)
            seg_start[r] = row
            delta = 0
            for L in lens:
                cs.append(row + delta)
                cl.append(int(L))
                cd.append(delta)
                cr.append(r)
                delta += int(L)
            ctx_len[r] = delta
            row += delta + int(self.q_lens[r])
        seg_start[R] = row
        self.seg_start = seg_start
        self.ctx_len = ctx_len
        self.chunk_start = np.asarray(cs, dtype=np.int32)
        self.chunk_len = np.asarray(cl, dtype=np.int32)
        self.chunk_delta = np.asarray(cd, dtype=np.int32)
        self.chunk_req = np.asarray(cr, dtype=np.int32)

    @property
    def sel_start(self) -> np.ndarray:
        """[R+1] offsets of the requests' selections in a packed list; the counts come from the function given
        to ``use_recompute_count`` (this module does not know how p = r * n is rounded)."""
        if self._sel_start is None:
            if _count_fn is None:
                raise RuntimeError("a3_synth.use_recompute_count(fn) has not been called")
            num, den = self.ratio
            k = [int(_count_fn(int(n), int(num), int(den))) for n in self.ctx_len]
            self._sel_start = np.concatenate([[0], np.cumsum(k)]).astype(np.int32)
        return self._sel_start

    @sel_start.setter
    def sel_start(self, value) -> None:
        self._sel_start = np.asarray(value, dtype=np.int32)

    # ---- sizes -------------------------------------------------------------------
    @property
    def n_req(self) -> int:
        return len(self.chunk_lens)

    @property
    def n_chunks(self) -> int:
        return int(self.chunk_start.shape[0])

    @property
    def total_tokens(self) -> int:
        return int(self.seg_start[-1])

    @property
    def total_ctx(self) -> int:
        return int(self.ctx_len.sum())

    @property
    def total_q(self) -> int:
        return int(self.q_lens.sum())

    @property
    def total_k(self) -> int:
        return int(self.sel_start[-1])

    # ---- index helpers (pure bookkeeping) -------------------------------------------
    def ctx_rows(self, r: int) -> np.ndarray:
        s = int(self.seg_start[r])
        return np.arange(s, s + int(self.ctx_len[r]), dtype=np.int32)

    def question_rows(self, r: int | None = None) -> np.ndarray:
        rs = range(self.n_req) if r is None else [r]
        out = []
        for i in rs:
            s = int(self.seg_start[i]) + int(self.ctx_len[i])
            out.append(np.arange(s, s + int(self.q_lens[i]), dtype=np.int32))
        return np.concatenate(out) if out else np.zeros(0, np.int32)

    def token_positions(self) -> np.ndarray:
        """Global position of every packed row inside its own request."""
        pos = np.zeros(self.total_tokens, dtype=np.int32)
        for r in range(self.n_req):
            s, e = int(self.seg_start[r]), int(self.seg_start[r + 1])
            pos[s:e] = np.arange(e - s, dtype=np.int32)
        return pos

    def token_local_positions(self) -> np.ndarray:
        """Position every context row had when its chunk was precomputed on its own
        (0..len-1 inside each chunk); question rows keep their global position."""
        pos = self.token_positions()
        for c in range(self.n_chunks):
            s, L = int(self.chunk_start[c]), int(self.chunk_len[c])
            pos[s:s + L] = np.arange(L, dtype=np.int32)
        return pos

    def token_requests(self) -> np.ndarray:
        req = np.zeros(self.total_tokens, dtype=np.int32)
        for r in range(self.n_req):
            req[int(self.seg_start[r]):int(self.seg_start[r + 1])] = r
        return req

    def planted_rows(self) -> np.ndarray:
        """Seeded packed rows that will carry planted relevant tokens: spread round-robin
        over the chunks of each request at seeded offsets."""
        if self.n_planted == 0:
            return np.zeros(0, np.int32)
        rng = np.random.Generator(np.random.PCG64(self.seed + 777_000))
        rows = []
        per_req = self.n_planted
        for r in range(self.n_req):
            cids = np.nonzero(self.chunk_req == r)[0]
            for i in range(per_req):
                c = cids[i % len(cids)]
                off = int(rng.integers(0, int(self.chunk_len[c])))
                rows.append(int(self.chunk_start[c]) + off)
        return np.unique(np.asarray(rows, dtype=np.int32))


def _fixed_chunks(n_chunks: int, chunk: int) -> np.ndarray:
    return np.full(n_chunks, chunk, dtype=np.int32)


def config(cfg: int, layer: int = 0, rope_layout: int = ROPE_INTERLEAVED) -> Workload:
    """The five benchmark configurations.  ``layer`` only changes the seed (config 3 is a
    stack of 32 independent layer problems with the same index structure)."""
    seed = 1000 * cfg + layer
    lay = np.random.Generator(np.random.PCG64(1000 * cfg + 500_000))   # layout stream: layer independent

    def with_layout(s: ModelShape) -> ModelShape:
        return replace(s, rope_layout=rope_layout)

    if cfg == 1:
        return Workload(with_layout(TINY), [_fixed_chunks(4, 128)], [32], (15, 100), 4, seed, "cfg1-tiny-f32")
    if cfg == 2:
        return Workload(with_layout(LLAMA3_8B), [_fixed_chunks(10, 512)], [64], (15, 100), 16, seed,
                        "cfg2-llama3-8b-5k")
    if cfg == 3:
        return Workload(with_layout(LLAMA3_8B), [_fixed_chunks(32, 512)], [64], (10, 100), 0, seed,
                        "cfg3-llama3-8b-16k")
    if cfg == 4:
        lens = lay.integers(256, 769, size=64).astype(np.int32)
        return Workload(with_layout(QWEN25_7B), [lens], [128], (20, 100), 32, seed, "cfg4-qwen2.5-7b-32k")
    if cfg == 5:
        chunk_lens, q_lens = [], []
        for _ in range(8):
            while True:   # "16 chunks of 256..1024 tokens totalling about 8K": redraw until 7168 <= N <= 9216
                lens = lay.integers(256, 1025, size=16).astype(np.int32)
                if 7168 <= int(lens.sum()) <= 9216:
                    break
            chunk_lens.append(lens)
            q_lens.append(int(lay.integers(32, 129)))
        return Workload(with_layout(LLAMA3_8B), chunk_lens, q_lens, (15, 100), 0, seed, "cfg5-llama3-8b-batched")
    raise ValueError(f"unknown config {cfg}")


def custom(shape: ModelShape, chunk_lens, q_lens, ratio=(15, 100), n_planted=0, seed=0, name="custom") -> Workload:
    return Workload(shape, [np.asarray(c, dtype=np.int32) for c in chunk_lens], q_lens, ratio, n_planted, seed, name)


# ---- value draws -----------------------------------------------------------------------

def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an array once to the storage type and return it widened to float32
    (bf16 values are exactly representable in float32)."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x32
    if dtype == "bf16":
        import torch
        return torch.from_numpy(x32).to(torch.bfloat16).to(torch.float32).numpy()
    raise ValueError(dtype)


@dataclass
class Tensors:
    x_pre: np.ndarray    # [T, h]  hidden states the stale chunk caches were computed from
    x_cur: np.ndarray    # [T, h]  true hidden states of the concatenated prompt at this layer
    wq: np.ndarray       # [Hq*d, h]
    wk: np.ndarray       # [Hkv*d, h]
    wv: np.ndarray       # [Hkv*d, h]


def draw_tensors(w: Workload, stale_equals_current: bool = False) -> Tensors:
    """hidden ~ N(0,1), weights ~ N(0, 0.02^2), all rounded once to the storage type.

    Context rows of ``x_cur`` differ from ``x_pre`` (the chunk-only prefill saw different
    hidden states than the full prompt produces): x_cur = (x_pre + 0.5 z) / sqrt(1.25).
    Question rows share a common component, x_j = 0.7 u + 0.7 z_j, so that their mean
    query is long enough for planted keys to align with it.
    """
    s = w.shape
    rng = np.random.Generator(np.random.PCG64(w.seed))
    T, h = w.total_tokens, s.hidden
    x_pre = rng.standard_normal((T, h), dtype=np.float32)
    if stale_equals_current:
        x_cur = x_pre.copy()
    else:
        z = rng.standard_normal((T, h), dtype=np.float32)
        x_cur = (x_pre + np.float32(0.5) * z) / np.float32(np.sqrt(1.25))
    for r in range(w.n_req):
        rows = w.question_rows(r)
        u = rng.standard_normal((1, h), dtype=np.float32)
        zq = rng.standard_normal((len(rows), h), dtype=np.float32)
        xq = np.float32(0.7) * u + np.float32(0.7) * zq
        x_pre[rows] = xq
        x_cur[rows] = xq
    wq = rng.standard_normal((s.n_q_heads * s.head_dim, h), dtype=np.float32) * np.float32(0.02)
    wk = rng.standard_normal((s.n_kv_heads * s.head_dim, h), dtype=np.float32) * np.float32(0.02)
    wv = rng.standard_normal((s.n_kv_heads * s.head_dim, h), dtype=np.float32) * np.float32(0.02)
    r2s = lambda a: round_to_storage(a, s.dtype)
    return Tensors(r2s(x_pre), r2s(x_cur), r2s(wq), r2s(wk), r2s(wv))


def draw_cache(w: Workload, which: str) -> np.ndarray:
    """A stale K or V cache drawn directly as N(0, sigma^2), sigma = 0.02 * sqrt(hidden):
    the standard deviation a projection of N(0,1) hidden states by N(0,0.02^2) weights has.
    For throughput runs, where synthesising the cache through a real projection would cost
    far more host time than the measurement itself."""
    s = w.shape
    rng = np.random.Generator(np.random.PCG64(w.seed + (111_000 if which == "k" else 222_000)))
    sigma = np.float32(0.02 * np.sqrt(s.hidden))
    x = rng.standard_normal((w.total_tokens, s.n_kv_heads, s.head_dim), dtype=np.float32) * sigma
    return round_to_storage(x, s.dtype)


def draw_stack_weights(w: Workload, n_layers: int) -> dict:
    """Weights of ``n_layers`` decoder blocks and the embedding output of every packed row, all rounded
    once to the storage type: projections and MLP ~ N(0, 0.02^2) (the output projections wo and w_down
    scaled by 1/sqrt(2 n_layers), the usual residual-branch scaling), norm weights 1 + 0.1 z, embedding
    rows ~ N(0,1) with the common question component of ``draw_tensors``.
    Returns dict(resid0 [T,h], g_final [h], layers=[dict(wq, wk, wv, wo, g_in, g_post, w_gate, w_up, w_down)])."""
    s = w.shape
    assert s.ffn > 0
    rng = np.random.Generator(np.random.PCG64(w.seed + 333_000))
    T, h, f = w.total_tokens, s.hidden, s.ffn
    r2s = lambda a: round_to_storage(a, s.dtype)
    resid0 = rng.standard_normal((T, h), dtype=np.float32)
    for r in range(w.n_req):
        rows = w.question_rows(r)
        u = rng.standard_normal((1, h), dtype=np.float32)
        resid0[rows] = np.float32(0.7) * u + np.float32(0.7) * rng.standard_normal((len(rows), h), dtype=np.float32)
    branch = np.float32(1.0 / np.sqrt(2.0 * n_layers))
    nrm = lambda *shape: rng.standard_normal(shape, dtype=np.float32) * np.float32(0.02)
    gain = lambda: np.float32(1.0) + np.float32(0.1) * rng.standard_normal(h, dtype=np.float32)
    layers = []
    for _ in range(n_layers):
        layers.append(dict(
            wq=r2s(nrm(s.n_q_heads * s.head_dim, h)), wk=r2s(nrm(s.n_kv_heads * s.head_dim, h)),
            wv=r2s(nrm(s.n_kv_heads * s.head_dim, h)), wo=r2s(nrm(h, s.n_q_heads * s.head_dim) * branch),
            g_in=r2s(gain()), g_post=r2s(gain()),
            w_gate=r2s(nrm(f, h)), w_up=r2s(nrm(f, h)), w_down=r2s(nrm(h, f) * branch)))
    return dict(resid0=r2s(resid0), g_final=r2s(gain()), layers=layers)
