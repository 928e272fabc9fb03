#!/usr/bin/env python3
"""Benchmark of the per-layer A^3 KV-cache fusion path on one MI355X.

A step is one pass of the whole path (question projection, key realign + scores, top-p,
selected projection with cache update, attention) over one layer of the 16K-context
configuration: Llama-3-8B-shaped layer, 32 chunks x 512 tokens + 64 question tokens,
recompute ratio 10%.  The 32 layers of that configuration are 32 independent sets of buffers
that the steps cycle through, so every step starts with its tensors cold in cache.

Prints ONE JSON line: fused-context tokens/s per layer, the roofline of the dominant kernel
(the attention kernel, against the dense bf16 MFMA peak) and the CPU oracle timed on the host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def draw_layer(torch, w, layer_idx, device):
    """Seeded synthetic tensors of one layer, drawn on the device (same distributions as the
    host generator: hidden ~ N(0,1) with a shared component on the question rows, weights
    ~ N(0, 0.02^2), stale cache ~ N(0, (0.02 sqrt(hidden))^2))."""
    s = w.shape
    g = torch.Generator(device=device)
    g.manual_seed(w.seed * 1000 + layer_idx)
    dt = torch.bfloat16 if s.dtype == "bf16" else torch.float32
    T, h = w.total_tokens, s.hidden
    x = torch.randn((T, h), generator=g, device=device, dtype=torch.float32)
    for r in range(w.n_req):
        rows = torch.as_tensor(w.question_rows(r), device=device, dtype=torch.long)
        u = torch.randn((1, h), generator=g, device=device)
        x[rows] = 0.7 * u + 0.7 * x[rows]
    sigma = 0.02 * (h ** 0.5)
    mk = lambda *shape, std=1.0: (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std).to(dt)
    return dict(
        x=x.to(dt),
        wq=mk(s.n_q_heads * s.head_dim, h, std=0.02),
        wk=mk(s.n_kv_heads * s.head_dim, h, std=0.02),
        wv=mk(s.n_kv_heads * s.head_dim, h, std=0.02),
        k_cat=mk(T, s.n_kv_heads, s.head_dim, std=sigma),
        v=mk(T, s.n_kv_heads, s.head_dim, std=sigma),
    )


def algorithmic_work(w, act_positions):
    """Flops / bytes per step that the method itself requires (not what a kernel happens to move)."""
    s = w.shape
    b = 2 if s.dtype == "bf16" else 4
    N, nq, k = w.total_ctx, w.total_q, w.total_k
    n_act = k + nq
    row = s.n_kv_heads * s.head_dim * b
    visible = int(sum(int(p) + 1 for p in act_positions))
    return {
        "realign_bytes": 2 * N * row,
        "scores_bytes": N * row,
        "scores_flops": 2 * sum(int(c) * int(q) for c, q in zip(w.ctx_len, w.q_lens)) * s.n_q_heads * s.head_dim,
        "proj_flops": 2 * n_act * s.hidden * (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim,
        "scatter_bytes": 4 * n_act * row,
        "attn_flops": 4 * s.n_q_heads * s.head_dim * visible,
        "visible_row_keys": visible,
    }


def measured_traffic(workload_name):
    """HBM bytes per launch of the attention kernel, from the committed summary of two rocprofv3 --pmc
    runs (FETCH_SIZE, WRITE_SIZE) scaled by the copy kernel of known size; None if there is none for
    this workload."""
    path = os.path.join(ROOT, "profiles", "attention_cfg3_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":", 1)
        vals[k.strip()] = v.strip()
    if vals.get("workload") != workload_name:
        return None
    try:
        return float(vals["traffic_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def cpu_baseline(cfg, max_seconds=60.0):
    """The CPU oracle, as it is (float64 NumPy), on layers of the same configuration, on the host's cores; plus
    the time of one layer of configurations 1 and 2 with the BLAS pool held to one thread."""
    import numpy as np
    from threadpoolctl import threadpool_info, threadpool_limits
    from oracle import a3_oracle as ora
    from oracle import workload as wl
    import a3_synth as synth

    def one_layer(w):
        t = synth.draw_tensors(w)
        k_cat, v_cat = synth.draw_cache(w, "k"), synth.draw_cache(w, "v")
        t0 = time.perf_counter()
        res = ora.fuse_layer(t.x_cur, k_cat, v_cat, t.wq, t.wk, t.wv, **wl.layout_kwargs(w))
        return time.perf_counter() - t0, int(len(res["sel_idx"]))

    dt, n_layers, n_sel = 0.0, 0, 0
    for layer_i in range(3):                     # three of the 32 layers: about 10 s of CPU work
        w = synth.config(cfg, layer=layer_i)
        sec, n_sel = one_layer(w)
        dt += sec
        n_layers += 1
        if dt > max_seconds:
            break
    threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] + [1])
    single = {}
    with threadpool_limits(limits=1):
        for c in (1, 2):
            single[f"cfg{c}"] = round(one_layer(synth.config(c))[0], 3)
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return {
        "value": n_layers * w.total_ctx / dt, "unit": "fused-context tokens/s/layer", "cores": int(threads), "kind": "oracle",
        "sample": f"{n_layers} of the 32 layers of {w.name} (float64 NumPy oracle, all steps, stale cache drawn directly), "
                  f"{dt:.1f} s wall",
        "seconds": dt, "n_selected": n_sel, "oracle_dtype": "float64", "nproc": os.cpu_count(), "usable_cpus": usable,
        "blas_threads": int(threads), "one_thread_seconds_per_layer": single,
    }


def stack_main(args):
    """--stack L: the A^3 schedule over L decoder blocks (block 0 on every row, selection at layer 1, rows
    [Re, Q] afterwards) against the plain prefill of the same stack, both through the same library.  Weights,
    embedding output and chunk caches are drawn on the device (N(0, 0.02^2) weights, N(0, 1) rows, caches with
    the matched standard deviation)."""
    import numpy as np
    import torch
    import a3_synth as synth
    from paper_2511_17560_amd import api, stack
    synth.use_recompute_count(api.a3_recompute_count)

    w = synth.config(args.config)
    s = w.shape
    dt = api.torch_dtype(s.dtype)
    lay = api.Layout.from_workload(w)
    T, h, f, qd, kd = w.total_tokens, s.hidden, s.ffn, s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    g = torch.Generator(device="cuda").manual_seed(1000 * args.config + 7)
    mk = lambda *shape, std=0.02: (torch.randn(*shape, device="cuda", generator=g) * std).to(dt)
    branch = 1.0 / (2.0 * args.stack) ** 0.5
    layers = [dict(wq=mk(qd, h), wk=mk(kd, h), wv=mk(kd, h), wo=mk(h, qd, std=0.02 * branch), g_in=mk(h, std=0.1) + 1,
                   g_post=mk(h, std=0.1) + 1, w_gate=mk(f, h), w_up=mk(f, h), w_down=mk(h, f, std=0.02 * branch))
              for _ in range(args.stack)]
    g_final = mk(h, std=0.1) + 1
    resid0 = mk(T, h, std=1.0)
    sigma = 0.02 * h ** 0.5
    k_cat = [None, None] + [mk(T, s.n_kv_heads, s.head_dim, std=sigma) for _ in range(args.stack - 2)]
    v_cat = [None, None] + [mk(T, s.n_kv_heads, s.head_dim, std=sigma) for _ in range(args.stack - 2)]
    q_rows = w.question_rows()
    resid = torch.empty_like(resid0)

    def timed(fn, steps, warmup):
        ms = []
        for i in range(warmup + steps):
            resid.copy_(resid0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            out = fn()
            e1.record()
            torch.cuda.synchronize()
            if i >= warmup:
                ms.append(e0.elapsed_time(e1))
        return float(np.mean(ms)), out

    steps, warmup = max(1, min(args.steps, 16)), max(1, min(args.warmup, 2))
    fuse_ms, out = timed(lambda: stack.fuse_stack(lay, s, layers, g_final, resid, k_cat, v_cat, w.sel_start, q_rows),
                         steps, warmup)
    act = out["act_idx"].cpu().numpy()
    assert out["n_act"] == w.total_k + w.total_q and np.all(np.diff(act) > 0)
    assert bool(torch.isfinite(out["hidden"][out["act_idx"].long()].float()).all())
    full_ms, _ = timed(lambda: stack.prefill_stack(lay, s, layers, g_final, resid), max(1, steps // 4), 1)
    streamed_ms = streamed_q8_ms = file_q8_ms = None
    if args.stream_caches:
        from paper_2511_17560_amd import loader
        host_k = [None if c is None else [c[s0:s0 + n].cpu().pin_memory() for s0, n in zip(w.chunk_start, w.chunk_len)]
                  for c in k_cat]
        host_v = [None if c is None else [c[s0:s0 + n].cpu().pin_memory() for s0, n in zip(w.chunk_start, w.chunk_len)]
                  for c in v_cat]
        cs = loader.ChunkCacheStream(lay, s, w.chunk_start, w.chunk_len, host_k, host_v, depth=2)
        streamed_ms, _ = timed(lambda: stack.fuse_stack(lay, s, layers, g_final, resid, None, None, w.sel_start, q_rows,
                                                        cache_stream=cs), steps, warmup)
        del cs, host_k, host_v
        # the same with 8-bit blocks (quantised once by a3_quantize_q8, as a chunk store would hold them)
        row = api.a3_q8_row_bytes(lay)
        host_q8 = []
        for kc, vc in zip(k_cat, v_cat):
            if kc is None:
                host_q8.append(None)
                continue
            rec = torch.empty((T, row), dtype=torch.uint8, device="cuda")
            api.a3_quantize_q8(lay, kc, vc, rec)
            rec = rec.cpu()
            host_q8.append([rec[s0:s0 + n].contiguous().pin_memory() for s0, n in zip(w.chunk_start, w.chunk_len)])
        cs8 = loader.ChunkCacheStream(lay, s, w.chunk_start, w.chunk_len, host_q8, None, depth=2)
        streamed_q8_ms, _ = timed(lambda: stack.fuse_stack(lay, s, layers, g_final, resid, None, None, w.sel_start,
                                                           q_rows, cache_stream=cs8), steps, warmup)
        del cs8
        # and with the records in files (one per chunk, layer after layer; written just now, so the reads are served
        # from the page cache: what is timed is the path, not a disk)
        import os
        import tempfile
        with tempfile.TemporaryDirectory() as tmp:
            paths = []
            for ci in range(len(w.chunk_start)):
                paths.append(os.path.join(tmp, f"chunk{ci}.q8"))
                with open(paths[-1], "wb") as fh:
                    for blocks_l in host_q8:
                        if blocks_l is not None:
                            fh.write(blocks_l[ci].numpy().tobytes())
            fs = loader.ChunkFileStream(lay, s, w.chunk_start, w.chunk_len, paths, args.stack, depth=3, io_threads=8)
            try:
                file_q8_ms, _ = timed(lambda: stack.fuse_stack(lay, s, layers, g_final, resid, None, None, w.sel_start,
                                                               q_rows, cache_stream=fs), steps, warmup)
            finally:
                fs.close()
    n_act = out["n_act"]
    # H(.) alone at the active rows: the call that dominates a layer once the rows are few
    attn_out = mk(n_act, s.n_q_heads, s.head_dim, std=1.0)
    ws = torch.empty(api.a3_block_tail_ws_bytes(lay, f, n_act), dtype=torch.uint8, device="cuda")
    lw = layers[2 % args.stack]
    hid = torch.empty_like(resid)
    call = lambda: api.a3_block_tail(lay, attn_out, out["act_idx"], n_act, lw["wo"], lw["g_post"], lw["w_gate"],
                                     lw["w_up"], lw["w_down"], g_final, s.rms_eps, resid, hid, ws)
    for _ in range(3):
        call()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        call()
    e1.record()
    torch.cuda.synchronize()
    tail_us = e0.elapsed_time(e1) * 1e3 / 20
    tail_flops = 2.0 * n_act * (qd * h + 3 * h * f)
    # eviction extension on one layer's cache: votes of the question window, retention at C = 1024 per KV head
    # (system prompt of 32 rows and the question always kept), compaction of K and V
    C, S = 1024, 32
    budget = [min(max(C - S - int(q), 0), int(n) - S) for n, q in zip(w.ctx_len, w.q_lens)]
    keep_start = np.concatenate([[0], np.cumsum([S + b + int(q) for b, q in zip(budget, w.q_lens)])]).astype(np.int32)
    total_keep = int(keep_start[-1])
    dev_i32 = lambda a: torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device="cuda")
    sys_len_d, keep_start_d = dev_i32([S] * w.n_req), dev_i32(keep_start)
    q_question = mk(w.total_q, s.n_q_heads, s.head_dim, std=1.0)
    kc = k_cat[2] if args.stack > 2 else mk(T, s.n_kv_heads, s.head_dim, std=sigma)
    vc = v_cat[2] if args.stack > 2 else mk(T, s.n_kv_heads, s.head_dim, std=sigma)
    votes = torch.empty((s.n_kv_heads, T), dtype=torch.float32, device="cuda")
    keep = torch.empty((s.n_kv_heads, total_keep), dtype=torch.int32, device="cuda")
    k_ev = torch.empty((total_keep, s.n_kv_heads, s.head_dim), dtype=dt, device="cuda")
    v_ev = torch.empty_like(k_ev)
    ws_e = lay.workspace(0)

    def evict():
        api.a3_window_votes(lay, q_question, kc, votes, ws_e)
        api.a3_evict_select(lay, votes, sys_len_d, keep_start_d, total_keep, keep)
        api.a3_evict_compact(lay, kc, vc, keep, total_keep, k_ev, v_ev)

    for _ in range(3):
        evict()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        evict()
    e1.record()
    torch.cuda.synchronize()
    evict_us = e0.elapsed_time(e1) * 1e3 / 20
    print(json.dumps({
        "metric": f"time of the A^3 schedule over {args.stack} decoder blocks (embedding output to final hidden "
                  "states of the rows [Re, Q])",
        "value": fuse_ms, "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": fuse_ms,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": s.dtype, "data": "synthetic",
        "config": {"workload": w.name, "blocks": args.stack, "ctx_tokens": w.total_ctx, "question_tokens": w.total_q,
                   "selected_tokens": w.total_k, "requests": w.n_req,
                   "shape": f"h{s.hidden}/Hq{s.n_q_heads}/Hkv{s.n_kv_heads}/d{s.head_dim}/ffn{s.ffn}"},
        "full_prefill_ms": full_ms, "speedup_over_full_prefill": full_ms / fuse_ms,
        "streamed_caches_ms": streamed_ms,
        "streamed_cache_bytes": None if streamed_ms is None else
        2 * (args.stack - 2) * int(w.total_ctx) * kd * (2 if s.dtype == "bf16" else 4),
        "streamed_q8_caches_ms": streamed_q8_ms,
        "file_q8_caches_ms": file_q8_ms,
        "streamed_q8_cache_bytes": None if streamed_q8_ms is None else
        (args.stack - 2) * int(w.total_ctx) * row,
        "block_tail": {"us_per_call": round(tail_us, 1), "rows": n_act, "flops_per_call": tail_flops,
                       "achieved_TFLOPs": round(tail_flops / tail_us / 1e6, 1),
                       "frac_of_mfma_peak": tail_flops / tail_us / 1e6 / PEAK_BF16_TFLOPS},
        "eviction": {"capacity": C, "system_prompt_rows": S, "us_per_layer": round(evict_us, 1),
                     "ms_all_layers": round(evict_us * args.stack / 1e3, 3), "rows_kept_per_head": total_keep},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--config", type=int, default=3, help="workload configuration 1..5 (3 = the 16K-context metric)")
    ap.add_argument("--layers", type=int, default=0, help="independent layer buffer sets to cycle (0 = 32 for config 3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stream-caches", action="store_true",
                    help="with --stack: also time the schedule with the chunk caches streamed from pinned host memory "
                         "layer by layer (a3_chunk_cache_load on a copy stream) instead of resident in HBM")
    ap.add_argument("--two-streams", action="store_true",
                    help="also time the same steps issued alternately on two streams (derived.two_streams_us_per_step; "
                         "never the headline value)")
    ap.add_argument("--stack", type=int, default=0,
                    help="L >= 2: time the A^3 schedule over L decoder blocks against the plain prefill of the same "
                         "stack instead of the per-layer hot path (not the headline metric)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB float32 copy kernel (torch.mul by 1) three times: the known-size "
                         "dispatch that scales the HBM byte counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.stack:
        if args.stack < 2:
            print("bench.py: --stack needs at least 2 blocks", file=sys.stderr)
            sys.exit(2)
        return stack_main(args)

    import numpy as np
    import torch
    import a3_synth as synth
    from paper_2511_17560_amd import api, layer
    synth.use_recompute_count(api.a3_recompute_count)

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    api.lib()                                   # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    w = synth.config(args.config)
    s = w.shape
    n_layers = args.layers or (32 if args.config == 3 else 4)
    lay = api.Layout.from_workload(w)
    layers = [draw_layer(torch, w, i, dev) for i in range(n_layers)]
    bufs = [layer.make_buffers(lay, w.sel_start, w.question_rows(), s) for _ in range(n_layers)]
    torch.cuda.synchronize()

    def step(i):
        L, B = layers[i % n_layers], bufs[i % n_layers]
        layer.fuse_layer(lay, B, L["x"], L["k_cat"], L["v"], L["wq"], L["wk"], L["wv"])

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # set-up, outside the warm-up / steps accounting: every buffer set is run once, so that first-use costs (page
    # mappings of the 32 sets, kernel attributes) do not land in the timed region when --warmup is small
    for i in range(n_layers):
        step(i)
    torch.cuda.synchronize()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly --steps steps.  Inside it the dominant call is bracketed twice on the stream the
    # kernels run on: torch events around the whole a3_fused_attention_planned call (main kernel + the kernel that
    # merges partial results; the work layout was made by a3_topk_select_plan), raw HIP events recorded by the
    # library right before / after the main kernel alone.
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")

    def raw_event():
        e = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def raw_elapsed_ms(e0, e1):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
        return ms.value

    attn_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    main_ev = [(raw_event(), raw_event()) for _ in range(args.steps)]
    attn_name = "a3_fused_attention_planned"
    orig_attn = getattr(api, attn_name)
    cur = {"i": 0}

    def timed_attn(layout, q_act, act_idx, n_act, k_fused, v_fused, out, ws, stream=None):
        e0, e1 = attn_ev[cur["i"]]
        m0, m1 = main_ev[cur["i"]]
        e0.record()
        api.a3_fused_attention_planned_events(layout, q_act, act_idx, n_act, k_fused, v_fused, out, ws, m0.value, m1.value,
                                              stream=stream)
        e1.record()

    setattr(api, attn_name, timed_attn)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        cur["i"] = i
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    setattr(api, attn_name, orig_attn)
    attn_ms = float(np.mean([a.elapsed_time(b) for a, b in attn_ev]))
    attn_main_ms = float(np.mean([raw_elapsed_ms(a, b) for a, b in main_ev]))
    for a, b in main_ev:
        hip.hipEventDestroy(a)
        hip.hipEventDestroy(b)

    # ---- the same steps on two streams, alternately (outside the timed region) -----------------
    two_streams_ms = None
    if args.two_streams and n_layers >= 2:
        pair = [torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)]      # default priority
        torch.cuda.synchronize()

        def step2(i):
            L, B = layers[i % n_layers], bufs[i % n_layers]
            layer.fuse_layer(lay, B, L["x"], L["k_cat"], L["v"], L["wq"], L["wk"], L["wv"], stream=pair[i % 2])

        for i in range(min(args.warmup, 8)):
            step2(i)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for i in range(args.steps):
            step2(i)
        torch.cuda.synchronize()
        two_streams_ms = (time.perf_counter() - t2) * 1e3 / args.steps

    # ---- per-call breakdown (outside the timed region) ----------------------------------------
    # once with the sequence that was timed (one call for realign + scores, projections write K/V
    # straight into the caches) and once with the plain six-call sequence (a3_rope_realign,
    # a3_question_scores, a3_selected_qkv_proj + a3_kv_scatter), so every entry point is reported
    names = ["a3_selected_qkv_proj", "a3_selected_qkv_proj_scatter", "a3_rope_realign", "a3_question_scores", "a3_realign_scores",
             "a3_topk_select", "a3_topk_select_plan", "a3_active_rows", "a3_kv_scatter", "a3_fused_attention",
             "a3_fused_attention_planned"]
    originals = {n: getattr(api, n) for n in names}
    reps = min(args.steps, 2 * n_layers)

    def breakdown(fused):
        per_call = {}

        def wrap(n):
            def f(*a, **kw):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                originals[n](*a, **kw)
                e1.record()
                per_call.setdefault(n, []).append((e0, e1))
            return f

        for n in names:
            setattr(api, n, wrap(n))
        for i in range(reps):
            L, B = layers[i % n_layers], bufs[i % n_layers]
            layer.fuse_layer(lay, B, L["x"], L["k_cat"], L["v"], L["wq"], L["wk"], L["wv"], fused_scatter=fused,
                             fused_realign=fused, fused_plan=fused)
        torch.cuda.synchronize()
        for n in names:
            setattr(api, n, originals[n])
        out = {}
        for n, evs in per_call.items():
            tot = sum(a.elapsed_time(b) for a, b in evs) * 1e3 / reps
            out[n] = {"us_per_step": round(tot, 2), "calls_per_step": len(evs) // reps}
        return out

    per_call_us = breakdown(True)

    # what a plain device copy of the realign's size reaches on this machine (read + write): the practical
    # ceiling the HBM-bound kernels are up against, next to the nominal peak
    src = layers[0]["k_cat"]
    dsts = [torch.empty_like(src) for _ in range(4)]
    for d in dsts:
        d.copy_(src)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for i in range(32):
        dsts[i % 4].copy_(layers[i % n_layers]["k_cat"])
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * src.numel() * src.element_size() / (c0.elapsed_time(c1) * 1e-3 / 32) / 1e9
    del dsts
    per_call_plain = breakdown(False)

    # ---- sanity: the pass produced a full, finite result --------------------------------------------
    B0 = bufs[0]
    act = B0.act_idx.cpu().numpy()[:B0.n_act]
    assert np.all(np.diff(act) > 0) and B0.n_act == w.total_k + w.total_q
    assert bool(torch.isfinite(B0.out[:B0.n_act].float()).all())
    pos = w.token_positions()[act]

    work = algorithmic_work(w, pos)
    ms_per_step = elapsed * 1e3 / args.steps
    value = w.total_ctx / (ms_per_step * 1e-3)
    attn_tflops = work["attn_flops"] / (attn_main_ms * 1e-3) / 1e12          # the main kernel alone
    attn_call_tflops = work["attn_flops"] / (attn_ms * 1e-3) / 1e12          # main kernel + merge of partial results
    derived = {
        "realign_GBs": work["realign_bytes"] / (per_call_plain["a3_rope_realign"]["us_per_step"] * 1e-6) / 1e9,
        "scores_GBs": work["scores_bytes"] / (per_call_plain["a3_question_scores"]["us_per_step"] * 1e-6) / 1e9,
        # one call: the stale keys are read once and the realigned cache written once
        "realign_scores_GBs": work["realign_bytes"] / (per_call_us["a3_realign_scores"]["us_per_step"] * 1e-6) / 1e9,
        "scatter_GBs": work["scatter_bytes"] / (per_call_plain["a3_kv_scatter"]["us_per_step"] * 1e-6) / 1e9,
        # both projection calls of a step (Q of the question rows, then Q/K/V of the rows [Re, Q])
        "proj_TFLOPs": work["proj_flops"] / ((per_call_us["a3_selected_qkv_proj_scatter"]["us_per_step"] +
                                               per_call_us["a3_selected_qkv_proj"]["us_per_step"]) * 1e-6) / 1e12,
        "attn_TFLOPs": work["attn_flops"] / (per_call_us[attn_name]["us_per_step"] * 1e-6) / 1e12,
        # the method's own work: one Q K^T (the two passes of the kernel form every logit twice)
        "scores_TFLOPs": work["scores_flops"] / (per_call_plain["a3_question_scores"]["us_per_step"] * 1e-6) / 1e12,
        "plain_copy_same_size_GBs": copy_gbs,
        # the same steps issued alternately on two streams (the layer problems of this workload are independent
        # of each other): what the launch floors of the dozen small kernels of a step cost when nothing fills them.
        # Reported beside the figure above, never as `value`.
        "two_streams_us_per_step": None if two_streams_ms is None else two_streams_ms * 1e3,
    }
    result = {
        "metric": "fused-context tokens/sec per layer at 16K ctx" if args.config == 3
                  else "fused-context tokens/sec per layer",
        "value": value, "unit": "tokens/s/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": s.dtype, "data": "synthetic",
        "config": {"workload": w.name, "ctx_tokens": w.total_ctx, "question_tokens": w.total_q,
                   "selected_tokens": w.total_k, "layers_cycled": n_layers, "requests": w.n_req,
                   "shape": f"h{s.hidden}/Hq{s.n_q_heads}/Hkv{s.n_kv_heads}/d{s.head_dim}"},
        # `achieved` / `frac`: the dominant kernel alone (attn_bf16_kernel, HIP events recorded by the library around it
        # inside the timed region); `whole_call_*`: the a3_fused_attention_planned call (that kernel plus the merge
        # of partial results)
        "roofline": {"bound": "mfma", "kernel": "attn_bf16_kernel (main kernel of a3_fused_attention_planned)",
                     "achieved": attn_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": attn_tflops / PEAK_BF16_TFLOPS, "frac_is": "main kernel alone",
                     "traffic": measured_traffic(w.name), "avg_launch_ms": attn_main_ms,
                     "flops_per_launch": work["attn_flops"], "whole_call_ms": attn_ms,
                     "whole_call_achieved": attn_call_tflops, "whole_call_frac": attn_call_tflops / PEAK_BF16_TFLOPS},
        "per_call_us": per_call_us,
        "per_call_us_plain_sequence": per_call_plain,
        "derived": {k: (None if v is None else round(v, 2)) for k, v in derived.items()},
        "fraction_of_peak": {
            "realign_hbm": derived["realign_GBs"] / PEAK_HBM_GBS, "scores_hbm": derived["scores_GBs"] / PEAK_HBM_GBS,
            "realign_scores_hbm": derived["realign_scores_GBs"] / PEAK_HBM_GBS,
            "scores_mfma": derived["scores_TFLOPs"] / PEAK_BF16_TFLOPS,
            "scatter_hbm": derived["scatter_GBs"] / PEAK_HBM_GBS, "proj_mfma": derived["proj_TFLOPs"] / PEAK_BF16_TFLOPS,
            "attn_mfma": derived["attn_TFLOPs"] / PEAK_BF16_TFLOPS},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args.config)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
