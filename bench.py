#!/usr/bin/env python3
"""Benchmark of the re-positioned cached-KV prefill path on one MI355X.

Headline (the default line): Alg. 2, Phase 1 over the LLaMA-2-7B-shaped layer stack — 32 layers, a 32-token
shared prefix, 30 cached documents x 160 tokens, a 48-token query, bf16, every layer with K/V buffers of its own
(2.5 GB in all: every layer streams from HBM), a prune event after layers 8/16/24/32 that keeps 60 % of the
candidates and re-allocates the positions.  A step is the whole stack: the initial allocation plus 32
cf_prefill_layer calls (keys re-positioned on the fly, attention, per-document mass, S += mass, and at the prune
layers ranking, allocation and the next layer's table).  The value is KV tokens per second per layer: the key
positions attended, summed over the 32 layers, over the step's time.

The same JSON line carries, under "configs", the single-layer workloads (LLaMA-2-7B layer, Qwen2-7B layer, Qwen2-1.5B
batch of 64), each timed the same way: K back-to-back steps between two synchronisations, five repeats, the median.
The dominant kernel's duration comes from start/stop events the library attaches to its dispatches on the launch
stream.  "measured_peaks" holds what plain read / copy / dense-MFMA kernels sustain on this GPU in the same run;
fractions are given against the nominal peaks (8 TB/s, 2.5 PFLOP/s) and against those.  Inputs are seeded and
synthetic and resident in HBM before any timing.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0      # dense bf16 / fp16
HEADLINE = "llama2_7b_stack"
REPEATS = 5
# HBM bytes per launch of each workload's dominant kernel (read + written), from the FETCH_SIZE and WRITE_SIZE
# counter runs summarised under profiles/ (one file per kernel and workload, with the commands; both counters
# scaled by what they read for a copy kernel of known size: FETCH_SIZE reads half the bytes of a 1 GiB copy, hence
# the factor 2 on it, WRITE_SIZE reads them all; both are in KiB).  None: not measured for the kernels as they stand.
TRAFFIC_BYTES_PER_LAUNCH = {
    "llama2_7b_stack": int((2 * 23409.1 + 3534.0) * 1024),      # mean of the stack's 32 launches
    "llama2_7b_layer": int((2 * 15087.3 + 3432.0) * 1024),
    "qwen2_7b_layer": int((2 * 16987.6 + 10612.0) * 1024),
    "qwen2_1p5b_batch": int((2 * 103534.6 + 20736.0) * 1024),
}


def _median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


def timed_repeats(step, steps: int, warmup: int, repeats: int = REPEATS):
    """`warmup` untimed steps, then `repeats` blocks of exactly `steps` back-to-back steps, each block bracketed by
    a device synchronisation on both sides.  Returns (median ms per step, every block's ms per step)."""
    import torch
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    per_step = []
    n = warmup
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(n + i)
        torch.cuda.synchronize()
        per_step.append(1e3 * (time.perf_counter() - t0) / steps)
        n += steps
    return _median(per_step), per_step


def attention_kernel_ms(step, n_steps: int, launches_per_step: int, batches: int = REPEATS):
    """Duration of the attention kernel's launches, from start/stop events that the library attaches to those
    dispatches on the launch stream: `batches` batches of up to `n_steps` more steps (at most 1024 launches are kept
    per batch), each batch's mean taken, the median of the batch means returned with the number of launches timed."""
    import torch
    from paper_2502_11101_amd import binding as cf
    n_steps = max(1, min(n_steps, 1000 // launches_per_step))
    means, total = [], 0
    for _ in range(batches):
        cf.cf_profile_kernel_events(True)
        for i in range(n_steps):
            step(i)
        torch.cuda.synchronize()
        ms, n = cf.cf_profile_kernel_ms()
        cf.cf_profile_kernel_events(False)
        assert n == n_steps * launches_per_step, (n, n_steps, launches_per_step)
        means.append(ms)
        total += n
    return _median(means), total


def single_step_latency_ms(step, n: int = 20) -> float:
    """Isolated latency: one step between two synchronisations, the median of n."""
    import torch
    lat = []
    for i in range(n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step(i)
        torch.cuda.synchronize()
        lat.append(1e3 * (time.perf_counter() - t0))
    return _median(lat)


def measure_peaks() -> dict:
    """What plain kernels of known size sustain on this GPU (cf_calibrate): a streaming read and a copy of 2 GiB
    (eight times the 256 MB last-level cache), and a dense 32x32x16 MFMA loop on every SIMD."""
    import torch
    from paper_2502_11101_amd import binding as cf
    nbytes = 2 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    src.fill_(1)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(64, dtype=torch.uint8, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def best(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return _median(ts)

    out = {}
    wgs = 256 * 16
    out["hbm_read_gbs"] = nbytes / (best(lambda: cf.cf_calibrate(cf.CF_CALIB_READ, src, None, nbytes, wgs, 0, sink)) * 1e-3) / 1e9
    out["hbm_copy_gbs"] = 2 * nbytes / (best(lambda: cf.cf_calibrate(cf.CF_CALIB_COPY, src, dst, nbytes, wgs, 0, sink)) * 1e-3) / 1e9
    for name, kind in (("mfma_bf16_tflops", cf.CF_CALIB_MFMA_BF16), ("mfma_f16_tflops", cf.CF_CALIB_MFMA_F16)):
        flops = [0.0]

        def run(kind=kind):
            flops[0] = cf.cf_calibrate(kind, None, None, 0, 256 * 8, 400, sink)
        ms = best(run)
        out[name] = flops[0] / (ms * 1e-3) / 1e12
    out["what"] = ("cf_calibrate: read and copy of 2 GiB (copy counts read + written bytes), 4096 workgroups; "
                   "MFMA: 2048 workgroups x 4 wavefronts x 400 x 64 v_mfma_f32_32x32x16, no memory traffic")
    del src, dst
    torch.cuda.empty_cache()
    return out


def roofline_entry(workload: str, kernel: str, kernel_ms: float, launches: int, bytes_per_launch: float,
                   flops_per_launch: float, bound: str, peaks: dict, dtype: str) -> dict:
    if bound == "hbm":
        achieved = bytes_per_launch / (kernel_ms * 1e-3) / 1e9
        peak, unit, measured = HBM_PEAK_GBS, "GB/s", peaks.get("hbm_read_gbs") if peaks else None
    else:
        achieved = flops_per_launch / (kernel_ms * 1e-3) / 1e12
        peak, unit = MFMA_PEAK_TFLOPS, "TFLOP/s"
        measured = peaks.get("mfma_f16_tflops" if dtype == "f16" else "mfma_bf16_tflops") if peaks else None
    r = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
         "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(workload), "kernel": kernel, "ms_per_launch": kernel_ms,
         "launches_timed": launches, "algorithmic_bytes_per_launch": bytes_per_launch}
    if flops_per_launch:
        r["algorithmic_flops_per_launch"] = flops_per_launch
    if measured:
        r["measured_peak"] = measured
        r["frac_of_measured_peak"] = achieved / measured
    return r


def setup_stack(args):
    """Alg. 2 Phase 1 over the whole layer stack (LLaMA-2-7B geometry): returns (step, info)."""
    import math

    import torch
    from paper_2502_11101_amd import binding as cf
    from paper_2502_11101_amd import pipeline as pl
    from paper_2502_11101_amd import workloads as wl

    cfg = wl.CONFIGS["llama2_7b_stack"]
    g = cfg.geometry
    st = wl.build_structure(cfg)
    ts, hs = pl.store_strides(st.n_store_tokens, g.n_kv_heads, g.head_dim, args.store_layout)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions,
                        store_token_stride=ts, store_head_stride=hs)
    pb = pl.PrefillBatch(desc, st.doc_off[:-1][st.query_docs], st.doc_lens[st.query_docs], cfg.tq, cfg.prefix_len,
                         cfg.doc_stored_start, st.n_store_tokens)
    layers = []
    for layer in range(cfg.n_layers):
        t = wl.build_layer(cfg, st, layer)
        layers.append({k: (pl.store_to_device(v, g.dtype, args.store_layout) if k in ("k_store", "v_store")
                           else pl.to_device(v, g.dtype)) for k, v in t.items()})
    out = torch.empty_like(layers[0]["q"])
    keeps, alive, k = {}, [], cfg.docs_per_query
    for layer in range(cfg.n_layers):
        alive.append(k)
        if layer in cfg.prune_layers:
            k = max(1, math.ceil(cfg.keep_frac * k))
            keeps[layer] = k
    doc_len = int(st.doc_lens[0])
    kv_tokens = sum(cfg.prefix_len + n * doc_len + cfg.tq for n in alive)
    cand0 = torch.arange(pb.stride, dtype=torch.int32, device="cuda").repeat(pb.batch, 1)

    def step(_: int) -> None:
        pb.cand.copy_(cand0)
        pb.n_cand.fill_(pb.stride)
        pb.score.zero_()
        pb.n_alive = pb.stride
        pb.allocate_initial()
        for layer, L in enumerate(layers):
            # Alg. 2 reads S only at the prune events: the layers in between leave their scores pending
            pb.layer(L["q"], L["k_self"], L["v_self"], L["k_store"], L["v_store"], out, keep=keeps.get(layer),
                     strategy=cf.CF_ALLOC_SORT, defer=layer not in keeps)
            if layer in keeps:
                pb.advance()

    def check() -> None:
        assert pb.flags() == 0 and int(pb.n_cand[0].item()) == k

    info = dict(cfg=cfg, st=st, kv_tokens=kv_tokens, launches_per_step=cfg.n_layers, bound="hbm", check=check,
                kernel="attn_tile_kernel<bf16,1,32,2,true>, the 32 launches of a step taken together",
                config={"workload": "llama2_7b_stack", "layers": cfg.n_layers, "documents_per_layer": alive,
                        "kv_tokens_per_step": kv_tokens, "q_heads": g.n_q_heads, "kv_heads": g.n_kv_heads,
                        "head_dim": g.head_dim, "tq": cfg.tq, "batch": 1, "store_layout": args.store_layout,
                        "step": "initial allocation + 32 x cf_prefill_layer (prune events after layers 8, 16, 24, 32: "
                                "keep 60 %, positions re-allocated; the seven layers before each event defer their scores "
                                "to it)"})
    return step, info


def setup_layer(name: str, args):
    """One layer of a single-layer workload per step (cf_prefill_layer with its prune event), cycling through
    distinct layer buffers whose total exceeds twice the 256 MB last-level cache: returns (step, info)."""
    import torch
    from paper_2502_11101_amd import binding as cf
    from paper_2502_11101_amd import pipeline as pl
    from paper_2502_11101_amd import workloads as wl

    cfg = wl.CONFIGS[name]
    g = cfg.geometry
    n_layers = args.layers
    if args.batch > 1 and name == "llama2_7b_layer":
        cfg = wl.scaled(cfg, batch=args.batch, n_store_docs=args.batch * cfg.docs_per_query)
        per_layer = args.batch * cfg.docs_per_query * cfg.doc_len_range[1] * 2 * g.n_kv_heads * g.head_dim * 2
        n_layers = max(2, min(n_layers, int(3.0e9 // per_layer)))
    st = wl.build_structure(cfg)
    # enough distinct layer buffers that what a step reads was evicted since its last use: twice the 256 MB cache
    store_bytes = 2 * st.n_store_tokens * g.n_kv_heads * g.head_dim * 2
    n_layers = max(n_layers, min(96, -(-2 * (256 << 20) // store_bytes)))
    ts, hs = pl.store_strides(st.n_store_tokens, g.n_kv_heads, g.head_dim, args.store_layout)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions,
                        store_token_stride=ts, store_head_stride=hs)
    pb = pl.PrefillBatch(desc, st.doc_off[:-1][st.query_docs], st.doc_lens[st.query_docs], cfg.tq, cfg.prefix_len,
                         cfg.doc_stored_start, st.n_store_tokens)
    layers = []
    values = "seeded NumPy draws (workloads.build_layer)"
    if name == "qwen2_1p5b_batch":
        # 1.5 M store tokens: the store of each layer copy is drawn on the device (N(0,1), seeded), the queries' own
        # tensors on the host as everywhere else; two copies (3.1 GB) are cycled through
        n_layers = 2
        values = "store: torch.randn on the device (seeded); q / own block: seeded NumPy draws"
        dt = pl.TORCH_DTYPE[g.dtype]
        gen = torch.Generator(device="cuda").manual_seed(5000)
        shape = (st.n_store_tokens, g.n_kv_heads, g.head_dim) if args.store_layout == "token" else \
            (g.n_kv_heads, st.n_store_tokens, g.head_dim)
        rng = np.random.default_rng(5001)
        nq = cfg.batch * cfg.tq
        for _ in range(n_layers):
            L = {k: torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(dt) for k in ("k_store", "v_store")}
            for k, h in (("q", g.n_q_heads), ("k_self", g.n_kv_heads), ("v_self", g.n_kv_heads)):
                L[k] = pl.to_device(wl.round_to_dtype(rng.standard_normal((nq, h, g.head_dim), dtype=np.float32), g.dtype), g.dtype)
            layers.append(L)
    else:
        for layer in range(n_layers):
            t = wl.build_layer(cfg, st, layer)
            layers.append({k: (pl.store_to_device(v, g.dtype, args.store_layout) if k in ("k_store", "v_store")
                               else pl.to_device(v, g.dtype)) for k, v in t.items()})
    out = torch.empty_like(layers[0]["q"])
    pb.allocate_initial()
    torch.cuda.synchronize()
    kv_tokens = wl.kv_tokens_per_call(cfg, st)

    def step(i: int) -> None:
        L = layers[i % len(layers)]
        # attention + mass + S += mass + prune + allocation + next layer's table (this layer's table stays in use)
        pb.layer(L["q"], L["k_self"], L["v_self"], L["k_store"], L["v_store"], out, keep=cfg.keep,
                 strategy=cf.CF_ALLOC_SORT)

    def check() -> None:
        assert pb.flags() == 0, f"device flag {pb.flags()}"

    mha = g.n_q_heads == g.n_kv_heads
    kernel = ("attn_tile_kernel" if mha else "attn_pipe_kernel") + f"<{g.dtype}> (first kernel of cf_prefill_layer)"
    info = dict(cfg=cfg, st=st, kv_tokens=kv_tokens, launches_per_step=1, bound="hbm" if mha else "mfma", check=check,
                kernel=kernel,
                config={"workload": name, "batch": cfg.batch, "kv_tokens_per_step": kv_tokens, "q_heads": g.n_q_heads,
                        "kv_heads": g.n_kv_heads, "head_dim": g.head_dim, "tq": cfg.tq, "docs": cfg.docs_per_query,
                        "keep": cfg.keep, "layer_buffers": len(layers), "store_layout": args.store_layout, "values": values,
                        "step": "cf_prefill_layer: attention + mass + prune_topk + assign_positions + gather_segments"})
    return step, info


def run_workload(name: str, args, steps: int, warmup: int, peaks: dict) -> dict:
    step, info = setup_stack(args) if name == HEADLINE else setup_layer(name, args)
    cfg = info["cfg"]
    g = cfg.geometry
    ms_per_step, repeats = timed_repeats(step, steps, warmup)
    info["check"]()
    kernel_ms, launches = attention_kernel_ms(step, steps, info["launches_per_step"])
    latency_ms = single_step_latency_ms(step)
    info["check"]()
    kv_tokens = info["kv_tokens"]
    bytes_per_token = 2 * g.n_kv_heads * g.head_dim * (4 if g.dtype == "f32" else 2)
    n_launch = info["launches_per_step"]
    bytes_per_launch = kv_tokens * bytes_per_token / n_launch
    flops_per_launch = kv_tokens * 4.0 * cfg.tq * g.head_dim * g.n_q_heads / n_launch
    roof = roofline_entry(name, info["kernel"], kernel_ms, launches, bytes_per_launch, flops_per_launch, info["bound"], peaks, g.dtype)
    step_gbs = kv_tokens * bytes_per_token / (ms_per_step * 1e-3) / 1e9
    step_tflops = flops_per_launch * n_launch / (ms_per_step * 1e-3) / 1e12
    cfg_out = dict(info["config"])
    cfg_out.update({"whole_step_gbs": step_gbs, "whole_step_tflops": step_tflops,
                    "whole_step_frac_of_peak": step_gbs / HBM_PEAK_GBS if info["bound"] == "hbm" else step_tflops / MFMA_PEAK_TFLOPS})
    return {"value": kv_tokens / (ms_per_step * 1e-3), "ms_per_step": ms_per_step, "ms_per_step_repeats": repeats,
            "single_step_latency_ms": latency_ms, "dtype": g.dtype, "config": cfg_out, "roofline": roof,
            "_cfg": cfg, "_st": info["st"]}


def cpu_baseline(cfg, st, workload: str, budget_s: float = 12.0) -> dict:
    """The oracle as it stands, on the host cores, on as many layer passes of the same workload as fit the time
    budget (at least one): for the layer stack its first layers (all 30 documents alive), for a batch its first query.
    A pass is the oracle's attention with per-document mass, the ranking and the allocation of the survivors."""
    from oracle import cachefocus_oracle as orc
    from paper_2502_11101_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    g = cfg.geometry
    lens = [int(st.doc_lens[d]) for d in st.query_docs[0]]
    slots = list(range(cfg.docs_per_query))
    tokens = 0
    passes = 0
    t0 = time.perf_counter()
    while True:
        t = wl.build_layer(cfg, st, layer=passes)
        t1 = time.perf_counter()
        new_start, q_start, _ = orc.assign_positions(lens, slots, cfg.prefix_len, g.max_positions - cfg.tq)
        segs = []
        if cfg.prefix_len:
            segs.append(orc.Segment(0, cfg.prefix_len, 0, 0, orc.KIND_PREFIX, -1))
        for s in slots:
            doc = int(st.query_docs[0, s])
            segs.append(orc.Segment(int(st.doc_off[doc]), lens[s], cfg.doc_stored_start, new_start[s],
                                    orc.KIND_DOC, s))
        segs.append(orc.Segment(0, cfg.tq, 0, q_start, orc.KIND_SELF, -1))
        q = np.asarray(t["q"][:cfg.tq], dtype=np.float64)
        _, mass = orc.prefill_attention(q, 0, q_start, t["k_store"], t["v_store"], t["k_self"], t["v_self"],
                                        segs, g.n_kv_heads, g.rope_base)
        score = np.zeros(cfg.docs_per_query)
        for sg, m in zip(segs, mass):
            if sg.kind == orc.KIND_DOC:
                score[sg.doc] += m
        ranked = orc.prune_topk(score, lens, slots, cfg.keep)
        orc.assign_positions(lens, ranked, cfg.prefix_len, g.max_positions - cfg.tq)
        spent = time.perf_counter() - t1
        tokens += sum(s.len for s in segs)
        passes += 1
        cpu_time = spent if passes == 1 else cpu_time + spent
        if time.perf_counter() - t0 > budget_s:
            break
    return {"value": tokens / cpu_time, "unit": "KV tokens/s per layer", "cores": int(cores), "kind": "oracle",
            "sample": f"{passes} layer pass(es) of {workload} (its first layers, one query, {cfg.docs_per_query} documents alive), input generation excluded"}


def bench_assemble(args) -> int:
    """Final Re-Positioning (Alg. 2, Phase 2): one step gathers and re-positions one layer's prefix, surviving
    documents and query block (LLaMA-2-7B stack geometry, 160-token documents) into a head-major decode cache.
    Algorithmic bytes per gathered token: K and V read once and written once = 4 * Hkv * d * sizeof."""
    import torch
    from paper_2502_11101_amd import binding as cf
    from paper_2502_11101_amd import pipeline as pl
    from paper_2502_11101_amd import workloads as wl

    base = wl.CONFIGS["llama2_7b_stack"]
    cfg = wl.scaled(base, n_store_docs=args.assemble_docs, docs_per_query=args.assemble_docs,
                    n_planted=min(3, args.assemble_docs))
    g = cfg.geometry
    st = wl.build_structure(cfg)
    ts, hs = pl.store_strides(st.n_store_tokens, g.n_kv_heads, g.head_dim, args.store_layout)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions,
                        store_token_stride=ts, store_head_stride=hs)
    pb = pl.PrefillBatch(desc, st.doc_off[:-1][st.query_docs], st.doc_lens[st.query_docs], cfg.tq, cfg.prefix_len,
                         cfg.doc_stored_start, st.n_store_tokens)
    pb.allocate_initial()
    tokens = wl.kv_tokens_per_call(cfg, st)
    n_buf = max(2, min(args.layers, int(1.2e9 // (tokens * 2 * g.n_kv_heads * g.head_dim * 2 * 2))))
    layers = []
    for layer in range(n_buf):
        t = wl.build_layer(cfg, st, layer)
        layers.append({k: (pl.store_to_device(v, g.dtype, args.store_layout) if k in ("k_store", "v_store")
                           else pl.to_device(v, g.dtype)) for k, v in t.items() if k != "q"})
    fts, fhs = pl.store_strides(tokens, g.n_kv_heads, g.head_dim, "head")
    finals = [(torch.empty((g.n_kv_heads, tokens, g.head_dim), dtype=pl.TORCH_DTYPE[g.dtype], device="cuda"),
               torch.empty((g.n_kv_heads, tokens, g.head_dim), dtype=pl.TORCH_DTYPE[g.dtype], device="cuda"))
              for _ in range(n_buf)]
    final_off = torch.zeros(1, dtype=torch.int64, device="cuda")
    final_len = torch.zeros(1, dtype=torch.int32, device="cuda")
    max_seg = int(max(st.doc_lens.max(), cfg.prefix_len, cfg.tq))

    if args.path == "reposition":
        # the documents' keys of one layer moved to their allocated positions, out of place (Eq. 5 as its own pass)
        doc_segs = cf.segments_to_device(cf.segments_array(
            [(int(st.doc_off[d]), int(st.doc_lens[d]), cfg.doc_stored_start, cfg.doc_stored_start + 7 + 3 * j, cf.CF_SEG_DOC, j)
             for j, d in enumerate(st.query_docs[0])]))
        n_docs = len(st.query_docs[0])
        moved = int(np.sum(st.doc_lens[st.query_docs[0]]))
        outs = [torch.empty_like(L["k_store"]) for L in layers]

        def rstep(i: int) -> None:
            cf.cf_reposition_keys(desc, layers[i % n_buf]["k_store"], outs[i % n_buf], doc_segs, n_docs, st.n_store_tokens,
                                  max_seg, pb.dev_flag)

        for i in range(args.warmup):
            rstep(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(args.steps):
            rstep(args.warmup + i)
        e1.record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        assert pb.flags() == 0
        ms_per_step = 1e3 * elapsed / args.steps
        call_ms = e0.elapsed_time(e1) / args.steps
        nbytes = moved * 2 * g.n_kv_heads * g.head_dim * 2          # read + write of every moved key
        achieved = nbytes / (call_ms * 1e-3) / 1e9
        print(json.dumps({
            "metric": "key tokens/s per layer, stand-alone re-positioning", "value": moved / (ms_per_step * 1e-3),
            "unit": "key tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": g.dtype, "data": "synthetic",
            "config": {"workload": "llama2_7b_stack documents, one layer", "documents": n_docs, "key_tokens_per_step": moved,
                       "kv_heads": g.n_kv_heads, "head_dim": g.head_dim, "layer_buffers": n_buf, "store_layout": args.store_layout,
                       "step": "cf_reposition_keys, out of place"},
            "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                         "traffic": None, "kernel": "reposition_kernel", "ms_per_launch": call_ms,
                         "algorithmic_bytes_per_launch": nbytes}}))
        return 0

    def step(i: int) -> None:
        L, (kf, vf) = layers[i % n_buf], finals[i % n_buf]
        cf.cf_assemble_cache(desc, L["k_store"], L["v_store"], st.n_store_tokens, L["k_self"], L["v_self"], pb.q_off, pb.segs,
                             pb.n_seg, pb.seg_stride, 1, cfg.tq, max_seg, final_off, tokens, fts, fhs, kf, vf, final_len,
                             None, pb.dev_flag)

    if args.path == "decode":
        # every layer's cache is assembled once; a step is then the attention of one new token (already carrying RoPE
        # for its position, right after the query block) over one layer's cache and over itself
        for i in range(n_buf):
            step(i)
        torch.cuda.synchronize()
        assert pb.flags() == 0 and int(final_len.item()) == tokens
        ddesc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions,
                             store_token_stride=fts, store_head_stride=fhs)
        p_new = int(pb.q_start.item()) + cfg.tq
        table = cf.segments_to_device(cf.segments_array([(0, tokens, 0, 0, cf.CF_SEG_PREFIX, -1),
                                                         (0, 1, p_new, p_new, cf.CF_SEG_SELF, -1)]))
        n_seg = torch.full((1,), 2, dtype=torch.int32, device="cuda")
        q_off = torch.tensor([0, 1], dtype=torch.int32, device="cuda")
        q_new = torch.full((1,), p_new, dtype=torch.int32, device="cuda")
        gen = torch.Generator(device="cuda").manual_seed(5)
        new_tok = [tuple(torch.randn(shape, generator=gen, device="cuda").to(pl.TORCH_DTYPE[g.dtype])
                         for shape in ((1, g.n_q_heads, g.head_dim), (1, g.n_kv_heads, g.head_dim), (1, g.n_kv_heads, g.head_dim)))
                   for _ in range(n_buf)]
        dout = torch.empty_like(new_tok[0][0])
        dmass = torch.zeros((1, 2), dtype=torch.float32, device="cuda")
        ws_bytes = cf.cf_prefill_workspace_bytes(ddesc, 1, 1, 2, tokens + 1)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

        def step(i: int) -> None:                                                  # noqa: F811
            (kf, vf), (q1, k1, v1) = finals[i % n_buf], new_tok[i % n_buf]
            cf.cf_prefill_attention(ddesc, q1, q_off, p_new, q_new, kf, vf, tokens, k1, v1, table, n_seg, 2, 1, 1, tokens + 1,
                                    dout, None, None, 1, ws, ws_bytes, pb.dev_flag)           # outputs only: no mass

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert pb.flags() == 0 and int(final_len.item()) == tokens
    if args.path == "decode":
        assert bool(torch.isfinite(dout.float()).all())
        ms_per_step = 1e3 * elapsed / args.steps
        call_ms = e0.elapsed_time(e1) / args.steps
        bytes_per_token = 2 * g.n_kv_heads * g.head_dim * 2
        achieved = (tokens + 1) * bytes_per_token / (call_ms * 1e-3) / 1e9
        cf.cf_profile_kernel_events(True)                       # the attention kernel's own dispatches
        for i in range(min(args.steps, 1000)):
            step(i)
        torch.cuda.synchronize()
        kernel_ms, n_bracketed = cf.cf_profile_kernel_ms()
        cf.cf_profile_kernel_events(False)
        print(json.dumps({
            "metric": "KV tokens/s per layer, decode-step attention over the assembled cache",
            "value": (tokens + 1) / (ms_per_step * 1e-3), "unit": "KV tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": g.dtype, "data": "synthetic",
            "config": {"workload": "llama2_7b_stack final survivors, one layer, one new token", "documents": args.assemble_docs,
                       "kv_tokens_per_step": tokens + 1, "kv_heads": g.n_kv_heads, "head_dim": g.head_dim, "layer_buffers": n_buf,
                       "step": "cf_prefill_attention (Tq = 1)"},
            "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                         "traffic": None, "kernel": "whole call: attn_tile_kernel + attn_combine_kernel (no mass asked for)",
                         "ms_per_launch": call_ms, "algorithmic_bytes_per_launch": (tokens + 1) * bytes_per_token,
                         "attention_kernel_ms": kernel_ms, "attention_kernel_launches_timed": n_bracketed,
                         "attention_kernel_gbs": (tokens + 1) * bytes_per_token / (kernel_ms * 1e-3) / 1e9}}))
        return 0
    ms_per_step = 1e3 * elapsed / args.steps
    kernel_ms = e0.elapsed_time(e1) / args.steps
    bytes_per_token = 4 * g.n_kv_heads * g.head_dim * 2
    achieved = tokens * bytes_per_token / (kernel_ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "KV tokens/s per layer, final re-positioning (cache assembly)", "value": tokens / (ms_per_step * 1e-3),
        "unit": "KV tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": g.dtype, "data": "synthetic",
        "config": {"workload": "llama2_7b_stack final survivors, one layer", "documents": args.assemble_docs,
                   "kv_tokens_per_step": tokens, "kv_heads": g.n_kv_heads, "head_dim": g.head_dim,
                   "layer_buffers": n_buf, "store_layout": args.store_layout, "step": "cf_assemble_cache"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": "assemble_kernel<bf16, half>",
                     "ms_per_launch": kernel_ms, "algorithmic_bytes_per_launch": tokens * bytes_per_token}}))
    return 0


def bench_encode(args) -> int:
    """Query-independent parallel document caching (Sec. 2.2) for one layer: a step encodes the documents of the
    LLaMA-2-7B stack geometry (each attends to the 32-token prefix in the store and causally to itself) and writes
    their keys, moved to the cached positions, and values into the store: cf_prefill_attention + cf_assemble_cache.
    The attention is a dense contraction: 4 * d * Hq flops per (query row, visible key) pair."""
    import torch
    from paper_2502_11101_amd import binding as cf
    from paper_2502_11101_amd import pipeline as pl
    from paper_2502_11101_amd import workloads as wl

    base = wl.CONFIGS["llama2_7b_stack"]
    cfg = wl.scaled(base, n_store_docs=args.assemble_docs, docs_per_query=args.assemble_docs,
                    n_planted=min(3, args.assemble_docs))
    g = cfg.geometry
    st = wl.build_structure(cfg)
    ts, hs = pl.store_strides(st.n_store_tokens, g.n_kv_heads, g.head_dim, args.store_layout)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions,
                        store_token_stride=ts, store_head_stride=hs)
    lens = st.doc_lens.astype(np.int64)
    sb = pl.StoreBuilder(desc, st.doc_off[:-1], lens, np.full(len(lens), cfg.doc_stored_start), cfg.prefix_len,
                         st.n_store_tokens)
    doc_tokens = int(lens.sum())
    n_buf = max(2, min(args.layers, 8))
    dt = pl.TORCH_DTYPE[g.dtype]
    gen = torch.Generator(device="cuda").manual_seed(11)
    shape = (st.n_store_tokens, g.n_kv_heads, g.head_dim) if args.store_layout == "token" else \
        (g.n_kv_heads, st.n_store_tokens, g.head_dim)
    bufs = []
    for _ in range(n_buf):
        fresh = [torch.randn((doc_tokens, h, g.head_dim), generator=gen, device="cuda").to(dt)
                 for h in (g.n_q_heads, g.n_kv_heads, g.n_kv_heads)]
        stores = [torch.randn(shape, generator=gen, device="cuda").to(dt) for _ in range(2)]     # the prefix rows matter
        bufs.append((fresh, stores))
    out = torch.empty_like(bufs[0][0][0])

    def step(i: int) -> None:
        (q, k, v), (ks, vs) = bufs[i % n_buf]
        sb.attend(q, k, v, ks, vs, out)
        sb.write(k, v, ks, vs, ts, hs)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert sb.flags() == 0 and bool(torch.isfinite(out.float()).all())
    ms_per_step = 1e3 * elapsed / args.steps
    cf.cf_profile_kernel_events(True)
    for i in range(min(args.steps, 1000)):
        step(i)
    torch.cuda.synchronize()
    kernel_ms, n_bracketed = cf.cf_profile_kernel_ms()
    cf.cf_profile_kernel_events(False)
    pairs = float(sum(int(n) * cfg.prefix_len + int(n) * (int(n) + 1) // 2 for n in lens))     # (row, visible key)
    flops = 4.0 * g.head_dim * g.n_q_heads * pairs
    tflops = flops / (kernel_ms * 1e-3) / 1e12
    print(json.dumps({
        "metric": "document tokens/s per layer, offline document encoding into the cache store",
        "value": doc_tokens / (ms_per_step * 1e-3), "unit": "document tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": g.dtype, "data": "synthetic",
        "config": {"workload": "llama2_7b_stack documents, one layer", "documents": len(lens), "document_tokens_per_step": doc_tokens,
                   "prefix": cfg.prefix_len, "q_heads": g.n_q_heads, "kv_heads": g.n_kv_heads, "head_dim": g.head_dim,
                   "layer_buffers": n_buf, "store_layout": args.store_layout,
                   "step": "cf_prefill_attention (each document over the prefix and causally over itself) + cf_assemble_cache into the store"},
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / MFMA_PEAK_TFLOPS, "traffic": None,
                     "kernel": f"attn_pipe_kernel<{g.dtype},2> (first kernel of cf_prefill_attention)",
                     "ms_per_launch": kernel_ms, "launches_timed": n_bracketed, "algorithmic_flops_per_launch": flops}}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100,
                    help="steps per timed block of the headline workload (a step is the whole 32-layer stack)")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=24, help="distinct layer buffers the single-layer workloads cycle through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="headline only: skip the single-layer workloads")
    ap.add_argument("--no-peaks", action="store_true", help="skip the calibration kernels")
    ap.add_argument("--workload", choices=[HEADLINE, "llama2_7b_layer", "qwen2_7b_layer", "qwen2_1p5b_batch"], default=HEADLINE,
                    help="the workload of the line's value (default: the layer stack, with the others nested under "
                         "\"configs\"); naming another one times that workload alone, e.g. for a profiler run")
    ap.add_argument("--batch", type=int, default=0,
                    help="queries per step for --workload llama2_7b_layer (default: the configuration's own, 1); each query "
                         "gets documents of its own, so the step streams batch times the K/V")
    ap.add_argument("--store-layout", choices=["head", "token"], default="head",
                    help="layout of the cache store: head-major [kv head][token][d] (default, the layout the "
                         "store is meant to be kept in) or token-major [token][kv head][d]")
    ap.add_argument("--path", choices=["prefill", "assemble", "decode", "reposition", "encode"], default="prefill",
                    help="prefill: the per-layer hot path (the headline metric).  assemble: Alg. 2 Phase 2, "
                         "cf_assemble_cache of one layer of the final survivor set into a decode cache.  decode: one "
                         "decode step's attention (one new token) over an assembled cache, Alg. 2 Phase 3.  reposition: "
                         "the stand-alone Eq. 5 call, cf_reposition_keys, out of place over the documents of one layer.  encode: offline "
                         "document encoding of one layer into the cache store (Sec. 2.2), --assemble-docs documents")
    ap.add_argument("--assemble-docs", type=int, default=5, help="surviving documents per query for --path assemble")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only 10 copies of 1 GiB (read 1 GiB + write 1 GiB each) through cf_calibrate: the known-size "
                         "kernel that scales the HBM byte counters of a profiler run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2502_11101_amd import binding as cf

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    cf.load()
    if args.copy_calibration:
        n = 1 << 30
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        sink = torch.zeros(64, dtype=torch.uint8, device="cuda")
        for _ in range(10):
            cf.cf_calibrate(cf.CF_CALIB_COPY, src, dst, n, 4096, 0, sink)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"kernel": "calib_copy_kernel", "launches": 10, "read_bytes": n, "write_bytes": n}}))
        return 0
    if args.path in ("assemble", "decode", "reposition"):
        return bench_assemble(args)
    if args.path == "encode":
        return bench_encode(args)

    peaks = None if args.no_peaks else measure_peaks()
    main_run = run_workload(args.workload, args, args.steps, args.warmup, peaks)
    result = {
        "metric": "KV tokens/s per layer, re-positioned cached-KV prefill",
        "value": main_run["value"],
        "unit": "KV tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_run["ms_per_step"],
        "ms_per_step_repeats": main_run["ms_per_step_repeats"],
        "single_step_latency_ms": main_run["single_step_latency_ms"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": main_run["dtype"],
        "data": "synthetic",
        "config": main_run["config"],
        "roofline": main_run["roofline"],
    }
    if peaks:
        result["measured_peaks"] = peaks
    if args.workload == HEADLINE and not args.no_configs:
        # the single-layer workloads: >= 200 back-to-back steps per block, five blocks, the median
        sub_steps = max(200, args.steps)
        result["configs"] = []
        for name in ("llama2_7b_layer", "qwen2_7b_layer", "qwen2_1p5b_batch"):
            r = run_workload(name, args, sub_steps, 50, peaks)
            result["configs"].append({"workload": name, "value": r["value"], "unit": "KV tokens/s", "steps": sub_steps,
                                      "ms_per_step": r["ms_per_step"], "ms_per_step_repeats": r["ms_per_step_repeats"],
                                      "single_step_latency_ms": r["single_step_latency_ms"], "dtype": r["dtype"],
                                      "config": r["config"], "roofline": r["roofline"]})
            torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(main_run["_cfg"], main_run["_st"], args.workload)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
