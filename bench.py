#!/usr/bin/env python3
"""Benchmark of the TurboRAG online-prefill hot path on one MI355X.

A step is one pass of the online path for one request of configuration 4 (Llama-3-8B attention
shape, 32 chunks x 1024 tokens, 256 query tokens, reordered positions), one layer: gather plan ->
tr_kv_assemble_append (KV gather with RoPE re-rotation, and the query tokens' own rows, one
launch) -> tr_prefill_attn.  Steps cycle through 4 requests with different chunk orders, their own
cache buffers and two copies of the store, so that the store is read from HBM rather than from a
warm cache.  The K timed steps are captured once in a HIP graph (the way a serving loop would
issue them) and replayed between two synchronisations; `eager_us_per_step` is the same loop driven
call by call from Python, host-side plan included.

The JSON line starts with a summary (kernel@workload -> [us, fraction of peak, bound]) and also
carries the roofline of the dominant kernel of the step, the rooflines of the other kernels at
the sizes where they are bandwidth- or MFMA-bound (configurations 2, 3 and 5, the one-pass
sequence form, decode, short queries), what a plain copy and a bare matrix-instruction loop reach
on the same GPU in the same run, and the CPU oracle timed on the host cores.
"""
import argparse
import gc
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published

def _events(torch, n):
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _time_calls(torch, fn, iters, warmup=3, reps=5):
    """Average duration (us) of fn's GPU work.  `iters` calls are captured into one HIP graph, so that they run
    back to back without host launch gaps, and each replay is bracketed by one HIP event pair on the launching
    stream.  Returns (mean, median, min) over `reps` replays of the per-call average."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(iters):
            fn()
    graph.replay()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = _events(torch, 2)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e3 / iters)
    ts.sort()
    return float(np.mean(ts)), float(ts[len(ts) // 2]), float(ts[0])


def source_digest():
    """SHA-256 over the kernel sources: counter figures measured on other kernels than these are not reported."""
    import hashlib
    here = os.path.dirname(os.path.abspath(__file__))
    csrc = os.path.join(here, "paper_2410_07590_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(f for f in os.listdir(csrc) if f.endswith((".hip", ".h"))):
        h.update(name.encode())
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def load_traffic():
    """HBM bytes per launch from the rocprofv3 counter runs summarised under profiles/ (written there by
    `python -m paper_2410_07590_amd.profile_summary`).  Empty when the kernels have changed since they were taken."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return {}, None
    if rec.get("csrc_sha256") != source_digest():
        return {}, None
    return rec.get("bytes_per_launch", {}), rec.get("commit")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations and the CPU baseline")
    ap.add_argument("--no-graph", action="store_true", help="time the eager loop instead of a HIP graph replay")
    ap.add_argument("--host-store", action="store_true",
                    help="time the host-resident store over all 28 layers, three times (the default run does 8 layers once)")
    ap.add_argument("--case", default=None,
                    help="profiling aid: run only one kernel path --iters times, eagerly, and print nothing but a note "
                         "(step2, assemble2, asmapp2, attn2, step4, assemble4, asmapp4, raw4, attn4, batched3, offline5, sequence4, "
                         "decode2, shortq, shortq16, linear2, linearqkv2, copy, mfmaloop)")
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_07590_amd import accounting as acct
    from paper_2410_07590_amd import build as trbuild
    from paper_2410_07590_amd import synth
    if not os.path.exists(trbuild.LIB):
        trbuild.build()
    from paper_2410_07590_amd import binding as B
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    B.lib()
    torch.cuda.set_device(0)
    if args.case:
        run_case(torch, B, synth, args.case, args.iters)
        return

    traffic, traffic_commit = load_traffic()

    def hbm_roof(name, workload, nbytes, t_us):
        a = nbytes / (t_us[0] * 1e-6) / 1e9
        return {"kernel": name, "workload": workload, "bound": "hbm", "achieved": round(a, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(a / HBM_PEAK_GBS, 4), "traffic": traffic.get("%s@%s" % (name, workload)),
                "avg_us": round(t_us[0], 2), "median_us": round(t_us[1], 2), "algorithmic_bytes": nbytes}

    def mfma_roof(name, workload, flops, t_us, nbytes):
        a = flops / (t_us[0] * 1e-6) / 1e12
        return {"kernel": name, "workload": workload, "bound": "mfma", "achieved": round(a, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(a / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic.get("%s@%s" % (name, workload)),
                "avg_us": round(t_us[0], 2), "median_us": round(t_us[1], 2), "algorithmic_flops": flops,
                "algorithmic_bytes": nbytes, "hbm_gbs": round(nbytes / (t_us[0] * 1e-6) / 1e9, 1)}

    # headline: the step at configuration 4, the largest single-GPU configuration
    cfg = synth.CONFIGS[4]
    head = bench_step(torch, B, synth, acct, cfg, N_VARIANTS[4], args.steps, args.warmup, args.no_graph, hbm_roof, mfma_roof)
    us_per_step = head["eager_us"] if args.no_graph else head["graph_us"]
    sh = cfg.shape
    result = {
        "summary": None,   # filled below; first, so that a truncated record keeps every kernel's figure
        "metric": "us/layer query-prefill over assembled KV (gather plan + assemble and append + prefill attention); `value` is a "
                  "HIP-graph replay of the K steps, which holds the kernels only: the host-side plan and argument marshalling "
                  "ran at capture; eager_us_per_step is the same K steps driven call by call from Python, plan included",
        "value": round(us_per_step, 3), "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us_per_step / 1e3, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 4: %s (%d q heads, %d kv heads, head_dim %d, 32 chunks x 1024 tokens, 256 query tokens, reordered positions)"
                               % (cfg.name, sh.n_q_heads, sh.n_kv_heads, sh.head_dim),
                   "timed_as": "eager" if args.no_graph else "hip_graph_replay", "request_variants": N_VARIANTS[4]},
        "eager_us_per_step": round(head["eager_us"], 3),
        "kernel_us": head["kernel_us"],
        "roofline": head["roofline"],
        "traffic_measured_at_commit": traffic_commit,
    }
    roof_extra = head["roof_extra"]

    if not args.no_extra:
        c2 = bench_step(torch, B, synth, acct, synth.CONFIGS[2], N_VARIANTS[2], 256, 16, args.no_graph, hbm_roof, mfma_roof)
        roof_extra.append({"kernel": "step (assemble and append + prefill attention)", "workload": synth.CONFIGS[2].name,
                           "graph_replay_us": round(c2["graph_us"], 2), "eager_us": round(c2["eager_us"], 2), "steps": 256,
                           "kernel_us": c2["kernel_us"]})
        roof_extra += [c2["roofline"]] + c2["roof_extra"]
        roof_extra += bench_config3(torch, B, synth, acct, hbm_roof, mfma_roof)
        roof_extra += bench_config5(torch, B, synth, acct, mfma_roof)
        roof_extra += bench_sequence(torch, B, synth, acct, mfma_roof)
        roof_extra += bench_decode(torch, B, synth, hbm_roof)
        roof_extra += bench_short_query(torch, B, synth, hbm_roof)
        roof_extra += bench_host_store(torch, B, synth, acct, *((H2D_LAYERS, 3) if args.host_store else (8, 1)))
        result["layer_context"], lin_roofs = bench_layer_context(torch, B, synth, hbm_roof)
        roof_extra += lin_roofs
        result["table4_batch_scaling"] = bench_table4_batches(torch, B, synth)
        ceil = {"hbm_copy_gbs": measured_copy_rate(torch)}
        ceil.update(measured_mfma_loop(torch, B))
        result["measured_ceilings"] = ceil
        result["hbm_copy_ceiling_gbs"] = ceil["hbm_copy_gbs"]
        notes = {"batched-serving-16req": "one batch replayed: 390 MB of caches, more than the 256 MB last-level cache holds",
                 "offline-64x512": "cold by size: 840 MB of q, k, v, k' and out per call",
                 "32x1024-chunks-plus-256-query-llama3-8b": "cold by size: 850 MB per call",
                 "decode-%dx%d-qwen2-7b" % (DECODE_BATCH, DECODE_KV): "cold by size: 537 MB of cache rows per call",
                 "short-query-16-tokens-over-12288-rows-qwen2-7b": "cold: twelve caches of 25 MB in turn",
                 "short-query-16req-x-16-tokens-over-12288-rows-qwen2-7b": "cold: two sets of caches of 403 MB in turn",
                 "qwen2-7b-qkv-projection-64-tokens": "cold: the weights of ten layers in turn (587 MB)",
                 "qwen2-7b-output-projection-64-tokens": "cold: the weights of ten layers in turn (587 MB)"}
        for r in roof_extra:
            if "memory" not in r and r.get("workload") in notes:
                r["memory"] = notes[r["workload"]]
        for r in [result["roofline"]] + roof_extra:   # the same fractions against what the chip delivered in this run
            if r.get("bound") == "mfma":
                r["frac_of_measured_loop"] = round(r["achieved"] / ceil["mfma_loop_tflops_random_operands"], 4)
            elif r.get("bound") == "hbm":
                r["frac_of_measured_copy"] = round(r["achieved"] / ceil["hbm_copy_gbs"], 4)
        result["cpu_baseline"] = cpu_baseline(synth, cfg)
    result["roofline_extra"] = roof_extra
    result["summary"] = {"%s@%s" % (r["kernel"], r["workload"]): [r["avg_us"], r["frac"], r["bound"]]
                         for r in [result["roofline"]] + roof_extra if "frac" in r and "avg_us" in r}
    print(json.dumps(result))


N_VARIANTS = {2: 16, 4: 4}


def bench_step(torch, B, synth, acct, cfg, n_variants, steps, warmup, eager_only, hbm_roof, mfma_roof):
    """The step (gather plan -> tr_kv_assemble_append -> tr_prefill_attn, one layer) for one request of `cfg`.
    Steps cycle through n_variants requests with different chunk ids, their own cache buffers and one of two copies
    of the store, so that a step reads its chunks from HBM rather than from a warm cache."""
    sh = cfg.shape
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    store = synth.make_store(cfg)
    stores = [B.Store(gs, store.k.cuda(), store.v.cuda(), store.row_start) for _ in range(2)]
    base_req = synth.make_requests(cfg, store)[0]
    rng = synth.rng_for(cfg, 9)
    variants = []
    for i in range(n_variants):
        if i == 0:
            ids = base_req.chunk_ids
        elif cfg.id_draw == "shuffle_all":
            ids = rng.permutation(cfg.store_chunks).astype(np.int32)
        else:
            ids = rng.choice(cfg.store_chunks, size=cfg.chunks_per_request, replace=False).astype(np.int32)
        sd = stores[i % 2]
        offsets, _ = B.tr_plan(sd, ids, base_req.pos_mode, want_pos_ids=False)
        n_doc = int(offsets[-1])
        kv_len = n_doc + base_req.n_q
        variants.append(dict(
            sd=sd, ids=ids, n_doc=n_doc, kv_len=kv_len,
            cache_k=torch.empty((kv_len, sh.n_kv_heads, sh.head_dim), dtype=sh.torch_dtype, device="cuda"),
            cache_v=torch.empty((kv_len, sh.n_kv_heads, sh.head_dim), dtype=sh.torch_dtype, device="cuda"),
            out=torch.empty((base_req.n_q, sh.n_q_heads, sh.head_dim), dtype=sh.torch_dtype, device="cuda")))
    q, k_q, v_q = base_req.q.cuda(), base_req.k_q.cuda(), base_req.v_q.cuda()
    q_pos = torch.from_numpy(base_req.q_pos).cuda()
    n_q = base_req.n_q
    ws = B.workspace(B.tr_prefill_attn_workspace_size(gs, n_q, variants[0]["kv_len"]))

    def assemble(v):
        offsets, _ = B.tr_plan(v["sd"], v["ids"], base_req.pos_mode, want_pos_ids=False)   # the gather plan (host)
        B.tr_kv_assemble(v["sd"], v["ids"], offsets, base_req.pos_mode, v["cache_k"], v["cache_v"])

    def assemble_raw(v):   # the same bytes moved from a store read as un-rotated keys, each turned once at its position id
        offsets, _ = B.tr_plan(v["sd"], v["ids"], base_req.pos_mode, want_pos_ids=False)
        B.tr_kv_assemble_raw(v["sd"], v["ids"], offsets, base_req.pos_mode, v["cache_k"], v["cache_v"])

    def append(v):
        B.tr_kv_append(gs, k_q, v_q, q_pos, v["cache_k"], v["cache_v"], v["n_doc"])

    def attn(v):
        B.tr_prefill_attn(gs, q, v["cache_k"], v["cache_v"], q_pos, v["kv_len"], v["out"], ws)

    def assemble_append(v):
        offsets, _ = B.tr_plan(v["sd"], v["ids"], base_req.pos_mode, want_pos_ids=False)   # the gather plan (host)
        B.tr_kv_assemble_append(v["sd"], v["ids"], offsets, base_req.pos_mode, k_q, v_q, q_pos, v["cache_k"], v["cache_v"])

    def step(i):
        v = variants[i % n_variants]
        assemble_append(v)
        attn(v)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()

    # eager loop (host-driven).  Python's cyclic collector is paused for it: with torch loaded one full collection
    # takes about 40 ms, many steps' worth, and it would fire a few times inside the loop.
    gc.collect()
    gc.disable()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    eager_us = (time.perf_counter() - t0) / steps * 1e6
    gc.enable()

    graph_us = None
    if not eager_only:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(steps):
                step(i)
        graph.replay()               # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) / steps * 1e6

    # per-kernel durations, HIP events around graph replays
    it = 64 if cfg.number == 2 else 24
    cyc = {"i": 0}

    def cyc_call(fn):
        def f():
            cyc["i"] += 1
            fn(variants[cyc["i"] % n_variants])
        return f

    t_asm = _time_calls(torch, cyc_call(assemble), it)
    t_app = _time_calls(torch, cyc_call(append), it)
    t_raw = _time_calls(torch, cyc_call(assemble_raw), it) if cfg.number == 4 else None
    t_asa = _time_calls(torch, cyc_call(assemble_append), it)   # last: the caches hold the pre-rotated store's rows again
    t_att = _time_calls(torch, cyc_call(attn), it)

    kv_len, n_doc = variants[0]["kv_len"], variants[0]["n_doc"]
    eb = sh.elem_bytes
    asm_bytes = acct.assemble_bytes(n_doc, sh.n_kv_heads, sh.head_dim, eb)
    att_flops = acct.attn_flops(sh.n_q_heads, sh.head_dim, acct.visible_pairs_prefix(n_q, kv_len))
    att_bytes = acct.prefill_attn_bytes(n_q, kv_len, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, eb)
    # dominant kernel of the step: query-prefill attention (prefix_attn_kernel + its split-KV combine)
    roofline = mfma_roof("tr_prefill_attn", cfg.name, att_flops, t_att, att_bytes)
    asa_bytes = asm_bytes + acct.append_bytes(n_q, sh.n_kv_heads, sh.head_dim, eb)
    roof_extra = [hbm_roof("tr_kv_assemble_append", cfg.name, asa_bytes, t_asa),
                  hbm_roof("tr_kv_assemble", cfg.name, asm_bytes, t_asm),
                  {"kernel": "tr_kv_append", "workload": cfg.name, "avg_us": round(t_app[0], 2), "median_us": round(t_app[1], 2)}]
    if t_raw:
        roof_extra.append(hbm_roof("tr_kv_assemble_raw", cfg.name, asm_bytes, t_raw))
    touched = (2 * store.k.numel() * store.k.element_size() * 2 + sum(2 * v["cache_k"].numel() * v["cache_k"].element_size() for v in variants)) // 1000000
    for r in [roofline] + roof_extra:
        r["memory"] = "cold: %d request variants in turn, %d MB of store copies and caches per cycle (last-level cache: 256 MB)" % (n_variants, touched)
    kernel_us = {"assemble_append": round(t_asa[0], 2), "prefill_attn": round(t_att[0], 2),
                 "assemble_alone": round(t_asm[0], 2), "append_alone": round(t_app[0], 2)}
    return {"graph_us": graph_us, "eager_us": eager_us, "kernel_us": kernel_us, "roofline": roofline, "roof_extra": roof_extra}


def run_case(torch, B, synth, case, iters):
    """One kernel path, a few eager launches: what the rocprofv3 counter runs under profiles/ execute."""
    if case == "copy":
        # calibration for the HBM counters: a plain device copy of known size (256 MiB read, 256 MiB written)
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(iters):
            dst.copy_(src)
        torch.cuda.synchronize()
        print("case copy: %d launches of a %d-byte device copy" % (iters, src.numel()))
        return
    if case == "linear2":
        # the query projection of configuration 2's layer: 64 tokens, 3584 x 3584 weight
        gen = torch.Generator(device="cuda")
        gen.manual_seed(3)
        rnd = lambda *shape: torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        x, w = rnd(64, 3584), rnd(3584, 3584)
        y = torch.empty((64, 3584), dtype=torch.bfloat16, device="cuda")
        ws = B.workspace(B.tr_linear_workspace_size(64, [3584], 3584))
        for _ in range(iters):
            B.tr_linear(x, w, y, ws)
        torch.cuda.synchronize()
        print("case linear2: %d calls" % iters)
        return
    if case == "linearqkv2":
        # query, key and value projections of configuration 2's layer in one launch: 64 tokens, 3584 + 512 + 512 features
        gen = torch.Generator(device="cuda")
        gen.manual_seed(4)
        rnd = lambda *shape: torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        x, w = rnd(64, 3584), [rnd(3584, 3584), rnd(512, 3584), rnd(512, 3584)]
        y = [torch.empty((64, wj.shape[0]), dtype=torch.bfloat16, device="cuda") for wj in w]
        ws = B.workspace(B.tr_linear_workspace_size(64, [3584, 512, 512], 3584))
        for _ in range(iters):
            B.tr_linear(x, w, y, ws)
        torch.cuda.synchronize()
        print("case linearqkv2: %d calls" % iters)
        return
    if case == "mfmaloop":
        sink = torch.empty(B.tr_probe_mfma_loop_sink_bytes() // 4, dtype=torch.float32, device="cuda")
        for _ in range(iters):
            B.tr_probe_mfma_loop(30000, 0, sink)
            B.tr_probe_mfma_loop(30000, 1, sink)
        torch.cuda.synchronize()
        print("case mfmaloop: %d launches with constant and %d with random operands, 30000 loop trips each" % (iters, iters))
        return
    if case in ("shortq", "shortq16"):
        att, _ = _short_query_setup(torch, B, synth, 16 if case == "shortq16" else 1)
        for _ in range(iters):
            att()
        torch.cuda.synchronize()
        print("case %s: %d calls" % (case, iters))
        return
    if case == "batched3":
        _, _, asm, app, att = _config3_setup(torch, B, synth)
        for _ in range(iters):
            asm(); app(); att()
        torch.cuda.synchronize()
        print("case batched3: %d iterations of assemble, append, attention" % iters)
        return
    if case == "sequence4":
        run = _sequence_setup(torch, B, synth)[-1]
        for _ in range(iters):
            run()
        torch.cuda.synchronize()
        print("case sequence4: %d calls" % iters)
        return
    if case == "decode2":
        run, _ = _decode_setup(torch, B, synth)
        for _ in range(iters):
            run()
        torch.cuda.synchronize()
        print("case decode2: %d calls" % iters)
        return
    if case == "offline5":
        cfg = synth.CONFIGS[5]
        sh = cfg.shape
        gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
        pc = synth.make_packed_chunks(cfg)
        q, k, v = pc.q.cuda(), pc.k.cuda(), pc.v.cuda()
        cu = torch.from_numpy(pc.cu).cuda()
        max_len = int(np.diff(pc.cu).max())
        out, k_rot = torch.empty_like(q), torch.empty_like(k)
        ws = B.workspace(B.tr_chunk_prefill_attn_workspace_size(gs, q.shape[0], max_len))
        for _ in range(iters):
            B.tr_chunk_prefill_attn(gs, q, k, v, cu, pc.cu.size - 1, max_len, out, k_rot, ws)
        torch.cuda.synchronize()
        print("case offline5: %d calls" % iters)
        return
    cfg = synth.CONFIGS[int(case[-1])]
    sh = cfg.shape
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    store = synth.make_store(cfg)
    sd = B.Store(gs, store.k.cuda(), store.v.cuda(), store.row_start)
    req = synth.make_requests(cfg, store)[0]
    offsets, _ = B.tr_plan(sd, req.chunk_ids, req.pos_mode, want_pos_ids=False)
    n_doc, kv_len = int(offsets[-1]), int(offsets[-1]) + req.n_q
    ck = torch.empty((kv_len, sh.n_kv_heads, sh.head_dim), dtype=sh.torch_dtype, device="cuda")
    cv = torch.empty_like(ck)
    q, k_q, v_q = req.q.cuda(), req.k_q.cuda(), req.v_q.cuda()
    q_pos = torch.from_numpy(req.q_pos).cuda()
    out = torch.empty_like(q)
    ws = B.workspace(B.tr_prefill_attn_workspace_size(gs, req.n_q, kv_len))
    asm = lambda: B.tr_kv_assemble(sd, req.chunk_ids, offsets, req.pos_mode, ck, cv)
    app = lambda: B.tr_kv_append(gs, k_q, v_q, q_pos, ck, cv, n_doc)
    att = lambda: B.tr_prefill_attn(gs, q, ck, cv, q_pos, kv_len, out, ws)
    asm(); app()
    fused = lambda: B.tr_kv_assemble_append(sd, req.chunk_ids, offsets, req.pos_mode, k_q, v_q, q_pos, ck, cv)
    raw = lambda: B.tr_kv_assemble_raw(sd, req.chunk_ids, offsets, req.pos_mode, ck, cv)
    what = {"assemble": [asm], "attn": [att], "step": [fused, att], "asmapp": [fused], "raw": [raw]}[case[:-1]]
    for _ in range(iters):
        for f in what:
            f()
    torch.cuda.synchronize()
    print("case %s: %d iterations" % (case, iters))


def _config3_setup(torch, B, synth):
    """Batched serving: 16 requests x 10 chunks (bounded Zipf ids over 1000 chunks of 256..1024 rows), 32..128 query
    tokens each, composite and reordered positions mixed; one launch per stage for the whole batch."""
    cfg = synth.CONFIGS[3]
    sh = cfg.shape
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    store = synth.make_store(cfg)
    sd = B.Store(gs, store.k.cuda(), store.v.cuda(), store.row_start)
    reqs = synth.make_requests(cfg, store)
    ids = np.concatenate([r.chunk_ids for r in reqs]).astype(np.int32)
    cu_chunks = np.concatenate([[0], np.cumsum([r.chunk_ids.size for r in reqs])]).astype(np.int32)
    modes = np.array([r.pos_mode for r in reqs], np.int32)
    crs = np.concatenate([[0], np.cumsum([r.n_doc + r.n_q for r in reqs])]).astype(np.int64)
    cu_q = np.concatenate([[0], np.cumsum([r.n_q for r in reqs])]).astype(np.int32)
    total = int(crs[-1])
    ck = torch.empty((total, sh.n_kv_heads, sh.head_dim), dtype=sh.torch_dtype, device="cuda")
    cv = torch.empty_like(ck)
    q = torch.cat([r.q for r in reqs]).cuda()
    k_q = torch.cat([r.k_q for r in reqs]).cuda()
    v_q = torch.cat([r.v_q for r in reqs]).cuda()
    q_pos = torch.from_numpy(np.concatenate([r.q_pos for r in reqs]).astype(np.int32)).cuda()
    out = torch.empty_like(q)
    ws = B.workspace(B.tr_prefill_attn_batched_workspace_size(gs, cu_q, crs))
    asm = lambda: B.tr_kv_assemble_batched(sd, ids, cu_chunks, modes, crs, ck, cv)
    app = lambda: B.tr_kv_append_batched(gs, k_q, v_q, q_pos, cu_q, crs, ck, cv)
    att = lambda: B.tr_prefill_attn_batched(gs, q, ck, cv, q_pos, cu_q, crs, out, ws)
    return cfg, reqs, asm, app, att


def bench_config3(torch, B, synth, acct, hbm_roof, mfma_roof):
    cfg, reqs, asm, app, att = _config3_setup(torch, B, synth)
    sh = cfg.shape
    asm(); app()
    t_asm, t_app, t_att = _time_calls(torch, asm, 20), _time_calls(torch, app, 30), _time_calls(torch, att, 30)
    eb = sh.elem_bytes
    n_doc = sum(r.n_doc for r in reqs)
    flops = sum(acct.attn_flops(sh.n_q_heads, sh.head_dim, acct.visible_pairs_prefix(r.n_q, r.n_doc + r.n_q)) for r in reqs)
    nbytes = sum(acct.prefill_attn_bytes(r.n_q, r.n_doc + r.n_q, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, eb) for r in reqs)
    return [hbm_roof("tr_kv_assemble_batched", cfg.name, acct.assemble_bytes(n_doc, sh.n_kv_heads, sh.head_dim, eb), t_asm),
            {"kernel": "tr_kv_append_batched", "workload": cfg.name, "avg_us": round(t_app[0], 2), "median_us": round(t_app[1], 2)},
            mfma_roof("tr_prefill_attn_batched", cfg.name, flops, t_att, nbytes)]


def bench_config5(torch, B, synth, acct, mfma_roof):
    cfg = synth.CONFIGS[5]
    sh = cfg.shape
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    pc = synth.make_packed_chunks(cfg)
    T = pc.q.shape[0]
    q, k, v = pc.q.cuda(), pc.k.cuda(), pc.v.cuda()
    cu = torch.from_numpy(pc.cu).cuda()
    max_len = int(np.diff(pc.cu).max())
    out = torch.empty(q.shape, dtype=sh.torch_dtype, device="cuda")
    k_rot = torch.empty(k.shape, dtype=sh.torch_dtype, device="cuda")
    ws = B.workspace(B.tr_chunk_prefill_attn_workspace_size(gs, T, max_len))

    def run():
        B.tr_chunk_prefill_attn(gs, q, k, v, cu, pc.cu.size - 1, max_len, out, k_rot, ws)

    t = _time_calls(torch, run, 20)
    flops = acct.attn_flops(sh.n_q_heads, sh.head_dim, acct.visible_pairs_blockdiag(np.diff(pc.cu)))
    nbytes = acct.chunk_prefill_bytes(T, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.elem_bytes)
    r = mfma_roof("tr_chunk_prefill_attn", cfg.name, flops, t, nbytes)
    r["note"] = "whole call: position table + key rotation + block-diagonal attention kernels"
    return [r]


def _sequence_setup(torch, B, synth):
    """The fine-tuning / whole-prefill form of configuration 4 in one pass: 32 chunks x 1024 tokens that attend
    inside their own chunk, then 256 query tokens that attend everything (reordered position ids)."""
    cfg = synth.CONFIGS[4]
    sh = cfg.shape
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    lens, n_tail = [1024] * 32, 256
    seg, pos = B.tr_sequence_plan(lens, n_tail, synth.POS_REORDERED)
    T = seg.size
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20241011)
    mk = lambda h: torch.randn((T, h, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(sh.torch_dtype)
    q, k, v = mk(sh.n_q_heads), mk(sh.n_kv_heads), mk(sh.n_kv_heads)
    out, k_rot = torch.empty_like(q), torch.empty_like(k)
    seg_d, pos_d = torch.from_numpy(seg).cuda(), torch.from_numpy(pos).cuda()
    ws = B.workspace(B.tr_sequence_prefill_attn_workspace_size(gs, seg, T))
    run = lambda: B.tr_sequence_prefill_attn(gs, q, k, v, seg_d, pos_d, out, k_rot, seg_start_host=seg, workspace=ws)
    return sh, lens, n_tail, T, run


def bench_sequence(torch, B, synth, acct, mfma_roof):
    sh, lens, n_tail, T, run = _sequence_setup(torch, B, synth)
    t = _time_calls(torch, run, 10)
    n_doc = sum(lens)
    pairs = acct.visible_pairs_blockdiag(lens) + acct.visible_pairs_prefix(n_tail, n_doc + n_tail)
    r = mfma_roof("tr_sequence_prefill_attn", "32x1024-chunks-plus-256-query-llama3-8b",
                  acct.attn_flops(sh.n_q_heads, sh.head_dim, pairs), t,
                  acct.chunk_prefill_bytes(T, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.elem_bytes))
    r["note"] = "whole call: key rotation at the position ids + one attention pass over documents and query"
    return [r]


def bench_layer_context(torch, B, synth, hbm_roof):
    """The attention block of one layer around the step: query/key/value projections of the query tokens' hidden
    states (Eq. 1), the step (assemble and append + prefill attention), the output projection, at the Qwen2-7B shape
    with random weights; biases, norms and the MLP are not part of it.  Two workloads: configuration 2, and the shape
    of the paper's Table 4 (16 chunks x 512 tokens, 128 query tokens)."""
    sh = synth.QWEN2_7B
    hidden = sh.n_q_heads * sh.head_dim
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20241013)
    rnd = lambda *shape, scale=1.0: (torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32) * scale).to(torch.bfloat16)
    # the weights of N_LAYERS layers are used in turn, as a model walks through them: 587 MB (257 MB of output
    # weights alone), more than the 256 MB last-level cache holds, so that no call finds its weights cached
    N_LAYERS = 10
    layers = [(rnd(hidden, hidden, scale=hidden ** -0.5), rnd(sh.n_kv_heads * sh.head_dim, hidden, scale=hidden ** -0.5),
               rnd(sh.n_kv_heads * sh.head_dim, hidden, scale=hidden ** -0.5), rnd(hidden, hidden, scale=hidden ** -0.5))
              for _ in range(N_LAYERS)]    # (wq, wk, wv, wo), each [out_features, in_features]
    wq, wk, wv, wo = layers[0]
    turn = {"i": 0}

    def next_layer():
        turn["i"] += 1
        return layers[turn["i"] % N_LAYERS]
    rows, roofs = [], []
    for name, n_chunks, n_q in (("qwen2-7b-8x512-q64", 8, 64), ("table4-shape-16x512-q128", 16, 128)):
        n_store = 64
        ks, vs = rnd(n_store * 512, sh.n_kv_heads, sh.head_dim), rnd(n_store * 512, sh.n_kv_heads, sh.head_dim)
        sd = B.Store(gs, ks, vs, np.arange(n_store + 1, dtype=np.int64) * 512)
        ids = np.random.default_rng(7).permutation(n_store)[:n_chunks].astype(np.int32)
        n_doc = n_chunks * 512
        kv_len = n_doc + n_q
        x = rnd(n_q, hidden)
        q, o = torch.empty((n_q, sh.n_q_heads, sh.head_dim), dtype=torch.bfloat16, device="cuda"), None
        kq, vq = (torch.empty((n_q, sh.n_kv_heads, sh.head_dim), dtype=torch.bfloat16, device="cuda") for _ in range(2))
        ck = torch.empty((kv_len, sh.n_kv_heads, sh.head_dim), dtype=torch.bfloat16, device="cuda")
        cv, att = torch.empty_like(ck), torch.empty_like(q)
        o = torch.empty((n_q, hidden), dtype=torch.bfloat16, device="cuda")
        q_pos = torch.arange(n_doc, kv_len, dtype=torch.int32, device="cuda")
        ws = B.workspace(B.tr_prefill_attn_workspace_size(gs, n_q, kv_len))

        def step():
            offsets, _ = B.tr_plan(sd, ids, synth.POS_REORDERED, want_pos_ids=False)
            B.tr_kv_assemble_append(sd, ids, offsets, synth.POS_REORDERED, kq, vq, q_pos, ck, cv)
            B.tr_prefill_attn(gs, q, ck, cv, q_pos, kv_len, att, ws)

        def layer_library():
            wq, wk, wv, wo = next_layer()
            torch.matmul(x, wq.t(), out=q.view(n_q, hidden))
            torch.matmul(x, wk.t(), out=kq.view(n_q, -1))
            torch.matmul(x, wv.t(), out=vq.view(n_q, -1))
            step()
            torch.matmul(att.view(n_q, hidden), wo.t(), out=o)

        ws_qkv = B.workspace(B.tr_linear_workspace_size(n_q, [wq.shape[0], wk.shape[0], wv.shape[0]], hidden))
        ws_o = B.workspace(B.tr_linear_workspace_size(n_q, [hidden], hidden))

        def layer():
            wq, wk, wv, wo = next_layer()
            B.tr_linear(x, [wq, wk, wv], [q, kq, vq], ws_qkv)
            step()
            B.tr_linear(att.view(n_q, hidden), wo, o, ws_o)

        def projections():
            wq, wk, wv, wo = next_layer()
            B.tr_linear(x, [wq, wk, wv], [q, kq, vq], ws_qkv)
            B.tr_linear(att.view(n_q, hidden), wo, o, ws_o)

        def proj_qkv():
            wq, wk, wv, _ = next_layer()
            B.tr_linear(x, [wq, wk, wv], [q, kq, vq], ws_qkv)

        def proj_o():
            B.tr_linear(att.view(n_q, hidden), next_layer()[3], o, ws_o)

        t_layer = _time_calls(torch, layer, 24)
        t_lib = _time_calls(torch, layer_library, 24)
        t_step = _time_calls(torch, step, 20)
        t_proj = _time_calls(torch, projections, 24)
        if n_q == 64:   # roofline rows for the two launches: weights, x and y moved once
            n_qkv = wq.shape[0] + wk.shape[0] + wv.shape[0]
            t_qkv = _time_calls(torch, proj_qkv, 24)
            t_o = _time_calls(torch, proj_o, 24)
            roofs.append(hbm_roof("tr_linear", "qwen2-7b-qkv-projection-64-tokens", 2 * (n_qkv * hidden + n_q * hidden + n_q * n_qkv), t_qkv))
            roofs.append(hbm_roof("tr_linear", "qwen2-7b-output-projection-64-tokens", 2 * (hidden * hidden + 2 * n_q * hidden), t_o))
        w_bytes = 2 * (wq.numel() + wk.numel() + wv.numel() + wo.numel())
        rows.append({"workload": name, "attention_block_us": round(t_layer[0], 2), "step_us": round(t_step[0], 2),
                     "tr_linear_us": round(t_proj[0], 2), "weight_bytes": w_bytes,
                     "weight_stream_gbs": round(w_bytes / (t_proj[0] * 1e-6) / 1e9, 1),
                     "attention_block_with_library_gemms_us": round(t_lib[0], 2)})
    return {"what": "attention block of one layer: q/k/v projection (tr_linear, one launch for the three weights, random weights) + "
                    "step + output projection (tr_linear); the same block with torch.matmul for the projections beside it; "
                    "the weights of %d layers are used in turn (%d MB, more than the last-level cache holds)" % (N_LAYERS, N_LAYERS * 58720256 // 1000000),
            "rows": rows}, roofs


def _short_query_setup(torch, B, synth, n_req):
    """A few query tokens over a long context (the shape of the paper's Table 2 workloads, Sec. 4.4: 7.5k-16k context
    tokens, 6-20 query tokens): n_req requests of 16 query tokens over 12288 document rows each, Qwen2-7B heads.
    Every key is read once, so the rows are priced against HBM; enough caches are cycled that the keys do not sit in
    the last-level cache."""
    sh = synth.QWEN2_7B
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20241012)
    rnd = lambda *shape: torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    n_q, n_doc = 16, 12288
    kv_len = n_doc + n_q
    n_caches = 12 if n_req == 1 else 2
    caches = [(rnd(n_req * kv_len, sh.n_kv_heads, sh.head_dim), rnd(n_req * kv_len, sh.n_kv_heads, sh.head_dim)) for _ in range(n_caches)]
    q = rnd(n_req * n_q, sh.n_q_heads, sh.head_dim)
    out = torch.empty_like(q)
    q_pos = torch.arange(n_doc, kv_len, dtype=torch.int32, device="cuda").repeat(n_req)
    cu_q = (np.arange(n_req + 1) * n_q).astype(np.int32)
    crs = np.arange(n_req + 1, dtype=np.int64) * kv_len
    if n_req == 1:
        ws = B.workspace(B.tr_prefill_attn_workspace_size(gs, n_q, kv_len))
    else:
        ws = B.workspace(B.tr_prefill_attn_batched_workspace_size(gs, cu_q, crs))
    c = {"i": 0}

    def att():
        c["i"] += 1
        ck, cv = caches[c["i"] % len(caches)]
        if n_req == 1:
            B.tr_prefill_attn(gs, q, ck, cv, q_pos, kv_len, out, ws)
        else:
            B.tr_prefill_attn_batched(gs, q, ck, cv, q_pos, cu_q, crs, out, ws)

    nbytes = n_req * (2 * kv_len * sh.n_kv_heads * sh.head_dim * 2 + 2 * n_q * sh.n_q_heads * sh.head_dim * 2)
    return att, nbytes


def bench_short_query(torch, B, synth, hbm_roof):
    rows = []
    for n_req, name, kernel in ((1, "short-query-16-tokens-over-12288-rows-qwen2-7b", "tr_prefill_attn"),
                                (16, "short-query-16req-x-16-tokens-over-12288-rows-qwen2-7b", "tr_prefill_attn_batched")):
        att, nbytes = _short_query_setup(torch, B, synth, n_req)
        rows.append(hbm_roof(kernel, name, nbytes, _time_calls(torch, att, 24 if n_req == 1 else 12)))
    return rows


def bench_table4_batches(torch, B, synth):
    """The step at the shape of the paper's Table 4 (8192 document tokens = 16 chunks x 512, 128 query tokens per
    request, Qwen2-7B heads) for batches of 1, 2, 4 and 8 requests, one launch per stage for the whole batch, the
    store resident on the device (the table's "w/o h2d" column; --host-store times the transfer)."""
    sh = synth.QWEN2_7B
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20241010)
    rnd = lambda *shape: torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    n_store, n_chunks, n_q = 256, 16, 128
    sd = B.Store(gs, rnd(n_store * 512, sh.n_kv_heads, sh.head_dim), rnd(n_store * 512, sh.n_kv_heads, sh.head_dim),
                 np.arange(n_store + 1, dtype=np.int64) * 512)
    rng = np.random.default_rng(11)
    rows = []
    for batch in (1, 2, 4, 8):
        ids = np.concatenate([rng.permutation(n_store)[:n_chunks] for _ in range(batch)]).astype(np.int32)
        cu_chunks = (np.arange(batch + 1) * n_chunks).astype(np.int32)
        modes = np.full(batch, synth.POS_REORDERED, np.int32)
        kv_len = n_chunks * 512 + n_q
        crs = (np.arange(batch + 1, dtype=np.int64) * kv_len)
        cu_q = (np.arange(batch + 1) * n_q).astype(np.int32)
        ck = torch.empty((batch * kv_len, sh.n_kv_heads, sh.head_dim), dtype=torch.bfloat16, device="cuda")
        cv = torch.empty_like(ck)
        q, k_q, v_q = rnd(batch * n_q, sh.n_q_heads, sh.head_dim), rnd(batch * n_q, sh.n_kv_heads, sh.head_dim), rnd(batch * n_q, sh.n_kv_heads, sh.head_dim)
        q_pos = torch.arange(n_chunks * 512, kv_len, dtype=torch.int32, device="cuda").repeat(batch)
        out = torch.empty_like(q)
        ws = B.workspace(B.tr_prefill_attn_batched_workspace_size(gs, cu_q, crs))

        def step():
            B.tr_kv_assemble_batched(sd, ids, cu_chunks, modes, crs, ck, cv)
            B.tr_kv_append_batched(gs, k_q, v_q, q_pos, cu_q, crs, ck, cv)
            B.tr_prefill_attn_batched(gs, q, ck, cv, q_pos, cu_q, crs, out, ws)

        t = _time_calls(torch, step, 20)
        rows.append({"batch": batch, "step_us": round(t[0], 2), "us_per_request": round(t[0] / batch, 2)})
    return {"what": "step (assemble, append, prefill attention; one layer) at Table 4's shape, 8192 document + 128 query tokens per request",
            "rows": rows}


DECODE_BATCH, DECODE_KV = 64, 4096


def _decode_setup(torch, B, synth):
    sh = synth.CONFIGS[2].shape
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20241007)
    rows = DECODE_BATCH * DECODE_KV
    k = torch.randn((rows, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(sh.torch_dtype)
    v = torch.randn((rows, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(sh.torch_dtype)
    q = torch.randn((DECODE_BATCH, sh.n_q_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(sh.torch_dtype)
    crs = np.arange(DECODE_BATCH + 1, dtype=np.int64) * DECODE_KV
    q_pos = torch.full((DECODE_BATCH,), DECODE_KV - 1, dtype=torch.int32, device="cuda")
    out = torch.empty_like(q)
    ws = B.workspace(B.tr_decode_attn_workspace_size(gs, crs))
    nbytes = (2 * rows * sh.n_kv_heads + 2 * DECODE_BATCH * sh.n_q_heads) * sh.head_dim * sh.elem_bytes
    return (lambda: B.tr_decode_attn(gs, q, k, v, q_pos, crs, out, ws)), nbytes


def bench_decode(torch, B, synth, hbm_roof):
    """Decode step: one new token for each of 64 requests, 4096 cache rows each, Qwen2-7B shape (random cache
    contents: the kernel's time does not depend on the values)."""
    run, nbytes = _decode_setup(torch, B, synth)
    t = _time_calls(torch, run, 20)
    return [hbm_roof("tr_decode_attn", "decode-%dx%d-qwen2-7b" % (DECODE_BATCH, DECODE_KV), nbytes, t)]


H2D_LAYERS = 28
PCIE_PEAK_GBS = 63.0   # PCIe 5.0 x16, per direction, after encoding


def bench_host_store(torch, B, synth, acct, layers, reps):
    """Host-resident store (the chunk caches stay in pinned host memory, as in the paper's end-to-end runs): the
    assemble kernel reads the chunks across PCIe and writes the rotated cache rows in one pass.  `layers` layers of
    configuration 2 (Sec. 4.5, Table 4's "with h2d" column), the same request each layer, `reps` times; `serial` runs assemble+append and attention of a layer back to back
    on one stream, `overlapped` assembles layer l+1 on a second stream while layer l's attention runs (two cache
    buffers).  Eager launches, wall clock."""
    cfg = synth.CONFIGS[2]
    sh = cfg.shape
    gs = B.make_shape(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, sh.rope_base)
    store = synth.make_store(cfg)
    sd = B.Store(gs, store.k.pin_memory(), store.v.pin_memory(), store.row_start)
    req = synth.make_requests(cfg, store)[0]
    offsets, _ = B.tr_plan(sd, req.chunk_ids, req.pos_mode, want_pos_ids=False)
    n_doc, kv_len = int(offsets[-1]), int(offsets[-1]) + req.n_q
    caches = [(torch.empty((kv_len, sh.n_kv_heads, sh.head_dim), dtype=sh.torch_dtype, device="cuda"),
               torch.empty((kv_len, sh.n_kv_heads, sh.head_dim), dtype=sh.torch_dtype, device="cuda")) for _ in range(2)]
    q, k_q, v_q = req.q.cuda(), req.k_q.cuda(), req.v_q.cuda()
    q_pos = torch.from_numpy(req.q_pos).cuda()
    out = torch.empty_like(q)
    ws = B.workspace(B.tr_prefill_attn_workspace_size(gs, req.n_q, kv_len))
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in range(2)]
    free = [torch.cuda.Event() for _ in range(2)]

    def fetch(l, stream):
        ck, cv = caches[l % 2]
        B.tr_kv_assemble_append(sd, req.chunk_ids, offsets, req.pos_mode, k_q, v_q, q_pos, ck, cv, stream=stream)

    def attend(l, stream):
        ck, cv = caches[l % 2]
        B.tr_prefill_attn(gs, q, ck, cv, q_pos, kv_len, out, ws, stream=stream)

    def serial():
        for l in range(layers):
            fetch(l, main)
            attend(l, main)

    def overlapped():
        for e in free:
            e.record(main)
        for l in range(layers):
            side.wait_event(free[l % 2])
            fetch(l, side)
            ready[l % 2].record(side)
            main.wait_event(ready[l % 2])
            attend(l, main)
            free[l % 2].record(main)

    res = {}
    for name, fn in (("serial", serial), ("overlapped", overlapped)):
        fn()
        torch.cuda.synchronize()
        gc.collect()
        gc.disable()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) / (reps * layers) * 1e6
        gc.enable()
    nbytes = acct.assemble_bytes(n_doc, sh.n_kv_heads, sh.head_dim, sh.elem_bytes) // 2   # bytes that cross PCIe per layer
    rate = nbytes / (res["overlapped"] * 1e-6) / 1e9
    return [{"kernel": "tr_kv_assemble_append + tr_prefill_attn, host-resident store", "workload": cfg.name, "bound": "pcie",
             "achieved": round(rate, 1), "peak": PCIE_PEAK_GBS, "unit": "GB/s", "frac": round(rate / PCIE_PEAK_GBS, 4),
             "us_per_layer_serial": round(res["serial"], 1), "us_per_layer_overlapped": round(res["overlapped"], 1),
             "pcie_bytes_per_layer": nbytes, "layers": layers, "reps": reps,
             "note": "PCIe-inclusive; never part of `value`, which is measured with the store resident in HBM"}]


def measured_copy_rate(torch):
    """What a plain device-to-device copy of 256 MiB reaches on this GPU (read + written bytes per second, GB/s):
    the practical ceiling the HBM-bound kernels are up against, next to the published 8 TB/s."""
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    t = _time_calls(torch, lambda: dst.copy_(src), 10)
    return round(2 * src.numel() / (t[0] * 1e-6) / 1e9, 1)


def measured_mfma_loop(torch, B):
    """What a bare loop of the attention kernels' matrix instruction reaches on this GPU in this run (TFLOP/s): 8
    waves on every compute unit, operands from LDS, no softmax and no memory traffic.  Constant operands, and bf16
    operands of random sign and mantissa; the second is the ceiling attention over real data is up against."""
    sink = torch.empty(B.tr_probe_mfma_loop_sink_bytes() // 4, dtype=torch.float32, device="cuda")
    res = {}
    for key, rnd in (("mfma_loop_tflops_constant_operands", 0), ("mfma_loop_tflops_random_operands", 1)):
        B.tr_probe_mfma_loop(2000, rnd, sink)
        torch.cuda.synchronize()
        rates = []
        for _ in range(3):
            e0, e1 = _events(torch, 2)
            e0.record()
            flops = B.tr_probe_mfma_loop(30000, rnd, sink)
            e1.record()
            torch.cuda.synchronize()
            rates.append(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        res[key] = round(sorted(rates)[1], 1)
    return res


def cpu_baseline(synth, cfg):
    """The CPU oracle as it stands on one whole request of the headline configuration (the whole step: plan,
    assemble, append, attention), timed once."""
    import oracle
    store = synth.make_store(cfg)
    req = synth.make_requests(cfg, store)[0]
    bits = synth.as_oracle_array
    ks, vs = bits(store.k), bits(store.v)
    qb, kqb, vqb = bits(req.q), bits(req.k_q), bits(req.v_q)
    t0 = time.perf_counter()
    oracle.online_prefill(ks, vs, store.row_start, req.chunk_ids, req.pos_mode, qb, kqb, vqb, req.q_pos, cfg.shape.rope_base)
    dt = time.perf_counter() - t0
    return {"value": round(dt * 1e6, 1), "unit": "us/layer", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "one full request of configuration %d in %.1f s (plan, assemble, append, attention over %d keys for %d "
                      "query tokens); fp64, attention loops on all threads, gather and RoPE single-threaded"
                      % (cfg.number, dt, int(req.n_doc + req.n_q), int(req.n_q))}


if __name__ == "__main__":
    main()
