#!/usr/bin/env python3
"""Benchmark of the DDD draft round on one MI355X.

A "step" is one whole draft round (Algorithm 1 of the paper end to end: reset, up to D draft
calls each = stand-in draft body + LM-head kernel + merge/beam/stop kernel, final tree,
stand-in target, accept walk).  By default the host paces the draft calls (ddd_round_run);
`--launch graph` replays one captured HIP graph per round instead, and the default run times
that form too, beside the headline.  Inputs are seeded and synthetic (7B-shaped by default)
and resident in HBM before the timed region starts.

Prints ONE JSON line: draft rounds/s plus us per executed depth step, the roofline of the
dominant kernel (the LM-head weight stream at B = 1: HBM; the MFMA GEMM at B = 64), the
round-level HBM fraction, the CPU oracle timed on a bounded sample, and - in the default
run - a `secondary` list with the other workloads of the metric (7B shape at B = 64, 13B
shape, large vocabulary), each measured the same way on fewer rounds.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E peak
MFMA_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 MFMA peak
CACHE_BYTES = 256 * 2**20   # memory-side cache (Infinity Cache)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(wl, W_bits, plant_dir, threshold, budget_s):
    """The CPU oracle, as it stands, on a bounded sample of the same rounds: sequence after sequence of round 0,
    then of round 1, ... until the time budget is used."""
    from oracle import synth_round as SR
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    t0 = time.perf_counter()
    n = steps = 0
    while True:
        res, _, _ = SR.oracle_round(wl, W_bits, plant_dir, n % wl.B, n // wl.B, threshold=threshold)
        n += 1
        steps += res.steps
        el = time.perf_counter() - t0
        if el > budget_s or n >= 64:
            break
    what = (f"{n} rounds of sequence 0, rounds 0..{n - 1}" if wl.B == 1 else
            f"{n} sequence-rounds (sequences 0..{min(n, wl.B) - 1} of round 0" + (", then round 1 ..." if n > wl.B else "") + ")")
    return {"value": n / el, "unit": "rounds/s" if wl.B == 1 else "sequence-rounds/s", "cores": int(threads),
            "kind": "oracle", "sample": f"{what}, {steps} depth steps, {el:.1f} s",
            "us_per_depth_step": 1e6 * el / steps}


def time_tree_attention(torch, D, g, wl, L, side):
    """ddd_tree_attention on the workload's final trees (as left by the last round), random q / k / v."""
    B, T, nh = wl.B, wl.m + 1, wl.H // 128
    Tp, Lp = (T + 31) // 32 * 32, (L + 31) // 32 * 32
    rnd = lambda *s: torch.randn(*s, device="cuda").to(torch.bfloat16)
    q, kt = rnd(B, T, nh, 128), rnd(B, T, nh, 128)
    vtt = torch.zeros(B, nh, 128, Tp, device="cuda", dtype=torch.bfloat16)
    vtt[..., :T] = rnd(B, nh, 128, T)
    kpk = torch.empty(B * nh * (Lp // 32) * 4096, device="cuda", dtype=torch.bfloat16)
    vpk = torch.empty_like(kpk)
    D.ddd_kv_pack(g.ctx, rnd(B, L, nh, 128), rnd(B, L, nh, 128), L, nh, kpk, vpk)
    ws = torch.empty(max(1, D.ddd_tree_attention_workspace(g.ctx, nh, L) // 4), dtype=torch.float32, device="cuda")
    res = torch.empty(B, T, nh, 128, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    n = 50
    with torch.cuda.stream(side):
        for _ in range(5):
            D.ddd_tree_attention(g.ctx, g.tree, q, kt, vtt, kpk, vpk, L, nh, ws, res, stream=side.cuda_stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(side)
        for _ in range(n):
            D.ddd_tree_attention(g.ctx, g.tree, q, kt, vtt, kpk, vpk, L, nh, ws, res, stream=side.cuda_stream)
        e1.record(side)
        side.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / n
    alg = 2 * B * (L + T) * nh * 256 + B * T * nh * 128 * (2 + 4)   # keys and values once, queries in, fp32 rows out
    return {"us_per_call": us, "B": B, "tree_nodes": T, "heads": nh, "prompt_len": L, "algorithmic_bytes": alg,
            "GBs": alg / us / 1e3, "hbm_frac": alg / us / 1e3 / HBM_PEAK_GBS}


def time_verify_sample(torch, D, g, wl, temperature, side):
    """ddd_verify_sample on the workload's final trees (as left by the last round): target logits N(0, 2) over the
    vocabulary, most tree nodes favouring the token of one of their children (what synth.make_target_logits does on
    the host, written here with device tensors because the 7b_b64 shape is 500 MB of logits)."""
    B, T, V = wl.B, wl.m + 1, wl.V
    gen = torch.Generator(device="cuda").manual_seed(1234)
    logits = torch.randn(B, T, V, device="cuda", generator=gen) * 2.0
    tok, par = g.tree_t["tree_token"].view(B, T).long(), g.tree_t["parent_idx"].view(B, T).long()
    n_sel = g.tree_t["n_sel"].view(B).long()
    idx = torch.arange(T, device="cuda")
    valid = (idx[None, :] >= 1) & (idx[None, :] <= n_sel[:, None])
    # every valid node proposes itself to its parent with a random priority; the parent's row favours the winner
    prio = torch.rand(B, T, device="cuda", generator=gen).masked_fill(~valid, -1.0)
    best = torch.full((B, T), -1.0, device="cuda").scatter_reduce(1, par.clamp(min=0), prio, "amax", include_self=True)
    win = valid & (prio == best.gather(1, par.clamp(min=0))) & (torch.rand(B, T, device="cuda", generator=gen) < 0.8)
    bsel, csel = torch.nonzero(win, as_tuple=True)
    logits[bsel, par[bsel, csel], tok[bsel, csel]] += 13.0
    ua = torch.rand(B, T, device="cuda", dtype=torch.float64, generator=gen)
    ub = torch.rand(B, T, device="cuda", dtype=torch.float64, generator=gen)
    alen = torch.zeros(B, dtype=torch.int32, device="cuda")
    apath = torch.zeros(B, wl.D + 1, dtype=torch.int32, device="cuda")
    bonus = torch.zeros(B, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    call = lambda: D.ddd_verify_sample(g.ctx, g.tree, logits, temperature, ua, ub, alen, apath, bonus, stream=side.cuda_stream)
    n = 50
    with torch.cuda.stream(side):
        for _ in range(5):
            call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(side)
        for _ in range(n):
            call()
        e1.record(side)
        side.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / n
    rows = int((alen.long() + 1).sum())
    alg = rows * V * 4            # one pass over the logit row of every node on the accepted paths
    return {"us_per_call": us, "B": B, "tree_nodes": T, "temperature": temperature,
            "mean_accept_len": float(alen.float().mean()), "rows_read": rows,
            "rows_longest_path": int(alen.max()) + 1, "algorithmic_bytes": alg,
            "GBs": alg / us / 1e3, "hbm_frac": alg / us / 1e3 / HBM_PEAK_GBS}


def time_rounds(torch, g, launch, steps, warmup, side):
    """`warmup` untimed rounds, then exactly `steps` timed ones between synchronisations; returns wall seconds,
    the event time and the histograms the rounds' post hook kept on the device."""
    torch.cuda.synchronize()
    g.set_round(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(warmup):
            launch()
        side.synchronize()
        g.depth_hist.zero_()
        g.accept_hist.zero_()
        g.batch_depth_hist.zero_()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        e0.record(side)
        for _ in range(steps):
            launch()
        e1.record(side)
        side.synchronize()
        torch.cuda.synchronize()
        wall = time.perf_counter() - w0
    depth_hist = g.depth_hist.cpu().numpy()
    return {"wall": wall, "ev_ms": e0.elapsed_time(e1), "depth_hist": depth_hist,
            "accept_hist": g.accept_hist.cpu().numpy(),
            "exec_steps": int(sum(d * int(c) for d, c in enumerate(depth_hist))),
            # a depth step of the batch = one LM-head pass: a round executes as many as its deepest sequence
            "batch_steps": int(sum(d * int(c) for d, c in enumerate(g.batch_depth_hist.cpu().numpy())))}


def trace_rounds(torch, D, g, wl, n_rounds, launch, side):
    """Device-timestamp breakdown of the draft calls (B = 1 weight-stream workloads): `n_rounds` rounds with the
    context's trace on, read back after every round.  Times in microseconds (100 MHz wall clock, 10 ns steps):
    where a call's time goes inside the weight-stream launch (workgroup start skew, first tile, steady stream,
    last workgroup's lag), between the launches, and inside the bookkeeping launch."""
    import numpy as np
    D.ddd_trace_enable(g.ctx, True)
    acc = {}

    def add(name, v):
        acc.setdefault(name, []).append(float(v) / 100.0)

    nsl = D.ddd_num_slices(g.ctx)
    per_slice = []
    try:
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            for _ in range(n_rounds):
                launch()
                side.synchronize()
                steps = int(g.st_t["steps"][0])
                tr = D.ddd_trace_read(g.ctx).astype(np.int64)
                prev_end = None
                for s in range(steps):
                    st = tr[s, :nsl * 8].reshape(nsl, 8)
                    bk = tr[s, 256 * 8:256 * 8 + 8]
                    if (st[:, :6] == 0).any() or (bk[:6] == 0).any():
                        continue
                    t0, t1, t2, t3 = st[:, 0], st[:, 1], st[:, 2], st[:, 5]
                    if (st[:, 6] != 0).all():
                        add("stream: last tile multiplied by wave 0 -> by every wave (barrier), median", np.median(st[:, 6] - t2))
                        add("stream: -> folded into the row statistics, median", np.median(st[:, 3] - st[:, 6]))
                    else:
                        add("stream: last tile multiplied -> folded into the row statistics, median", np.median(st[:, 3] - t2))
                    add("stream: -> the lanes' lists exchanged through LDS, median", np.median(st[:, 4] - st[:, 3]))
                    add("stream: -> k merge rounds, partials written, median", np.median(st[:, 5] - st[:, 4]))
                    per_slice.append((t3 - t0.min()) / 100.0)
                    add("stream: launch span (first workgroup in -> last out)", t3.max() - t0.min())
                    add("stream: workgroup start skew (last in - first in)", t0.max() - t0.min())
                    add("stream: entry -> first tile multiplied, median", np.median(t1 - t0))
                    add("stream: first -> last tile, median", np.median(t2 - t1))
                    add("stream: last tile -> partials written, median", np.median(t3 - t2))
                    add("stream: median workgroup in -> out", np.median(t3 - t0))
                    add("stream: last workgroup out - median out", t3.max() - np.median(t3))
                    add("gap: stream out -> bookkeeping in", bk[0] - t3.max())
                    add("bookkeeping: entry -> slice keys arrived", bk[1] - bk[0])
                    add("bookkeeping: merge of the rows", bk[2] - bk[1])
                    add("bookkeeping: beam update + stop test", bk[3] - bk[2])
                    if bk[4] - bk[3] > 20:                      # a tree was built in this call (more than 0.2 us)
                        add("bookkeeping: final tree (stopping call)", bk[4] - bk[3])
                    add("bookkeeping: entry -> exit", bk[5] - bk[0])
                    if prev_end is not None:
                        add("gap: bookkeeping out -> next stream in (draft body between)", t0.min() - prev_end[0])
                        add("call period (stream in -> next stream in)", t0.min() - prev_end[1])
                    prev_end = (bk[5], t0.min())
    finally:
        D.ddd_trace_enable(g.ctx, False)
    out = {k: {"mean_us": float(np.mean(v)), "min_us": float(np.min(v)), "max_us": float(np.max(v)), "n": len(v)}
           for k, v in acc.items()}
    for k, v in out.items():
        log(f"[trace] {k:78s} mean {v['mean_us']:7.2f}  min {v['min_us']:7.2f}  max {v['max_us']:7.2f}  (n={v['n']})")
    if per_slice:
        # is the lag of the last workgroups a property of where they run?  mean finish time per workgroup index
        ps = np.mean(np.stack(per_slice), axis=0)
        by8 = [float(np.mean(ps[i::8])) for i in range(8)]
        out["finish_us_by_workgroup_mod_8"] = by8
        order = np.argsort(ps)
        log(f"[trace] mean finish time after the first entry, by workgroup index mod 8: {[round(x, 2) for x in by8]}")
        log(f"[trace] earliest workgroups {order[:8].tolist()} ({ps[order[:8]].round(2).tolist()}), latest "
            f"{order[-8:].tolist()} ({ps[order[-8:]].round(2).tolist()}); spread of the per-workgroup means "
            f"{float(ps.max() - ps.min()):.2f} us")
        out["finish_us_spread_of_workgroup_means"] = float(ps.max() - ps.min())
    return out


def kernel_roofline(torch, D, SD, g, wl, iters, side, traffic_path):
    """The LM-head kernel alone: HIP events around stand-alone launches on the stream they run on (all B*k rows
    active; <= 16 rows: the weight stream, HBM-bound; more: the MFMA GEMM), in three settings - as consecutive
    draft calls run it (alternating sweep direction: a launch starts in what its predecessor left in the memory-side
    cache), every launch sweeping forward, and every launch after a 1 GB read of other memory (nothing of W
    cached) - plus a plain read-stream kernel and, for MFMA-bound shapes, a register-resident MFMA loop as the
    practical ceilings."""
    n_rows = wl.B * wl.k
    w_bytes = wl.V * wl.H * 2
    mean_ms, min_ms = D.ddd_profile_lmhead(g.ctx, g.W, g.hid, n_rows, iters, stream=side.cuda_stream)
    if n_rows <= 16 and wl.k <= 16:
        kernel_name = "lmhead_stream_kernel"
        alg_bytes = w_bytes + n_rows * wl.H * 2 + n_rows * D.ddd_num_slices(g.ctx) * (wl.k * 8 + 4)
    else:
        kernel_name = "lmhead_gemm_kernel"
        alg_bytes = w_bytes + n_rows * wl.H * 2 + n_rows * (wl.k * 8 + 4)   # W, hidden rows, k keys + lse per row
    alg_flops = 2.0 * wl.V * wl.H * n_rows
    achieved = alg_bytes / (mean_ms * 1e-3) / 1e9
    achieved_tflops = alg_flops / (mean_ms * 1e-3) / 1e12
    mfma_bound = alg_flops / (MFMA_PEAK_TFLOPS * 1e12) > alg_bytes / (HBM_PEAK_GBS * 1e9)

    # the same launch with every call sweeping forward, and with the memory-side cache emptied before each launch
    cfg_fwd = D.make_config(wl.B, wl.H, wl.V, wl.k, wl.D, wl.m, wl.threshold, wl.check_mask, D.DDD_FLAG_FORWARD_SWEEPS)
    ctx_fwd = D.ddd_create(cfg_fwd)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    try:
        if g.packed:
            D.ddd_weights_pack(ctx_fwd, g.W, stream=side.cuda_stream)
        fwd_ms, _ = D.ddd_profile_lmhead(ctx_fwd, g.W, g.hid, n_rows, iters, stream=side.cuda_stream)
        other = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        other.zero_()
        cold = []
        for _ in range(24):
            SD.N.ddd_synth_read_stream(other, other.numel(), sink, 4096, stream=side.cuda_stream)
            cold.append(D.ddd_profile_lmhead(ctx_fwd, g.W, g.hid, n_rows, 1, stream=side.cuda_stream)[0])
        cold_ms = sum(cold[4:]) / len(cold[4:])
        del other
    finally:
        D.ddd_destroy(ctx_fwd)

    # plain read stream over the same bytes: the practical ceiling of an HBM-bound kernel
    with torch.cuda.stream(side):
        best = None
        for blocks in (2048, 4096, 8192):
            for _ in range(3):
                SD.N.ddd_synth_read_stream(g.W, w_bytes, sink, blocks, stream=side.cuda_stream)
            r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            r0.record(side)
            for _ in range(20):
                SD.N.ddd_synth_read_stream(g.W, w_bytes, sink, blocks, stream=side.cuda_stream)
            r1.record(side)
            side.synchronize()
            gbs = 20 * w_bytes / (r0.elapsed_time(r1) * 1e-3) / 1e9
            best = gbs if best is None else max(best, gbs)
    # register-resident MFMA loop on random operands: the practical matrix-core ceiling
    mfma_ceiling = None
    if mfma_bound:
        fsink = torch.zeros(1, dtype=torch.float32, device="cuda")
        with torch.cuda.stream(side):
            it, blocks = 4000, 512             # 2 waves per SIMD; 512*4*4000*8 MFMAs of 32768 flop
            SD.N.ddd_synth_mfma_rate(fsink, 200, blocks, stream=side.cuda_stream)
            m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            m0.record(side)
            SD.N.ddd_synth_mfma_rate(fsink, it, blocks, stream=side.cuda_stream)
            m1.record(side)
            side.synchronize()
        mfma_ceiling = blocks * 4 * it * 8 * 32768.0 / (m0.elapsed_time(m1) * 1e-3) / 1e12

    # a plain device-to-device copy of W (known size: reads and writes V*H*2 bytes): the reference the
    # rocprofv3 FETCH_SIZE / WRITE_SIZE counters are scaled by
    with torch.cuda.stream(side):
        wcopy = torch.empty_like(g.W)
        for _ in range(3):
            wcopy.copy_(g.W)
        side.synchronize()
        del wcopy

    # HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload (null if none)
    traffic, source = None, None
    if os.path.exists(traffic_path):
        with open(traffic_path) as f:
            tj = json.load(f)
        traffic = tj.get("bytes")
        source = (f"{os.path.relpath(traffic_path, ROOT)}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                  f"scaled by a copy of known size (committed; not measured in this run; see {tj.get('source')})")
    if mfma_bound:
        roof = {"bound": "mfma", "achieved": achieved_tflops, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved_tflops / MFMA_PEAK_TFLOPS, "hbm_GBs": achieved, "hbm_frac": achieved / HBM_PEAK_GBS,
                "frac_forward_sweep": alg_flops / (fwd_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                "frac_cache_flushed": alg_flops / (cold_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS}
    else:
        roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS,
                "frac_forward_sweep": alg_bytes / (fwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "frac_cache_flushed": alg_bytes / (cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "mfma_TFLOPs": achieved_tflops}
    roof.update({"traffic": traffic, "traffic_source": source, "kernel": kernel_name, "rows": n_rows,
                 "sweep_of_frac": "alternating (memory-side cache included when W is within its reach: "
                                  f"W = {w_bytes / 2**20:.0f} MiB, cache = 256 MiB)",
                 "us_per_launch": mean_ms * 1e3, "us_per_launch_min": min_ms * 1e3,
                 "us_per_launch_forward_sweep": fwd_ms * 1e3, "us_per_launch_cache_flushed": cold_ms * 1e3,
                 "algorithmic_bytes_per_launch": alg_bytes, "algorithmic_flops_per_launch": alg_flops,
                 "launches_timed": iters, "read_stream_ceiling_GBs": best, "mfma_loop_ceiling_TFLOPs": mfma_ceiling})
    log(f"[bench] {wl.name}: {kernel_name} ({n_rows} rows): {mean_ms * 1e3:.2f} us per launch (min {min_ms * 1e3:.2f}; "
        f"forward sweeps {fwd_ms * 1e3:.2f}; cache flushed {cold_ms * 1e3:.2f}); {alg_bytes / 1e6:.2f} MB -> {achieved:.0f} GB/s "
        f"({100 * achieved / HBM_PEAK_GBS:.1f}% of 8 TB/s); {alg_flops / 1e9:.1f} GFLOP -> {achieved_tflops:.0f} TFLOP/s "
        f"({100 * achieved_tflops / MFMA_PEAK_TFLOPS:.1f}% of {MFMA_PEAK_TFLOPS:.0f}); read stream {best:.0f} GB/s"
        + (f"; MFMA loop {mfma_ceiling:.0f} TFLOP/s" if mfma_ceiling else ""))
    return roof


def run_workload(torch, D, synth, SD, wl, thr, args, steps, warmup, launch_mode, also_graph, cpu_budget, W_cache,
                 with_kernel=True):
    """One workload measured end to end; returns the fields of its JSON object.  with_kernel=False skips the
    stand-alone timing of the LM-head kernel (variants of a workload whose kernel launch is the same)."""
    log(f"[bench] workload {wl.name}: B={wl.B} H={wl.H} V={wl.V} k={wl.k} D={wl.D} m={wl.m} t={thr} gain={wl.gain}")
    t0 = time.perf_counter()
    key = (wl.V, wl.H, wl.sigma_w, wl.seed, wl.dup_pairs)
    g = SD.GpuWorkload(wl, W_bits=W_cache.get(key), threshold=thr, debug=False,
                       flags=D.DDD_FLAG_FORWARD_SWEEPS if args.sweep == "forward" else 0)
    W_cache.clear()                 # keep one matrix at most (the 7B head serves both 7B workloads)
    W_cache[key] = g.W_bits
    log(f"[bench] inputs generated and uploaded in {time.perf_counter() - t0:.1f} s; "
        f"stream slices={D.ddd_num_slices(g.ctx)}")
    if args.body == "layer":
        F = args.ffn if args.ffn is not None else (13824 if wl.H == 5120 else 11008)
        t1 = time.perf_counter()
        g.use_layer_body(F, args.prompt_len)
        log(f"[bench] draft layer: F={F}, prompt length {args.prompt_len}, {g.body_bytes / 1e6:.1f} MB of layer weights "
            f"streamed per call ({time.perf_counter() - t1:.1f} s to generate and upload)")
    uses_gemm = wl.B * wl.k > 16 or wl.k > 16
    g.packed = args.pack_weights == "on" or (args.pack_weights == "auto" and uses_gemm and wl.V * wl.H * 2 > CACHE_BYTES)
    if g.packed:
        D.ddd_weights_pack(g.ctx, g.W)
        torch.cuda.synchronize()
        log("[bench] GEMM path reads W from its tile-major copy (ddd_weights_pack)")
    side = torch.cuda.Stream()
    launchers = {"paced": lambda: g.run_round(side.cuda_stream), "eager": lambda: g.enqueue_round(side.cuda_stream),
                 "graph": lambda: g.launch(side.cuda_stream)}
    also_graph = also_graph and args.graph_rounds > 0
    if launch_mode == "graph" or also_graph:
        g.capture(side)
    r = time_rounds(torch, g, launchers[launch_mode], steps, warmup, side)
    n_round_seq = int(r["depth_hist"].sum())
    assert n_round_seq == steps * wl.B, (n_round_seq, steps, wl.B)
    wall = r["wall"]
    rounds_per_s = steps * wl.B / wall
    w_bytes = wl.V * wl.H * 2
    log(f"[bench] {steps} rounds ({launch_mode}) in {wall * 1e3:.2f} ms wall ({r['ev_ms']:.2f} ms by events): "
        f"{rounds_per_s:.1f} {'rounds' if wl.B == 1 else 'sequence-rounds'}/s, {1e6 * wall / steps:.1f} us/round, "
        f"{1e6 * wall / max(1, r['batch_steps']):.1f} us per executed depth step")
    log(f"[bench] depth histogram (steps -> sequences): { {d: int(c) for d, c in enumerate(r['depth_hist']) if c} }")
    log(f"[bench] accept-length histogram: { {d: int(c) for d, c in enumerate(r['accept_hist']) if c} }")
    launch_names = {"graph": "one hipGraph per round", "eager": "stream launches",
                    "paced": "stream launches paced by the host (ddd_round_run)"}
    modes = {launch_mode: {"rounds_per_s": rounds_per_s, "us_per_round": 1e6 * wall / steps, "rounds_timed": steps}}
    if launch_mode == "paced":
        modes["paced"]["host_waits"] = D.ddd_round_run_stats(g.ctx)
    if also_graph and launch_mode != "graph":
        n2 = max(steps, args.graph_rounds)
        r2 = time_rounds(torch, g, launchers["graph"], n2, warmup, side)
        modes["graph"] = {"rounds_per_s": n2 * wl.B / r2["wall"], "us_per_round": 1e6 * r2["wall"] / n2, "rounds_timed": n2}
        log(f"[bench] the same rounds as one hipGraph each: {modes['graph']['rounds_per_s']:.1f}/s, "
            f"{modes['graph']['us_per_round']:.1f} us/round")

    traffic_path = args.traffic or os.path.join(ROOT, "profiles", f"traffic_{wl.name}.json")
    roof = kernel_roofline(torch, D, SD, g, wl, args.profile_iters, side, traffic_path) if with_kernel else {}
    # round level: one pass over W per executed depth step of the batch is what the method has to move
    roof["round_frac"] = r["batch_steps"] * w_bytes / wall / 1e9 / HBM_PEAK_GBS
    roof["round_GBs"] = r["batch_steps"] * w_bytes / wall / 1e9
    out = {
        "value": rounds_per_s,
        "unit": "rounds/s" if wl.B == 1 else "sequence-rounds/s",
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": 1e3 * wall / steps,
        "config": {"workload": wl.name, "B": wl.B, "H": wl.H, "V": wl.V, "k": wl.k, "max_depth": wl.D, "m": wl.m,
                   "threshold": thr, "check_mask": int(wl.check_mask), "mode": args.mode, "hidden_gain": wl.gain,
                   "launch": launch_names[launch_mode], "launch_modes": modes,
                   "paced_timeouts": modes.get("paced", {}).get("host_waits", {}).get("timeouts"),
                   "packed_weights": bool(g.packed), "sweep": args.sweep, "body": args.body,
                   "body_weight_bytes_per_call": int(getattr(g, "body_bytes", 0)),
                   "depth_hist": {str(d): int(c) for d, c in enumerate(r["depth_hist"]) if c},
                   "accept_len_hist": {str(d): int(c) for d, c in enumerate(r["accept_hist"]) if c},
                   "executed_depth_steps": r["exec_steps"], "executed_batch_steps": r["batch_steps"],
                   "us_per_depth_step": 1e6 * wall / max(1, r["batch_steps"]),
                   "mean_depth": r["exec_steps"] / max(1, n_round_seq)},
        "roofline": roof,
    }
    if args.trace > 0 and not uses_gemm:
        g.set_round(0)
        out["trace"] = trace_rounds(torch, D, g, wl, args.trace, launchers["paced" if launch_mode == "graph" else launch_mode], side)
    if args.tree_attention > 0:
        out["tree_attention"] = time_tree_attention(torch, D, g, wl, args.tree_attention, side)
        log(f"[bench] tree attention: {out['tree_attention']}")
    if args.verify_sample > 0:
        out["verify_sample"] = time_verify_sample(torch, D, g, wl, args.verify_sample, side)
        log(f"[bench] sampled acceptance: {out['verify_sample']}")
    if cpu_budget > 0:
        log(f"[bench] timing the CPU oracle for about {cpu_budget:.0f} s ...")
        out["cpu_baseline"] = cpu_baseline(wl, g.W_bits, g.plant_dir_np if wl.n_plant else None, thr, cpu_budget)
        log(f"[bench] oracle: {out['cpu_baseline']}")
    g.close()
    del g
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000, help="timed draft rounds")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="7b_b1", help="synthetic workload name (see synth/inputs.py)")
    ap.add_argument("--threshold", type=float, default=None, help="stop threshold t (default: the workload's)")
    ap.add_argument("--k", type=int, default=None, help="beam width override (wide beams above 16; Appendix, Table 2)")
    ap.add_argument("--max-depth", type=int, default=None, help="maximum number of draft calls override")
    ap.add_argument("--m", type=int, default=None, help="final tree size override")
    ap.add_argument("--mode", choices=["default", "paper", "strict", "eagle2"], default="default",
                    help="paper: the paper's setting n=11, S={5,7,9}, x=-0.3 (t=exp(x)) of Section 3.2; strict: the same "
                         "with the test after every call (Table 1's DDD + Strict row, Section 3.4); eagle2: fixed depth "
                         "6, no stop test (Section 3.2)")
    ap.add_argument("--cpu-budget", type=float, default=15.0, help="seconds of oracle time for cpu_baseline (0 = skip)")
    ap.add_argument("--profile-iters", type=int, default=200)
    ap.add_argument("--launch", choices=["paced", "graph", "eager"], default="paced",
                    help="paced (default): ddd_round_run, the host queues draft call s once call s-2 has reported that a "
                         "sequence is still active; graph: one captured hipGraph of all max_depth calls per round; eager: "
                         "plain stream launches of all max_depth calls")
    ap.add_argument("--body", choices=["hash", "layer"], default="hash",
                    help="draft body between the LM-head calls: the hash-based hidden-state generator of the workload "
                         "(default: the LM head and the bookkeeping are all a round does), or the stand-in draft layer "
                         "(embedding + FC + one decoder layer with tree attention, synthetic weights; weight streams for up "
                         "to 16 rows per call, the MFMA path for batched rounds)")
    ap.add_argument("--ffn", type=int, default=None, help="MLP width of the draft layer (default 11008, 13824 for H=5120)")
    ap.add_argument("--lm-sigma", type=float, default=None, help="std of the LM-head weights with --body layer (default 0.07)")
    ap.add_argument("--prompt-len", type=int, default=256, help="prompt positions every draft row attends to")
    ap.add_argument("--tree-attention", type=int, default=0, metavar="L",
                    help="also time ddd_tree_attention (the consumer of the tree mask) for the workload's B and m, H/128 "
                         "heads and a prompt of L positions; adds a tree_attention object to the JSON line")
    ap.add_argument("--sweep", choices=["alternate", "forward"], default="alternate",
                    help="direction in which the weight-stream kernel walks W: alternating between consecutive draft calls "
                         "(default; a call starts in what the previous one left in the memory-side cache) or always forward")
    ap.add_argument("--verify-sample", type=float, default=0.0, metavar="T",
                    help="also time ddd_verify_sample (sampled acceptance at temperature T > 0) on the workload's final "
                         "trees with synthetic target logits; adds a verify_sample object to the JSON line")
    ap.add_argument("--pack-weights", choices=["auto", "on", "off"], default="auto",
                    help="tile-major copy of W for the GEMM path (ddd_weights_pack); auto: when the GEMM path is used "
                         "and W is larger than the 256 MB Infinity Cache, i.e. really streams from HBM")
    ap.add_argument("--traffic", default=None,
                    help="JSON file with the HBM bytes per launch from rocprofv3 --pmc runs "
                         "(default: profiles/traffic_<workload>.json)")
    ap.add_argument("--graph-rounds", type=int, default=200,
                    help="rounds (at least) of the second timing leg, the same rounds launched as one hipGraph each; 0 skips it")
    ap.add_argument("--trace", type=int, default=0, metavar="N",
                    help="also run N rounds with the context's device-timestamp trace on (B*k <= 16 workloads) and add the "
                         "breakdown of a draft call - inside the weight-stream launch, between launches, inside the "
                         "bookkeeping launch - as a trace object to the JSON line")
    ap.add_argument("--secondary", choices=["auto", "on", "off"], default="auto",
                    help="also measure, into a `secondary` list, the other thresholds and the paper's parameter modes at the "
                         "7B shape, the other workloads of the metric (7b_b64, 13b_b1, large_vocab; 200 rounds each) and "
                         "the rounds with the stand-in draft layer; auto: in the plain default run only (no workload, "
                         "mode, shape or body option)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import numpy as np  # noqa: F401
    import torch
    import paper_2409_00142_amd as D
    import synth
    from synth import device as SD

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a gfx950 GPU (the HIP path has no CPU fallback)")
    D.load_library()
    wl = synth.WORKLOADS[args.workload]
    if args.mode != "default":    # Section 3.2's parameters / Table 1's strict variant / EAGLE-2's fixed depth
        wl = synth.paper_mode(wl, args.mode)
    over = {n: v for n, v in (("k", args.k), ("D", args.max_depth), ("m", args.m)) if v is not None}
    if over:
        wl = wl.with_(**over)
    if args.body == "layer":
        # the layer's output rows have an rms of about 1.4, not the hash body's gain of 3.5: a wider LM head
        # gives the logits the same spread (std about 4.5), so that rounds again stop at mixed depths
        wl = wl.with_(sigma_w=args.lm_sigma if args.lm_sigma is not None else 0.07)
    thr = wl.threshold if args.threshold is None else args.threshold
    plain = (args.workload == "7b_b1" and args.mode == "default" and not over and args.body == "hash"
             and args.threshold is None and args.launch == "paced" and args.sweep == "alternate")
    secondary = args.secondary == "on" or (args.secondary == "auto" and plain)

    W_cache = {}
    res = run_workload(torch, D, synth, SD, wl, thr, args, args.steps, args.warmup, args.launch,
                       also_graph=True, cpu_budget=args.cpu_budget, W_cache=W_cache)
    out = {
        "metric": "DDD draft rounds/sec (7B-shaped synthetic draft round, whole hot path per round)",
        "value": res["value"],
        "unit": res["unit"],
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
    }
    out.update({k: v for k, v in res.items() if k not in out})
    if secondary:
        import copy
        out["secondary"] = []

        def variant(label, name, steps, full, **over):
            a2 = copy.copy(args)
            a2.tree_attention, a2.verify_sample, a2.trace = 0, 0.0, 0
            w2 = synth.WORKLOADS[name]
            thr2 = over.pop("threshold", None)
            for key, val in over.items():
                setattr(a2, key, val)
            if a2.mode != "default":
                w2 = synth.paper_mode(w2, a2.mode)
            if a2.body == "layer":
                w2 = w2.with_(sigma_w=0.07)
            sec = run_workload(torch, D, synth, SD, w2, w2.threshold if thr2 is None else thr2, a2, steps, 10, "paced",
                               also_graph=True, cpu_budget=min(args.cpu_budget, 5.0) if full else 0.0, W_cache=W_cache,
                               with_kernel=full)
            sec["label"] = label
            out["secondary"].append(sec)

        # the other thresholds of the 7B B = 1 configuration, and the paper's own parameter settings (same kernel launch)
        variant("7b_b1, t = 0.1", "7b_b1", 1000, False, threshold=0.1)
        variant("7b_b1, t = 0.5", "7b_b1", 1000, False, threshold=0.5)
        variant("7b_b1, Section 3.2's parameters (n = 11, S = {5,7,9}, x = -0.3)", "7b_b1", 300, False, mode="paper")
        variant("7b_b1, the same checked after every call (Table 1: DDD + Strict)", "7b_b1", 300, False, mode="strict")
        variant("7b_b1, EAGLE-2's fixed depth 6", "7b_b1", 300, False, mode="eagle2")
        # the batched half of the metric, with the consumers of the tree on its trees
        variant("7b_b64", "7b_b64", 200, True, tree_attention=2048, verify_sample=1.0)
        variant("13b_b1", "13b_b1", 200, True)
        variant("large_vocab", "large_vocab", 200, True)
        # the stand-in draft layer between the LM-head calls (472 MB of layer weights per call)
        variant("7b_b1 with the stand-in draft layer", "7b_b1", 200, False, body="layer")
        variant("7b_b64 with the stand-in draft layer", "7b_b64", 30, False, body="layer")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
