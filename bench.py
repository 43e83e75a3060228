#!/usr/bin/env python3
"""Benchmark of the pre-gated MoE hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--also cfg5_top2,cfg2,...] [--all] [--no-sweep-k]

A "step" is one pass of the whole hot path over one batch: conventional gate of block 0,
pre-gates, migration of the pre-gated experts from pinned host memory, token grouping,
expert FFNs and weighted combine, for all L blocks of the stack.  Inputs (hidden states of
every step, gate weights) are resident in HBM before the timed region; the expert store is in
pinned host memory (offloaded workloads) or in HBM (resident workloads), as the workload says.

Prints ONE JSON line.  The headline numbers are those of --workload (default: the largest
configuration, the Switch-Large-128 decode stack with top-1 routing, 25.8 GB of experts in pinned
host memory); --also adds abbreviated results of other workloads under "other_workloads" (same
measurement, fewer steps); the top-2 run of the same model shares the headline's expert store.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # dense bf16, published
HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
LINK_PEAK_GBPS = 64.0       # PCIe gen5 x16, per direction, nominal


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, steps_sample, host_threads):
    """Time the CPU oracle (as it stands) on a bounded sample of the same workload: once on one
    thread and once on all the threads OpenMP gives it here (it parallelises over tokens, so it can
    use at most T of them)."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import workloads as W
    from oracle import reference as R

    gates = W.gate_tensors(w)
    cache = {}

    def gen(be):
        if be not in cache:
            w1, w2 = W.expert_weights(w, *be)
            cache[be] = (W.to_bf16_bits(w1), W.to_bf16_bits(w2)) if w.dtype == "bf16" else (w1, w2)

    xs = [W.step_input(w, s) for s in range(steps_sample)]
    # untimed pass: the same chain block by block, generating the experts each block's routing asks
    # for on a thread pool (weight generation is not part of what is timed)
    with ThreadPoolExecutor(max_workers=max(1, host_threads)) as pool:
        for x0 in xs:
            hs = [np.asarray(x0, np.float64)]
            for i, (gw, gb) in enumerate(gates):
                g = R.gate(hs[R.routing_source(i)], gw, gb, w.top_k)
                need = [(i, int(e)) for e in np.unique(g["idx"])]
                list(pool.map(gen, need))
                y = R.block(hs[i], g["p"], g["idx"], {e: cache[(b, e)] for b, e in need}, w.d_ff)
                hs.append(hs[i] + y)

    def timed(threads):
        t0 = time.perf_counter()
        for x in xs:
            R.stack_forward(x, gates, w.top_k, lambda b, e: cache[(b, e)], w.d_ff, threads=threads)
        return time.perf_counter() - t0

    n_all = int(min(R.max_threads(), w.tokens))
    dt1 = timed(1)
    dtn = timed(n_all) if n_all > 1 else dt1
    tok = w.tokens * steps_sample
    return {"value": tok / dtn, "unit": "tokens/s", "cores": n_all, "kind": "oracle",
            "sample": f"{steps_sample} steps x {w.n_blocks} blocks x {w.tokens} tokens of {w.name} (fp64, routed): "
                      f"{dtn:.2f} s on {n_all} threads, {dt1:.2f} s on one; expert weight generation excluded",
            "ms_per_token_per_layer": 1e3 * dtn / (tok * w.n_blocks),
            "single_thread": {"value": tok / dt1, "unit": "tokens/s", "cores": 1,
                              "ms_per_token_per_layer": 1e3 * dt1 / (tok * w.n_blocks)},
            "host": {"cpu_model": cpu_model(), "threads_openmp_offers": int(R.max_threads()),
                     "logical_cpus": os.cpu_count()}}


def measured_peaks():
    """Plain-copy rates of this machine, for context next to the nominal peaks (torch copies only)."""
    import torch
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device="cuda")
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    h = torch.empty(256 << 20, dtype=torch.uint8, pin_memory=True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    b.copy_(a)
    a[: h.numel()].copy_(h, non_blocking=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(5):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    d2d = 2.0 * n * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    e0.record()
    for _ in range(4):
        a[: h.numel()].copy_(h, non_blocking=True)
    e1.record()
    torch.cuda.synchronize()
    h2d = h.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return {"hbm_copy_read_plus_write_GBps": d2d, "h2d_pinned_256MiB_GBps": h2d}


def vendor_gemm_context(w):
    """Context only, never part of `value`: what the vendor's GEMM library (hipBLASLt behind torch.bmm)
    needs for the same two products with the rows dealt evenly to the experts, and for one large
    square product: how much of the published matrix-core peak a tuned library delivers on this
    box for this shape and for its best case."""
    import torch
    E, M, d, f = w.n_experts, w.tokens * w.top_k // w.n_experts, w.d_model, w.d_ff

    def timed(fn, n=40):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n * 1e3

    g = torch.Generator(device="cuda").manual_seed(1)
    x = torch.randn(E, M, d, device="cuda", dtype=torch.bfloat16, generator=g)
    w1 = torch.randn(E, d, f, device="cuda", dtype=torch.bfloat16, generator=g) * 0.02
    w2 = torch.randn(E, f, d, device="cuda", dtype=torch.bfloat16, generator=g) * 0.02
    h = torch.empty(E, M, f, device="cuda", dtype=torch.bfloat16)
    y = torch.empty(E, M, d, device="cuda", dtype=torch.bfloat16)
    up = timed(lambda: torch.bmm(x, w1, out=h))
    down = timed(lambda: torch.bmm(h, w2, out=y))
    n = 8192
    a = torch.randn(n, n, device="cuda", dtype=torch.bfloat16, generator=g)
    c = torch.empty(n, n, device="cuda", dtype=torch.bfloat16)
    sq = timed(lambda: torch.mm(a, a, out=c), 10)
    flops = 4.0 * E * M * d * f
    return {"up_us": up, "down_us": down, "both_TFLOPs": flops / (up + down) / 1e6,
            "both_frac_of_mfma_peak": flops / (up + down) / 1e6 / MFMA_BF16_PEAK_TFLOPS,
            "square_8192_TFLOPs": 2.0 * n ** 3 / sq / 1e6, "square_8192_frac_of_mfma_peak": 2.0 * n ** 3 / sq / 1e6 / MFMA_BF16_PEAK_TFLOPS,
            "note": f"torch.bmm (vendor GEMM library) on [{E}, {M}, {d}] x [{E}, {d}, {f}] and [{E}, {M}, {f}] x [{E}, {f}, {d}], "
                    "back-to-back launches, no ReLU, no routing; and torch.mm on 8192^3: a measuring stick for the peak, not a code path"}


def pmc_traffic(workload_name):
    """HBM bytes per FFN launch from the committed rocprofv3 --pmc summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "expert_ffn_hbm_traffic.md")
    try:
        m = re.search(r"^traffic_bytes_per_launch\[%s\]\s*=\s*([0-9.eE+]+)" % re.escape(workload_name),
                      open(path).read(), flags=re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def run_workload(name, K, Wm, host_threads, with_cpu, cpu_steps, trace_steps, gpu_only=True, systems=False,
                 cache_frac=0.2, store=None, graphs=False, fetch_mode="auto", extras=None):
    """systems: also the paper's comparison systems on this workload; extras (default: as systems): also the
    other migration engine, pre-gate distance 2/3 and the non-MoE stand-in rows."""
    extras = systems if extras is None else extras
    import numpy as np
    import torch

    import workloads as W
    from paper_2308_12066_amd import harness as H

    w = W.CONFIGS[name]
    K = K if K is not None else w.steps
    Wm = Wm if Wm is not None else max(2, min(16, K // 8))
    L, T, k, E = w.n_blocks, w.tokens, w.top_k, w.n_experts

    t0 = time.perf_counter()
    cfg = H.config_for(w)
    own_store = store is None
    if own_store:
        store = H.ExpertStore(w, cfg, threads=host_threads)
    from paper_2308_12066_amd import binding as B
    # migration engine: the library's own choice by default (copy engines for large per-block
    # migrations, the device-side pull kernel for small ones), or forced from the command line
    mig_flags = {"auto": B.FLAG_FETCH_AUTO, "pull": 0, "memcpy": B.FLAG_FETCH_MEMCPY}[fetch_mode]
    stack = H.Stack(w, store, flags=mig_flags)
    engine = stack.ctx.migration_engine if w.offloaded else "none"
    # Every timed step gets its own hidden-state block (slice 0 pre-filled with that step's
    # input) and its own routing-index slice, so the timed loop holds library calls only.
    n_in = min(K, max(1, (1 << 30) // ((L + 1) * T * w.d_model * w.elem_bytes)))   # distinct inputs kept in HBM
    x_all = torch.zeros((n_in, L + 1, T, w.d_model), dtype=stack.x_states.dtype, device="cuda")
    for s in range(n_in):
        x_all[s, 0].copy_(H.to_device(W.step_input(w, s % max(w.steps, 1)), w.dtype))
    idx_log = torch.zeros((K, L, T, k), dtype=torch.int32, device="cuda")
    step_bufs = [stack.ctx.make_step_buffers(stack.gate_w, stack.gate_b, x_all[s % n_in], stack.y_blocks, idx_log[s],
                                             stack.topk_prob, stack.row_of, stack.expert_offsets, stack.x_perm,
                                             stack.y_perm, stack.workspace) for s in range(K)]
    torch.cuda.synchronize()
    log(f"[bench] {w.name}: store {store.host.numel() / 2**30:.2f} GiB built in {time.perf_counter() - t0:.1f} s")

    def two_passes(stk, bufs):
        """pass 1: K steps, nothing but the hot path on the streams (-> step time);
        pass 2: the same K steps with an event pair around every expert-FFN kernel launch (each
        pair costs several microseconds on the stream, which is why pass 1 runs without)."""
        def run(count):
            for s in range(count):
                stk.ctx.stack_step(bufs[s % K], T, stk.compute, stk.copy)
        run(Wm)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(K)
        torch.cuda.synchronize()
        dt_clean = time.perf_counter() - t0
        stk.ctx.ffn_timing_begin(K * L)
        t1 = time.perf_counter()
        run(K)
        torch.cuda.synchronize()
        dt_ev = time.perf_counter() - t1
        n_t, ms, oh = stk.ctx.ffn_timing_end()
        assert stk.ctx.device_flags() == 0
        return dt_clean, dt_ev, n_t, ms, oh

    dt, dt_events, n_timed, ffn_ms, overhead_us = two_passes(stack, step_bufs)

    def graph_replay(stk, buf, x_buf):
        """One step captured into a HIP graph (pgmoe_stack_step only enqueues) and replayed K times,
        each time after copying that step's input into the captured input buffer: what a serving
        loop that re-uses its buffers runs.  Same work per step as the eager loop (gates,
        migration, FFNs, fresh routing per step)."""
        g = torch.cuda.CUDAGraph()
        saved = x_buf.clone()
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=stk.compute):
            stk.ctx.stack_step(buf, T, stk.compute, stk.copy)
        torch.cuda.synchronize()
        with torch.cuda.stream(stk.compute):
            for s in range(Wm):
                x_buf.copy_(x_all[(s + 1) % n_in, 0], non_blocking=True)
                g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(K):
                x_buf.copy_(x_all[(s + 1) % n_in, 0], non_blocking=True)
                g.replay()
            torch.cuda.synchronize()
            dtg = time.perf_counter() - t0
        del g
        x_buf.copy_(saved)          # step 0's own input back in place for the later passes
        torch.cuda.synchronize()
        return {"tokens_per_s": T * K / dtg, "ms_per_step": 1e3 * dtg / K}

    # algorithmic bytes of the FFN launches: weights of the distinct experts each launch touches
    # plus its activation rows in and out
    idx_host = idx_log.cpu().numpy()
    uniq = np.array([[len(np.unique(idx_host[s, b])) for b in range(L)] for s in range(K)])
    act_bytes = 2 * T * k * w.d_model * w.elem_bytes
    ffn_bytes = float(uniq.sum()) * w.expert_bytes + float(K * L) * act_bytes
    raw_us = 1e3 * ffn_ms / max(n_timed, 1)
    ffn_avg_us = max(raw_us - overhead_us, 1e-3)
    per_launch = ffn_bytes / max(n_timed, 1)
    ffn_gbps = per_launch / (ffn_avg_us * 1e-6) / 1e9 if n_timed else 0.0
    h2d_bytes = float(uniq.sum()) * w.expert_bytes if w.offloaded else 0.0

    out = {
        "metric": "tokens/s through the pre-gated MoE stack (all layers; ms/token/layer alongside)",
        "value": T * K / dt,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": 1e3 * dt / K,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: L={L} d_model={w.d_model} d_ff={w.d_ff} E={E} top{k} T={T}/step, "
                               f"experts {'offloaded to pinned host memory' if w.offloaded else 'resident in HBM'}",
                   "tokens_per_step": T, "blocks": L,
                   "migration": {"copy_engine": "copy engines: one hipMemcpyAsync per expert, issued by the host once it has read "
                                                "the routing back", "pull": "device-side pull kernel", "none": "none"}[engine]
                                + (" (the library's choice for this configuration)" if fetch_mode == "auto" and w.offloaded else "")},
        "ms_per_token": 1e3 * dt / (T * K),
        "ms_per_token_per_layer": 1e3 * dt / (T * K * L),
        "block_latency_us": 1e6 * dt / (K * L),
        "roofline": {"bound": "hbm", "achieved": ffn_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": ffn_gbps / HBM_PEAK_GBPS, "traffic": pmc_traffic(w.name),
                     "kernel": stack.ctx.ffn_kernel_name(T * k),
                     "launches": n_timed, "avg_launch_us": ffn_avg_us, "event_pair_us": raw_us,
                     "event_overhead_us": overhead_us, "algorithmic_bytes_per_launch": per_launch,
                     "ms_per_step_with_events": 1e3 * dt_events / K},
        "host_link": {"bytes_per_step": h2d_bytes / K, "achieved_GBps": h2d_bytes / dt / 1e9,
                      "peak_GBps": LINK_PEAK_GBPS, "frac": h2d_bytes / dt / 1e9 / LINK_PEAK_GBPS,
                      "mean_unique_experts_per_block": float(uniq.mean())},
    }

    # stream pairs (compute, copy, the library's own copy stream) that share a hardware queue after
    # the harness has asked the library to check and replaced streams: 0 = all run side by side
    out["streams"] = {"pairs_sharing_a_hardware_queue": stack.shared_streams}
    if out["roofline"]["kernel"].startswith("ffn_gemm"):
        # hundreds of rows per expert: the two tiled GEMMs are bound by the matrix cores, not by
        # HBM (arithmetic intensity = rows per expert); the timed region spans both GEMM kernels
        flops = 4.0 * T * k * w.d_model * w.d_ff
        tf = flops / (ffn_avg_us * 1e-6) / 1e12
        out["roofline"].update({"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "flops_per_launch": flops,
                                "hbm_achieved_GBps": ffn_gbps, "hbm_frac": ffn_gbps / HBM_PEAK_GBPS})
        if gpu_only:     # not in the --main-only runs the profiler summaries are taken from
            out["roofline"]["vendor_library_context"] = vendor_gemm_context(w)
    if graphs and engine != "copy_engine":   # the host-issued migration cannot be captured
        out["graph_replay"] = graph_replay(stack, step_bufs[0], x_all[0, 0])
    if w.offloaded and trace_steps > 0:
        # pass 3: instrumented steps for the overlap figures (per-block events on both streams)
        stack.ctx.trace(True)
        busy = busy0 = stall = stall0 = comp = fsum = csum = cbytes = 0.0
        for s in range(trace_steps):
            stack.ctx.stack_step(step_bufs[s % K], T, stack.compute, stack.copy)
            torch.cuda.synchronize()
            tr = [stack.ctx.block_trace(b) for b in range(L)]
            # time with at least one migration in flight (the pull kernels of consecutive blocks
            # may share the link, so their durations must not simply be added)
            iv = sorted((t.fetch_start_ms, t.fetch_end_ms) for t in tr)
            end = -1e30
            for a, b in iv:
                busy += max(0.0, b - max(a, end))
                end = max(end, b)
            busy0 += tr[0].fetch_ms
            stall += sum(t.stall_ms for t in tr)
            stall0 += tr[0].stall_ms
            comp += sum(t.compute_ms for t in tr)
            fsum += sum(t.fetch_ms for t in tr)
            csum += sum(t.copy_ms for t in tr)
            cbytes += float(uniq[s % K].sum()) * w.expert_bytes
        stack.ctx.trace(False)
        n = float(trace_steps)
        out["overlap"] = {
            "steps": trace_steps,
            "link_busy_ms_per_step": busy / n, "stall_ms_per_step": stall / n, "compute_ms_per_step": comp / n,
            "sum_of_fetch_durations_ms_per_step": fsum / n,
            # the copies alone (the pull kernel's own clock readings, without its wait for the turn on the
            # link; with the copy engines the events around a block's copies): bytes / time = link rate
            "sum_of_copy_times_ms_per_step": csum / n,
            "link_GBps_while_copying": cbytes / max(csum, 1e-9) / 1e6,
            "hidden_frac": 1.0 - stall / busy,
            "hidden_frac_without_block0": 1.0 - (stall - stall0) / max(busy - busy0, 1e-9),
            "hidden_frac_upper_bound": min(1.0, comp / busy),
            "overlap_efficiency": (busy - stall) / max(min(comp, busy), 1e-9),
            "note": "hidden = share of the time with a migration in flight during which the compute stream was not "
                    "waiting for experts; compute = the MoE blocks only (no attention or other non-MoE layers exist "
                    "here to hide behind); block 0's fetch is exposed by construction",
        }
    if w.offloaded and gpu_only:
        # The paper's GPU-only design point on the same workload: every expert resident in HBM,
        # nothing migrates.  Also gives the FFN kernel's duration without a migration kernel
        # running next to it.
        w2 = w.replace(offloaded=False)
        stack2 = H.Stack(w2, store)
        bufs2 = [stack2.ctx.make_step_buffers(stack2.gate_w, stack2.gate_b, x_all[s % n_in], stack2.y_blocks, idx_log[s],
                                              stack2.topk_prob, stack2.row_of, stack2.expert_offsets, stack2.x_perm,
                                              stack2.y_perm, stack2.workspace) for s in range(K)]
        dt2, _, n2, ms2, oh2 = two_passes(stack2, bufs2)
        us2 = max(1e3 * ms2 / max(n2, 1) - oh2, 1e-3)
        out["gpu_only"] = {"value": T * K / dt2, "unit": "tokens/s", "ms_per_step": 1e3 * dt2 / K,
                           "ffn_avg_launch_us": us2, "ffn_achieved_GBps": per_launch / (us2 * 1e-6) / 1e9,
                           "ffn_frac_of_hbm_peak": per_launch / (us2 * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                           "note": "same workload and routing with all experts resident in HBM (no migration); a "
                                   "decode-sized expert launch here also carries the next block's pre-gate as one extra "
                                   "workgroup, so its duration is that of the combined launch"}
        if w.dtype == "bf16":
            # The expert-FFN kernel on its own: the primitive calls (pgmoe_permute, pgmoe_expert_ffn) over
            # the K steps' routings, block after block, so that every launch reads other experts than the
            # one before it (the same expert launched back to back is served by the 256 MB last-level
            # cache, not by HBM); no migration beside it, no pre-gate on board.
            ctx2 = stack2.ctx
            ctx2.ffn_timing_begin(K * L)
            for s_ in range(K):
                for b in range(L):
                    ctx2.permute(x_all[s_ % n_in, b], idx_log[s_, b], T, stack2.x_perm, stack2.row_of[b], stack2.expert_offsets[b],
                                 stack2.compute)
                    ctx2.expert_ffn(b, stack2.x_perm, stack2.expert_offsets[b], T * k, stack2.y_perm, stack2.workspace,
                                    stack2.compute)
            torch.cuda.synchronize()
            n3, ms3, oh3 = ctx2.ffn_timing_end()
            us3 = max(1e3 * ms3 / max(n3, 1) - oh3, 1e-3)
            alone = {"avg_launch_us": us3, "achieved_GBps": per_launch / (us3 * 1e-6) / 1e9,
                     "frac_of_hbm_peak": per_launch / (us3 * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                     "note": "pgmoe_permute + pgmoe_expert_ffn over the same routings with resident experts, one block after "
                             "the other: the kernel with no migration beside it and no pre-gate on board"}
            if ctx2.ffn_kernel_name(T * k).startswith("ffn_gemm"):
                alone["achieved_TFLOPs"] = 4.0 * T * k * w.d_model * w.d_ff / (us3 * 1e-6) / 1e12
                alone["frac_of_mfma_peak"] = alone["achieved_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
            out["roofline"]["kernel_alone"] = alone
        if graphs:
            out["gpu_only"]["graph_replay"] = graph_replay(stack2, bufs2[0], x_all[0, 0])
        stack2.close()
        del stack2, bufs2
    if w.offloaded and extras:
        # The other migration engine on the same workload, same passes: what the choice costs and buys.
        other = "pull" if engine == "copy_engine" else "copy_engine"
        stk = H.Stack(w, store, flags=0 if other == "pull" else B.FLAG_FETCH_MEMCPY)
        bufs = [stk.ctx.make_step_buffers(stk.gate_w, stk.gate_b, x_all[s % n_in], stk.y_blocks, idx_log[s], stk.topk_prob,
                                          stk.row_of, stk.expert_offsets, stk.x_perm, stk.y_perm, stk.workspace) for s in range(K)]
        dto, _, no, mso, oho = two_passes(stk, bufs)
        uso = max(1e3 * mso / max(no, 1) - oho, 1e-3)
        stk.close()
        del stk, bufs

        def engine_row(dt_, us_):
            return {"tokens_per_s": T * K / dt_, "ms_per_step": 1e3 * dt_ / K, "host_link_GBps": h2d_bytes / dt_ / 1e9,
                    "ffn_avg_launch_us": us_, "ffn_frac_of_hbm_peak": per_launch / (us_ * 1e-6) / 1e9 / HBM_PEAK_GBPS}
        out["migration_engines"] = {engine: engine_row(dt, ffn_avg_us), other: engine_row(dto, uso), "used_for_value": engine}
    if w.offloaded and cache_frac > 0:
        # Expert cache on top of the migration (the paper's caching study: a fraction of each
        # block's experts kept in HBM across steps; LRU here, all three policies for the headline
        # workload).  A labelled extra: `value` above is the base design without a cache.
        C = max(1, min(B.MAX_CACHE_SLOTS, int(np.ceil(cache_frac * E))))
        out["expert_cache"] = {"slots_per_block": C, "fraction_of_experts": C / E}
        pols = (("lru", B.CACHE_LRU), ("lfu", B.CACHE_LFU), ("lifo", B.CACHE_LIFO)) if systems else (("lru", B.CACHE_LRU),)
        for pname, pol in pols:
            stk = H.Stack(w, store, cache_slots=C, cache_policy=pol)     # the cache is kept by the pull kernel
            bufs = [stk.ctx.make_step_buffers(stk.gate_w, stk.gate_b, x_all[s % n_in], stk.y_blocks, idx_log[s],
                                              stk.topk_prob, stk.row_of, stk.expert_offsets, stk.x_perm, stk.y_perm,
                                              stk.workspace) for s in range(K)]
            for s in range(Wm):
                stk.ctx.stack_step(bufs[s % K], T, stk.compute, stk.copy)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(K):
                stk.ctx.stack_step(bufs[s], T, stk.compute, stk.copy)
            torch.cuda.synchronize()
            dtc = time.perf_counter() - t0
            # hit rate of a few further steps, read back step by step
            hits = sel = 0
            for s in range(min(K, 16)):
                stk.ctx.stack_step(bufs[s], T, stk.compute, stk.copy)
                torch.cuda.synchronize()
                for b in range(L):
                    fs = stk.ctx.fetch_stats(b)
                    hits += fs.cache_hits
                    sel += fs.n_unique
            out["expert_cache"][pname] = {"tokens_per_s": T * K / dtc, "ms_per_step": 1e3 * dtc / K,
                                          "speedup_vs_no_cache": dt / dtc, "hit_rate": hits / max(sel, 1)}
            if "migration_engines" in out:    # against the uncached pull engine too (the cache lives in the pull kernel)
                out["expert_cache"][pname]["speedup_vs_uncached_pull"] = \
                    out["migration_engines"]["pull"]["ms_per_step"] / (1e3 * dtc / K)
            stk.close()
            del stk, bufs
    if w.offloaded and systems:
        # The paper's comparison systems on the same kernels and the same workload (conventional
        # wiring): experts fetched on demand after the gate, or all experts of the next block
        # prefetched.  Block latency is what the paper's latency figure compares.
        Ks = min(K, 32)
        comp = {"pregated": {"block_latency_us": 1e6 * dt / (K * L), "tokens_per_s": T * K / dt,
                             "peak_resident_expert_MB": float((uniq[:, :-1] + uniq[:, 1:]).max() if L > 1 else uniq.max())
                             * w.expert_bytes / 1e6}}
        for sname, sched in (("on_demand", B.SCHED_ON_DEMAND), ("prefetch_all", B.SCHED_PREFETCH_ALL)):
            stk = H.Stack(w, store, slots_per_gen=E if sched == B.SCHED_PREFETCH_ALL else 0, flags=mig_flags)
            stk.ctx.set_schedule(sched)
            bufs = [stk.ctx.make_step_buffers(stk.gate_w, stk.gate_b, x_all[s % n_in], stk.y_blocks, idx_log[s],
                                              stk.topk_prob, stk.row_of, stk.expert_offsets, stk.x_perm, stk.y_perm,
                                              stk.workspace) for s in range(Ks)]
            for s in range(2):
                stk.ctx.stack_step(bufs[s], T, stk.compute, stk.copy)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(Ks):
                stk.ctx.stack_step(bufs[s], T, stk.compute, stk.copy)
            torch.cuda.synchronize()
            dts = time.perf_counter() - t0
            u2 = np.array([[len(np.unique(r)) for r in step] for step in idx_log[:Ks].cpu().numpy()])
            peak = 2 * E if sched == B.SCHED_PREFETCH_ALL else int(u2.max())
            comp[sname] = {"block_latency_us": 1e6 * dts / (Ks * L), "tokens_per_s": T * Ks / dts,
                           "peak_resident_expert_MB": peak * w.expert_bytes / 1e6}
            stk.close()
            del stk, bufs
        if "gpu_only" in out:
            comp["gpu_only"] = {"block_latency_us": 1e3 * out["gpu_only"]["ms_per_step"] / L,
                                "tokens_per_s": out["gpu_only"]["value"],
                                "peak_resident_expert_MB": L * E * w.expert_bytes / 1e6}
        base = comp["pregated"]["block_latency_us"]
        for v in comp.values():
            v["block_latency_vs_pregated"] = v["block_latency_us"] / base
        out["systems"] = comp
    if w.offloaded and systems and extras:
        # Pre-gate looking N = 2 / 3 blocks ahead (the paper's activation-level study, system
        # side): experts are requested N blocks early and N + 1 generations stay resident.
        dist = {"1": {"tokens_per_s": T * K / dt, "block_latency_us": 1e6 * dt / (K * L),
                      "resident_generations": 2}}
        for N in (2, 3):
            if N >= L:
                continue
            stk = H.Stack(w, store, pregate_distance=N, flags=mig_flags)
            bufs = [stk.ctx.make_step_buffers(stk.gate_w, stk.gate_b, x_all[s % n_in], stk.y_blocks, idx_log[s],
                                              stk.topk_prob, stk.row_of, stk.expert_offsets, stk.x_perm, stk.y_perm,
                                              stk.workspace) for s in range(K)]
            for s in range(Wm):
                stk.ctx.stack_step(bufs[s % K], T, stk.compute, stk.copy)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(K):
                stk.ctx.stack_step(bufs[s], T, stk.compute, stk.copy)
            torch.cuda.synchronize()
            dtn = time.perf_counter() - t0
            assert stk.ctx.device_flags() == 0
            dist[str(N)] = {"tokens_per_s": T * K / dtn, "block_latency_us": 1e6 * dtn / (K * L),
                            "resident_generations": N + 1}
            stk.close()
            del stk, bufs
        out["pregate_distance"] = dist
        # Sensitivity row, separately labelled and not part of `value`: the non-MoE layers that sit
        # between two MoE blocks in the real model (and that the paper's migration also hides
        # behind) replaced by a kernel that only keeps the compute stream busy for a given time per
        # block.  Shows where the design's benefit comes from: once the work per block reaches the
        # migration time, the migration of every block but the first disappears behind it.
        sens = {}
        Kq = min(K, 32 if 1e3 * dt / K < 5.0 else 8)
        # one Stack for every row: the same streams, hence the same hardware queues, throughout
        stk = H.Stack(w, store, flags=mig_flags)
        bufs = [stk.ctx.make_step_buffers(stk.gate_w, stk.gate_b, x_all[s % n_in], stk.y_blocks, idx_log[s],
                                          stk.topk_prob, stk.row_of, stk.expert_offsets, stk.x_perm, stk.y_perm,
                                          stk.workspace) for s in range(Kq)]
        # stand-in durations: none, then about 0.6, 1.2 and 2.4 times this workload's block latency
        # (100 / 200 / 400 us for the batch-1 decode stack, whose block takes 170 us)
        unit_us = max(100.0, 100.0 * round(0.6 * 1e6 * dt / (K * L) / 100.0))
        for us in (0.0, unit_us, 2.0 * unit_us, 4.0 * unit_us):
            row = {}
            for sname, sched in (("pregated", B.SCHED_PREGATED), ("on_demand", B.SCHED_ON_DEMAND)):
                stk.ctx.set_schedule(sched)
                stk.ctx.set_nonmoe_standin(us)
                for s in range(2):
                    stk.ctx.stack_step(bufs[s], T, stk.compute, stk.copy)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for s in range(Kq):
                    stk.ctx.stack_step(bufs[s], T, stk.compute, stk.copy)
                torch.cuda.synchronize()
                dts = time.perf_counter() - t0
                row[sname + "_block_latency_us"] = 1e6 * dts / (Kq * L)
                if sched == B.SCHED_PREGATED:
                    stk.ctx.trace(True)
                    busy = stall = busy0 = stall0 = 0.0
                    for s in range(4):
                        stk.ctx.stack_step(bufs[s], T, stk.compute, stk.copy)
                        torch.cuda.synchronize()
                        tr = [stk.ctx.block_trace(b) for b in range(L)]
                        end = -1e30
                        for a, b in sorted((t.fetch_start_ms, t.fetch_end_ms) for t in tr):
                            busy += max(0.0, b - max(a, end))
                            end = max(end, b)
                        busy0 += tr[0].fetch_ms
                        stall += sum(t.stall_ms for t in tr)
                        stall0 += tr[0].stall_ms
                    stk.ctx.trace(False)
                    row["hidden_frac"] = 1.0 - stall / busy
                    row["hidden_frac_without_block0"] = 1.0 - (stall - stall0) / max(busy - busy0, 1e-9)
            row["on_demand_vs_pregated"] = row["on_demand_block_latency_us"] / row["pregated_block_latency_us"]
            sens[str(int(us))] = row
        stk.close()
        del stk, bufs
        out["nonmoe_standin_sensitivity"] = {
            "note": "NOT the headline: a clock-watching kernel of the given microseconds per block stands in for the "
                    "non-MoE layers of the real model; block latency includes it",
            "by_standin_us": sens}
    if with_cpu:
        # about 10 s of oracle time on one thread (2.1 ms per token and block at d_model 768, d_ff 3072,
        # in proportion to d_model * d_ff elsewhere), then the same steps on all threads
        per_step_s = 2.1e-3 * T * L * k * (w.d_model * w.d_ff) / (768.0 * 3072.0)
        sample = cpu_steps or max(1, min(1000, int(round(10.0 / per_step_s))))
        log(f"[bench] {w.name}: timing the CPU oracle on {sample} steps")
        out["cpu_baseline"] = cpu_baseline(w, sample, host_threads)
    stack.close()
    if own_store:
        store.device = None
    del stack, store, x_all, step_bufs
    torch.cuda.empty_cache()
    return out


def activated_expert_sweep(host_threads, steps):
    """Block latency of the four systems against the number of activated experts on the
    Switch-Base-64 shape at batch 1 (the paper's micro-benchmark, Sec. VI-D), each normalised to
    GPU-only at the same k.  One expert store serves every k (same seed index)."""
    import workloads as W
    from paper_2308_12066_amd import harness as H

    first = W.CONFIGS[f"sweep64_k{W.SWEEP_K[0]}"]
    store = H.ExpertStore(first, H.config_for(first), threads=host_threads)
    rows = {}
    # from the largest k down: the first point then migrates every expert of every block, so no
    # later point pays the first access to a blob of the pinned store inside its timed steps
    # (with one expert per block and step, the two warm-up steps would leave most blobs untouched)
    for k in sorted(W.SWEEP_K, reverse=True):
        r = run_workload(f"sweep64_k{k}", steps, 2, host_threads, False, None, 0, systems=True, cache_frac=0.0, store=store,
                         extras=False)
        sysm = r["systems"]
        g = sysm["gpu_only"]["block_latency_us"]
        rows[str(k)] = {n: {"block_latency_us": v["block_latency_us"], "vs_gpu_only": v["block_latency_us"] / g,
                            "peak_resident_expert_MB": v["peak_resident_expert_MB"]} for n, v in sysm.items()}
        rows[str(k)]["link_GBps"] = r["host_link"]["achieved_GBps"]
        log(f"[bench] sweep k={k}: " + ", ".join(f"{n} {v['block_latency_us']:.0f} us" for n, v in sysm.items()))
    del store
    return {"shape": "Switch-Base-64 (d_model 768, d_ff 3072, 64 experts, 6 blocks), 1 token per step",
            "steps": steps, "by_top_k": {str(k): rows[str(k)] for k in W.SWEEP_K}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg5")
    ap.add_argument("--also", default="cfg5_top2,cfg2,cfg3,cfg4,base8_prefill",
                    help="comma list of further workloads to summarise ('' for none); base8_prefill is the supplementary "
                         "shape with ~512 rows per expert, where the FFN is bound by the matrix cores")
    ap.add_argument("--all", action="store_true", help="also run the offloaded Switch-Base-128 prefill")
    ap.add_argument("--fetch", default="auto", choices=("auto", "pull", "memcpy"),
                    help="migration engine of the offloaded workloads: the library's choice by configuration (default), the "
                         "device-side pull kernel, or one hipMemcpyAsync per expert issued by the host")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-steps", type=int, default=None)
    ap.add_argument("--trace-steps", type=int, default=8)
    ap.add_argument("--host-threads", type=int, default=16)
    ap.add_argument("--main-only", action="store_true",
                    help="only the timed passes of --workload (no GPU-only, cache, comparison-system or distance passes): "
                         "what the rocprofv3 summaries under profiles/ are taken from")
    ap.add_argument("--no-sweep-k", action="store_true",
                    help="leave out the activated-expert sweep (top-1..64 on the Switch-Base-64 shape, four systems)")
    ap.add_argument("--sweep-steps", type=int, default=8)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    import workloads as W
    from paper_2308_12066_amd import harness as H

    others = [n for n in args.also.split(",") if n and n != args.workload]
    if args.all:
        others += [n for n in ("cfg4_offloaded",) if n not in others]
    # workloads with the same seed index have the same expert weights (Switch-Large-128 top-1 and
    # top-2; the resident and the offloaded prefill): they share one expert store
    stores = {}

    def store_for(name):
        w = W.CONFIGS[name]
        users = [n for n in [args.workload] + others if W.CONFIGS[n].index == w.index]
        if len(users) < 2:
            return None
        if w.index not in stores:
            t0 = time.perf_counter()
            stores[w.index] = H.ExpertStore(w, H.config_for(w), threads=args.host_threads)
            log(f"[bench] shared expert store of {', '.join(users)}: built in {time.perf_counter() - t0:.1f} s")
        return stores[w.index]

    def drop_store(name):
        """The last user of a shared store has run: give its pinned and device memory back."""
        w = W.CONFIGS[name]
        rest = [n for n in pending if W.CONFIGS[n].index == w.index]
        if not rest and w.index in stores:
            stores.pop(w.index).device = None
            torch.cuda.empty_cache()

    pending = list(others)
    if args.main_only:
        out = run_workload(args.workload, args.steps, args.warmup, args.host_threads, not args.no_cpu_baseline,
                           args.cpu_sample_steps, args.trace_steps, gpu_only=False, systems=False, cache_frac=0.0,
                           store=store_for(args.workload), fetch_mode=args.fetch)
    else:
        out = run_workload(args.workload, args.steps, args.warmup, args.host_threads, not args.no_cpu_baseline,
                           args.cpu_sample_steps, args.trace_steps, systems=True, graphs=True, store=store_for(args.workload),
                           fetch_mode=args.fetch)
    drop_store(args.workload)
    out["measured_peaks"] = measured_peaks()
    short = {"cfg1": 8, "cfg2": 32, "cfg3": 24, "cfg4": 4, "cfg4_offloaded": 2, "cfg5": 6, "cfg5_top2": 6, "base8_prefill": 4}
    keep = ("value", "unit", "steps", "ms_per_step", "ms_per_token_per_layer", "block_latency_us", "config", "roofline",
            "host_link", "overlap", "gpu_only", "expert_cache")
    out["other_workloads"] = {}
    for n in others:
        pending.remove(n)
        r = run_workload(n, short.get(n, 8), 2, args.host_threads, False, None, min(args.trace_steps, 2), store=store_for(n),
                         fetch_mode=args.fetch)
        drop_store(n)
        out["other_workloads"][n] = {k: r[k] for k in keep if k in r}
    if not args.no_sweep_k and not args.main_only:
        out["activated_expert_sweep"] = activated_expert_sweep(args.host_threads, args.sweep_steps)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
