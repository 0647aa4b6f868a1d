#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: for every layer,
append the new token's K/V and run paged-attention decode (and, in the swap leg,
prefetch the next layer's host-resident blocks behind it and write dirty blocks
back).  The headline number is decode tokens/s on the Llama-2-7B-shaped fp16
workload with all KV resident (inputs already in HBM).  The same line carries
the roofline of the attention kernel, the float64 oracle timed on the host's
cores on a sample, and the swap leg: 30 % of every sequence's blocks in pinned
host memory, reporting host-link GB/s, kernel-latency inflation and stall; and
a second, short leg with 0.5 % on the host, below the fraction the link can hide.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
LINK_PEAK_GBS = 63.0           # PCIe Gen5 x16, per direction, before protocol overhead


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg4", "cfg5"])
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers (diagnostics only)")
    ap.add_argument("--ctx-fixed", type=int, default=0, help="diagnostics: give every sequence this context length")
    ap.add_argument("--partition", type=int, default=0, help="attention partition size in tokens (0 = library default)")
    ap.add_argument("--swap-fraction", type=float, default=0.30)
    ap.add_argument("--swap-steps", type=int, default=3)
    ap.add_argument("--below-knee-fraction", type=float, default=0.005,
                    help="host-resident fraction of the second, short swap leg (below link rate / attention rate)")
    ap.add_argument("--swap-path", type=int, default=0)
    ap.add_argument("--swap-wgs", type=int, default=0, help="workgroups of the gather / scatter kernel (0 = library default)")
    ap.add_argument("--attn-vector-alu", action="store_true",
                    help="MHA workloads: the attention's products on the vector ALU instead of the matrix cores (A/B)")
    ap.add_argument("--no-swap", action="store_true")
    ap.add_argument("--no-extra", action="store_true",
                    help="leave out the compact legs of the 8B-shaped and 70B-shaped workloads (cfg4, cfg5) that the "
                         "default line carries beside the headline")
    ap.add_argument("--scatter-link-fraction", type=float, default=0.02,
                    help="host fraction of the transfer-bound point of the gather-kernel leg")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=64)
    ap.add_argument("--cpu-layers", type=int, default=6)
    ap.add_argument("--sweep", default="", help="comma-separated host-resident fractions to run in fixed-fraction mode "
                    "(e.g. 0,0.005,0.01,0.02,0.05,0.1,0.2,0.3,0.4,0.5,0.6); adds a 'sweep' list to the line")
    ap.add_argument("--adaptive-steps", type=int, default=0,
                    help="run the adaptive-expansion controller from f = 0 for this many decode steps; adds 'adaptive'")
    ap.add_argument("--adaptive-units", type=int, default=0, help="controller levels per 100 %% (default 8 x layers)")
    ap.add_argument("--layer-fifo", type=int, default=0,
                    help="also run the paper's layer-granular protocol with this many layers starting in CPU memory "
                         "(GPU layer slots = layers - m, CPU slots = m + 2); adds 'layer_fifo'")
    ap.add_argument("--elastic", type=int, default=0,
                    help="also run the chunked layer caches with this many layers asked to stay in CPU memory: the "
                         "caches of the others grow to a / (n - m); adds 'elastic'")
    ap.add_argument("--t-other-us", type=float, default=0.0,
                    help="experiments only: keep the compute stream busy this long after each layer's attention, standing "
                         "for the rest of a transformer layer (default 0 = the measured path; -1 = the time to read the "
                         "layer's weights once at the rate the stream probe measures on this workload)")
    ap.add_argument("--serve", type=int, default=0,
                    help="experiment instead of the benchmark line: serve this many synthetic requests (Poisson arrivals, "
                         "iteration-level scheduling) on a GPU pool of --serve-gpu-blocks blocks per layer at the expansion "
                         "levels in --serve-levels and with the controller; prints its own JSON line")
    ap.add_argument("--serve-elastic", action="store_true",
                    help="with --serve: the paper's own unit - whole layers move and the caches of the layers that stay "
                         "grow; --serve-levels are then numbers of layers kept in CPU memory, --serve-gpu-blocks a "
                         "layer's cache while everything is on the GPU")
    ap.add_argument("--serve-chunk-blocks", type=int, default=256)
    ap.add_argument("--serve-rates", default="", help="with --serve-elastic: also serve at these request rates, given as "
                    "shares of the rate the first level sustains when saturated (e.g. 0.7,1.0,1.15), at the first and "
                    "at the last of --serve-levels")
    ap.add_argument("--serve-gpu-blocks", type=int, default=16384)
    ap.add_argument("--serve-levels", default="0,1,2,4,8", help="budget levels; one level = 1/64 of the GPU pool")
    ap.add_argument("--serve-load", type=float, default=0.8,
                    help="arrival rate of the latency legs as a share of the level-0 saturated request rate")
    ap.add_argument("--link-sweep", action="store_true",
                    help="experiment instead of the benchmark line: host-link rate against transfer size, copy engine and "
                         "gather kernel, and the flavours of page-locked memory; prints its own JSON line")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run a plain elementwise copy of this many MiB (a known-size reference for HBM counters)")
    return ap.parse_args()


def timed_steps(dw, streams, n, pf, dirty):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, pf, dirty, dw.out, *streams)
    dw.pool.sync()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def step_distribution(dw, streams, n, pf, dirty):
    """p10 / p50 / p90 of single steps, each bracketed by a synchronisation (ms)."""
    import torch
    ts = []
    for _ in range(n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, pf, dirty, dw.out, *streams)
        dw.pool.sync()
        ts.append((time.perf_counter() - t0) * 1e3)
    return [float(np.percentile(ts, q)) for q in (10, 50, 90)]


def measured_link_peak(mib=512):
    """One large pinned-host to device copy: the link's measured large-transfer rate (GB/s)."""
    import torch
    src = torch.empty(mib << 20, dtype=torch.uint8, pin_memory=True)
    dst = torch.empty(mib << 20, dtype=torch.uint8, device="cuda:0")
    best = 0.0
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        best = max(best, (mib << 20) / (time.perf_counter() - t0) / 1e9)
    return best


def layer_profile(dw, streams, pf, dirty, reps=3):
    """Per-layer event times (ms), median over a few timed steps."""
    acc = {}
    dw.pool.set_timing(True)
    for _ in range(reps):
        dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, pf, dirty, dw.out, *streams)
        dw.pool.sync()
        lt = dw.pool.layer_times()
        st = dw.pool.stats()
        for k, v in lt.items():
            acc.setdefault(k, []).append(v.copy())
        acc.setdefault("step_ms", []).append(st.step_ms)
        acc.setdefault("bytes_in", []).append(st.bytes_in)
        acc.setdefault("bytes_out", []).append(st.bytes_out)
    dw.pool.set_timing(False)
    out = {k: np.median(np.stack(v), axis=0) for k, v in acc.items() if k not in ("step_ms", "bytes_in", "bytes_out")}
    out["step_ms"] = float(np.median(acc["step_ms"]))
    out["bytes_in"] = int(acc["bytes_in"][-1])
    out["bytes_out"] = int(acc["bytes_out"][-1])
    return out


def leg_metrics(w, dw, sp, s_per_step, base_kernel_ms, base_step_ms, achieved):
    """Numbers of one swap leg from its per-layer profile `sp` and its untimed seconds per step."""
    st = dw.pool.stats()
    t_in = float(np.mean(sp["swap_in"]))
    in_gbs = sp["bytes_in"] / w.n_layers / (t_in * 1e-3) / 1e9 if t_in > 0 else 0.0
    return {
        "host_fraction": st.host_fraction, "host_blocks": st.host_blocks_in_use,
        "expansion_simple": st.expansion_simple, "expansion_staged": st.expansion_staged,
        "tokens_per_s": w.batch / s_per_step, "ms_per_step": s_per_step * 1e3,
        "bytes_in_per_layer": sp["bytes_in"] // w.n_layers, "bytes_out_per_layer": sp["bytes_out"] // w.n_layers,
        "swap_in_ms_per_layer": t_in, "swap_out_ms_per_layer": float(np.mean(sp["swap_out"])),
        "host_link_GBps": in_gbs, "host_link_peak_GBps": LINK_PEAK_GBS, "host_link_frac": in_gbs / LINK_PEAK_GBS,
        "attn_kernel_ms_per_layer": float(np.mean(sp["kernel"])),
        "inflation_kernel": float(np.median(sp["kernel"]) / np.median(base_kernel_ms) - 1.0),
        "stall_ms_per_step": float(np.sum(sp["stall"])),
        "inflation_e2e": s_per_step * 1e3 / base_step_ms - 1.0,
        "transparent_fraction_bound": in_gbs / achieved if achieved > 0 else None,
    }


def fixed_fraction_leg(w, dw, streams, f, n_steps, base_kernel_ms, base_step_ms, achieved):
    """Fixed-fraction mode: the first round(f * blocks) handles of the seeded order live on the host."""
    dw.pool.set_host_fraction(f, dw.order, streams[1])
    dw.pool.sync()
    pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
    timed_steps(dw, streams, 1, pf, dirty)
    s_total = timed_steps(dw, streams, n_steps, pf, dirty)
    sp = layer_profile(dw, streams, pf, dirty, reps=2)
    assert dw.pool.check_errors() == 0
    m = leg_metrics(w, dw, sp, s_total / n_steps, base_kernel_ms, base_step_ms, achieved)
    keep = ("host_fraction", "tokens_per_s", "ms_per_step", "swap_in_ms_per_layer", "attn_kernel_ms_per_layer",
            "host_link_GBps", "inflation_kernel", "inflation_e2e", "stall_ms_per_step", "expansion_simple")
    return {k: m[k] for k in keep}


def host_time_in_step(dw, streams, pf, dirty, n=10):
    """How long the caller's thread spends inside pie_step, when it enqueues the step itself (on the copy-engine
    path it then paces the GPU) and when the pool's own thread does (pie_set_async_submit); and the step time
    with the latter."""
    import torch
    res = {}
    for name, on in (("caller_enqueues_ms", False), ("async_submit_ms", True)):
        dw.pool.set_async_submit(on)
        timed_steps(dw, streams, 2, pf, dirty)
        ts = []
        for _ in range(n):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, pf, dirty, dw.out, *streams)
            ts.append((time.perf_counter() - t0) * 1e3)
            dw.pool.sync()
        res[name] = float(np.median(ts))
        if on:
            res["ms_per_step_async_submit"] = timed_steps(dw, streams, n, pf, dirty) / n * 1e3
    dw.pool.set_async_submit(False)
    return res


def dirty_tail_leg(w, dw, streams, f, tail_share, base_step_ms, n_steps=10):
    """Below the knee, with write-backs: the same number of host blocks as the fixed-fraction leg, but a share of
    them are tail blocks (they receive the step's token, so every layer stages them, appends to the staged copy
    and writes them back).  The seeded demotion order rarely names a tail at such a small fraction, so that leg
    has nothing to write back; this one says what the write-back costs.  All blocks must be GPU-homed on entry
    and are again on return."""
    from paper_2411_09317_amd import binding as B
    T = w.block_tokens
    n_host = int(round(f * dw.total_blocks))
    n_tail = max(1, int(round(tail_share * n_host)))
    tails = [int(dw.table[b, (int(dw.ctx_lens[b]) - 1) // T]) for b in range(w.batch)][:n_tail]
    tail_set = set(tails)
    others = [int(h) for h in dw.order if int(h) not in tail_set][:n_host - len(tails)]
    hs = np.asarray(tails + others, dtype=np.int32)
    dw.pool.migrate(hs, B.HOST, streams[1])
    dw.pool.sync()
    pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
    assert len(dirty) == len(tails) and len(pf) == len(hs)
    timed_steps(dw, streams, 2, pf, dirty)
    s = timed_steps(dw, streams, n_steps, pf, dirty) / n_steps
    assert dw.pool.check_errors() == 0
    dw.pool.migrate(hs, B.GPU, streams[1])
    dw.pool.sync()
    return {"host_blocks": len(hs), "dirty_tail_blocks": len(tails), "ms_per_step": s * 1e3,
            "tokens_per_s": w.batch / s, "inflation_e2e": s * 1e3 / base_step_ms - 1.0,
            "bytes_out_per_layer": len(tails) * w.block_bytes}


def scattered_kernel_leg(w, dw, streams, f_small, f_link, base_kernel_ms, base_step_ms, achieved):
    """The gather kernel on a host pool full of holes: twice the blocks go to the host and every other one comes
    back, so a layer's prefetch is as many pieces as blocks and the copy engine would pay its per-call cost for
    each.  Two points: f_small (below what the link hides: what the path costs a step) and f_link (transfer-bound:
    the link rate the kernel reaches, and the decode kernel's slowdown with the gather beside it all the time)."""
    from paper_2411_09317_amd import binding as B
    out = {"swap_path": "gather kernel (PIE_SWAP_KERNEL), library defaults"}
    for name, f in (("below_knee", f_small), ("link_bound", f_link)):
        k = int(round(2 * f * len(dw.order)))
        dw.pool.migrate(dw.order[:k], B.HOST, streams[1])
        dw.pool.migrate(dw.order[1:k:2], B.GPU, streams[1])
        dw.pool.sync()
        pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
        slots = np.asarray(dw.pool.block_where(pf)[1])
        dw.pool.set_swap_path(B.SWAP_KERNEL)
        timed_steps(dw, streams, 1, pf, dirty)
        n = 10 if name == "below_knee" else 3
        s_total = timed_steps(dw, streams, n, pf, dirty)
        sp = layer_profile(dw, streams, pf, dirty, reps=3)
        assert dw.pool.check_errors() == 0
        m = leg_metrics(w, dw, sp, s_total / n, base_kernel_ms, base_step_ms, achieved)
        keep = ("host_fraction", "tokens_per_s", "ms_per_step", "bytes_in_per_layer", "swap_in_ms_per_layer",
                "host_link_GBps", "attn_kernel_ms_per_layer", "inflation_kernel", "inflation_e2e", "stall_ms_per_step")
        out[name] = {k_: m[k_] for k_ in keep}
        out[name]["pieces_per_layer"] = 1 + int((np.diff(slots) != 1).sum())
        dw.pool.set_swap_path(B.SWAP_AUTO)
        dw.pool.migrate(dw.order[:k], B.GPU, streams[1])
        dw.pool.sync()
    return out


def roofline_of(w, dw, streams, steps, warmup):
    """All-resident steps of a workload: throughput and the decode kernel's roofline numbers."""
    none = np.zeros(0, dtype=np.int32)
    timed_steps(dw, streams, 1, none, none)
    probe_ms = float(np.mean([dw.pool.attn_stream_probe(l % w.n_layers, dw.d_table, dw.d_ctx, streams[0])
                              for l in range(2 * min(w.n_layers, 8))][2:]))
    timed_steps(dw, streams, warmup, none, none)
    s = timed_steps(dw, streams, steps, none, none) / steps
    prof = layer_profile(dw, streams, none, none)
    assert dw.pool.check_errors() == 0
    k_ms = float(np.mean(prof["kernel"]))
    achieved = dw.kv_bytes_per_layer / (k_ms * 1e-3) / 1e9
    traffic, source = traffic_from_profile(f"attn_decode_{w.name}_pmc.txt")
    res = {"tokens_per_s": w.batch / s, "ms_per_step": s * 1e3, "layers": w.n_layers,
           "attn_partition_tokens": dw.pool.attn_partition(),
           "roofline": {"bound": "hbm", "kernel": "k_attn_decode_mfma", "achieved": achieved, "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": source,
                        "kernel_ms": k_ms, "algorithmic_bytes_per_launch": dw.kv_bytes_per_layer,
                        "stream_probe_ms": probe_ms, "frac_of_stream_probe": probe_ms / k_ms}}
    return res, prof["kernel"].copy(), s * 1e3, achieved


def compact_cfg4(steps, warmup):
    """The 8B-shaped GQA workload in the default line: roofline at the full shape, fixed host fractions around
    the knee and at 30 %, and the controller's operating point next to the best fixed point (the criterion the
    paper's ablation applies to its adaptive expansion: close to the exhaustive optimum)."""
    import torch
    from paper_2411_09317_amd import inputs as I
    from paper_2411_09317_amd import workload as WL
    w = I.CONFIGS["cfg4"]
    dw = WL.build(w, host_capacity_fraction=0.32)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    res, base_k, base_ms, achieved = roofline_of(w, dw, streams, steps, warmup)
    res["workload"] = (f"cfg4: {w.n_layers} layers, batch {w.batch}, {w.n_q_heads} q heads / {w.n_kv_heads} kv heads, "
                       f"head_dim {w.head_dim}, bf16, ctx lognormal(median {w.ctx_median}, sigma {w.ctx_sigma}) clipped to "
                       f"[{w.ctx_lo},{w.ctx_hi}], {int(dw.ctx_lens.sum())} context tokens")
    pts = [{"host_fraction": 0.0, "tokens_per_s": res["tokens_per_s"], "ms_per_step": res["ms_per_step"],
            "inflation_kernel": 0.0, "inflation_e2e": 0.0, "stall_ms_per_step": 0.0, "expansion_simple": 1.0}]
    for f in (0.0025, 0.005, 0.0075, 0.01, 0.30):
        pts.append(fixed_fraction_leg(w, dw, streams, f, 3, base_k, base_ms, achieved))
    res["fixed_fraction"] = pts
    units = 8 * w.n_layers
    ad = adaptive_leg(w, dw, streams, 160, units, int(0.04 * units))
    # the controller's own signal, tokens/s x expansion, at every fixed point and where the controller ended
    signal = lambda p: p["tokens_per_s"] * p["expansion_simple"]
    best = max(pts[:-1], key=signal)
    at = min(pts[:-1], key=lambda p: abs(p["host_fraction"] - ad["final_host_fraction"]))
    res["adaptive"] = {k: ad[k] for k in ("units", "steps", "final_level", "final_host_fraction", "level_min_second_half",
                                          "level_max_second_half", "monitoring_overhead")}
    res["adaptive"].update({"best_fixed_host_fraction": best["host_fraction"],
                            "signal_at_final_over_best_fixed": signal(at) / signal(best),
                            "signal": "tokens/s x 1/(1-f), evaluated on the fixed-fraction points nearest to each f"})
    dw.pool.close()
    del dw
    torch.cuda.empty_cache()
    return res


def compact_cfg5(steps, warmup, layers=16, overflow=0.215):
    """The 70B-shaped long-context workload: 343.6 GB of KV do not fit 288 GB of HBM, so at least 21.5 % must live
    on the host.  One GPU shows the real per-layer shape (batch 32 x 32768 tokens, 64 / 8 heads, 4.29 GB per
    layer) on `layers` of the 80 layers: the roofline of the kernel, and the pipeline with the overflow share of
    every sequence's blocks in pinned memory."""
    import torch
    from paper_2411_09317_amd import binding as B
    from paper_2411_09317_amd import inputs as I
    from paper_2411_09317_amd import workload as WL
    w0 = I.CONFIGS["cfg5"]
    dw = WL.build(w0, host_capacity_fraction=overflow + 0.01, n_layers=layers)
    w = dw.w
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    res, base_k, base_ms, achieved = roofline_of(w, dw, streams, steps, warmup)
    res["workload"] = (f"cfg5 per-layer shape on {layers} of {w0.n_layers} layers: batch {w.batch} x {w.ctx_hi} tokens, "
                       f"{w.n_q_heads} q heads / {w.n_kv_heads} kv heads, head_dim {w.head_dim}, bf16")
    res["aliasing"] = (f"{layers} physical layers stand for {w0.n_layers}: per-layer numbers are real, a whole step would "
                       f"take {w0.n_layers}/{layers} times ms_per_step; the full cache ({w0.n_layers} x "
                       f"{dw.kv_bytes_per_layer / 1e9:.2f} GB = {w0.n_layers * dw.kv_bytes_per_layer / 1e9:.1f} GB) does not fit one GPU")
    res["tokens_per_s_whole_model_extrapolated"] = res["tokens_per_s"] * layers / w0.n_layers
    hs = WL.per_sequence_host_order(dw, overflow)
    dw.pool.migrate(hs, B.HOST, streams[1])
    dw.pool.sync()
    pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
    timed_steps(dw, streams, 1, pf, dirty)
    s = timed_steps(dw, streams, 2, pf, dirty) / 2
    sp = layer_profile(dw, streams, pf, dirty, reps=2)
    assert dw.pool.check_errors() == 0
    m = leg_metrics(w, dw, sp, s, base_k, base_ms, achieved)
    keep = ("host_fraction", "tokens_per_s", "ms_per_step", "bytes_in_per_layer", "swap_in_ms_per_layer", "host_link_GBps",
            "host_link_frac", "attn_kernel_ms_per_layer", "inflation_kernel", "inflation_e2e", "stall_ms_per_step")
    res["overflow_on_host"] = {k: m[k] for k in keep}
    res["overflow_on_host"]["tokens_per_s_whole_model_extrapolated"] = m["tokens_per_s"] * layers / w0.n_layers
    dw.pool.close()
    del dw
    torch.cuda.empty_cache()
    return res


def adaptive_leg(w, dw, streams, n_steps, units, k_max):
    """The controller in the loop: it starts at f = 0, sees every step's per-layer times, and moves the host
    fraction one level at a time.  The throughput signal is tokens/s x expansion: a larger effective cache
    admits a proportionally larger batch (the premise of the method); the batch itself is fixed here."""
    from paper_2411_09317_amd import binding as B
    # a level must bring at least half the capacity it adds to count as scaling (with levels finer than 1 % the
    # default threshold of 1 % could never be met)
    ctl = B.Controller(units, k_max, plateau_eps=min(0.01, 0.5 / units))
    dw.pool.set_host_fraction(0.0, dw.order, streams[1])
    dw.pool.sync()
    none = np.zeros(0, dtype=np.int32)
    cost = {}
    for name, mode in (("off", B.TIMING_OFF), ("device_clock", B.TIMING_CLOCK), ("events", B.TIMING_EVENTS)):
        dw.pool.set_timing(mode)                   # what the monitoring itself costs, nothing on the host
        timed_steps(dw, streams, 2, none, none)
        cost[name] = timed_steps(dw, streams, 10, none, none) / 10 * 1e3
    dw.pool.set_timing(B.TIMING_CLOCK)
    level, traj = 0, []
    for step in range(n_steps):
        pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
        t0 = time.perf_counter()
        dw.pool.step(dw.q, dw.k_new, dw.v_new, dw.d_table, dw.d_ctx, pf, dirty, dw.out, *streams)
        dw.pool.sync()
        dt = time.perf_counter() - t0
        st = dw.pool.stats()
        f_next = ctl.update_from_pool(dw.pool, w.batch / dt * st.expansion_simple)
        traj.append((level, round(dt * 1e3, 3)))
        new_level = int(round(f_next * units))
        if new_level != level:
            dw.pool.set_host_fraction(new_level / units, dw.order, streams[1])
            dw.pool.sync()
            level = new_level
    dw.pool.set_timing(False)
    assert dw.pool.check_errors() == 0
    k, ceiling = ctl.level()
    ctl.close()
    levels = [t[0] for t in traj]
    tail = levels[len(levels) // 2:]
    return {"units": units, "k_max": k_max, "steps": n_steps, "monitoring": "device clock",
            "monitoring_overhead": {"ms_per_step_unmonitored": cost["off"],
                                    "device_clock": cost["device_clock"] / cost["off"] - 1.0,
                                    "events": cost["events"] / cost["off"] - 1.0},
            "final_level": k, "ceiling": ceiling,
            "final_host_fraction": k / units, "level_min_second_half": min(tail), "level_max_second_half": max(tail),
            "levels": levels, "ms_per_step_last": traj[-1][1]}


def layer_fifo_leg(w, dw, m, n_steps, t_other_us, base_step_ms):
    """The paper's own unit: whole layers move.  n - m GPU layer slots, m + 2 CPU layer slots, the last m
    layers start in CPU memory.  Content is random (only timing is measured here; parity is in the tests)."""
    import torch
    from paper_2411_09317_amd import binding as B
    n = w.n_layers
    inner = B.Pool(n - m, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, dw.total_blocks + 64, 0, 0,
                   max_batch=w.batch, max_blocks_per_seq=dw.table.shape[1])
    hs = np.asarray(inner.block_alloc(B.GPU, dw.total_blocks), dtype=np.int32)
    table = np.full_like(dw.table, -1)
    table[dw.table >= 0] = hs                                  # same shape of table, this pool's handles
    inner.gpu_image().view(torch.int16).copy_(dw.pool.gpu_image()[: n - m, : inner.n_slots].view(torch.int16))
    lp = B.LayerPool(inner, n, m + 2, list(range(n - m, n)))
    for l in range(n - m, n):
        lp.layer_image(l).copy_(dw.pool.gpu_image()[l, : inner.n_slots])
    if t_other_us:
        inner.set_layer_compute_us(t_other_us)
    d_table = torch.from_numpy(table).to(dw.q.device)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    out = torch.empty_like(dw.q)
    def run(k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            lp.step(dw.q, dw.k_new, dw.v_new, d_table, dw.d_ctx, out, *streams)
        inner.sync()
        return time.perf_counter() - t0
    run(1)
    s0 = lp.stats()
    dt = run(n_steps)
    s1 = lp.stats()
    assert inner.check_errors() == 0
    res = {"layers_on_cpu": m, "gpu_layer_slots": n - m, "cpu_layer_slots": m + 2, "expansion_simple": n / (n - m),
           "expansion_buffered": (n + 4) / (n - m + 2), "layer_MB": lp.layer_bytes / 1e6,
           "tokens_per_s": w.batch * n_steps / dt, "ms_per_step": dt / n_steps * 1e3,
           "inflation_e2e": dt / n_steps * 1e3 / base_step_ms - 1.0,
           "swap_ins_per_step": (s1.n_swap_in - s0.n_swap_in) / n_steps,
           "swap_outs_per_step": (s1.n_swap_out - s0.n_swap_out) / n_steps,
           "forced_ins_per_step": (s1.n_forced_in - s0.n_forced_in) / n_steps,
           "host_wait_ms_per_step": (s1.stall_ms - s0.stall_ms) / n_steps,
           "link_GBps_in": (s1.bytes_in - s0.bytes_in) / dt / 1e9, "link_GBps_out": (s1.bytes_out - s0.bytes_out) / dt / 1e9}
    lp.close()
    inner.close()
    return res


def traffic_from_profile(name):
    """HBM bytes per launch measured with rocprofv3 counters, as a committed summary states them: (bytes, where
    that number comes from).  It is a figure from an earlier, separate profiler run of the same command (counters
    cannot be collected inside this run), so the line names the file and its date beside it."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch"):
            stamp = time.strftime("%Y-%m-%d", time.gmtime(os.path.getmtime(path)))
            return float(line.split("=")[1].split()[0]), (f"profiles/{name} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, separate "
                                                          f"earlier runs, file dated {stamp}; not measured in this run)")
    return None, None


def cpu_baseline(dw, n_seqs, n_layers):
    """The float64 oracle on a sample: the first n_layers layers of the first n_seqs sequences, with the very
    bytes the GPU holds.  Also checks the GPU's output for those sequences against it."""
    import torch
    from threadpoolctl import threadpool_info
    from oracle.pool_model import PoolModel
    w = dw.w
    n_seqs = min(n_seqs, w.batch)
    nb = dw.n_blocks[:n_seqs]
    total = int(nb.sum())
    n_layers = min(n_layers, w.n_layers)
    mod = PoolModel(n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, total, 0, 0)
    handles = mod.block_alloc(0, total)
    table = np.full((n_seqs, int(nb.max())), -1, dtype=np.int32)
    where, slots = dw.pool.block_where(dw.table[:n_seqs][dw.table[:n_seqs] >= 0])
    assert all(x == 0 for x in where)
    src = torch.as_tensor(np.asarray(slots, dtype=np.int64), device=dw.q.device)
    for l in range(n_layers):
        blocks = dw.pool.gpu_image()[l].index_select(0, src).cpu().numpy()       # [total][block_bytes]
        mod.gpu[l, :total] = mod.blocks_from_bytes(blocks)
    i = 0
    for b in range(n_seqs):
        for j in range(int(nb[b])):
            table[b, j] = handles[i]
            i += 1
    q_dev = dw.q[:n_layers, :n_seqs]
    q = q_dev.view(torch.int16).cpu().numpy().view(np.uint16) if w.dtype == 2 else q_dev.cpu().numpy()
    dt, rel = 0.0, 0.0
    for l in range(n_layers):
        t0 = time.perf_counter()
        ref = mod.attn_decode(l, q[l], table, dw.ctx_lens[:n_seqs])
        dt += time.perf_counter() - t0
        got = dw.out[l, :n_seqs].to(torch.float64).cpu().numpy()
        num = np.abs(got - ref).max(axis=-1)
        den = np.abs(ref).max(axis=-1)
        rel = max(rel, float((num / np.where(den == 0, 1, den)).max()))
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    tokens_per_s = n_seqs / (dt * w.n_layers / n_layers)     # n_layers timed; a step has w.n_layers of them
    return {"value": tokens_per_s, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"float64 oracle, first {n_layers} of {w.n_layers} layers, first {n_seqs} of {w.batch} sequences "
                      f"({int(dw.ctx_lens[:n_seqs].sum())} context tokens per layer), {dt:.2f} s; scaled by "
                      f"{w.n_layers}/{n_layers} layers to a whole step", "host_cpus": os.cpu_count(),
            "gpu_vs_oracle_rowwise_rel_err": rel}


def elastic_leg(w, dw, m, n_steps, t_other_us, base_step_ms, chunk_blocks=256):
    """Layer caches made of chunks: m layers are asked to stay in CPU memory, the chunks they leave go to the
    layers that stay (a / (n - m) per layer), and the steps are timed once that is complete."""
    import torch
    from paper_2411_09317_amd import binding as B
    n = w.n_layers
    k0 = (dw.total_blocks + chunk_blocks - 1) // chunk_blocks
    k_cap = (n * k0) // (n - m)
    inner = B.Pool(n, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, k0 * chunk_blocks, 0, 0,
                   max_batch=w.batch, max_blocks_per_seq=dw.table.shape[1])
    table = np.full_like(dw.table, -1)
    table[dw.table >= 0] = np.arange(dw.total_blocks, dtype=np.int32)      # block indices of a layer's cache
    inner.gpu_image()[:, : dw.total_blocks].view(torch.int16).copy_(
        dw.pool.gpu_image()[:, : dw.total_blocks].view(torch.int16))
    ep = B.ElasticPool(inner, chunk_blocks, k_cap, m + 2)
    if t_other_us:
        inner.set_layer_compute_us(t_other_us)
    d_table = torch.from_numpy(table).to(dw.q.device)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    out = torch.empty_like(dw.q)
    def run(k):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k):
            ep.step(dw.q, dw.k_new, dw.v_new, d_table, dw.d_ctx, out, *streams)
        inner.sync()
        return time.perf_counter() - t0
    run(1)
    resident_ms = run(n_steps) / n_steps * 1e3                       # everything on the GPU, through the block maps
    ep.set_live_blocks(dw.total_blocks)                          # a leaving layer takes along only the chunks in use
    ep.set_layers_on_cpu(m, dw.total_blocks, streams[0])
    steps_to_visible = 0
    while ep.capacity()[0] < ep.capacity()[1] and steps_to_visible < 4 * n:
        run(1)
        steps_to_visible += 1
    s0 = ep.stats()
    dt = run(n_steps)
    s1 = ep.stats()
    assert inner.check_errors() == 0
    vis, tgt, _ = ep.capacity()
    res = {"layers_on_cpu": m, "chunk_blocks": chunk_blocks, "chunk_MB": chunk_blocks * w.block_bytes / 1e6,
           "chunks_per_layer_before": k0, "chunks_per_layer_after": vis // chunk_blocks,
           "blocks_per_layer_before": k0 * chunk_blocks, "blocks_per_layer_visible": vis, "blocks_per_layer_target": tgt,
           "expansion": vis / (k0 * chunk_blocks), "steps_until_visible": steps_to_visible,
           "ms_per_step_all_resident": resident_ms, "ms_per_step": dt / n_steps * 1e3,
           "tokens_per_s": w.batch * n_steps / dt, "inflation_e2e": dt / n_steps * 1e3 / base_step_ms - 1.0,
           "swap_ins_per_step": (s1.n_swap_in - s0.n_swap_in) / n_steps,
           "swap_outs_per_step": (s1.n_swap_out - s0.n_swap_out) / n_steps,
           "forced_ins_per_step": (s1.n_forced_in - s0.n_forced_in) / n_steps,
           "host_wait_ms_per_step": (s1.stall_ms - s0.stall_ms) / n_steps,
           "link_GBps_in": (s1.bytes_in - s0.bytes_in) / dt / 1e9, "link_GBps_out": (s1.bytes_out - s0.bytes_out) / dt / 1e9}
    ep.close()
    inner.close()
    return res


def link_sweep_mode(args):
    """The host link against transfer size (the paper's Section 2.4 measurement on its machine: bandwidth against
    access size, large accesses needed for the link's rate): single copy-engine transfers host to device and
    device to host, 64 KiB to 1 GiB, and the gather / scatter kernel moving the same bytes as 64 KiB blocks,
    alone on the GPU; then the 256 MiB point again for the flavours of page-locked memory hipHostMalloc offers,
    given to the library as its host pool.  Prints its own JSON line."""
    import ctypes
    import torch
    from paper_2411_09317_amd import binding as B
    hip = ctypes.CDLL("libamdhip64.so.7")                          # the copy torch has loaded
    hip.hipHostMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t, ctypes.c_uint]
    hip.hipHostFree.argtypes = [ctypes.c_void_p]
    hip.hipMemcpyAsync.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    GiB = 1 << 30
    blk = 64 << 10                                                 # 8 kv heads x 16 tokens x 128 dims x 2 bytes x (K, V)
    sizes = [64 << 10, 256 << 10, 1 << 20, 4 << 20, 16 << 20, 64 << 20, 256 << 20, GiB]
    stream = torch.cuda.Stream()
    d_buf = torch.empty(GiB, dtype=torch.uint8, device="cuda:0")

    def timed(fn, reps):
        ts = []
        for _ in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            e1.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e-3)
        return float(np.median(ts[1:]))                            # the first pass through fresh memory is slow

    def copies(h_ptr, size, reps):
        s = ctypes.c_void_p(stream.cuda_stream)
        h2d = timed(lambda: hip.hipMemcpyAsync(ctypes.c_void_p(d_buf.data_ptr()), ctypes.c_void_p(h_ptr), size, 1, s), reps)
        d2h = timed(lambda: hip.hipMemcpyAsync(ctypes.c_void_p(h_ptr), ctypes.c_void_p(d_buf.data_ptr()), size, 2, s), reps)
        return size / h2d / 1e9, size / d2h / 1e9

    def gather(h_ptr, n_blocks_total, points, reps):
        """pie_swap_in / pie_swap_out of the first n blocks of a pool whose host pool is the given memory."""
        pool = B.Pool(1, 32, 8, 128, 16, 2, 8, n_blocks_total, n_blocks_total, host_ptr=h_ptr, host_bytes=n_blocks_total * blk)
        hs = np.asarray(pool.block_alloc(B.HOST, n_blocks_total), dtype=np.int32)
        pool.set_swap_path(B.SWAP_KERNEL)
        out = []
        for size in points:
            n = size // blk
            t_in = timed(lambda: pool.swap_in(0, hs[:n], stream), reps)
            t_out = timed(lambda: pool.swap_out(0, hs[:n], stream), reps)
            out.append((size / t_in / 1e9, size / t_out / 1e9))
        pool.sync()
        pool.close()
        return out

    reps_of = lambda size: 20 if size <= (4 << 20) else (6 if size <= (64 << 20) else 3)
    pinned = torch.empty(GiB, dtype=torch.uint8, pin_memory=True)
    pinned.zero_()
    rows = []
    g = gather(pinned.data_ptr(), GiB // blk, sizes, 3)
    for size, (gi, go) in zip(sizes, g):
        h2d, d2h = copies(pinned.data_ptr(), size, reps_of(size))
        rows.append({"bytes": size, "copy_engine_h2d_GBps": h2d, "copy_engine_d2h_GBps": d2h,
                     "gather_kernel_h2d_GBps": gi, "scatter_kernel_d2h_GBps": go})
        print(f"# {size >> 10:8d} KiB: copy engine {h2d:5.1f} / {d2h:5.1f} GB/s   kernel {gi:5.1f} / {go:5.1f} GB/s",
              file=sys.stderr, flush=True)
    big = rows[-1]["copy_engine_h2d_GBps"]
    knee = next((r["bytes"] for r in rows if r["copy_engine_h2d_GBps"] >= 0.95 * big), None)
    del pinned
    flavours = []
    size = 256 << 20
    for name, flags in (("hipHostMallocDefault", 0x0), ("hipHostMallocCoherent", 0x40000000),
                        ("hipHostMallocNonCoherent", 0x80000000), ("hipHostMallocWriteCombined", 0x4),
                        ("hipHostMallocNumaUser", 0x20000000)):
        ptr = ctypes.c_void_p(0)
        rc = hip.hipHostMalloc(ctypes.byref(ptr), size, flags)
        if rc != 0 or not ptr.value:
            flavours.append({"flavour": name, "error": f"hipHostMalloc returned {rc}"})
            continue
        ctypes.memset(ptr, 0, size)
        h2d, d2h = copies(ptr.value, size, 3)
        (gi, go), = gather(ptr.value, size // blk, [size], 3)
        flavours.append({"flavour": name, "bytes": size, "copy_engine_h2d_GBps": h2d, "copy_engine_d2h_GBps": d2h,
                         "gather_kernel_h2d_GBps": gi, "scatter_kernel_d2h_GBps": go})
        print(f"# {name}: copy engine {h2d:5.1f} / {d2h:5.1f} GB/s   kernel {gi:5.1f} / {go:5.1f} GB/s", file=sys.stderr, flush=True)
        torch.cuda.synchronize()
        hip.hipHostFree(ptr)
    print(json.dumps({"experiment": "host link against transfer size", "link_peak_GBps_theoretical": LINK_PEAK_GBS,
                      "memory": "torch pin_memory (hipHostMalloc default flags), 1 GiB", "sweep": rows,
                      "bytes_for_95_percent_of_large_transfer_rate_h2d": knee,
                      "gather_kernel": "library defaults, alone on the GPU, 64 KiB blocks in ascending slots",
                      "pinned_memory_flavours_at_256MiB": flavours}))


def serving_elastic_mode(args):
    """The same in the paper's own unit: whole layers move, the caches of the layers that stay grow, and the
    scheduler admits against the size the pool shows.  Fixed numbers of layers in CPU memory, then the
    controller; every request waiting from the start."""
    import torch
    from paper_2411_09317_amd import binding as B
    from paper_2411_09317_amd import inputs as I
    from paper_2411_09317_amd import serving as S
    from paper_2411_09317_amd import workload as WL
    w = I.scaled(I.CONFIGS[args.workload], batch=0, n_layers=args.layers or I.CONFIGS[args.workload].n_layers)
    n, C = w.n_layers, args.serve_chunk_blocks
    k0 = args.serve_gpu_blocks // C
    ms = [int(x) for x in args.serve_levels.split(",")]
    m_max = max(ms + [2])
    k_cap = (n * k0) // (n - m_max)
    out_lo, out_hi = 64, 256
    max_blocks = (w.ctx_hi + out_hi + w.block_tokens - 1) // w.block_tokens
    max_batch = 1024
    inner = B.Pool(n, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, k0 * C, 0, 0, max_batch=max_batch,
                   max_blocks_per_seq=max_blocks)
    img = inner.gpu_image()
    for l in range(n):
        layer = img[l].view(-1).view(WL.TORCH_DT[w.dtype])
        layer.copy_((torch.randn(layer.numel(), device=img.device, dtype=torch.float32) * w.value_scale).to(layer.dtype))
    if args.t_other_us:
        inner.set_layer_compute_us(args.t_other_us)

    def stream(rate):
        a, p, o = I.draw_requests(w, args.serve, rate, out_lo, out_hi)
        return [S.Request(i, float(a[i]), int(p[i]), int(o[i])) for i in range(args.serve)]

    def run(m, adaptive=False, rate=1e9):
        ep = B.ElasticPool(inner, C, k_cap, m_max + 2)
        ctl = B.Controller(n, m_max, k_up=8, k_down=2, probe_period=256) if adaptive else None
        t0 = time.perf_counter()
        r = S.serve_elastic(ep, w, stream(rate), max_batch, max_blocks, controller=ctl, layers_on_cpu=m,
                            progress=lambda it, now, done: print(f"#   iteration {it}: {done} requests done, {now:.1f} s",
                                                                 file=sys.stderr, flush=True))
        r["wall_s"] = round(time.perf_counter() - t0, 2)
        r["mode"] = "adaptive" if adaptive else f"{m} layers on the CPU"
        r["requests_per_s_offered"] = rate if rate < 1e8 else None
        if ctl:
            ctl.close()
        ep.close()
        print(f"# serve elastic {r['mode']} at {rate:.3g} req/s: {r['tokens_per_s']:.0f} tok/s, batch {r['mean_batch']:.1f}, "
              f"latency {r['latency_s_mean']:.1f} s (queue {r['queue_s_mean']:.1f}), "
              f"{r['ms_per_iteration']:.2f} ms/iter, blocks per layer {r['blocks_per_layer_mean']:.0f}, "
              f"waits {r['host_wait_ms']:.0f} ms", file=sys.stderr, flush=True)
        return r

    res = {"experiment": "serving on layer caches that grow and shrink",
           "workload": f"{w.name} shape, {n} layers, {k0} chunks of {C} blocks ({C * w.block_bytes / 1e6:.0f} MB) per layer "
                       f"while everything is on the GPU ({n * k0 * C * w.block_bytes / 1e9:.1f} GB)",
           "requests": args.serve, "prompt": f"{w.ctx_dist} [{w.ctx_lo},{w.ctx_hi}]", "output": f"uniform [{out_lo},{out_hi}]",
           "t_other_us": args.t_other_us, "data": "synthetic"}
    res["saturated"] = [run(m) for m in ms] + [run(0, adaptive=True)]
    if args.serve_rates:
        # offered load as a share of what the caches at their base size sustain: both sizes at every rate
        base = res["saturated"][0]
        full = base["requests"] / base["makespan_s"]
        res["by_rate"] = [{"share_of_base_rate": x, "requests_per_s": x * full,
                           "base": run(ms[0], rate=x * full), "expanded": run(ms[-1], rate=x * full)}
                          for x in [float(v) for v in args.serve_rates.split(",")]]
    inner.close()
    print(json.dumps(res))


def serving_mode(args):
    """Expansion turned into batch size: a request stream served at fixed budget levels and by the controller,
    first saturated (every request waiting from the start: throughput), then at a share of the level-0
    request rate (latency split into queueing and decoding)."""
    import torch
    from paper_2411_09317_amd import binding as B
    from paper_2411_09317_amd import inputs as I
    from paper_2411_09317_amd import serving as S
    w = I.scaled(I.CONFIGS[args.workload], batch=0)
    n_gpu, units = args.serve_gpu_blocks, 64
    unit = n_gpu // units
    levels = [int(x) for x in args.serve_levels.split(",")]
    k_max = max(levels + [16])
    out_lo, out_hi = 64, 256
    max_blocks = (w.ctx_hi + out_hi + w.block_tokens - 1) // w.block_tokens
    max_batch = 1024
    pool = B.Pool(w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.block_tokens, w.dtype, n_gpu, unit * k_max,
                  unit * k_max, max_batch=max_batch, max_blocks_per_seq=max_blocks)
    from paper_2411_09317_amd import workload as WL
    img = pool.gpu_image()
    for l in range(w.n_layers):                                  # "prompts already in the cache": finite random values
        layer = img[l].view(-1).view(WL.TORCH_DT[w.dtype])
        layer.copy_((torch.randn(layer.numel(), device=img.device, dtype=torch.float32) * w.value_scale).to(layer.dtype))
    pool.host_image().zero_()
    if args.t_other_us:
        pool.set_layer_compute_us(args.t_other_us)

    def stream(rate):
        a, p, o = I.draw_requests(w, args.serve, rate, out_lo, out_hi)
        return [S.Request(i, float(a[i]), int(p[i]), int(o[i])) for i in range(args.serve)]

    def run(level, rate, adaptive=False):
        bud = S.BlockBudget(n_gpu, unit, k_max)
        ctl = None
        if adaptive:
            ctl = B.Controller(units, k_max)
        else:
            bud.set_level(level)
        t0 = time.perf_counter()
        r = S.serve(pool, w, stream(rate), bud, max_batch, max_blocks, controller=ctl,
                    progress=lambda it, now, done: print(f"#   iteration {it}: {done} requests done, {now:.1f} s",
                                                         file=sys.stderr, flush=True))
        r["wall_s"] = round(time.perf_counter() - t0, 2)
        r["mode"] = "adaptive" if adaptive else f"level {level}"
        if ctl:
            ctl.close()
        print(f"# serve {r['mode']} rate {rate:.3g}/s: {r['tokens_per_s']:.0f} tok/s, batch {r['mean_batch']:.1f}, "
              f"{r['ms_per_iteration']:.2f} ms/iter, latency {r['latency_s_mean']:.2f} s", file=sys.stderr, flush=True)
        return r

    res = {"experiment": "serving", "workload": f"{w.name} shape, {w.n_layers} layers, GPU pool {n_gpu} blocks per layer "
           f"({n_gpu * w.block_bytes * w.n_layers / 1e9:.1f} GB), one level = {unit} host blocks per layer",
           "requests": args.serve, "prompt": f"{w.ctx_dist} [{w.ctx_lo},{w.ctx_hi}]", "output": f"uniform [{out_lo},{out_hi}]",
           "t_other_us": args.t_other_us, "data": "synthetic"}
    res["saturated"] = [run(k, 1e9) for k in levels] + [run(0, 1e9, adaptive=True)]
    base = res["saturated"][0]
    rate = args.serve_load * base["requests"] / base["makespan_s"]
    res["at_load"] = {"requests_per_s": rate, "runs": [run(0, rate), run(0, rate, adaptive=True)]}
    pool.close()
    print(json.dumps(res))


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py measures one GPU; --gpus {args.gpus} is not supported in this build "
              "(the path would shard by sequence, each GPU with its own pools, host link and controller, no exchange step)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2411_09317_amd import binding as B
    from paper_2411_09317_amd import inputs as I
    from paper_2411_09317_amd import workload as WL

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.link_sweep:
        return link_sweep_mode(args)
    if args.serve:
        return serving_elastic_mode(args) if args.serve_elastic else serving_mode(args)
    w = I.CONFIGS[args.workload]
    if args.ctx_fixed:
        w = I.scaled(w, name=w.name + "-fixedctx", ctx_dist="fixed", ctx_lo=args.ctx_fixed, ctx_hi=args.ctx_fixed)
    swap_leg = not args.no_swap and args.swap_fraction > 0
    host_cap = args.swap_fraction if swap_leg else 0.0
    if args.sweep:
        host_cap = max([host_cap] + [float(f) for f in args.sweep.split(",")])
    if args.adaptive_steps:
        host_cap = max(host_cap, 0.10)
    t_build = time.perf_counter()
    dw = WL.build(w, host_capacity_fraction=(host_cap + 0.02) if host_cap > 0 else 0.0, n_layers=args.layers)
    w = dw.w
    t_build = time.perf_counter() - t_build
    if args.partition:
        dw.pool.set_attn_partition(args.partition)
    dw.pool.set_swap_path(args.swap_path)
    if args.attn_vector_alu:
        dw.pool.set_attn_vector_alu(True)
    if args.swap_wgs:
        dw.pool.set_swap_workgroups(args.swap_wgs)
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    none = np.zeros(0, dtype=np.int32)
    timed_steps(dw, streams, 1, none, none)       # first touch of everything
    probe_ms = float(np.mean([dw.pool.attn_stream_probe(l % w.n_layers, dw.d_table, dw.d_ctx, streams[0])
                              for l in range(2 * min(w.n_layers, 8))][2:]))
    if args.t_other_us < 0:                       # the rest of a layer as the time to stream its weights once
        args.t_other_us = w.layer_weight_bytes / (dw.kv_bytes_per_layer / probe_ms) * 1e3
    if args.t_other_us:
        dw.pool.set_layer_compute_us(args.t_other_us)

    if args.calib_copy_mib:
        n = args.calib_copy_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)          # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del src, dst

    # ---- all-resident: the headline ---------------------------------------------------------------
    timed_steps(dw, streams, args.warmup, none, none)
    total_s = timed_steps(dw, streams, args.steps, none, none)
    ms_per_step = total_s / args.steps * 1e3
    tokens_per_s = w.batch / (total_s / args.steps)
    prof = layer_profile(dw, streams, none, none)
    p10, p50, p90 = step_distribution(dw, streams, min(args.steps, 100), none, none)
    assert dw.pool.check_errors() == 0
    k_ms = float(np.mean(prof["kernel"]))
    bytes_layer = dw.kv_bytes_per_layer
    achieved = bytes_layer / (k_ms * 1e-3) / 1e9
    elem = {0: "f32", 1: "f16", 2: "bf16"}[w.dtype]
    result = {
        "metric": "decode tokens/s", "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": elem, "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_layers} layers, batch {w.batch}, {w.n_q_heads} q heads / "
                               f"{w.n_kv_heads} kv heads, head_dim {w.head_dim}, block 16, ctx {w.ctx_dist} "
                               f"[{w.ctx_lo},{w.ctx_hi}], all KV GPU-resident",
                   "context_tokens": int(dw.ctx_lens.sum()), "kv_bytes_per_layer": bytes_layer,
                   "kv_blocks_per_layer": dw.total_blocks, "attn_partition_tokens": dw.pool.attn_partition(),
                   "attn_partition_chosen_by": "caller" if args.partition else "planning kernel",
                   "t_other_us": args.t_other_us, "layer_weight_bytes": w.layer_weight_bytes,
                   "build_s": round(t_build, 1),
                   # where each part of the named metric ("decode tokens/s & HBM GB/s at X% host-resident KV;
                   # per-layer latency inflation") is in this line
                   "metric_parts": {"decode tokens/s": "value (0 % host-resident), swap.tokens_per_s, "
                                                       "swap_below_knee.tokens_per_s, swap_kernel.*.tokens_per_s, "
                                                       "cfg4.fixed_fraction[].tokens_per_s, cfg5.*.tokens_per_s",
                                    "HBM GB/s": "roofline.achieved, cfg4.roofline.achieved, cfg5.roofline.achieved",
                                    "X% host-resident": "swap.host_fraction, swap_below_knee.host_fraction, "
                                                        "cfg4.fixed_fraction[].host_fraction, "
                                                        "cfg5.overflow_on_host.host_fraction",
                                    "per-layer latency inflation": "inflation_kernel (the attention kernel's own "
                                                                   "slowdown) and inflation_e2e (step time, waits "
                                                                   "included) in swap, swap_below_knee, swap_kernel.*, "
                                                                   "cfg4.fixed_fraction[], cfg5.overflow_on_host"}},
        "roofline": {"bound": "hbm", "kernel": "k_attn_decode_mfma", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic_from_profile(f"attn_decode_{w.name}_pmc.txt")[0],
                     "traffic_source": traffic_from_profile(f"attn_decode_{w.name}_pmc.txt")[1],
                     "kernel_ms": k_ms, "algorithmic_bytes_per_launch": bytes_layer,
                     "stream_probe_ms": probe_ms, "stream_probe_GBps": bytes_layer / (probe_ms * 1e-3) / 1e9,
                     "frac_of_stream_probe": probe_ms / k_ms},
        "per_layer_ms": {"attn_total": float(np.mean(prof["attn"])), "attn_kernel": k_ms,
                         "step_ms_events": prof["step_ms"],
                         "single_step_ms_p10_p50_p90": [p10, p50, p90]},
    }
    base_kernel_ms = prof["kernel"].copy()
    base_step_ms = ms_per_step

    # ---- the oracle on the host's cores -----------------------------------------------------------------
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(dw, args.cpu_seqs, args.cpu_layers)

    # ---- swap leg: a fraction of every sequence's blocks in pinned host memory ------------------------------
    if swap_leg:
        hs = WL.per_sequence_host_order(dw, args.swap_fraction, I.CONFIGS.get("cfg3") if w.name == "cfg2" else None)
        t0 = time.perf_counter()
        dw.pool.migrate(hs, B.HOST, streams[1])
        dw.pool.sync()
        t_mig = time.perf_counter() - t0
        pf, dirty = dw.pool.prefetch_list(dw.table, dw.ctx_lens)
        timed_steps(dw, streams, 1, pf, dirty)
        s_total = timed_steps(dw, streams, args.swap_steps, pf, dirty)
        sp = layer_profile(dw, streams, pf, dirty, reps=2)
        assert dw.pool.check_errors() == 0
        result["swap"] = leg_metrics(w, dw, sp, s_total / args.swap_steps, base_kernel_ms, base_step_ms, achieved)
        result["swap"].update({"migrate_s": round(t_mig, 2), "swap_path": args.swap_path,
                               "host_link_measured_peak_GBps": measured_link_peak()})
        dw.pool.migrate(hs, B.GPU, streams[1])
        dw.pool.sync()
        # the same path below the link's knee: what the swaps cost when every transfer hides behind a layer
        result["swap_below_knee"] = fixed_fraction_leg(w, dw, streams, args.below_knee_fraction, 10, base_kernel_ms,
                                                       base_step_ms, achieved)
        result["swap_below_knee"]["host_time_in_pie_step"] = host_time_in_step(
            dw, streams, *dw.pool.prefetch_list(dw.table, dw.ctx_lens))
        dw.pool.set_host_fraction(0.0, dw.order, streams[1])
        dw.pool.sync()
        # the same number of host blocks with a quarter of them tail blocks: what the dirty write-back costs
        result["swap_below_knee"]["with_dirty_tails"] = dirty_tail_leg(w, dw, streams, args.below_knee_fraction, 0.25,
                                                                       base_step_ms)
        # and through the gather kernel, on a host pool full of holes
        result["swap_kernel"] = scattered_kernel_leg(w, dw, streams, args.below_knee_fraction, args.scatter_link_fraction,
                                                     base_kernel_ms, base_step_ms, achieved)

    # ---- optional: fixed-fraction sweep and the adaptive controller ---------------------------------------
    if args.sweep:
        result["sweep"] = [fixed_fraction_leg(w, dw, streams, float(f), args.swap_steps, base_kernel_ms, base_step_ms,
                                              achieved) for f in args.sweep.split(",")]
    if args.layer_fifo:
        result["layer_fifo"] = layer_fifo_leg(w, dw, args.layer_fifo, args.swap_steps, args.t_other_us, base_step_ms)
    if args.elastic:
        result["elastic"] = elastic_leg(w, dw, args.elastic, args.swap_steps, args.t_other_us, base_step_ms)
    if args.adaptive_steps:
        units = args.adaptive_units or 8 * w.n_layers
        k_max = int(host_cap * units)
        result["adaptive"] = adaptive_leg(w, dw, streams, args.adaptive_steps, units, k_max)
    dw.pool.close()
    headline = args.workload == "cfg2" and not args.layers and not args.ctx_fixed
    del dw
    torch.cuda.empty_cache()
    # ---- the other two named workloads, compact (each builds and frees its own pools) ------------------------
    if headline and not args.no_extra:
        result["cfg4"] = compact_cfg4(10, 2)
        result["cfg5"] = compact_cfg5(5, 1)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
