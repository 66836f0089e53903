#!/usr/bin/env python3
"""Benchmark of the Task-KV hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
for every layer of the workload, semantic separator + cache compression of
the resident prefill K/V, then the workload's decode steps (append + ragged
attention) over every layer.  Inputs are generated on the GPU before the timed
region.  The reported value is the decode part's effective KV bandwidth:
bytes of kept K and V rows that each decode step must read (sum over units of
len * d * 2 * sizeof) divided by the GPU time of the decode calls.

The default run reports the load-imbalance stress workload (cfg5) as `value`
and adds short measurements of the other bf16 workloads as `also_cfg2`,
`also_cfg4` and `also_cfg3` (the 32-layer stack, with one decode call per
layer and with one call for the whole stack), and of two 32-layer stacks on
the paper's layer schedule as `also_schedules`; `--only` leaves them out.

Prints ONE JSON line.
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

HBM_PEAK_GBS = 8000.0
INT8_PEAK_TOPS = 5000.0
# HBM bytes per launch of the decode attention kernel from rocprofv3 --pmc runs
# (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size).  These are
# figures from the committed profile files, not counters read in this run.
PROFILED_TRAFFIC = {
    "cfg5": (573.2e6, "profiles/decode_stream_kernel_cfg5_hbm_traffic.txt"),
}
# Matrix-core utilisation of the row-statistics kernel by counter, same caveat.
PROFILED_MFMA_UTIL = {
    "cfg5": (0.323, "profiles/score_kernels_cfg5_mfma_utilisation.txt"),
}
ALSO_FIELDS = ("config", "value", "unit", "pct_hbm_peak", "decode_us_per_step", "compress_ms_per_layer",
               "roofline")


def n_long_units(wl, n_het):
    n_long = min(n_het, wl.n_kv_heads)
    if wl.add_centre_head and n_long < wl.n_kv_heads:
        n_long += 1
    if wl.n_sink + wl.n_recent >= wl.ctx_len:
        n_long = wl.n_kv_heads
    return n_long


def kept_tokens_total(wl, n_het, n_mid):
    """Tokens held by one layer's ragged cache right after compression."""
    n_long = n_long_units(wl, n_het)
    middle = max(wl.ctx_len - wl.n_sink - wl.n_recent, 0)
    short = wl.n_sink + min(n_mid, middle) + wl.n_recent
    return wl.batch * (n_long * wl.ctx_len + (wl.n_kv_heads - n_long) * short)


def _oracle_leg(wl, ld, budget_s):
    """One batch element of one layer through the oracle: compression once, then
    decode steps (no append) until the time budget is used."""
    import numpy as np
    from oracle import taskkv_oracle as orc
    from taskkv_synth import to_numpy
    q, k, v = to_numpy(ld.q_win[0]), to_numpy(ld.k[0]), to_numpy(ld.v[0])
    t0 = time.perf_counter()
    sep = orc.separate(q, k, v, wl.top_t, ld.n_hetero, bool(wl.add_centre_head))
    kept, kc, vc = orc.compress(k, v, sep["scores"], sep["mask"], wl.n_sink, wl.n_recent, ld.n_middle,
                                wl.pool_kernel)
    t_comp = time.perf_counter() - t0
    kc = [a.astype(np.float64) for a in kc]
    vc = [a.astype(np.float64) for a in vc]
    esize = 4 if wl.dtype == "f32" else 2
    nbytes, steps, t_dec = 0, 0, 0.0
    while steps < wl.decode_steps and (steps < 2 or t_dec < budget_s):
        qs, _, _ = ld.decode_inputs(steps)
        qb = to_numpy(qs[0])
        t0 = time.perf_counter()
        orc.decode_attention(qb, kc, vc)
        t_dec += time.perf_counter() - t0
        nbytes += sum(len(a) for a in kc) * wl.head_dim * 2 * esize
        steps += 1
    return {"decode_gbs": nbytes / t_dec / 1e9, "decode_steps": steps, "units": len(kc),
            "compress_ms_one_batch_element": t_comp * 1e3}


def cpu_baseline(wl, layers, budget_s=5.0):
    """The CPU oracle, as it stands, on a bounded sample (batch element 0 of
    layer 0), in two legs: the numerical library held to one thread, and with
    the threads it takes by default on this host."""
    from threadpoolctl import threadpool_info, threadpool_limits
    ld = layers[0]
    with threadpool_limits(limits=1):
        single = _oracle_leg(wl, ld, budget_s)
    pools = threadpool_info()
    threads = max([p.get("num_threads", 1) for p in pools] or [1])
    multi = _oracle_leg(wl, ld, budget_s)
    return {"value": multi["decode_gbs"], "unit": "GB/s", "cores": int(threads), "kind": "oracle",
            "nproc": os.cpu_count(),
            "sample": f"batch element 0 of layer 0, fp64 numpy: one compression, then {multi['decode_steps']} decode "
                      f"steps over its {multi['units']} units (no append); `value` is the leg with the numerical "
                      f"library's default thread pool ({threads} threads), `single_thread` the same with the pool "
                      f"held to one thread ({single['decode_steps']} decode steps)",
            "compress_ms_per_layer_scaled": multi["compress_ms_one_batch_element"] * wl.batch,
            "single_thread": {"value": single["decode_gbs"], "unit": "GB/s", "cores": 1,
                              "compress_ms_per_layer_scaled": single["compress_ms_one_batch_element"] * wl.batch},
            "note": "the oracle is plain numpy (no OpenMP C++ build exists); its own Python loops run on one "
                    "core in both legs, only the library routines inside use the pool"}


def exact_vector_leg(ctx_len=8192, reps=3):
    """The window approximation against the definition it replaces (Eq. 12-15 against Eq. 1-2) on the
    8192-token workload's shapes: the separator with the workload's window (L, t), and with L = N, t = N,
    where its vector is the exact one.  Both on the same queries (the window is their last L rows)."""
    import dataclasses
    import torch
    from paper_2501_15113_amd import session
    from taskkv_synth import WORKLOADS, make_layer

    base = WORKLOADS["cfg2"]
    wl_full = dataclasses.replace(base, name="cfg2_exact", ctx_len=ctx_len, obs_window=ctx_len, top_t=ctx_len)
    wl_win = dataclasses.replace(base, name="cfg2_window", ctx_len=ctx_len)
    ld = make_layer(wl_full, 0, "cuda:0")
    q_win = ld.q_win[:, :, ctx_len - wl_win.obs_window:, :].contiguous()
    res = {}
    for tag, wl, q in (("exact", wl_full, ld.q_win), ("window", wl_win, q_win)):
        cfg = session.cfg_from_workload(wl)
        bufs = session.LayerBuffers(cfg, 0)
        with session.Context([cfg], 0) as ctx:
            bufs.separate(ctx, q, ld.k, ld.v)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                bufs.separate(ctx, q, ld.k, ld.v)
            e1.record()
            torch.cuda.synchronize()
        res[tag] = (bufs.sem_vec[0].clone(), bufs.mask[0].clone(), e0.elapsed_time(e1) / reps)
    v, vw = res["exact"][0], res["window"][0]
    rel = ((vw - v).norm(dim=1) / v.norm(dim=1)).cpu()
    cos = ((vw * v).sum(dim=1) / (vw.norm(dim=1) * v.norm(dim=1))).cpu()
    agree = int((res["exact"][1] == res["window"][1]).sum().item())
    return {"workload": f"cfg2 shapes, batch 1, N={ctx_len}: window L={wl_win.obs_window}, t={wl_win.top_t} "
                        f"against L=N, t=N",
            "rel_err_mean": float(rel.mean()), "rel_err_max": float(rel.max()),
            "cosine_mean": float(cos.mean()), "cosine_min": float(cos.min()),
            "note": "Eq. 15 sums the top-t tokens' share of the attention mass only, so the window's vector is "
                    "shorter than the exact one by about that share; the head ranking is what it has to keep",
            "mask_agreement": f"{agree}/{wl_win.n_kv_heads} heads",
            "separator_ms_exact": res["exact"][2], "separator_ms_window": res["window"][2]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg5", help="cfg1..cfg5 (default cfg5: largest context, "
                    "the load-imbalance stress case); llama40 / llama60 / mistral40 / mistral60: 32-layer stacks "
                    "on the paper's layer schedule at a 40 %% / 60 %% budget")
    ap.add_argument("--layer-batched", action="store_true",
                    help="workloads with several layers: keep all layers' caches in one allocation and "
                         "serve a decode step of the whole stack with one taskkv_decode_attn call")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 1 GiB device copies (a kernel of known traffic against which "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled)")
    ap.add_argument("--only", action="store_true",
                    help="with the default workload: leave out the short extra measurements of the other "
                         "workloads that are reported beside it")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU path exists)")
    out = measure(args, args.workload, not args.no_cpu_baseline, args.layer_batched, args.steps, args.warmup)
    if args.workload == "cfg5" and not args.only:
        # The other workloads, a few passes each.  The 8192-token layer moves 9.6 MB per decode step
        # (1.2 us at peak) and the 65536-token one 71 MB: they measure latency more than bandwidth.  The
        # 32-layer stack moves more per step than the headline workload, but as 32 calls.
        k_extra, w_extra = min(args.steps, 5), min(args.warmup, 1)
        pick = lambda m: {k: m[k] for k in ALSO_FIELDS}
        out["also_cfg2"] = pick(measure(args, "cfg2", False, False, k_extra, w_extra))
        out["also_cfg4"] = pick(measure(args, "cfg4", False, False, k_extra, w_extra))
        out["also_cfg3"] = {"per_layer": pick(measure(args, "cfg3", False, False, min(k_extra, 3), w_extra)),
                            "stacked": pick(measure(args, "cfg3", False, True, min(k_extra, 3), w_extra))}
        # The 32-layer stacks on the paper's layer schedule (Eq. 16-17) at a 40 % budget, Llama- and
        # Mistral-shaped: heterogeneous head counts and middle budgets differ from layer to layer.
        out["also_schedules"] = {
            name: {"per_layer": pick(measure(args, name, False, False, min(k_extra, 2), w_extra)),
                   "stacked": pick(measure(args, name, False, True, min(k_extra, 2), w_extra))}
            for name in ("llama40", "mistral40")}
        out["exact_semantic_vector"] = exact_vector_leg()
    print(json.dumps(out))


def measure(args, workload, with_cpu_baseline, layer_batched, steps, warmup):
    """One workload: warm-up passes, the timed passes, the same passes again with the kernel's own
    events, and (optionally) the oracle on the host.  Returns the fields of the JSON line."""
    import torch
    import paper_2501_15113_amd as tk
    from paper_2501_15113_amd import session
    from taskkv_synth import WORKLOADS, make_layer

    wl = WORKLOADS[workload]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    esize = 4 if wl.dtype == "f32" else 2
    steps_dec = wl.decode_steps
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free0, _ = torch.cuda.mem_get_info()

    plan = [None] * wl.n_layers
    if wl.schedule is not None:
        # stacks on the paper's layer schedule: per-layer counts from the library's plan (Eq. 16-17)
        beta, m_top, frac = wl.schedule
        plan = tk.taskkv_layer_plan(wl.n_kv_heads, beta, m_top, wl.n_layers, frac, wl.ctx_len, wl.n_sink, wl.n_recent)
    layers = [make_layer(wl, r, dev, plan=plan[r]) for r in range(wl.n_layers)]
    torch.cuda.synchronize()
    torch.cuda.empty_cache()          # the generators' fp32 temporaries are not part of the path
    cfgs = [session.cfg_from_workload(wl, ld.n_hetero, ld.n_middle) for ld in layers]
    batched = layer_batched and wl.n_layers > 1
    if batched:
        stack = session.LayerStack(cfgs, steps_dec, dev)
        bufs = stack.layers
        dec_in = []
        for s in range(steps_dec):
            parts = [ld.decode_inputs(s) for ld in layers]
            dec_in.append(tuple(torch.cat([p[i] for p in parts]) for i in range(3)))
    else:
        bufs = [session.LayerBuffers(c, steps_dec, dev) for c in cfgs]
        dec_in = [[ld.decode_inputs(s) for s in range(steps_dec)] for ld in layers]
    ctx = session.Context(cfgs + ([stack.cfg] if batched else []), steps_dec)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()

    tokens0 = sum(kept_tokens_total(wl, ld.n_hetero, ld.n_middle) for ld in layers)
    units = wl.batch * wl.n_kv_heads * wl.n_layers
    # bytes the decode steps of one pass must read: lens grow by one per step (append first)
    step_bytes = [(tokens0 + (s + 1) * units) * wl.head_dim * 2 * esize for s in range(steps_dec)]
    pass_bytes = float(sum(step_bytes))

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def compress_all():
        for ld, b in zip(layers, bufs):
            b.separate(ctx, ld.q_win, ld.k, ld.v)
            b.compress(ctx, ld.k, ld.v)
        if batched:
            stack.rebase(ctx)

    def one_pass(record):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        compress_all()
        e1.record()
        for s in range(steps_dec):
            if batched:
                stack.decode(ctx, *dec_in[s])
            else:
                for li, b in enumerate(bufs):
                    q, kn, vn = dec_in[li][s]
                    b.decode(ctx, q, kn, vn)
        e2.record()
        if record is not None:
            record.append((e0, e1, e2))

    for _ in range(warmup):
        one_pass(None)
    torch.cuda.synchronize()

    def timed(k_steps):
        rec = []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(k_steps):
            one_pass(rec)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        comp_ms = sum(a.elapsed_time(b) for a, b, _ in rec)
        dec_ms = sum(b.elapsed_time(c) for _, b, c in rec)
        return wall, comp_ms, dec_ms

    wall, comp_ms, dec_ms = timed(steps)
    value = pass_bytes * steps / (dec_ms * 1e-3) / 1e9

    # same region again with the library's own HIP events around the dominant kernel
    tk.taskkv_profile_enable(ctx.handle, 1)
    wall_p, _, dec_ms_p = timed(steps)
    kern_ms, launches = tk.taskkv_profile_read(ctx.handle)
    tk.taskkv_profile_enable(ctx.handle, 0)
    total_launches = steps * steps_dec * (1 if batched else wl.n_layers)
    bytes_per_launch = pass_bytes * steps / total_launches
    avg_kernel_ms = kern_ms / max(launches, 1)
    achieved = bytes_per_launch / (avg_kernel_ms * 1e-3) / 1e9
    assert tk.taskkv_last_async_error(ctx.handle) == 0
    traffic, traffic_src = PROFILED_TRAFFIC.get(wl.name, (None, None))

    out = {
        "metric": "ragged-cache decode attn: effective KV GB/s (% HBM peak) + compress ms/layer",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(wall * 1e3 / steps, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.batch} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
                               f"N={wl.ctx_len} layers={wl.n_layers} sinks/recent={wl.n_sink}/{wl.n_recent} "
                               f"decode_steps={steps_dec}" + (" (one decode call per step for all layers)"
                                                              if batched else ""),
                   "kept_tokens_after_compress": tokens0, "kv_bytes_per_decode_step": step_bytes[0]},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "decode_us_per_step": round(dec_ms * 1e3 / (steps * steps_dec), 3),
        "compress_ms_per_layer": round(comp_ms / (steps * wl.n_layers), 4),
        "roofline": {"bound": "hbm", "kernel": "decode_stream_kernel" if wl.dtype == "bf16" else "decode_f32_kernel",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "traffic_source": (traffic_src + " (a committed rocprofv3 --pmc reading, not a counter of this run)")
                     if traffic_src else None,
                     "avg_kernel_us": round(avg_kernel_ms * 1e3, 3), "launches_timed": int(launches),
                     "launches_run": int(total_launches),
                     "value_with_kernel_events": round(pass_bytes * steps / (dec_ms_p * 1e-3) / 1e9, 1)},
    }
    if workload == args.workload:
        # the separator's dominant kernel (row statistics, Eq. 12) with its own events, compress passes only
        if wl.dtype == "bf16":
            tk.taskkv_profile_enable(ctx.handle, 2)
            for _ in range(steps):
                compress_all()
            st_ms, st_n = tk.taskkv_profile_read(ctx.handle)
            tk.taskkv_profile_enable(ctx.handle, 0)
            if st_n:
                t_s = st_ms / st_n * 1e-3
                macs = wl.batch * wl.n_q_heads * wl.obs_window * wl.ctx_len * wl.head_dim
                k_bytes = wl.batch * wl.n_kv_heads * wl.ctx_len * wl.head_dim * esize
                util, util_src = PROFILED_MFMA_UTIL.get(wl.name, (None, None))
                out["roofline_scoring"] = {
                    "bound": "mfma", "kernel": "score_i8_stats_kernel", "dtype": "int8",
                    "achieved": round(16 * 2 * macs / t_s / 1e12, 1), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                    "frac": round(16 * 2 * macs / t_s / 1e12 / INT8_PEAK_TOPS, 4),
                    "ops_counted": "16 int8 digit products per bf16 product of Eq. 12 (all-zero digit blocks that "
                                   "the kernel skips are counted as done)",
                    "method_tflops": round(2 * macs / t_s / 1e12, 1),
                    "hbm_gbs": round(k_bytes / t_s / 1e9, 1), "avg_kernel_us": round(t_s * 1e6, 1),
                    "launches_timed": int(st_n),
                    "mfma_util_counter": util,
                    "mfma_util_source": (util_src + " (a committed rocprofv3 --pmc reading, not a counter of this run)")
                    if util_src else None}
        # device memory held while full K/V and the ragged cache coexist (the peak of compress + decode)
        kv_full = sum(ld.k.numel() + ld.v.numel() for ld in layers) * esize
        cache = (stack.k_cache.numel() + stack.v_cache.numel()) * esize if batched else \
            sum(b.k_cache.numel() + b.v_cache.numel() for b in bufs) * esize
        out["peak_device_bytes"] = {
            "value": int(free0 - free1),
            "what": "device memory taken between the start of the workload and the timed region (hipMemGetInfo): "
                    "prefill Q window / K / V of every layer, separator outputs, ragged caches, decode inputs of "
                    "every step and the library workspace, all resident at once; nothing is allocated after that",
            "full_kv_bytes": int(kv_full), "ragged_cache_bytes": int(cache),
            "ragged_over_full": round(cache / kv_full, 4), "library_workspace_bytes": int(ctx.bytes),
            "held_after_prefill_release": int(cache + ctx.bytes)}
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if with_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, layers)
    ctx.close()
    del layers, bufs, dec_in
    if batched:
        del stack
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
