#!/usr/bin/env python3
"""Benchmark of the Task-KV hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
for every layer of the workload, semantic separator + cache compression of
the resident prefill K/V, then the workload's decode steps (append + ragged
attention) over every layer.  Inputs are generated on the GPU before the timed
region.  The reported value is the decode part's effective KV bandwidth:
bytes of kept K and V rows that each decode step must read (sum over units of
len * d * 2 * sizeof) divided by the GPU time of the decode calls.

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
# HBM bytes per launch of the decode attention kernel from rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE scaled by a copy kernel); None until measured for the
# default workload -- see profiles/.
MEASURED_TRAFFIC = {"cfg5": 573.2e6}  # profiles/decode_stream_kernel_cfg5_hbm_traffic.txt


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


def cpu_baseline(wl, layers, budget_s=12.0):
    """The CPU oracle, as it stands, on a bounded sample: batch element 0 of
    layer 0 -- one compression, then decode steps until the time budget."""
    import numpy as np
    from oracle import taskkv_oracle as orc
    from taskkv_synth import to_numpy
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    ld = layers[0]
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
    return {"value": nbytes / t_dec / 1e9, "unit": "GB/s", "cores": int(cores), "kind": "oracle",
            "sample": f"batch element 0 of layer 0: {steps} decode steps over its {len(kc)} units "
                      f"(no append), fp64 numpy; compression of that batch element took "
                      f"{t_comp * 1e3:.0f} ms",
            "compress_ms_per_layer_scaled": t_comp * 1e3 * wl.batch}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg5", help="cfg1..cfg5 (default cfg5: largest context, "
                    "the load-imbalance stress case)")
    ap.add_argument("--layer-batched", action="store_true",
                    help="workloads with several layers: keep all layers' caches in one allocation and "
                         "serve a decode step of the whole stack with one taskkv_decode_attn call")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 1 GiB device copies (a kernel of known traffic against which "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled)")
    ap.add_argument("--only", action="store_true",
                    help="with the default workload: leave out the short extra measurement of cfg2 "
                         "(the 8192-token single layer) that is reported beside it")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU path exists)")
    out = measure(args, args.workload, not args.no_cpu_baseline)
    if args.workload == "cfg5" and not args.only:
        # the 8192-token layer moves 9.6 MB per decode step (1.2 us at peak): it measures latency, not
        # bandwidth, so it is reported beside the headline workload rather than as `value`
        small = measure(args, "cfg2", False)
        out["also_cfg2"] = {k: small[k] for k in ("config", "value", "unit", "pct_hbm_peak", "decode_us_per_step",
                                                  "compress_ms_per_layer", "roofline")}
    print(json.dumps(out))


def measure(args, workload, with_cpu_baseline):
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

    layers = [make_layer(wl, r, dev) for r in range(wl.n_layers)]
    cfgs = [session.cfg_from_workload(wl, ld.n_hetero, ld.n_middle) for ld in layers]
    batched = args.layer_batched and wl.n_layers > 1
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
    torch.cuda.synchronize()

    tokens0 = sum(kept_tokens_total(wl, ld.n_hetero, ld.n_middle) for ld in layers)
    units = wl.batch * wl.n_kv_heads * wl.n_layers
    # bytes the decode steps of one pass must read: lens grow by one per step (append first)
    step_bytes = [(tokens0 + (s + 1) * units) * wl.head_dim * 2 * esize for s in range(steps_dec)]
    pass_bytes = float(sum(step_bytes))

    ctx = session.Context(cfgs + ([stack.cfg] if batched else []), steps_dec)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def one_pass(record):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        for ld, b in zip(layers, bufs):
            b.separate(ctx, ld.q_win, ld.k, ld.v)
            b.compress(ctx, ld.k, ld.v)
        if batched:
            stack.rebase()
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

    for _ in range(args.warmup):
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

    wall, comp_ms, dec_ms = timed(args.steps)
    value = pass_bytes * args.steps / (dec_ms * 1e-3) / 1e9

    # same region again with the library's own HIP events around the dominant kernel
    tk.taskkv_profile_enable(ctx.handle, True)
    wall_p, _, dec_ms_p = timed(args.steps)
    kern_ms, launches = tk.taskkv_profile_read(ctx.handle)
    tk.taskkv_profile_enable(ctx.handle, False)
    total_launches = args.steps * steps_dec * (1 if batched else wl.n_layers)
    bytes_per_launch = pass_bytes * args.steps / total_launches
    avg_kernel_ms = kern_ms / max(launches, 1)
    achieved = bytes_per_launch / (avg_kernel_ms * 1e-3) / 1e9
    assert tk.taskkv_last_async_error(ctx.handle) == 0

    out = {
        "metric": "ragged-cache decode attn: effective KV GB/s (% HBM peak) + compress ms/layer",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall * 1e3 / args.steps, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.batch} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
                               f"N={wl.ctx_len} layers={wl.n_layers} sinks/recent={wl.n_sink}/{wl.n_recent} "
                               f"decode_steps={steps_dec}" + (" (one decode call per step for all layers)"
                                                              if batched else ""),
                   "kept_tokens_after_compress": tokens0, "kv_bytes_per_decode_step": step_bytes[0]},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "decode_us_per_step": round(dec_ms * 1e3 / (args.steps * steps_dec), 3),
        "compress_ms_per_layer": round(comp_ms / (args.steps * wl.n_layers), 4),
        "roofline": {"bound": "hbm", "kernel": "decode_stream_kernel" if wl.dtype == "bf16" else "decode_f32_kernel",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC.get(wl.name),
                     "avg_kernel_us": round(avg_kernel_ms * 1e3, 3), "launches_timed": int(launches),
                     "value_with_kernel_events": round(pass_bytes * args.steps / (dec_ms_p * 1e-3) / 1e9, 1)},
    }
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
    return out


if __name__ == "__main__":
    main()
