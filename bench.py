#!/usr/bin/env python3
"""Benchmark: one step = spherical neighborhood attention forward + backward (all hot-path
kernels) on one batch of synthetic input, on ONE MI355X.

Prints one JSON line: whole-job throughput in output-points*heads per second, the roofline
of the dominant kernel (measured live with HIP events on the launch stream) and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks used for the roofline (fp32 vector, HBM3E, dense bf16 MFMA)
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0

# HBM bytes per launch (FETCH_SIZE + WRITE_SIZE from rocprofv3 --pmc, scaled by the factors a plain
# copy gives: see profiles/), keyed by (workload, kernel name).  Measured offline; None if not measured.
TRAFFIC_BYTES = {
    (3, "nattn_fwd_mfma"): 280e6, (3, "nattn_fwd_stream"): 747e6,
    (3, "nattn_bwd_dq_mfma"): 333e6, (3, "nattn_bwd_dq_stream"): 1023e6,
    (3, "nattn_bwd_dkdv_mfma"): 349e6, (3, "nattn_bwd_dkdv_stream"): 1058e6,
    (4, "nattn_fwd_tiled<8 waves>"): 981e6, (4, "nattn_fwd_tiled<1 wave>"): 228e6,
    (4, "nattn_bwd_dq_tiled<8 waves>"): 534e6, (4, "nattn_bwd_dq_tiled<1 wave>"): 290e6,
    (4, "nattn_bwd_dkdv2_tiled<8 waves>"): 159e6, (4, "nattn_bwd_dkdv2_tiled<1 wave>"): 1457e6,
    (6, "nattn_fwd_tiled<8 waves>"): 80e6, (6, "nattn_fwd_tiled<1 wave>"): 1425e6,
    (6, "nattn_bwd_dq_tiled<8 waves, classes>"): 66e6, (6, "nattn_bwd_dq_tiled<1 wave, classes>"): 2353e6,
    (6, "nattn_bwd_dkdv_tiled<8 waves, classes>"): 2853e6, (6, "nattn_bwd_dkdv_tiled<1 wave, classes>"): 902e6,
    (5, "global_fwd"): 160e6, (5, "global_bwd_dkdv"): 501e6, (5, "global_bwd_dq"): 287e6,
}


def copy_calibration():
    """Three 1 GiB device-to-device copies: what FETCH_SIZE / WRITE_SIZE read for a known transfer."""
    import torch
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    a.fill_(1.0)
    torch.cuda.synchronize()
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    print(json.dumps({"copy_calibration": {"bytes_per_copy": 1 << 30, "copies": 3}}))


def pairs_per_slice(S, g, c):
    """P = sum over output points of the neighborhood size (from the library's own lists)."""
    if c["nlon_out"] > c["nlon_in"]:
        # upsampling: one list per longitude class s = w mod r, each shared by nlon_in output longitudes
        r = c["nlon_out"] // c["nlon_in"]
        return sum(len(S.s2_grid_get_neighbors_at(g, h, s)) for h in range(c["nlat_out"]) for s in range(r)) * c["nlon_in"]
    row_ptr, _ = S.s2_grid_get_neighbors(g)
    return int(row_ptr[-1]) * c["nlon_out"]


def algorithmic(c, P):
    """Algorithmic flops and bytes per launch, fwd and bwd (recomputation not counted)."""
    bh, d = c["batch"] * c["heads"], c["d"]
    n_out, n_in = c["nlat_out"] * c["nlon_out"], c["nlat_in"] * c["nlon_in"]
    if c["kind"] == "global":
        fl_f, fl_b = 4.0 * n_out * n_in * d * bh, 10.0 * n_out * n_in * d * bh
        by_f = 2.0 * bh * (2 * n_out * d + 2 * n_in * d) + 4.0 * bh * n_out
        by_b = 2.0 * bh * (4 * n_out * d + 4 * n_in * d) + 4.0 * bh * n_out
    else:
        fl_f, fl_b = 4.0 * d * P * bh, 10.0 * d * P * bh
        by_f = 4.0 * bh * (2 * n_out * d + 2 * n_in * d + n_out)
        by_b = 4.0 * bh * (4 * n_out * d + 4 * n_in * d + n_out)
    return fl_f, fl_b, by_f, by_b


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="workload number (1-5; 6 = the extra upsampling workload), default 3 = 129x256 equiangular")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run three 1 GiB device copies (scale for the rocprofv3 HBM counters)")
    ap.add_argument("--cpu-slices", type=int, default=0, help="(batch*head) slices the oracle is timed on (0 = auto)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); batch*heads shards need no exchange, "
              "see DESIGN.md", file=sys.stderr)
        sys.exit(2)
    if args.copy_calibration:
        copy_calibration()
        return

    import numpy as np
    import torch

    import paper_2505_11157_amd as S
    from paper_2505_11157_amd.workloads import CONFIGS, grid_dict, make_inputs

    c, arrs = make_inputs(args.config)
    gd = grid_dict(args.config)
    B, H, d = c["batch"], c["heads"], c["d"]
    dev = torch.device("cuda:0")
    g = S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])
    scale = 1 / math.sqrt(d)
    is_global = c["kind"] == "global"
    tdt = torch.bfloat16 if c["dtype"] == "bf16" else torch.float32
    q, k, v, dout = (torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).to(tdt).contiguous() for a in arrs)

    if is_global:
        out = torch.empty_like(q)
        lse = torch.empty((B, H, q.shape[2]), dtype=torch.float32, device=dev)
        ws = torch.empty(max(S.s2_attn_global_bwd_workspace_bytes(g, B, H, d), 1), dtype=torch.uint8, device=dev)
        wsf = torch.empty(max(S.s2_attn_global_fwd_workspace_bytes(g, B, H, d), 1), dtype=torch.uint8, device=dev)
        fwd = lambda: S.s2_attn_global_fwd(g, q, k, v, scale, out=out, lse=lse, workspace=wsf)
        bwd = lambda: S.s2_attn_global_bwd(g, q, k, v, out, lse, dout, scale, dq=dq, dk=dk, dv=dv, workspace=ws)
    else:
        out = torch.empty((B, H, v.shape[2], c["nlat_out"], c["nlon_out"]), dtype=tdt, device=dev)
        lse = torch.empty((B, H, c["nlat_out"], c["nlon_out"]), dtype=torch.float32, device=dev)
        ws = torch.empty(max(S.s2_nattn_bwd_workspace_bytes(g, B, H, d, d), 1), dtype=torch.uint8, device=dev)
        fwd = lambda: S.s2_nattn_fwd(g, q, k, v, scale, out=out, lse=lse)
        bwd = lambda: S.s2_nattn_bwd(g, q, k, v, out, lse, dout, scale, dq=dq, dk=dk, dv=dv, workspace=ws)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

    def step():
        fwd()
        bwd()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps

    # per-phase device time with HIP events on the launch stream (the library launches on torch's current stream)
    def ev_time(fn, n):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) * 1e-3 / n

    n_ev = max(args.steps, 5)
    t_fwd, t_bwd = ev_time(fwd, n_ev), ev_time(bwd, n_ev)

    P = pairs_per_slice(S, g, c) if not is_global else c["nlat_in"] * c["nlon_in"] * c["nlat_out"] * c["nlon_out"]
    fl_f, fl_b, by_f, by_b = algorithmic(c, P)
    units = B * H * c["nlat_out"] * c["nlon_out"]

    # per-kernel device time: the library brackets each of its launches with HIP events on the launch
    # stream (s2_trace_*); the roofline object describes the launch with the largest average duration
    S.s2_trace_reset()
    S.s2_trace_enable(True)
    n_tr = max(min(args.steps, 10), 3)
    for _ in range(n_tr):
        step()
    torch.cuda.synchronize()
    S.s2_trace_enable(False)
    per = {}
    for name, ms, pairs in S.s2_trace_entries():
        a = per.setdefault(name, [0.0, 0, pairs])
        a[0] += ms
        a[1] += 1
    S.s2_trace_reset()

    def flops_per_pair(name):
        # algorithmic: forward 4d (QK^T, PV); dq launch 6d (s, dP, dq); dk/dv launch 4d (dk, dv)
        return (4.0 if "fwd" in name else 6.0 if "dq" in name else 4.0) * d

    peak = PEAK_BF16_TFLOPS if is_global else PEAK_FP32_TFLOPS
    kernels = {}
    for name, (tot, cnt, pairs) in per.items():
        ms = tot / cnt
        kernels[name] = {"ms": ms, "launches_per_step": cnt // n_tr, "pairs": pairs,
                         "TFLOPs": flops_per_pair(name) * pairs / (ms * 1e-3) / 1e12 if ms > 0 else None}
    dom = max(kernels, key=lambda n: kernels[n]["ms"])
    ach = kernels[dom]["TFLOPs"]
    roof = {"bound": "mfma" if is_global else "alu", "kernel": dom, "achieved": ach, "peak": peak,
            "unit": "TFLOP/s", "frac": ach / peak, "ms": kernels[dom]["ms"],
            "traffic": TRAFFIC_BYTES.get((args.config, dom))}
    roof["step"] = {"fwd_TFLOPs": fl_f / t_fwd / 1e12, "bwd_TFLOPs": fl_b / t_bwd / 1e12,
                    "fwd_frac": fl_f / t_fwd / 1e12 / peak, "bwd_frac": fl_b / t_bwd / 1e12 / peak,
                    "fwd_GBs": by_f / t_fwd / 1e9, "bwd_GBs": by_b / t_bwd / 1e9, "hbm_peak_GBs": PEAK_HBM_GBS}

    res = {
        "metric": "S2 neighborhood attn fwd+bwd: out-pts*heads/s" if not is_global else
                  "S2 global attn fwd+bwd: out-pts*heads/s",
        "value": units / t_step, "unit": "out-pts*heads/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if c["dtype"] == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": "cfg%d %s %dx%d->%dx%d theta=%.5f B%d H%d d%d" % (
            args.config, "LG" if c["grid_type"] else "equiangular-CC", c["nlat_in"], c["nlon_in"], c["nlat_out"],
            c["nlon_out"], c["theta"], B, H, d), "pairs_per_slice": P},
        "ms_fwd": t_fwd * 1e3, "ms_bwd": t_bwd * 1e3,
        "roofline": roof, "kernels": kernels,
    }

    if not args.no_cpu_baseline and not is_global and c["nlon_out"] > c["nlon_in"]:
        # the oracle handles upsampling grids only in its per-pair form (N_out * N_in bytes of mask): not timed here
        res["cpu_baseline"] = None
    elif not args.no_cpu_baseline:
        import oracle as O
        ns = args.cpu_slices or (24 if not is_global else 1)   # about 10-20 s of oracle time on 16 cores
        ns = min(ns, B * H)
        a64 = [a[:ns].astype(np.float64) for a in arrs]
        t0 = time.perf_counter()
        if is_global:
            O.global_fwd(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], a64[0], a64[1], a64[2], scale)
            O.global_bwd(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], *a64, scale)
        else:
            O.nattn_fwd(gd, a64[0], a64[1], a64[2], scale)
            O.nattn_bwd(gd, *a64, scale)
        t_cpu = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": ns * c["nlat_out"] * c["nlon_out"] / t_cpu, "unit": "out-pts*heads/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
                               "sample": "%d of %d (batch*head) slices of the same workload, fwd+bwd, %.1f s" % (
                                   ns, B * H, t_cpu)}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
