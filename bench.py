#!/usr/bin/env python3
"""Benchmark: one step = spherical attention forward + backward (all hot-path kernels) on one batch of
synthetic input, on ONE MI355X.

Prints one JSON line.  The headline figures are those of workload 3 (129x256 equiangular grid, the
shallow-water-sized layer): whole-job throughput in output-points*heads per second, the roofline of its dominant
kernel (measured live with HIP events on the launch stream) and the CPU oracle timed on a bounded sample of the
same workload.  `workloads` carries the same measurement (step time, dominant kernel, roofline fraction) for the
other full-size workloads: 2 (64x128 Gaussian grid), 4 (257x512 -> 129x256) and 5 (global attention, bf16).

Other modes: --peaks (measured device ceilings), --copy-calibration (a copy of known size for the HBM counters).
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

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy of known size: written by
# `python -m paper_2505_11157_amd.pmc_traffic` from the counter files of a profile run (the commands are in the
# file itself and in profiles/), keyed by workload number and kernel name as the library's trace reports it
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def load_traffic():
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f).get("bytes_per_launch", {})
    except (OSError, ValueError):
        return {}


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


def peaks():
    """Measured ceilings of this device (plain kernels of the library, see s2_peak_measure)."""
    import paper_2505_11157_amd as S
    res = {
        "stream_copy_GBs": S.s2_peak_measure(S.S2_PEAK_COPY),
        "v_fma_f32_TFLOPs": S.s2_peak_measure(S.S2_PEAK_FMA_F32),
        "mfma_f32_32x32x2_TFLOPs": S.s2_peak_measure(S.S2_PEAK_MFMA_F32),
        "mfma_bf16_32x32x16_TFLOPs": S.s2_peak_measure(S.S2_PEAK_MFMA_BF16),
        "lds_read_b128_TBs": S.s2_peak_measure(S.S2_PEAK_LDS_READ),
    }
    # bytes per clock and compute unit at the published 2.4 GHz and 256 units
    res["lds_read_B_per_clk_per_CU"] = res["lds_read_b128_TBs"] * 1e12 / 2.4e9 / 256
    res["published"] = {"hbm_GBs": PEAK_HBM_GBS, "fp32_vector_TFLOPs": PEAK_FP32_TFLOPS,
                        "fp32_mfma_TFLOPs": PEAK_FP32_TFLOPS, "bf16_mfma_TFLOPs": PEAK_BF16_TFLOPS}
    print(json.dumps({"peaks": res}))


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
    esz = 2.0 if c["dtype"] == "bf16" else 4.0
    if c["kind"] == "global":
        fl_f, fl_b = 4.0 * n_out * n_in * d * bh, 10.0 * n_out * n_in * d * bh
    else:
        fl_f, fl_b = 4.0 * d * P * bh, 10.0 * d * P * bh
    by_f = esz * bh * (2 * n_out * d + 2 * n_in * d) + 4.0 * bh * n_out
    by_b = esz * bh * (4 * n_out * d + 4 * n_in * d) + 4.0 * bh * n_out
    return fl_f, fl_b, by_f, by_b


def workload_name(cfg, c):
    return "cfg%d %s %dx%d->%dx%d theta=%.5f B%d H%d d%d %s" % (
        cfg, "LG" if c["grid_type"] else "equiangular-CC", c["nlat_in"], c["nlon_in"], c["nlat_out"],
        c["nlon_out"], c["theta"], c["batch"], c["heads"], c["d"], c["dtype"])


def measure(cfg, steps, warmup, traffic):
    """Time `steps` forward + backward passes of workload `cfg` (inputs resident in HBM) and the launches inside."""
    import torch

    import paper_2505_11157_amd as S
    from paper_2505_11157_amd.workloads import grid_dict, make_inputs

    c, arrs = make_inputs(cfg)
    gd = grid_dict(c)
    B, H, d = c["batch"], c["heads"], c["d"]
    dev = torch.device("cuda:0")
    g = S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])
    scale = 1 / math.sqrt(d)
    is_global = c["kind"] == "global"
    tdt = torch.bfloat16 if c["dtype"] == "bf16" else torch.float32
    q, k, v, dout = (torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).to(tdt).contiguous() for a in arrs)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

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
        ws = torch.empty(max(S.s2_nattn_bwd_workspace_bytes(g, B, H, d, d, S.S2_BF16 if c["dtype"] == "bf16" else S.S2_F32), 1),
                         dtype=torch.uint8, device=dev)
        fwd = lambda: S.s2_nattn_fwd(g, q, k, v, scale, out=out, lse=lse)
        bwd = lambda: S.s2_nattn_bwd(g, q, k, v, out, lse, dout, scale, dq=dq, dk=dk, dv=dv, workspace=ws)

    def step():
        fwd()
        bwd()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / steps

    # per-phase device time with HIP events on the launch stream (the library launches on torch's current stream)
    def ev_time(fn, n):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) * 1e-3 / n

    n_ev = max(steps, 5)
    t_fwd, t_bwd = ev_time(fwd, n_ev), ev_time(bwd, n_ev)

    P = pairs_per_slice(S, g, c) if not is_global else c["nlat_in"] * c["nlon_in"] * c["nlat_out"] * c["nlon_out"]
    fl_f, fl_b, by_f, by_b = algorithmic(c, P)
    units = B * H * c["nlat_out"] * c["nlon_out"]

    # per-kernel device time: the library brackets each of its launches with HIP events on the launch
    # stream (s2_trace_*); the roofline object describes the launch with the largest average duration
    S.s2_trace_reset()
    S.s2_trace_enable(True)
    n_tr = max(min(steps, 10), 3)
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
        # algorithmic: forward 4d (QK^T, PV); dq launch 6d (s, dP, dq); dk/dv launch 4d (dk, dv); a launch that
        # produces dq, dk and dv together 10d
        if "fwd" in name:
            return 4.0 * d
        if "dqkv" in name:
            return 10.0 * d
        return (6.0 if "dq" in name else 4.0) * d

    def launch_bytes(name):
        # algorithmic bytes of one launch of the neighborhood path: its inputs and outputs once
        esz = 2.0 if c["dtype"] == "bf16" else 4.0
        bh = B * H
        n_out, n_in = c["nlat_out"] * c["nlon_out"], c["nlat_in"] * c["nlon_in"]
        if "fwd" in name:
            return esz * bh * d * (2 * n_out + 2 * n_in) + 4.0 * bh * n_out
        if "dq" in name:
            return esz * bh * d * (4 * n_out + 2 * n_in) + 8.0 * bh * n_out
        return esz * bh * d * (2 * n_out + 4 * n_in) + 8.0 * bh * n_out

    on_mfma = is_global or c["dtype"] == "bf16"
    peak = PEAK_BF16_TFLOPS if on_mfma else PEAK_FP32_TFLOPS
    kernels = {}
    for name, (tot, cnt, pairs) in per.items():
        ms = tot / cnt
        kernels[name] = {"ms": ms, "launches_per_step": cnt // n_tr, "pairs": pairs,
                         "TFLOPs": flops_per_pair(name) * pairs / (ms * 1e-3) / 1e12 if ms > 0 and pairs > 0 else None}
    timed = {n: kk for n, kk in kernels.items() if kk["TFLOPs"] is not None}
    dom = max(timed, key=lambda n: timed[n]["ms"])
    ach = kernels[dom]["TFLOPs"]
    if not is_global and c["dtype"] == "bf16":
        # bf16 tensors: by the algorithmic figures (flop / 2.5 PFLOP/s against bytes / 8 TB/s) the path is bound by
        # HBM bandwidth, so the launch is priced by its bytes
        gbs = launch_bytes(dom) / (kernels[dom]["ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": dom, "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": gbs / PEAK_HBM_GBS, "ms": kernels[dom]["ms"], "traffic": traffic.get(str(cfg), {}).get(dom),
                "algorithmic_bytes": launch_bytes(dom), "TFLOPs": ach}
    else:
        roof = {"bound": "mfma" if on_mfma else "alu", "kernel": dom, "achieved": ach, "peak": peak,
                "unit": "TFLOP/s", "frac": ach / peak, "ms": kernels[dom]["ms"],
                "traffic": traffic.get(str(cfg), {}).get(dom)}
    roof["step"] = {"fwd_TFLOPs": fl_f / t_fwd / 1e12, "bwd_TFLOPs": fl_b / t_bwd / 1e12,
                    "fwd_frac": fl_f / t_fwd / 1e12 / peak, "bwd_frac": fl_b / t_bwd / 1e12 / peak,
                    "step_frac": (fl_f + fl_b) / (t_fwd + t_bwd) / 1e12 / peak,
                    "fwd_GBs": by_f / t_fwd / 1e9, "bwd_GBs": by_b / t_bwd / 1e9,
                    "hbm_frac": (by_f + by_b) / (t_fwd + t_bwd) / 1e9 / PEAK_HBM_GBS, "hbm_peak_GBs": PEAK_HBM_GBS}
    return {"c": c, "gd": gd, "arrs": arrs, "scale": scale, "t_step": t_step, "t_fwd": t_fwd, "t_bwd": t_bwd,
            "units": units, "P": P, "roofline": roof, "kernels": kernels, "is_global": is_global}


def measure_layers(steps):
    """Forward + backward of the two layers built around the kernels (Sec. 3.4, App. B.3) on the 129x256 grid of the
    headline workload, timed with HIP events on the launch stream: reported as they stand (no roofline: a chain of
    norm, projection, attention and split-K launches)."""
    import torch

    import paper_2505_11157_amd as S
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cpu").manual_seed(7)
    rnd = lambda *shape: torch.randn(*shape, generator=gen).to(dev)
    nlat, nlon, theta, B = 129, 256, 4 * math.pi / 128, 4
    g = S.s2_grid_init(0, nlat, nlon, nlat, nlon, theta)

    def ev_time(fn, n):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        b.synchronize()
        return a.elapsed_time(b) / n

    out = {}
    # attention sub-block with the head width of the SegFormer stages of App. C (embedding 128, 8 heads of 16)
    C, H = 128, 8
    x, dy = rnd(B, C, nlat, nlon), rnd(B, C, nlat, nlon)
    params = {"gamma": rnd(C), "beta": rnd(C), "pos": rnd(C, nlat, nlon)}
    for n in "qkvo":
        params["W" + n] = rnd(C, C) / math.sqrt(C)
        params["b" + n] = rnd(C)
    state = {}

    def mha_fwd():
        state["y"], state["ws"] = S.s2_mha_fwd(g, x, params, H)

    def mha_bwd():
        S.s2_mha_bwd(g, x, params, H, dy, state["ws"])

    t_f = ev_time(mha_fwd, steps)
    t_b = ev_time(mha_bwd, steps)
    out["mha"] = {"workload": "attention sub-block 129x256 B%d C%d heads%d d%d f32" % (B, C, H, C // H), "ms_fwd": t_f,
                  "ms_bwd": t_b, "ms_per_step": t_f + t_b}
    # DISCO convolution, 64 -> 64 channels, 9 radial basis functions, same grid
    cin = cout = 64
    dc = S.s2_disco_init(g, 9)
    xd, dyd = rnd(B, cin, nlat, nlon), rnd(B, cout, nlat, nlon)
    w, bias = rnd(cout, cin, 9) / math.sqrt(9 * cin), rnd(cout)

    def disco_fwd():
        state["yd"], state["wsd"] = S.s2_disco_fwd(dc, xd, w, bias)

    def disco_bwd():
        S.s2_disco_bwd(dc, xd, w, dyd, state["wsd"])

    t_f = ev_time(disco_fwd, steps)
    t_b = ev_time(disco_bwd, steps)
    out["disco"] = {"workload": "DISCO convolution 129x256 B%d %d->%d channels K9 f32" % (B, cin, cout), "ms_fwd": t_f,
                    "ms_bwd": t_b, "ms_per_step": t_f + t_b}
    return out


def cpu_baseline(m, cpu_slices):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    import numpy as np

    import oracle as O
    c, gd, arrs, scale = m["c"], m["gd"], m["arrs"], m["scale"]
    if not m["is_global"] and c["nlon_out"] > c["nlon_in"]:
        return None    # the oracle handles upsampling grids only in its per-pair form (N_out * N_in bytes of mask)
    nbh = c["batch"] * c["heads"]
    ns = min(cpu_slices or (24 if not m["is_global"] else 1), nbh)   # about 10-20 s of oracle time on 16 cores
    a64 = [a[:ns].astype(np.float64) for a in arrs]
    t0 = time.perf_counter()
    if m["is_global"]:
        O.global_fwd(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], a64[0], a64[1], a64[2], scale)
        O.global_bwd(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], *a64, scale)
    else:
        O.nattn_fwd(gd, a64[0], a64[1], a64[2], scale)
        O.nattn_bwd(gd, *a64, scale)
    t_cpu = time.perf_counter() - t0
    return {"value": ns * c["nlat_out"] * c["nlon_out"] / t_cpu, "unit": "out-pts*heads/s",
            "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
            "sample": "%d of %d (batch*head) slices of the same workload, fwd+bwd, %.1f s" % (ns, nbh, t_cpu)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3,
                    help="headline workload (1-5; 6 = upsampling, 7 = workload 3 with bf16 tensors), default 3 = 129x256 equiangular")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--force-band", action="store_true",
                    help="float32 d = 32 workloads on the band-tile matrix-core kernels that serve d = 16 and 64")
    ap.add_argument("--no-workloads", action="store_true", help="skip the extra `workloads` measurements")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run three 1 GiB device copies (scale for the rocprofv3 HBM counters)")
    ap.add_argument("--peaks", action="store_true", help="only measure the device ceilings (copy, FMA, MFMA, LDS)")
    ap.add_argument("--layers", action="store_true", help="only time the attention sub-block and the DISCO convolution")
    ap.add_argument("--cpu-slices", type=int, default=0, help="(batch*head) slices the oracle is timed on (0 = auto)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1): every (batch, head) slice is an independent "
              "problem, so several GPUs would each take a share of the slices with no exchange", file=sys.stderr)
        sys.exit(2)
    if args.copy_calibration:
        copy_calibration()
        return
    if args.peaks:
        peaks()
        return
    if args.layers:
        print(json.dumps({"layers": measure_layers(max(args.steps // 4, 3))}))
        return

    from paper_2505_11157_amd.workloads import CONFIGS
    if args.force_band:
        import torch                       # torch's HIP runtime first: the library must load into that process image
        torch.cuda.init()
        import paper_2505_11157_amd as S
        S.s2_debug_control(S.S2_DEBUG_FORCE_BAND, 0)

    traffic = load_traffic()
    m = measure(args.config, args.steps, args.warmup, traffic)
    c = m["c"]
    res = {
        "metric": "S2 neighborhood attn fwd+bwd: out-pts*heads/s" if not m["is_global"] else
                  "S2 global attn fwd+bwd: out-pts*heads/s",
        "value": m["units"] / m["t_step"], "unit": "out-pts*heads/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": m["t_step"] * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if c["dtype"] == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": workload_name(args.config, c), "pairs_per_slice": m["P"]},
        "ms_fwd": m["t_fwd"] * 1e3, "ms_bwd": m["t_bwd"] * 1e3,
        "roofline": m["roofline"], "kernels": m["kernels"],
    }
    if not args.no_workloads and args.config == 3:
        # the other full-size workloads, same measurement with fewer steps (a few hundred ms of GPU time in all)
        others = {}
        for cfg in (2, 4, 5, 7, 8, 9):
            if cfg not in CONFIGS:
                continue
            o = measure(cfg, max(args.steps // 2, 5), max(args.warmup, 2), traffic)
            r = o["roofline"]
            others["cfg%d" % cfg] = {
                "workload": workload_name(cfg, o["c"]), "ms_per_step": o["t_step"] * 1e3, "ms_fwd": o["t_fwd"] * 1e3,
                "ms_bwd": o["t_bwd"] * 1e3, "value": o["units"] / o["t_step"], "unit": "out-pts*heads/s",
                "dtype": o["c"]["dtype"], "dominant_kernel": r["kernel"], "bound": r["bound"], "frac": r["frac"],
                "achieved": r["achieved"], "peak": r["peak"], "traffic": r["traffic"],
                "step_frac": r["step"]["step_frac"], "hbm_frac": r["step"]["hbm_frac"],
                "kernels_ms": {n: kk["ms"] for n, kk in o["kernels"].items()}}
        res["workloads"] = others
        res["layers"] = measure_layers(5)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(m, args.cpu_slices)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
