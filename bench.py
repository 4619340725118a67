#!/usr/bin/env python3
"""Benchmark of the forward convolution layer (direct and Winograd) on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic layers: every layer of the
workload list below, each in the algorithm(s) named for it (tile pick, weight re-layout /
Winograd transforms, the matrix-core kernel, the store).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0

# (config name, algorithms run in a step)
WORKLOAD = [
    ("cfg2", ["wino2"]),
    ("cfg3", ["direct"]),
    ("cfg4", ["wino4"]),
    ("cfg5a", ["direct", "wino2", "wino4"]),
    ("cfg5b", ["direct", "wino2", "wino4"]),
    ("cfg5c", ["direct", "wino2", "wino4"]),
    ("cfg5d", ["direct", "wino2", "wino4"]),
]


def direct_flops(L):
    P = (L.H + 2 * L.pad - L.R) // L.stride + 1
    Q = (L.W + 2 * L.pad - L.S) // L.stride + 1
    return 2.0 * L.N * L.K * P * Q * L.C * L.R * L.S


def wino_product_flops(L, m):
    n = m + 2
    tiles = L.N * (-(-L.H // m)) * (-(-L.W // m))
    return 2.0 * n * n * tiles * L.C * L.K


def cpu_baseline(budget_s=15.0):
    """The CPU oracle as it stands, on a bounded sample: config 3 and config 4 whole, then images
    of config 5c in groups of 8 until about `budget_s` seconds of oracle time have been spent."""
    import numpy as np
    from oracle.conv_oracle import conv_ref
    from paper_2012_15667_amd.inputs import CONFIGS, layer_inputs
    flops, secs, threads = 0.0, 0.0, 0
    parts = []

    def timed(L, x, w, label):
        nonlocal flops, secs, threads
        t0 = time.perf_counter()
        _, threads = conv_ref(x, w, L.stride, L.pad, return_threads=True)
        secs += time.perf_counter() - t0
        flops += direct_flops(L) * (x.shape[0] / L.N)
        parts.append(label)

    for name in ("cfg3", "cfg4"):
        L = CONFIGS[name]
        x, w = layer_inputs(L)
        timed(L, x, w, name)
    extra = []
    for name in ("cfg5c", "cfg5d"):
        L = CONFIGS[name]
        x, w = layer_inputs(L)
        done = 0
        while done < L.N and secs < budget_s:
            timed(L, np.ascontiguousarray(x[done:done + 8]), w, "%s[%d:%d]" % (name, done, done + 8))
            done += 8
        if done:
            extra.append("the first %d images of %s" % (done, name))
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": "fp64 7-loop oracle on config 3 and config 4 (whole layers), %s: %.1f GFLOP in %.1f s"
                      % (" and ".join(extra), flops / 1e9, secs)}


TRAFFIC_FILE = os.path.join("profiles", "hbm_traffic_by_layer.txt")


def read_traffic_table():
    """Measured HBM bytes per layer call, from the committed rocprofv3 counter summary (written by
    `python -m paper_2012_15667_amd.traffic`): {(layer, algo, path): {"read": B, "written": B, "main_kernel": B}}.
    The figures are RECORDED ones (an earlier run of the same kernels), not measured by this run."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    table = {}
    if not os.path.exists(path):
        return table
    for line in open(path):
        if not line.startswith("row "):
            continue
        f = dict(kv.split("=", 1) for kv in line.split()[1:])
        table[(f["layer"], f["algo"], f["path"])] = {"read": float(f["read_bytes"]), "written": float(f["written_bytes"]),
                                                     "main_kernel": float(f["main_kernel_bytes"])}
    return table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", default="", help="comma-separated subset of config names (profiling runs)")
    ap.add_argument("--algos", default="", help="comma-separated subset of direct,wino2,wino3,wino4,wino6 (profiling runs; wino3 and wino6 are not part of the default step)")
    ap.add_argument("--wino-path", default="tuned", choices=["tuned", "fused", "unfused", "bound"],
                    help="Winograd tile: the tuner's pick, the first fused block, the first unfused tile of the "
                         "enumeration, or the bound-only pick (profiling runs)")
    ap.add_argument("--direct-pick", default="tuned", choices=["tuned", "bound"],
                    help="direct-convolution tile: the tuner's pick or the bound-only pick (profiling runs)")
    ap.add_argument("--profile", action="store_true",
                    help="run the selected layers --steps times and exit (for rocprofv3 runs: no warm-up beyond "
                         "--warmup, no per-layer repetitions, no ceiling probes, no JSON)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device copy (known size) to calibrate rocprofv3 FETCH_SIZE/WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (every figure is the one "
              "GPU's throughput)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2012_15667_amd import binding as B
    from paper_2012_15667_amd.inputs import CONFIGS, layer_inputs

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    B.lib()
    torch.cuda.set_device(0)

    if args.copy_calibration:
        n = 1 << 28                                   # 2^28 fp32 = 1 GiB read + 1 GiB written per copy
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 4 * n, "copy_bytes_written": 4 * n, "copies": 3}))
        return

    only_layers = set(filter(None, args.layers.split(",")))
    only_algos = set(filter(None, args.algos.split(",")))
    jobs = []           # (Layer, algo, x, w, y)
    for name, algos in WORKLOAD:
        if only_layers and name not in only_layers:
            continue
        L = CONFIGS[name]
        x, w = layer_inputs(L)
        xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        yd = torch.empty((L.N, L.K, L.H, L.W), dtype=torch.float32, device="cuda")
        for a in algos:
            if only_algos and a not in only_algos:
                continue
            jobs.append((L, a, xd, wd, yd))
    torch.cuda.synchronize()

    algo_ids = {"direct": B.DIRECT, "wino2": B.WINO_F2, "wino3": B.WINO_F3, "wino4": B.WINO_F4, "wino6": B.WINO_F6}

    def shape_of(L, a):
        return B.make_shape(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, algo_ids[a])

    def pick_tile(L, a, which):
        """None = let the library tune; otherwise an explicit tile."""
        sh = shape_of(L, a)
        if which == "tuned":
            return None
        if which == "bound":
            return B.iolb_tune_bound(sh)
        want = B.PATH_FUSED if which == "fused" else B.PATH_MFMA
        for t in B.iolb_enumerate(sh, 0, 0, False):
            if t["path"] == want:
                return t
        return None

    workspaces = {}

    def run(job, tile=None):
        L, a, xd, wd, yd = job
        if a == "direct":
            B.conv_direct(xd, wd, L.stride, L.pad, y=yd, cfg=tile)
        elif tile is None:
            B.conv_winograd(xd, wd, int(a[4:]), y=yd)
        else:
            m = int(a[4:])
            key = (L.name, m)
            if key not in workspaces:
                workspaces[key] = torch.empty(B.winograd_workspace_bytes(L.N, L.C, L.H, L.W, L.K, m), dtype=torch.uint8, device="cuda")
            B.conv_winograd(xd, wd, m, y=yd, cfg=tile, workspace=workspaces[key])

    forced = {id(j): pick_tile(j[0], j[1], args.direct_pick if j[1] == "direct" else args.wino_path) for j in jobs}

    def step():
        for job in jobs:
            run(job, forced[id(job)])

    if args.profile:
        for _ in range(args.warmup + args.steps):
            step()
        torch.cuda.synchronize()
        print("profiled %d calls of each of: %s" % (args.warmup + args.steps, ", ".join("%s[%s]" % (j[0].name, j[1]) for j in jobs)))
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly --steps steps, main kernels bracketed by HIP events ------------
    B.timing_read(B.TIME_DIRECT); B.timing_read(B.TIME_WINO_PRODUCT); B.timing_read(B.TIME_WINO_FUSED)
    B.timing_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    B.timing_enable(False)
    n_direct, ms_direct = B.timing_read(B.TIME_DIRECT)
    n_wino, ms_wino = B.timing_read(B.TIME_WINO_PRODUCT)
    n_fused, ms_fused = B.timing_read(B.TIME_WINO_FUSED)

    flops_step = sum(direct_flops(j[0]) for j in jobs)
    def tile_of(L, a):
        return B.iolb_tune(shape_of(L, a))

    # direct layers whose tile runs the matrix-core kernel (thin layers run a plain-FMA kernel of their own, which the
    # library does not time with them)
    def on_matrix_cores(j):
        return j[1] == "direct" and (forced[id(j)] or tile_of(j[0], "direct"))["path"] == B.PATH_MFMA
    direct_alg_flops = sum(direct_flops(j[0]) for j in jobs if on_matrix_cores(j))

    # Winograd layers by the kernel their tuned tile runs: unfused product, fused matrix-core kernel, or the thin
    # one-kernel FMA path (no matrix-core launch: nothing added to a roofline)
    wino_alg_flops = sum(wino_product_flops(j[0], int(j[1][4:])) for j in jobs
                         if j[1] != "direct" and tile_of(j[0], j[1])["path"] == B.PATH_MFMA)
    fused_alg_flops = sum(wino_product_flops(j[0], int(j[1][4:])) for j in jobs
                          if j[1] != "direct" and tile_of(j[0], j[1])["path"] == B.PATH_FUSED)

    # ---- per-layer figures (outside the timed region) ------------------------------------------
    traffic = read_traffic_table()
    path_names = {B.PATH_FMA: "fma", B.PATH_MFMA: "mfma", B.PATH_FUSED: "fused", B.PATH_POINT: "pointwise"}

    def timed(job, tile, reps=5):
        run(job, tile)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            run(job, tile)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    layers = []
    for job in jobs:
        L, a = job[0], job[1]
        shape = shape_of(L, a)
        tile = B.iolb_tune(shape)
        bound_tile = B.iolb_tune_bound(shape)
        ms = timed(job, None)
        ms_bound = ms if bound_tile == tile else timed(job, bound_tile)
        bnd = B.iolb_bounds(shape, 40960)
        keys = ("b", "x", "y", "z", "alpha", "threads", "path")
        rec = {
            "layer": L.name, "algo": a, "ms": round(ms, 4),
            "tflops_direct_equiv": round(direct_flops(L) / ms / 1e9, 2),
            "tile": {k: tile[k] for k in keys},
            "bound_pick": {"tile": {k: bound_tile[k] for k in keys}, "ms": round(ms_bound, 4),
                           "read_volume_over_tuned": round(bound_tile["q_read_elems"] / tile["q_read_elems"], 3)},
            "compulsory_MB": round(4 * bnd["compulsory_elems"] / 1e6, 2),
            "io_lower_bound_lead_MB_at_160KB": round(4 * bnd["q_lower_lead"] / 1e6, 2),
            "modelled_read_MB": round(4 * tile["q_read_elems"] / 1e6, 2),
        }
        if a != "direct":
            # the other Winograd path beside the tuned one (fused against unfused)
            other = pick_tile(L, a, "unfused" if tile["path"] == B.PATH_FUSED else "fused")
            if other is not None and tile["path"] != B.PATH_FMA:
                rec["other_path"] = {"path": path_names[other["path"]], "ms": round(timed(job, other), 4)}
        t = traffic.get((L.name, a, path_names[tile["path"]]))
        if t:
            denom = max(4 * bnd["compulsory_elems"], 4 * bnd["q_lower_lead"] if a != "direct" else 0)
            rec["hbm_MB_measured"] = round((t["read"] + t["written"]) / 1e6, 1)
            rec["hbm_over_bound"] = round((t["read"] + t["written"]) / denom, 3)
            rec["hbm_bound_MB"] = round(denom / 1e6, 1)
        layers.append(rec)

    # ---- measured ceilings of this GPU (outside the timed region) ------------------------------
    from paper_2012_15667_amd.ceilings import measure as measure_ceilings
    ceilings = measure_ceilings()

    ms_step = 1e3 * elapsed / args.steps
    value = flops_step / (elapsed / args.steps) / 1e12
    roofline = None
    if n_direct:
        achieved = direct_alg_flops * args.steps / (ms_direct * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "direct_mfma_kernel (all instantiations in the step)",
                    "achieved": round(achieved, 2), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_FP32_MFMA_TFLOPS, 4),
                    "frac_of_measured_mfma_loop": round(achieved / ceilings["mfma_f32_TFLOPs"], 4),
                    "avg_launch_ms": round(ms_direct / n_direct, 4), "launches": n_direct}
        per = [traffic[k]["main_kernel"] for k in traffic if k[1] == "direct" and any(j[0].name == k[0] and on_matrix_cores(j) for j in jobs)]
        roofline["traffic"] = round(sum(per) / len(per)) if per else None
        roofline["traffic_source"] = ("recorded: %s (rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of the same "
                                      "kernels, average over the direct launches of a step), not measured in this run" % TRAFFIC_FILE) if per else None
    wino_roofline = None
    if n_wino:
        achieved_w = wino_alg_flops * args.steps / (ms_wino * 1e-3) / 1e12
        wino_roofline = {"bound": "mfma", "kernel": "wino_product_kernel (all instantiations in the step)",
                         "achieved": round(achieved_w, 2), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(achieved_w / PEAK_FP32_MFMA_TFLOPS, 4),
                         "frac_of_measured_mfma_loop": round(achieved_w / ceilings["mfma_f32_TFLOPs"], 4),
                         "avg_launch_ms": round(ms_wino / n_wino, 4), "launches": n_wino}

    fused_roofline = None
    if n_fused:
        achieved_f = fused_alg_flops * args.steps / (ms_fused * 1e-3) / 1e12
        fused_roofline = {"bound": "mfma", "kernel": "wino_fused_mfma_kernel / wino_rows_kernel (fused Winograd layers of the step)",
                          "achieved": round(achieved_f, 2), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                          "frac": round(achieved_f / PEAK_FP32_MFMA_TFLOPS, 4),
                          "avg_launch_ms": round(ms_fused / n_fused, 4), "launches": n_fused}

    out = {
        "metric": "TFLOP/s per conv layer (direct & Winograd) + HBM bytes / I/O lower bound",
        "value": round(value, 3), "unit": "TFLOP/s (direct-conv-equivalent FLOPs, whole step)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs 2-5: " + ", ".join("%s[%s]" % (j[0].name, j[1]) for j in jobs),
                   "convs_per_step": len(jobs), "direct_equiv_gflop_per_step": round(flops_step / 1e9, 1)},
        "roofline": roofline,
        "roofline_winograd_product": wino_roofline,
        "roofline_winograd_fused": fused_roofline,
        "hbm_traffic_source": "recorded in %s by rocprofv3 counters, not measured in this run" % TRAFFIC_FILE,
        "measured_ceilings": ceilings,
        "layers": layers,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
