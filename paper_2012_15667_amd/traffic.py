"""HBM traffic per layer call, measured with rocprofv3 counters; writes profiles/hbm_traffic_by_layer.txt.

    python -m paper_2012_15667_amd.traffic            (on a box with an MI355X, from the repository root)

For every (layer, algorithm, path) of the list below it runs

    rocprofv3 --pmc <counter> --output-format csv -d rocprof_out/traffic -o <tag> -- \
        python3 bench.py --profile --warmup 0 --steps 2 --layers <layer> --algos <algo> [--wino-path <path>] [--direct-pick <pick>]

once per counter (FETCH_SIZE, WRITE_SIZE: KiB per dispatch between L2 and the fabric, so reads served by the
256 MB memory-side cache count like reads from HBM; optionally TCP_TCC_READ_REQ_sum / TCP_TCC_WRITE_REQ_sum:
requests between the compute units and L2; with --sq the matrix-core and LDS counters SQ_INSTS_MFMA,
SQ_VALU_MFMA_BUSY_CYCLES, SQ_LDS_BANK_CONFLICT, SQ_LDS_IDX_ACTIVE, SQ_BUSY_CYCLES, GRBM_GUI_ACTIVE), scales the counters by what they read for a plain 1 GiB copy
(`bench.py --copy-calibration`), and sums the library's kernels (names starting with iolb::) of one call.

bench.py reads the `row ...` lines of the summary for its per-layer `hbm_MB_measured`.
"""
import argparse
import collections
import csv
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT_DIR = os.path.join("rocprof_out", "traffic")
STEPS = 2

# (layer, algo, path): path "tuned"/"bound" for direct; "fused"/"unfused" for Winograd (thin layers: "tuned")
DEFAULT_RUNS = (
    [(l, "direct", "tuned") for l in ("cfg3", "cfg5a", "cfg5b", "cfg5c", "cfg5d")] +
    [("cfg2", "wino2", p) for p in ("unfused", "fused")] +
    [("cfg4", "wino4", p) for p in ("unfused", "fused")] +
    [("cfg5a", a, "tuned") for a in ("wino2", "wino4")] +
    [(l, a, p) for l in ("cfg5b", "cfg5c", "cfg5d") for a in ("wino2", "wino4") for p in ("unfused", "fused")]
)


REUSE = False      # --reuse: summarise the counter files of an earlier collection instead of running rocprofv3 again


def _rocprof(counters, tag, bench_args, timeout=180):
    cmd = ["rocprofv3", "--pmc"] + counters + ["--output-format", "csv", "-d", OUT_DIR, "-o", tag, "--",
                                               "python3", "bench.py"] + bench_args
    if REUSE:
        return " ".join(cmd)
    env = dict(os.environ, TMPDIR="/tmp")
    r = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=timeout)
    if r.returncode != 0:
        raise RuntimeError("rocprofv3 failed (%s):\n%s" % (" ".join(cmd), r.stdout[-2000:]))
    print("done: " + tag, flush=True)
    return " ".join(cmd)


def _rows(tag):
    files = glob.glob(os.path.join(ROOT, OUT_DIR, "**", tag + "_counter_collection.csv"), recursive=True)
    if not files:
        raise RuntimeError("no counter file for " + tag)
    with open(files[0]) as f:
        return list(csv.DictReader(f))


def _bench_args(layer, algo, path):
    args = ["--profile", "--warmup", "0", "--steps", str(STEPS), "--layers", layer, "--algos", algo]
    if algo == "direct":
        args += ["--direct-pick", path]
    elif path != "tuned":
        args += ["--wino-path", path]
    return args


def _path_label(layer, algo, path):
    """The path name bench.py looks a layer up under: the kernel path of the tile that ran."""
    from . import binding as B
    from .inputs import CONFIGS
    L = CONFIGS[layer]
    names = {B.PATH_FMA: "fma", B.PATH_MFMA: "mfma", B.PATH_FUSED: "fused", B.PATH_POINT: "pointwise"}
    if algo == "direct":
        if path != "tuned":
            return "bound"
        return names[B.iolb_tune(B.make_shape(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad))["path"]]
    if path == "tuned":
        sh = B.make_shape(L.N, L.C, L.H, L.W, L.K, algo={"wino2": B.WINO_F2, "wino4": B.WINO_F4}[algo])
        return {B.PATH_FMA: "fma", B.PATH_MFMA: "mfma", B.PATH_FUSED: "fused", B.PATH_POINT: "pointwise"}[B.iolb_tune(sh)["path"]]
    return {"unfused": "mfma", "fused": "fused"}[path]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=os.path.join("profiles", "hbm_traffic_by_layer.txt"))
    ap.add_argument("--l2", action="store_true", help="also collect the requests between the compute units and L2")
    ap.add_argument("--sq", action="store_true", help="also collect the matrix-core and LDS counters of the main kernels")
    ap.add_argument("--reuse", action="store_true", help="summarise the counter files already under rocprof_out/traffic")
    args = ap.parse_args()
    global REUSE
    REUSE = args.reuse
    from . import binding as B
    from .inputs import CONFIGS
    os.makedirs(os.path.join(ROOT, OUT_DIR), exist_ok=True)

    passes = [("FETCH_SIZE", ["FETCH_SIZE"]), ("WRITE_SIZE", ["WRITE_SIZE"])]
    if args.l2:
        passes.append(("L2REQ", ["TCP_TCC_READ_REQ_sum", "TCP_TCC_WRITE_REQ_sum"]))
    SQ = ["SQ_INSTS_MFMA", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE", "SQ_BUSY_CYCLES", "GRBM_GUI_ACTIVE"]
    layer_passes = list(passes) + ([("SQ", SQ)] if args.sq else [])

    # ---- calibration: what the counters read for a 1 GiB copy (3 copies per run)
    GiB_KiB = 1048576.0
    scale, raw, commands = {}, {}, []
    for pname, ctrs in passes:
        commands.append(_rocprof(ctrs, "copy_" + pname, ["--copy-calibration"]))
        for c in ctrs:
            v = [float(r["Counter_Value"]) for r in _rows("copy_" + pname)
                 if r["Counter_Name"] == c and float(r["Counter_Value"]) > 0 and
                 ("copy" in r["Kernel_Name"].lower() or "Cijk" in r["Kernel_Name"])]
            big = [x for x in v if x > 0.25 * max(v)]
            raw[c] = sum(big) / len(big)
    scale["FETCH_SIZE"] = GiB_KiB / raw["FETCH_SIZE"]
    scale["WRITE_SIZE"] = GiB_KiB / raw["WRITE_SIZE"]
    if args.l2:
        # bytes per request, from the same copy (2^30 bytes each way)
        scale["TCP_TCC_READ_REQ_sum"] = 2.0 ** 30 / raw["TCP_TCC_READ_REQ_sum"]
        scale["TCP_TCC_WRITE_REQ_sum"] = 2.0 ** 30 / raw["TCP_TCC_WRITE_REQ_sum"]

    # ---- the layers
    results = collections.OrderedDict()
    for layer, algo, path in DEFAULT_RUNS:
        per_kernel = collections.defaultdict(lambda: collections.defaultdict(float))
        for pname, ctrs in layer_passes:
            tag = "%s_%s_%s_%s" % (layer, algo, path, pname)
            commands.append(_rocprof(ctrs, tag, _bench_args(layer, algo, path)))
            for r in _rows(tag):
                k = r["Kernel_Name"]
                if "iolb::" not in k or (r["Counter_Name"] not in scale and r["Counter_Name"] not in SQ):
                    continue
                short = k.replace("(anonymous namespace)::", "").split("iolb::")[1].split("(")[0]
                per_kernel[short][r["Counter_Name"]] += float(r["Counter_Value"]) / STEPS
        results[(layer, algo, path)] = per_kernel

    lines = []
    w = lines.append
    w("HBM traffic per layer call (rocprofv3 counters FETCH_SIZE and WRITE_SIZE, one MI355X), by kernel.")
    w("")
    w("Written by:  python -m paper_2012_15667_amd.traffic%s%s   (from the repository root, on the GPU box)" % (" --l2" if args.l2 else "", " --sq" if args.sq else ""))
    w("which runs, each counter in a run of its own:")
    w("  " + commands[0])
    w("  rocprofv3 --pmc <counter> --output-format csv -d rocprof_out/traffic -o <tag> -- python3 bench.py --profile --warmup 0 "
      "--steps %d --layers <layer> --algos <algo> [--wino-path fused|unfused] [--direct-pick tuned]" % STEPS)
    w("")
    w("Calibration: a plain 1 GiB device copy (1048576 KiB each way) reads FETCH_SIZE = %.0f and WRITE_SIZE = %.0f," % (raw["FETCH_SIZE"], raw["WRITE_SIZE"]))
    w("so FETCH_SIZE is scaled by %.4f and WRITE_SIZE by %.4f.  The counters sit between L2 and the fabric: reads" % (scale["FETCH_SIZE"], scale["WRITE_SIZE"]))
    w("served by the 256 MB memory-side cache are included.  All figures are per call of the layer (average of %d)." % STEPS)
    if args.l2:
        w("L2 requests: the same copy gives %.0f bytes per TCP_TCC read request and %.0f per write request." %
          (scale["TCP_TCC_READ_REQ_sum"], scale["TCP_TCC_WRITE_REQ_sum"]))
    w("bound = max(compulsory bytes, leading term of the paper's lower bound at S_f = 40960 elements (160 KB)); for direct")
    w("convolution that term is below compulsory on every layer, for Winograd it is the printed expression of Sec. 4.3.")
    if args.sq:
        w("Matrix-core figures of a layer's main kernel: MFMA instructions against the algorithmic count (flop / 4096: one")
        w("v_mfma_f32_32x32x2_f32 is 4096 flop; direct 2 N K P Q C R S, Winograd 2 (m+2)^2 tiles C K) shows the work the kernel")
        w("adds (channel padding, idle slots); MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x GRBM_GUI_ACTIVE / 8 XCDs);")
        w("LDS conflicts = SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE.")
    w("")
    rows_out = []
    for (layer, algo, path), per_kernel in results.items():
        L = CONFIGS[layer]
        algo_id = {"direct": B.DIRECT, "wino2": B.WINO_F2, "wino4": B.WINO_F4}[algo]
        bnd = B.iolb_bounds(B.make_shape(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, algo_id), 40960)
        comp = 4.0 * bnd["compulsory_elems"]
        denom = max(comp, 4.0 * bnd["q_lower_lead"]) if algo != "direct" else comp
        label = _path_label(layer, algo, path)
        w("%s %s, path %s (%s):" % (layer, algo, label, path))
        tot_r = tot_w = 0.0
        main_bytes, main_name = 0.0, ""
        for k, c in per_kernel.items():
            rd = c["FETCH_SIZE"] * scale["FETCH_SIZE"] * 1024
            wr = c["WRITE_SIZE"] * scale["WRITE_SIZE"] * 1024
            extra = ""
            if args.l2:
                extra = "   L2 requests: %9.1f MB read %9.1f MB written" % (c["TCP_TCC_READ_REQ_sum"] * scale["TCP_TCC_READ_REQ_sum"] / 1e6,
                                                                          c["TCP_TCC_WRITE_REQ_sum"] * scale["TCP_TCC_WRITE_REQ_sum"] / 1e6)
            w("    %-46s read %9.1f MB   written %9.1f MB%s" % (k[:46], rd / 1e6, wr / 1e6, extra))
            tot_r += rd
            tot_w += wr
            if rd + wr > main_bytes and ("mfma" in k or "product" in k or "rows" in k or "fused" in k or "thin_kernel" in k):
                main_bytes, main_name = rd + wr, k
        if args.sq and main_name:
            c = per_kernel[main_name]
            m = {"direct": 0, "wino2": 2, "wino4": 4}[algo]
            if m:
                tiles = L.N * -(-L.H // m) * -(-L.W // m)
                flop = 2.0 * (m + 2) ** 2 * tiles * L.C * L.K
            else:
                P = (L.H + 2 * L.pad - L.R) // L.stride + 1
                Q = (L.W + 2 * L.pad - L.S) // L.stride + 1
                flop = 2.0 * L.N * L.K * P * Q * L.C * L.R * L.S
            if c["SQ_INSTS_MFMA"] > 0 and c["GRBM_GUI_ACTIVE"] > 0:
                w("    main kernel: %.0f MFMA instructions = %.3f x algorithmic;  MFMA busy %.3f;  LDS conflicts %.3f" % (
                    c["SQ_INSTS_MFMA"], c["SQ_INSTS_MFMA"] / (flop / 4096.0),
                    c["SQ_VALU_MFMA_BUSY_CYCLES"] / (1024.0 * c["GRBM_GUI_ACTIVE"] / 8.0),
                    c["SQ_LDS_BANK_CONFLICT"] / max(1.0, c["SQ_LDS_IDX_ACTIVE"])))
        w("    total %9.1f MB read + %9.1f MB written = %9.1f MB;  compulsory %8.1f MB (x %.2f);  bound %8.1f MB (x %.2f)" %
          (tot_r / 1e6, tot_w / 1e6, (tot_r + tot_w) / 1e6, comp / 1e6, (tot_r + tot_w) / comp, denom / 1e6, (tot_r + tot_w) / denom))
        w("")
        rows_out.append("row layer=%s algo=%s path=%s read_bytes=%.0f written_bytes=%.0f main_kernel_bytes=%.0f compulsory_bytes=%.0f bound_bytes=%.0f"
                        % (layer, algo, label, tot_r, tot_w, main_bytes, comp, denom))
    w("Machine-readable rows (bench.py reads these):")
    lines.extend(rows_out)
    with open(os.path.join(ROOT, args.out), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote " + args.out)


if __name__ == "__main__":
    main()
    sys.exit(0)
