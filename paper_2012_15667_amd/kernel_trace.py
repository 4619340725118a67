"""Kernel-trace summary of a bench.py run; writes profiles/bench_step_kernel_trace.md.

    python -m paper_2012_15667_amd.kernel_trace        (on a box with an MI355X, from the repository root)

runs  rocprofv3 --kernel-trace --stats --output-format csv -d rocprof_out/prof -o bench -- python3 bench.py --steps 5
--warmup 1 --no-cpu-baseline  and tabulates rocprofv3's per-kernel durations beside the HIP-event figures that the
same bench.py run printed (the average launch durations of the dominant kernels must agree).
"""
import csv
import glob
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CMD = ["rocprofv3", "--kernel-trace", "--stats", "--output-format", "csv", "-d", os.path.join("rocprof_out", "prof"), "-o", "bench",
       "--", "python3", "bench.py", "--steps", "5", "--warmup", "1", "--no-cpu-baseline"]


def main():
    out = os.path.join(ROOT, "profiles", "bench_step_kernel_trace.md")
    r = subprocess.run(CMD, cwd=ROOT, env=dict(os.environ, TMPDIR="/tmp"), stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    if r.returncode != 0:
        raise RuntimeError("rocprofv3 failed:\n" + r.stderr[-2000:])
    d = json.loads([l for l in r.stdout.splitlines() if l.startswith("{")][-1])
    stats = glob.glob(os.path.join(ROOT, "rocprof_out", "prof", "**", "bench_kernel_stats.csv"), recursive=True)[0]
    rows = list(csv.DictReader(open(stats)))
    with open(out, "w") as f:
        f.write("# rocprofv3 kernel-trace summary: bench.py step (configs 2-5, direct + Winograd F2/F4), one MI355X\n\n")
        f.write("Command (run from the repository root on the GPU box; written by `python -m paper_2012_15667_amd.kernel_trace`):\n\n    %s\n\n" % " ".join(CMD))
        f.write("Calls include the warm-up step and the per-layer timing loops of bench.py, not only the timed steps.\n\n")
        f.write("| kernel | calls | total ms | avg us | % |\n|---|---|---|---|---|\n")
        tot = {}
        for row in rows:
            name = row["Name"].replace("void ", "").replace("iolb::(anonymous namespace)::", "").replace("iolb::", "").split("(")[0]
            f.write("| %s | %s | %.3f | %.1f | %.2f |\n" % (name, row["Calls"], int(row["TotalDurationNs"]) / 1e6,
                                                         float(row["AverageNs"]) / 1e3, float(row["Percentage"])))
            t = tot.setdefault(name.split("<")[0], [0, 0])
            t[0] += int(row["Calls"])
            t[1] += int(row["TotalDurationNs"])
        f.write("\nPer kernel family:\n\n| family | calls | total ms | avg launch ms |\n|---|---|---|---|\n")
        for fam, (c, ns) in sorted(tot.items(), key=lambda kv: -kv[1][1]):
            f.write("| %s | %d | %.3f | %.4f |\n" % (fam, c, ns / 1e6, ns / 1e6 / c))
        f.write("\nbench.py's own HIP-event figures from the same run (timed steps only):\n\n")
        for key in ("roofline", "roofline_winograd_product", "roofline_winograd_fused"):
            rf = d.get(key)
            if rf:
                f.write("- %s: avg launch %.4f ms over %d launches, %.2f TFLOP/s (%.3f of the fp32 MFMA peak)\n" %
                        (rf["kernel"], rf["avg_launch_ms"], rf["launches"], rf["achieved"], rf["frac"]))
        f.write("- step: %.3f ms, %.1f TFLOP/s direct-equivalent\n\nPer layer (five back-to-back repetitions, outside the timed steps):\n\n" % (d["ms_per_step"], d["value"]))
        f.write("| layer | algo | path | tile b,x,y,z,alpha,threads | ms | TFLOP/s direct-eq. | bound-only pick ms | other Winograd path ms |\n|---|---|---|---|---|---|---|---|\n")
        for l in d["layers"]:
            t = l["tile"]
            other = l.get("other_path")
            f.write("| %s | %s | %s | %d,%d,%d,%d,%d,%d | %.4f | %.1f | %.4f | %s |\n" % (
                l["layer"], l["algo"], {0: "fma", 1: "mfma", 2: "fused"}[t["path"]], t["b"], t["x"], t["y"], t["z"], t["alpha"], t["threads"],
                l["ms"], l["tflops_direct_equiv"], l["bound_pick"]["ms"], "%s %.4f" % (other["path"], other["ms"]) if other else ""))
    print("wrote " + out)


if __name__ == "__main__":
    main()
    sys.exit(0)
