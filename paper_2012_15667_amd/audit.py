"""Audit of the tuner against measurement; writes profiles/tuner_vs_sweep.md.

    python -m paper_2012_15667_amd.audit        (on a box with an MI355X, from the repository root)

Part 1 -- exhaustive tile sweeps (paper_2012_15667_amd.sweep) of config 3 and configs 5a-d in direct convolution,
F(2x2) and F(4x4): how many tiles were timed, where the tuner's pick (modelled time) and the bound-only pick (least
reading volume inside the optimality box, the paper's objective alone) rank, and how far each is from the fastest.
Part 3 -- the fused Winograd kernels (all four steps in one kernel, Sec. 5.3) against the unfused path (four kernels
with the transformed tensors in memory) over layer shapes: both times, and whether the tuner's choice between
them is the faster one.
Part 2 -- the measured auto-tuning engine of Sec. 6 (paper_2012_15667_amd.autotune) with and without the
optimality box of Table 1: size of the searching domain, measurements until the search stops, best time found --
the analogue of the "search space" and "iterations" columns of Table 2.
"""
import contextlib
import io
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SWEEPS = [(l, a) for l in ("cfg3", "cfg5a", "cfg5b", "cfg5c", "cfg5d") for a in ("direct", "wino2", "wino4")]
CROSSOVER = ["cfg2", "cfg4", "cfg5b", "cfg5c", "cfg5d", "alex3", "alex4"] + \
            ["64,%d,56,56,%d,3,3,1,1" % (c, c) for c in (16, 32, 64, 128, 512)] + \
            ["64,%d,14,14,%d,3,3,1,1" % (c, c) for c in (64, 128, 512)] + ["8,128,28,28,128,3,3,1,1", "1,256,56,56,256,3,3,1,1"]
ENGINE_LAYERS = [("alex3", "direct"), ("alex2", "direct"), ("cfg3", "direct"), ("cfg5d", "direct")]
MAX_TILES = 300


def tile_text(t):
    return "%d,%d,%d,%d,%d,%d%s" % (t["b"], t["x"], t["y"], t["z"], t["alpha"], t["threads"],
                                    {0: " fma", 1: "", 2: " fused", 3: " pointwise"}[t["path"]])


def main():
    from . import binding as B
    from .autotune import autotune, gpu_domain_and_measure, with_stage_depths
    from .sweep import sweep
    lines = ["# The tuner against measurement (one MI355X)", "",
             "Written by `python -m paper_2012_15667_amd.audit` (run from the repository root on the GPU box).", "",
             "## Exhaustive tile sweeps", "",
             "Every tile of `iolb_enumerate` (whole domain; the %d evenly spaced in the tuner's order when there are more) timed with"
             % MAX_TILES,
             "`python -m paper_2012_15667_amd.sweep --layer <layer> --algo <algo> --max %d`.  *pick* = `iolb_tune` (modelled time," % MAX_TILES,
             "this build's heuristic); *bound-only* = `iolb_tune_bound` (least reading volume inside the optimality box of Table 1).",
             "Tiles are b,x,y,z,alpha,threads.  For Winograd the fused blocks are part of the domain.", "",
             "| layer | algo | tiles timed | fastest tile | ms | pick | ms | rank | pick / fastest | bound-only | ms | rank | bound-only / fastest |",
             "|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    for layer, algo in SWEEPS:
        with contextlib.redirect_stdout(io.StringIO()):
            r = sweep(layer, algo, MAX_TILES)
        lines.append("| %s | %s | %d | %s | %.4f | %s | %.4f | %d | %.3f | %s | %.4f | %d | %.3f |" % (
            layer, algo, r["tiles_timed"], tile_text(r["best_tile"]), r["best_ms"], tile_text(r["pick"]), r["pick_ms"], r["pick_rank"],
            r["pick_over_best"], tile_text(r["bound_pick"]), r["bound_pick_ms"], r["bound_pick_rank"], r["bound_pick_over_best"]))
        print("swept %s %s" % (layer, algo), flush=True)
    lines += ["", "## Measured search with and without the optimality box (Sec. 6.2)", "",
              "`python -m paper_2012_15667_amd.autotune --layer <layer> --algo direct [--no-box] --seed <s>`: random starts only (the",
              "analytical pick is not given to the search), n_s = 8 walks, patience 4; two seeds each.  *domain* counts tiles with",
              "every stage depth.  *to 3 %* = measurements made when the best time was first within 3 % of the search's final best.", "",
              "| layer | search | domain | share of whole domain | seed | measurements | to 3 % | best ms | tuner pick ms |",
              "|---|---|---|---|---|---|---|---|---|"]
    for layer, algo in ENGINE_LAYERS:
        for use_box in (True, False):
            shape, pick, dom, measure = gpu_domain_and_measure(layer, algo, use_box)
            full = with_stage_depths(B.iolb_enumerate(shape, 163840, 0, False), 4, shape.C)
            measure(pick)                      # first call of a process warms the clocks
            pick_ms = measure(pick)
            for seed in (0, 1):
                best, best_ms, history = autotune(dom, measure, 8, 4, seed=seed)
                to3 = next(n for n, t in history if t <= best_ms * 1.03)
                lines.append("| %s | %s | %d | %.1f %% | %d | %d | %d | %.4f | %.4f |" % (
                    layer, "box" if use_box else "whole domain", len(dom), 100.0 * len(dom) / max(1, len(full)), seed,
                    history[-1][0], to3, best_ms, pick_ms))
            print("searched %s %s box=%s" % (layer, algo, use_box), flush=True)
    import torch
    from .inputs import layer_inputs
    from .sweep import parse_layer, time_call
    lines += ["", "## Fused against unfused Winograd", "",
              "The first fused block and the first unfused tile of the enumeration (the tuner's order inside each path), five calls",
              "after two warm-up calls each.  Layers are configured names or N,C,H,W,K,R,S,stride,pad.", "",
              "| layer | F(m x m) | fused ms | unfused ms | unfused / fused | tuner picks | the faster one |",
              "|---|---|---|---|---|---|---|"]
    right = total = 0
    for name in CROSSOVER:
        L = parse_layer(name)
        x, w = layer_inputs(L)
        xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        y = torch.empty((L.N, L.K, L.H, L.W), dtype=torch.float32, device="cuda")
        for m in (2, 4):
            shape = B.make_shape(L.N, L.C, L.H, L.W, L.K, algo=B.WINO_ALGO[m])
            tiles = B.iolb_enumerate(shape, 0, 0, False)
            fused = [t for t in tiles if t["path"] == B.PATH_FUSED]
            unfused = [t for t in tiles if t["path"] == B.PATH_MFMA]
            if not fused or not unfused:
                continue
            ws = torch.empty(B.winograd_workspace_bytes(L.N, L.C, L.H, L.W, L.K, m), dtype=torch.uint8, device="cuda")
            ms = {}
            for label, t in (("fused", fused[0]), ("unfused", unfused[0])):
                ms[label] = time_call(torch, lambda: B.conv_winograd(xd, wd, m, y=y, cfg=t, workspace=ws), 5)
            pick = {B.PATH_FUSED: "fused", B.PATH_MFMA: "unfused", B.PATH_FMA: "thin-layer kernel"}[B.iolb_tune(shape)["path"]]
            faster = min(ms, key=ms.get)
            total += 1
            right += pick == faster
            lines.append("| %s | %d | %.4f | %.4f | %.2f | %s | %s |" % (name, m, ms["fused"], ms["unfused"], ms["unfused"] / ms["fused"], pick, faster))
        print("compared " + name, flush=True)
    lines += ["", "The tuner's choice is the faster path on %d of %d rows." % (right, total)]
    with open(os.path.join(ROOT, "profiles", "tuner_vs_sweep.md"), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote profiles/tuner_vs_sweep.md")


if __name__ == "__main__":
    main()
    sys.exit(0)
