"""Layer sets for the widening experiments of Sec. 7: the convolution layers of whole networks and the
shape sweeps of the two direct-convolution figures, as synthetic layers (shapes only; random inputs).

  * MODELS: the distinct convolution shapes of VGG-19, ResNet-18/34, SqueezeNet 1.0 and Inception-v3 (the
    networks of the end-to-end experiment of Sec. 7.3), each with the number of times the network runs it,
    written down from the architectures' published descriptions.  Layers that pad one axis only (the
    1x7 / 7x1 / 1x3 / 3x1 factorised kernels of Inception-v3) carry a (pad_h, pad_w) pair and run through
    conv_direct_pad2.
  * figure_sweep(): 3x3 kernels with C_in = 256 over input extents, output channels and strides (the sweep
    of the first figure of Sec. 7.1);
  * batch_sweep(): the same family at C_out = 256, stride 1, over batch sizes (the batched test of Sec. 7.1).

    python -m paper_2012_15667_amd.layersets --model vgg19 --batch 64
    python -m paper_2012_15667_amd.layersets --batch-sweep
    python -m paper_2012_15667_amd.layersets --figure-sweep --batch 32

Each line of output is one JSON record: the layer, the time and direct-equivalent TFLOP/s of every algorithm
that applies (direct always; Winograd F(2x2), F(4x4) for 3x3 stride-1 layers), and the fastest.  A final
record sums a network: time per image batch with the best algorithm per layer and with direct convolution
only.
"""
import argparse
import json
import sys
from collections import namedtuple

Conv = namedtuple("Conv", "name C H W K R S stride pad count")


def _c(name, C, HW, K, R, stride, pad, count=1):
    return Conv(name, C, HW, HW, K, R, R, stride, pad, count)


def _r(name, C, HW, K, R, S, count=1):
    """R x S kernel, stride 1, padded to keep the extents: pad = ((R-1)/2, (S-1)/2), one axis only for 1 x n."""
    return Conv(name, C, HW, HW, K, R, S, 1, ((R - 1) // 2, (S - 1) // 2), count)


def _inception_17(c, tag, times=1):
    """One InceptionC module at 17 x 17 with c channels in its 7-tap branches."""
    return [_c("mixed6%s_1x1_c" % tag, 768, 17, c, 1, 1, 0, 2 * times),
            _r("mixed6%s_1x7" % tag, c, 17, c, 1, 7, 2 * times), _r("mixed6%s_7x1" % tag, c, 17, c, 7, 1, 2 * times),
            _r("mixed6%s_7x1_out" % tag, c, 17, 192, 7, 1, times), _r("mixed6%s_1x7_out" % tag, c, 17, 192, 1, 7, times)]


MODELS = {
    # 16 convolutions, all 3x3 / stride 1 / pad 1
    "vgg19": [
        _c("conv1_1", 3, 224, 64, 3, 1, 1), _c("conv1_2", 64, 224, 64, 3, 1, 1),
        _c("conv2_1", 64, 112, 128, 3, 1, 1), _c("conv2_2", 128, 112, 128, 3, 1, 1),
        _c("conv3_1", 128, 56, 256, 3, 1, 1), _c("conv3_x", 256, 56, 256, 3, 1, 1, 3),
        _c("conv4_1", 256, 28, 512, 3, 1, 1), _c("conv4_x", 512, 28, 512, 3, 1, 1, 3),
        _c("conv5_x", 512, 14, 512, 3, 1, 1, 4),
    ],
    # basic blocks [2, 2, 2, 2]; the 1x1 stride-2 layers are the projection shortcuts
    "resnet18": [
        _c("conv1", 3, 224, 64, 7, 2, 3),
        _c("layer1", 64, 56, 64, 3, 1, 1, 4),
        _c("layer2_down", 64, 56, 128, 3, 2, 1), _c("layer2_proj", 64, 56, 128, 1, 2, 0), _c("layer2", 128, 28, 128, 3, 1, 1, 3),
        _c("layer3_down", 128, 28, 256, 3, 2, 1), _c("layer3_proj", 128, 28, 256, 1, 2, 0), _c("layer3", 256, 14, 256, 3, 1, 1, 3),
        _c("layer4_down", 256, 14, 512, 3, 2, 1), _c("layer4_proj", 256, 14, 512, 1, 2, 0), _c("layer4", 512, 7, 512, 3, 1, 1, 3),
    ],
    # basic blocks [3, 4, 6, 3]: the same shapes, run more often
    "resnet34": [
        _c("conv1", 3, 224, 64, 7, 2, 3),
        _c("layer1", 64, 56, 64, 3, 1, 1, 6),
        _c("layer2_down", 64, 56, 128, 3, 2, 1), _c("layer2_proj", 64, 56, 128, 1, 2, 0), _c("layer2", 128, 28, 128, 3, 1, 1, 7),
        _c("layer3_down", 128, 28, 256, 3, 2, 1), _c("layer3_proj", 128, 28, 256, 1, 2, 0), _c("layer3", 256, 14, 256, 3, 1, 1, 11),
        _c("layer4_down", 256, 14, 512, 3, 2, 1), _c("layer4_proj", 256, 14, 512, 1, 2, 0), _c("layer4", 512, 7, 512, 3, 1, 1, 5),
    ],
    # fire module = squeeze 1x1, then expand 1x1 and expand 3x3 side by side
    "squeezenet": [
        _c("conv1", 3, 227, 96, 7, 2, 0),
        _c("fire2_s", 96, 55, 16, 1, 1, 0), _c("fire2_e1", 16, 55, 64, 1, 1, 0, 2), _c("fire2_e3", 16, 55, 64, 3, 1, 1, 2),
        _c("fire3_s", 128, 55, 16, 1, 1, 0), _c("fire4_s", 128, 55, 32, 1, 1, 0),
        _c("fire4_e1", 32, 55, 128, 1, 1, 0), _c("fire4_e3", 32, 55, 128, 3, 1, 1),
        _c("fire5_s", 256, 27, 32, 1, 1, 0), _c("fire5_e1", 32, 27, 128, 1, 1, 0), _c("fire5_e3", 32, 27, 128, 3, 1, 1),
        _c("fire6_s", 256, 27, 48, 1, 1, 0), _c("fire6_e1", 48, 27, 192, 1, 1, 0, 2), _c("fire6_e3", 48, 27, 192, 3, 1, 1, 2),
        _c("fire7_s", 384, 27, 48, 1, 1, 0), _c("fire8_s", 384, 27, 64, 1, 1, 0),
        _c("fire8_e1", 64, 27, 256, 1, 1, 0), _c("fire8_e3", 64, 27, 256, 3, 1, 1),
        _c("fire9_s", 512, 13, 64, 1, 1, 0), _c("fire9_e1", 64, 13, 256, 1, 1, 0), _c("fire9_e3", 64, 13, 256, 3, 1, 1),
        _c("conv10", 512, 13, 1000, 1, 1, 0),
    ],
    # stem, the 35 x 35 stage, the 17 x 17 stage with its factorised 7-tap kernels, the 8 x 8 stage
    "inception_v3": [
        _c("stem_1", 3, 299, 32, 3, 2, 0), _c("stem_2", 32, 149, 32, 3, 1, 0), _c("stem_3", 32, 147, 64, 3, 1, 1),
        _c("stem_4", 64, 73, 80, 1, 1, 0), _c("stem_5", 80, 73, 192, 3, 1, 0),
        _c("mixed5b_1x1", 192, 35, 64, 1, 1, 0, 2), _c("mixed5b_1x1_48", 192, 35, 48, 1, 1, 0), _c("mixed5b_pool", 192, 35, 32, 1, 1, 0),
        _c("mixed5_5x5", 48, 35, 64, 5, 1, 2, 3), _c("mixed5_3x3a", 64, 35, 96, 3, 1, 1, 3), _c("mixed5_3x3b", 96, 35, 96, 3, 1, 1, 3),
        _c("mixed5c_1x1", 256, 35, 64, 1, 1, 0, 3), _c("mixed5c_1x1_48", 256, 35, 48, 1, 1, 0),
        _c("mixed5d_1x1", 288, 35, 64, 1, 1, 0, 3), _c("mixed5d_1x1_48", 288, 35, 48, 1, 1, 0),
        _c("mixed6a_3x3", 288, 35, 384, 3, 2, 0), _c("mixed6a_3x3b", 96, 35, 96, 3, 2, 0),
        _c("mixed6a_1x1", 288, 35, 64, 1, 1, 0), _c("mixed6a_3x3a", 64, 35, 96, 3, 1, 1),
        # 17 x 17: four modules (7-tap branches of 128, 160, 160, 192 channels); 1x1 to 192: twice per module
        _c("mixed6_1x1_192", 768, 17, 192, 1, 1, 0, 8),
    ] + _inception_17(128, "b") + _inception_17(160, "cd", 2) + _inception_17(192, "e") + [
        # reduction to 8 x 8
        _c("mixed7a_1x1", 768, 17, 192, 1, 1, 0, 2), _c("mixed7a_3x3", 192, 17, 320, 3, 2, 0),
        _r("mixed7a_1x7", 192, 17, 192, 1, 7), _r("mixed7a_7x1", 192, 17, 192, 7, 1), _c("mixed7a_3x3b", 192, 17, 192, 3, 2, 0),
        # 8 x 8: two modules, 1280 and 2048 input channels
        _c("mixed7b_1x1_320", 1280, 8, 320, 1, 1, 0), _c("mixed7b_1x1_384", 1280, 8, 384, 1, 1, 0),
        _c("mixed7b_1x1_448", 1280, 8, 448, 1, 1, 0), _c("mixed7b_1x1_192", 1280, 8, 192, 1, 1, 0),
        _c("mixed7c_1x1_320", 2048, 8, 320, 1, 1, 0), _c("mixed7c_1x1_384", 2048, 8, 384, 1, 1, 0),
        _c("mixed7c_1x1_448", 2048, 8, 448, 1, 1, 0), _c("mixed7c_1x1_192", 2048, 8, 192, 1, 1, 0),
        _r("mixed7_1x3", 384, 8, 384, 1, 3, 4), _r("mixed7_3x1", 384, 8, 384, 3, 1, 4), _c("mixed7_3x3", 448, 8, 384, 3, 1, 1, 2),
    ],
}
SKIPPED = {}


def figure_sweep():
    """3x3, C_in = 256: H_in = W_in in {14, 28, 56, 112}, C_out in {64, 128, 256, 512}, stride in {1, 2}."""
    return [Conv("hw%d_k%d_s%d" % (hw, k, st), 256, hw, hw, k, 3, 3, st, 1, 1)
            for hw in (14, 28, 56, 112) for k in (64, 128, 256, 512) for st in (1, 2)]


def batch_sweep():
    """(batch, layer) pairs: 3x3, C_in = C_out = 256, stride 1, batch 1...128 at four input extents."""
    return [(n, Conv("hw%d_n%d" % (hw, n), 256, hw, hw, 256, 3, 3, 1, 1, 1))
            for hw in (14, 28, 56, 112) for n in (1, 2, 4, 8, 16, 32, 64, 128)]


def pads(L):
    """(pad_h, pad_w) of a layer: its pad is one number for both axes or a pair."""
    return tuple(L.pad) if isinstance(L.pad, (tuple, list)) else (L.pad, L.pad)


def out_extents(L):
    ph, pw = pads(L)
    return (L.H + 2 * ph - L.R) // L.stride + 1, (L.W + 2 * pw - L.S) // L.stride + 1


def flops(N, L):
    P, Q = out_extents(L)
    return 2.0 * N * L.K * P * Q * L.C * L.R * L.S


def winograd_applies(L):
    return L.R == 3 and L.S == 3 and L.stride == 1 and not isinstance(L.pad, (tuple, list))


def time_layer(N, L, reps=5, seed=0):
    """Times every applicable algorithm on the GPU; returns {algo: ms}."""
    import torch
    from . import binding as B
    from .sweep import time_call
    g = torch.Generator(device="cuda").manual_seed(seed)
    x = torch.rand((N, L.C, L.H, L.W), generator=g, device="cuda", dtype=torch.float32)
    w = torch.randn((L.K, L.C, L.R, L.S), generator=g, device="cuda", dtype=torch.float32) * (2.0 / (L.R * L.S * L.C)) ** 0.5
    P, Q = out_extents(L)
    y = torch.empty((N, L.K, P, Q), device="cuda", dtype=torch.float32)
    def timed(fn):
        # short layers are timed over more calls: about two milliseconds of work, at least `reps` calls
        first = time_call(torch, fn, 3)
        return time_call(torch, fn, max(reps, min(100, int(2.0 / max(first, 1e-3)))), warmup=0)
    out = {"direct": timed(lambda: B.conv_direct(x, w, L.stride, L.pad, y=y))}
    if winograd_applies(L):
        for m in (2, 4):
            out["wino%d" % m] = timed(lambda m=m: B.conv_winograd(x, w, m, y=y, pad=L.pad))
    return out


def run(pairs, reps=5, out=sys.stdout):
    """pairs: iterable of (batch, Conv).  Prints one record per layer; returns the records."""
    records = []
    for N, L in pairs:
        ms = time_layer(N, L, reps)
        f = flops(N, L)
        best = min(ms, key=ms.get)
        rec = {"layer": L.name, "N": N, "C": L.C, "H": L.H, "W": L.W, "K": L.K, "R": L.R, "S": L.S,
               "stride": L.stride, "pad": list(pads(L)) if isinstance(L.pad, (tuple, list)) else L.pad, "count": L.count, "gflop": round(f / 1e9, 3),
               "ms": {a: round(t, 4) for a, t in ms.items()},
               "tflops_direct_equiv": {a: round(f / t / 1e9, 2) for a, t in ms.items()}, "best": best}
        records.append(rec)
        print(json.dumps(rec), file=out, flush=True)
    return records


def summarise(name, records):
    total_f = sum(r["gflop"] * r["count"] for r in records)
    t_best = sum(min(r["ms"].values()) * r["count"] for r in records)
    t_direct = sum(r["ms"]["direct"] * r["count"] for r in records)
    return {"model": name, "conv_layers": sum(r["count"] for r in records), "gflop": round(total_f, 2),
            "ms_best_per_layer": round(t_best, 3), "tflops_best": round(total_f / t_best, 2),
            "ms_direct_only": round(t_direct, 3), "tflops_direct_only": round(total_f / t_direct, 2),
            "skipped": SKIPPED.get(name, "")}


def report(path, reps=5):
    """Runs the three measurements and writes the summary (the tracked profiles/layer_sets.md)."""
    import io
    quiet = io.StringIO()
    w = []
    w.append("# Layer sets on one MI355X: whole networks' convolution layers, batch sweep, figure sweep\n")
    w.append("Written by `python -m paper_2012_15667_amd.layersets --report profiles/layer_sets.md` (run from the repository root")
    w.append("on the GPU box).  Timed with `torch.cuda.Event` around at least %d calls (about 2 ms of work for short layers) after warm-up calls, inputs resident in HBM, fp32;" % reps)
    w.append("TFLOP/s are direct-convolution-equivalent (2 N K P Q C R S / time); every call goes through the tuned tile.\n")
    w.append("## Networks (batch 64; distinct convolution shapes x how often the network runs them)\n")
    w.append("| network | conv layers | GFLOP | best algorithm per layer: ms / TFLOP/s | direct only: ms / TFLOP/s |")
    w.append("|---|---|---|---|---|")
    per_model = {}
    for name in sorted(MODELS):
        per_model[name] = run([(64, L) for L in MODELS[name]], reps, quiet)
        r = summarise(name, per_model[name])
        w.append("| %s | %d | %.1f | %.2f / %.1f | %.2f / %.1f |" % (r["model"], r["conv_layers"], r["gflop"], r["ms_best_per_layer"],
                                                               r["tflops_best"], r["ms_direct_only"], r["tflops_direct_only"]))
        print("timed " + name, flush=True)
    w.append("\nInception-v3: all 94 convolutions of the main path; the factorised 1x7 / 7x1 / 1x3 / 3x1 kernels pad one axis only "
             "(pad shown as h,w) and run through conv_direct_pad2; pad-0 3x3 layers reach Winograd through conv_winograd_pad.")
    ones = [q for recs in per_model.values() for q in recs if q["R"] == 1 and q["S"] == 1 and q["stride"] == 1 and q["gflop"] >= 1.0]
    tf = sorted(q["tflops_direct_equiv"]["direct"] for q in ones)
    w.append("\n1 x 1, stride-1 layers of at least 1 GFLOP (%d shapes): %.1f / %.1f / %.1f TFLOP/s lowest / median / highest; "
             "%d of them at 60 TFLOP/s or more." % (len(tf), tf[0], tf[len(tf) // 2], tf[-1], sum(1 for v in tf if v >= 60.0)))
    w.append("\nPer layer (ms; TFLOP/s in brackets):\n")
    w.append("| network | layer | C | H=W | K | RxS/stride/pad | count | GFLOP | direct | F(2x2) | F(4x4) |")
    w.append("|---|---|---|---|---|---|---|---|---|---|---|")
    for name in sorted(MODELS):
        for q in per_model[name]:
            f = lambda a: ("%.3f (%.0f)" % (q["ms"][a], q["tflops_direct_equiv"][a])) if a in q["ms"] else "-"
            pad = q["pad"] if not isinstance(q["pad"], list) else "%d,%d" % tuple(q["pad"])
            w.append("| %s | %s | %d | %d | %d | %dx%d/%d/%s | %d | %.2f | %s | %s | %s |" % (
                name, q["layer"], q["C"], q["H"], q["K"], q["R"], q["S"], q["stride"], pad, q["count"], q["gflop"],
                f("direct"), f("wino2"), f("wino4")))
    b = run(batch_sweep(), reps, quiet)
    print("timed the batch sweep", flush=True)
    ns = (1, 2, 4, 8, 16, 32, 64, 128)
    w.append("\n## Batch sweep (3x3, C = K = 256, stride 1, pad 1): TFLOP/s of the fastest algorithm, and of direct convolution\n")
    w.append("| H=W | " + " | ".join("N=%d" % n for n in ns) + " |")
    w.append("|---|" + "---|" * len(ns))
    for hw in (14, 28, 56, 112):
        row = [r for r in b if r["H"] == hw]
        w.append("| %d | " % hw + " | ".join("%.0f %s (direct %.0f)" % (max(r["tflops_direct_equiv"].values()), r["best"],
                                                                       r["tflops_direct_equiv"]["direct"]) for r in row) + " |")
    fg = run([(32, L) for L in figure_sweep()], reps, quiet)
    print("timed the figure sweep", flush=True)
    w.append("\n## Figure sweep (3x3, C = 256, batch 32): direct convolution TFLOP/s, stride 1 / stride 2; best Winograd at stride 1 in brackets\n")
    w.append("| H=W | K=64 | K=128 | K=256 | K=512 |")
    w.append("|---|---|---|---|---|")
    for hw in (14, 28, 56, 112):
        cells = []
        for k in (64, 128, 256, 512):
            s1 = [r for r in fg if r["H"] == hw and r["K"] == k and r["stride"] == 1][0]
            s2 = [r for r in fg if r["H"] == hw and r["K"] == k and r["stride"] == 2][0]
            wbest = max(v for a, v in s1["tflops_direct_equiv"].items() if a != "direct")
            cells.append("%.0f / %.0f (%.0f)" % (s1["tflops_direct_equiv"]["direct"], s2["tflops_direct_equiv"]["direct"], wbest))
        w.append("| %d | " % hw + " | ".join(cells) + " |")
    with open(path, "w") as f:
        f.write("\n".join(w) + "\n")
    print("wrote " + path)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--report", default="", help="run everything and write the markdown summary to this path")
    ap.add_argument("--model", default="", help="one of %s, or 'all'" % ", ".join(sorted(MODELS)))
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--batch-sweep", action="store_true")
    ap.add_argument("--figure-sweep", action="store_true")
    ap.add_argument("--reps", type=int, default=5)
    a = ap.parse_args()
    if a.report:
        report(a.report, a.reps)
        return 0
    if a.batch_sweep:
        run(batch_sweep(), a.reps)
    if a.figure_sweep:
        run([(a.batch, L) for L in figure_sweep()], a.reps)
    names = sorted(MODELS) if a.model == "all" else ([a.model] if a.model else [])
    for name in names:
        recs = run([(a.batch, L) for L in MODELS[name]], a.reps)
        print(json.dumps(summarise(name, recs)), flush=True)


if __name__ == "__main__":
    sys.exit(main())
