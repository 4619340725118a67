"""Measured auto-tuning engine over the tile domain (the engine of Sec. 6 of the paper, on this library).

Three parts, as in Sec. 6.1:
  * template manager  -- the kernels are the templates; `domain()` lists every configuration
    (`iolb_enumerate`, optionally only those inside the optimality-condition box of Sec. 6.2, plus
    shallower stage depths), and `measure()` runs one configuration on the GPU and times it;
  * cost model        -- gradient tree boosting on (configuration features -> log time), refitted as
    measurements accumulate (scikit-learn's GradientBoostingRegressor stands in for XGBoost);
  * configuration explorer -- n_s random walks over neighbouring configurations that drift towards a
    lower predicted cost; their end points are measured next (Sec. 6.2, "Searching Process").
The loop model training -> configuration searching -> dataset updating (Sec. 6.3) stops when the best
measured time has not improved for `patience` iterations.

    python -m paper_2012_15667_amd.autotune --layer alex3 --algo direct [--no-box] [--layouts]

With --layouts the tensor layout (CHW or HWC, Table 1) is one more parameter of the domain: every tile is
a candidate in both layouts and the engine reports which layout its best configuration uses.
"""
import argparse
import json
import math
import random
import sys

FEATURES = ("b", "x", "y", "z", "alpha", "threads", "waves_m", "waves_n", "lds_bytes_used",
            "acc_regs_per_thread", "q_read_elems")


def features(cfg):
    """Numeric description of a configuration for the cost model (logs of the integer fields)."""
    return [math.log2(max(1, cfg[k])) for k in FEATURES] + [math.log2(max(1, cfg["b"] * cfg["x"] * cfg["y"])),
                                                            float(cfg.get("layout", 0))]


def stage_depth_variant(t, a, C=None):
    """Tile t with the shallower stage depth a.  On the matrix-core path a tile whose single stage holds all
    C channels counts one LDS buffer; with a < C there are several stages and two buffers."""
    v = dict(t)
    buffers = 2 if C is not None and t["path"] == 1 and t["alpha"] >= C > a else 1
    v["lds_bytes_used"] = t["lds_bytes_used"] // t["alpha"] * a * buffers
    v["alpha"] = a
    return v


def with_stage_depths(tiles, min_alpha=4, C=None):
    """Each tile also with every shallower stage depth alpha/2, alpha/4, ... >= min_alpha (C: the layer's
    input channels, needed for the LDS figure of single-stage tiles)."""
    out = []
    for t in tiles:
        a = t["alpha"]
        if t["path"] not in (0, 1):          # the depths of the fused and 1 x 1 kernels are enumerated one by one
            out.append(t)
            continue
        while a >= min_alpha:
            out.append(stage_depth_variant(t, a, C))
            a //= 2
    return out


def with_layouts(tiles):
    """Each configuration in both tensor layouts (0: channels outermost, 1: channels innermost)."""
    # (the tiles of the 1 x 1 kernel and of the thin-layer kernel exist for channels-outermost tensors only)
    chw_only = lambda t: t["path"] == 3 or (t["path"] == 0 and t["wt_mode"] == 2)
    return [dict(t, layout=l) for t in tiles for l in (0, 1) if l == 0 or not chw_only(t)]


PARAMS = ("b", "x", "y", "z", "alpha", "layout")


def _params(cfg):
    return tuple(cfg.get(p, 0) for p in PARAMS)


def _key(cfg):
    return tuple(cfg[k] for k in ("b", "x", "y", "z", "alpha", "threads", "waves_m", "waves_n", "path")) + \
        (cfg.get("layout", 0),)


def neighbours(index, cfg):
    """Configurations of the domain that differ from cfg in ONE of (b, x, y, z, alpha, layout) by one
    step of that parameter's sorted value list.  `index` maps parameter tuples to domain entries."""
    out = []
    cur = _params(cfg)
    for i, p in enumerate(PARAMS):
        values = index["values"][p]
        j = values.index(cur[i])
        for jj in (j - 1, j + 1):
            if 0 <= jj < len(values):
                cand = list(cur)
                cand[i] = values[jj]
                hit = index["by_params"].get(tuple(cand))
                if hit is not None:
                    out.append(hit)
    return out


def build_index(dom):
    return {"values": {p: sorted({c.get(p, 0) for c in dom}) for p in PARAMS},
            "by_params": {_params(c): c for c in dom}}


class CostModel:
    """Gradient tree boosting on log time; before enough data exists it predicts a constant."""

    def __init__(self, min_points=8, seed=0):
        self.min_points = min_points
        self.seed = seed
        self.model = None
        self.default = 0.0

    def fit(self, cfgs, times):
        if not cfgs:
            return
        logs = [math.log(t) for t in times]
        self.default = sum(logs) / len(logs)
        if len(cfgs) < self.min_points:
            self.model = None
            return
        from sklearn.ensemble import GradientBoostingRegressor
        self.model = GradientBoostingRegressor(n_estimators=120, max_depth=3, learning_rate=0.1,
                                               subsample=1.0, random_state=self.seed)
        self.model.fit([features(c) for c in cfgs], logs)

    def predict(self, cfgs):
        if self.model is None:
            return [self.default] * len(cfgs)
        return list(self.model.predict([features(c) for c in cfgs]))


def explore(dom, index, model, measured, n_s, rng, walk_steps=16):
    """n_s random walks from random starts; each step looks at the neighbours and moves to a better
    predicted one (or, with small probability, to any neighbour).  Returns unmeasured end points."""
    picks = []
    seen = set()
    for _ in range(n_s):
        cur = rng.choice(dom)
        cur_cost = model.predict([cur])[0]
        for _ in range(walk_steps):
            nb = neighbours(index, cur)
            if not nb:
                break
            costs = model.predict(nb)
            best = min(range(len(nb)), key=lambda i: costs[i])
            if costs[best] < cur_cost or rng.random() < 0.1:
                j = best if costs[best] < cur_cost else rng.randrange(len(nb))
                cur, cur_cost = nb[j], costs[j]
            else:
                break
        k = _key(cur)
        if k not in measured and k not in seen:
            seen.add(k)
            picks.append(cur)
    # walks that ended on known ground are replaced by the best-predicted unmeasured configurations
    if len(picks) < n_s:
        rest = [c for c in dom if _key(c) not in measured and _key(c) not in seen]
        if rest:
            costs = model.predict(rest)
            order = sorted(range(len(rest)), key=lambda i: costs[i])
            for i in order[:n_s - len(picks)]:
                picks.append(rest[i])
    return picks


def autotune(dom, measure, n_s=8, patience=4, max_iterations=40, seed=0, seeds=()):
    """The tuning loop.  dom: list of configurations; measure(cfg) -> time; seeds: configurations to
    measure first (e.g. the analytical pick).  Returns (best_cfg, best_time, history) where history
    lists (measurement count, best time so far) after every iteration."""
    rng = random.Random(seed)
    index = build_index(dom)
    model = CostModel(seed=seed)
    measured = {}
    order = []

    def run(cfg):
        k = _key(cfg)
        if k not in measured:
            measured[k] = (cfg, measure(cfg))
            order.append(k)

    for c in seeds:
        run(c)
    for c in rng.sample(dom, min(n_s, len(dom))):
        run(c)
    history = []
    best = min(measured.values(), key=lambda ct: ct[1])
    history.append((len(measured), best[1]))
    stale = 0
    for _ in range(max_iterations):
        if len(measured) >= len(dom):
            break
        model.fit([measured[k][0] for k in order], [measured[k][1] for k in order])   # model training
        picks = explore(dom, index, model, measured, n_s, rng)                          # configuration searching
        if not picks:
            break
        for c in picks:                                                                # dataset updating
            run(c)
        now = min(measured.values(), key=lambda ct: ct[1])
        stale = stale + 1 if now[1] >= best[1] * 0.995 else 0
        best = now if now[1] < best[1] else best
        history.append((len(measured), best[1]))
        if stale >= patience:
            break
    return best[0], best[1], history


# ---------------------------------------------------------------------------------------------
# GPU front end
# ---------------------------------------------------------------------------------------------

def gpu_domain_and_measure(layer_name, algo, use_box=True, reps=3, layouts=False):
    import torch
    from . import binding as B
    from .inputs import layer_inputs
    from .sweep import parse_layer, time_call

    L = parse_layer(layer_name)          # a configured name or N,C,H,W,K,R,S,stride,pad
    x, w = layer_inputs(L)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    algo_id = {"direct": B.DIRECT, "wino2": B.WINO_F2, "wino3": B.WINO_F3, "wino4": B.WINO_F4, "wino6": B.WINO_F6}[algo]
    shape = B.make_shape(L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad, algo_id)
    pick = B.iolb_tune(shape)
    tiles = B.iolb_enumerate(shape, 163840, 0, use_box)
    dom = with_stage_depths(tiles, 4 if tiles and tiles[0]["path"] == B.PATH_MFMA else 1, L.C)
    P = (L.H + 2 * L.pad - L.R) // L.stride + 1
    Q = (L.W + 2 * L.pad - L.S) // L.stride + 1
    y = torch.empty((L.N, L.K, P, Q), dtype=torch.float32, device="cuda")
    ws = None
    if algo != "direct":
        ws = torch.empty(B.winograd_workspace_bytes(L.N, L.C, L.H, L.W, L.K, int(algo[4:])),
                         dtype=torch.uint8, device="cuda")
    if layouts and algo == "direct":
        dom = with_layouts(dom)
        x_hwc = xd.permute(0, 2, 3, 1).contiguous()
        y_hwc = torch.empty((L.N, P, Q, L.K), dtype=torch.float32, device="cuda")

    def measure(cfg):
        if algo == "direct" and cfg.get("layout", 0) == 1:
            return time_call(torch, lambda: B.conv_direct_layout(x_hwc, wd, L.stride, L.pad, B.LAYOUT_HWC, y=y_hwc,
                                                                 cfg=cfg), reps)
        if algo == "direct":
            return time_call(torch, lambda: B.conv_direct(xd, wd, L.stride, L.pad, y=y, cfg=cfg), reps)
        return time_call(torch, lambda: B.conv_winograd(xd, wd, int(algo[4:]), y=y, cfg=cfg,
                                                        workspace=ws), reps)

    # the first launches after an idle period run at lower clocks: warm up on the analytical pick
    for _ in range(3):
        measure(dict(pick, layout=0))
    return shape, pick, dom, measure


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layer", default="alex3")
    ap.add_argument("--algo", default="direct")
    ap.add_argument("--no-box", action="store_true", help="search the whole domain, not only the optimality box")
    ap.add_argument("--layouts", action="store_true", help="the tensor layout (CHW / HWC) is part of the domain")
    ap.add_argument("--n-s", type=int, default=8)
    ap.add_argument("--patience", type=int, default=4)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--exhaustive", action="store_true", help="also time every configuration for comparison")
    a = ap.parse_args()
    from . import binding as B
    shape, pick, dom, measure = gpu_domain_and_measure(a.layer, a.algo, not a.no_box, layouts=a.layouts)
    full = with_stage_depths(B.iolb_enumerate(shape, 163840, 0, False), 4 if dom and dom[0]["path"] == 1 else 1, shape.C)
    seeds = [c for c in dom if all(c[k] == pick[k] for k in ("b", "x", "y", "z", "alpha"))]
    best, best_ms, history = autotune(dom, measure, a.n_s, a.patience, seed=a.seed, seeds=seeds)
    pick_ms = measure(pick) if not seeds else measure(seeds[0])
    out = {"layer": a.layer, "algo": a.algo, "domain": len(dom), "full_domain": len(full),
           "domain_share_pct": round(100.0 * len(dom) / max(1, len(full)), 2),
           "measurements": history[-1][0], "iterations": len(history) - 1,
           "best_ms": round(best_ms, 4), "analytical_pick_ms": round(pick_ms, 4),
           "best_over_pick": round(best_ms / pick_ms, 3), "best": best, "history": history}
    if a.exhaustive:
        times = sorted(measure(c) for c in dom)
        out["exhaustive_best_ms"] = round(times[0], 4)
    print(json.dumps(out))


if __name__ == "__main__":
    sys.exit(main())
