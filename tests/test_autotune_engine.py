"""The measured auto-tuning loop (model training -> configuration searching -> dataset updating) on a
synthetic cost function: no GPU.  The domain is a real one from the library's enumeration."""
import math

from paper_2012_15667_amd import autotune as A
from paper_2012_15667_amd import binding as B


def _domain():
    shape = B.make_shape(64, 256, 56, 56, 256)
    tiles = B.iolb_enumerate(shape, 163840, 0, True)
    return A.with_stage_depths(tiles, 4)


def _synthetic_ms(cfg):
    """A smooth stand-in for a kernel time: read volume, a penalty for small workgroups, a stage-depth term."""
    npix = cfg["b"] * cfg["x"] * cfg["y"]
    return (1.0 + cfg["q_read_elems"] / 4e8 + 256.0 / cfg["threads"] + 4.0 / cfg["alpha"]
            + abs(math.log2(npix / (9.0 * cfg["z"]))) * 0.2)


def test_stage_depth_variants():
    dom = _domain()
    assert all(c["alpha"] % 4 == 0 and c["alpha"] >= 4 for c in dom)
    keys = {A._key(c) for c in dom}
    assert len(keys) == len(dom)


def test_neighbours_differ_in_one_parameter():
    dom = _domain()
    idx = A.build_index(dom)
    c = dom[len(dom) // 2]
    nb = A.neighbours(idx, c)
    assert nb
    for n in nb:
        diff = [p for p in ("b", "x", "y", "z", "alpha") if n[p] != c[p]]
        assert len(diff) == 1
        assert A._key(n) in {A._key(d) for d in dom}


def test_search_finds_a_near_optimal_configuration_with_few_measurements():
    dom = _domain()
    calls = []

    def measure(cfg):
        calls.append(1)
        return _synthetic_ms(cfg)

    best, best_ms, history = A.autotune(dom, measure, n_s=8, patience=4, seed=1)
    true_best = min(_synthetic_ms(c) for c in dom)
    assert len(calls) == history[-1][0] <= len(dom) // 2          # far fewer measurements than the domain
    assert best_ms <= true_best * 1.03
    assert [h[1] for h in history] == sorted((h[1] for h in history), reverse=True)   # best-so-far never rises


def test_seeds_are_measured_first_and_never_lost():
    dom = _domain()
    seed_cfg = dom[0]
    best, best_ms, _ = A.autotune(dom, _synthetic_ms, n_s=4, patience=1, max_iterations=1, seed=2, seeds=[seed_cfg])
    assert best_ms <= _synthetic_ms(seed_cfg)


def test_layout_is_a_parameter_of_the_domain():
    """Table 1 lists the tensor layout among the tunables: with it in the domain, a neighbour step may flip
    the layout alone, and the search settles on the layout that the measurements favour."""
    dom = A.with_layouts(_domain())
    assert len({A._key(c) for c in dom}) == len(dom)
    idx = A.build_index(dom)
    c = dom[len(dom) // 2]
    flips = [n for n in A.neighbours(idx, c) if n["layout"] != c["layout"]]
    assert len(flips) == 1 and all(flips[0][p] == c[p] for p in ("b", "x", "y", "z", "alpha"))

    def measure(cfg):
        return _synthetic_ms(cfg) * (0.8 if cfg["layout"] == 1 else 1.0)

    best, best_ms, _ = A.autotune(dom, measure, n_s=8, patience=4, seed=3)
    assert best["layout"] == 1
    assert best_ms <= min(measure(c) for c in dom) * 1.03


def test_shallower_stage_of_a_single_stage_tile_counts_two_buffers():
    """lds_bytes_used of a matrix-core tile whose one stage holds all C channels is one buffer; the same tile
    with fewer channels per stage has several stages and two buffers -- the figure the library checks."""
    from paper_2012_15667_amd.autotune import stage_depth_variant, with_stage_depths
    t = dict(path=1, alpha=16, lds_bytes_used=4 * 16 * 100)
    assert stage_depth_variant(t, 16, 16)["lds_bytes_used"] == 6400
    assert stage_depth_variant(t, 8, 16)["lds_bytes_used"] == 2 * 4 * 8 * 100
    assert stage_depth_variant(t, 8, 64)["lds_bytes_used"] == 3200      # C = 64: several stages to begin with, the figure just scales
    assert [v["alpha"] for v in with_stage_depths([t], 4, 16)] == [16, 8, 4]
    f = dict(path=0, alpha=4, lds_bytes_used=400)
    assert stage_depth_variant(f, 2, 3)["lds_bytes_used"] == 200                    # FMA path: single-buffered throughout
