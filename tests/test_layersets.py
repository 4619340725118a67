"""The layer tables of paper_2012_15667_amd/layersets.py against figures known from the networks' published
descriptions (multiply-accumulate counts of the convolution layers) and against the tuner.  CPU only."""
import pytest

from paper_2012_15667_amd import binding as B
from paper_2012_15667_amd import layersets as LS


def _macs(model):
    return sum(LS.flops(1, L) / 2 * L.count for L in LS.MODELS[model])


@pytest.mark.parametrize("model,gmacs,layers", [("vgg19", 19.51, 16), ("resnet18", 1.813, 20), ("resnet34", 3.66, 36),
                                                 ("inception_v3", 5.71, 94)])
def test_convolution_work_matches_the_published_totals(model, gmacs, layers):
    assert _macs(model) / 1e9 == pytest.approx(gmacs, rel=0.01)
    assert sum(L.count for L in LS.MODELS[model]) == layers


def test_squeezenet_fire_modules_chain():
    by = {L.name: L for L in LS.MODELS["squeezenet"]}
    # expand outputs are concatenated: the next squeeze layer sees e1 + e3 channels
    assert by["fire3_s"].C == by["fire2_e1"].K + by["fire2_e3"].K
    assert by["fire5_s"].C == by["fire4_e1"].K + by["fire4_e3"].K
    assert by["fire7_s"].C == by["fire6_e1"].K + by["fire6_e3"].K
    assert by["fire9_s"].C == by["fire8_e1"].K + by["fire8_e3"].K
    assert LS.out_extents(by["conv1"]) == (111, 111)
    assert sum(L.count for L in LS.MODELS["squeezenet"]) == 26


@pytest.mark.parametrize("model", sorted(LS.MODELS))
def test_every_layer_has_a_tile(model):
    for L in LS.MODELS[model]:
        P, Q = LS.out_extents(L)
        assert P >= 1 and Q >= 1
        ph, pw = LS.pads(L)
        if ph == pw:
            cfg = B.iolb_tune(B.make_shape(8, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, ph))
        else:       # per-axis padding: the library tunes the layer whose image already holds the zero borders
            cfg = B.iolb_tune(B.make_shape(8, L.C, L.H + 2 * ph, L.W + 2 * pw, L.K, L.R, L.S, L.stride, 0))
        if cfg["path"] == B.PATH_POINT:     # 1 x 1 layers: a block of the image taken as one row of pixels
            assert (L.R, L.S, ph, pw) == (1, 1, 0, 0)
            assert cfg["x"] in (128, 256, 512) and cfg["y"] == 1 and cfg["b"] == 1 and cfg["z"] in (32, 64)
            continue
        if cfg["path"] == B.PATH_FMA and cfg["wt_mode"] == 2:     # thin 3 x 3 layers: 256 lanes of 1 or 4 pixels each
            assert (L.R, L.S, L.stride) == (3, 3, 1) and L.C <= 4
            assert cfg["x"] == (1024 if Q % 4 == 0 else 256) and cfg["y"] == 1 and cfg["z"] == L.K
            continue
        Kz = -(-L.K // 32) * 32 if cfg["path"] == B.PATH_MFMA else L.K
        # tile extents: factors of the output extent or a balanced cut into up to 8 tiles
        fits = lambda n, t: n % t == 0 or any(t == -(-n // k) for k in range(1, 9))
        assert cfg["x"] >= 1 and fits(Q, cfg["x"]) and fits(P, cfg["y"]) and Kz % cfg["z"] == 0
        if LS.winograd_applies(L):
            for m in (2, 4):
                B.iolb_tune(B.make_shape(8, L.C, L.H, L.W, L.K, 3, 3, 1, L.pad, algo=B.WINO_ALGO[m]))


def test_sweeps_have_the_stated_shapes():
    fig = LS.figure_sweep()
    assert len(fig) == 4 * 4 * 2 and all(L.C == 256 and L.R == 3 for L in fig)
    bs = LS.batch_sweep()
    assert len(bs) == 32 and {n for n, _ in bs} == {1, 2, 4, 8, 16, 32, 64, 128}


def test_inception_modules_chain_and_keep_their_extents():
    """The factorised kernels pad one axis only and keep 17 x 17 / 8 x 8; the concatenated branch outputs give
    the next stage's input channels (64 + 64 + 96 + 32 = 256, ..., 4 x 192 = 768, 320 + 192 + 768 = 1280)."""
    by = {L.name: L for L in LS.MODELS["inception_v3"]}
    for name, L in by.items():
        if L.R != L.S:
            assert LS.out_extents(L) == (L.H, L.W), name
            assert sorted(LS.pads(L)) == [0, (max(L.R, L.S) - 1) // 2], name
    assert by["mixed5c_1x1"].C == 64 + 64 + 96 + 32 and by["mixed5d_1x1"].C == 64 + 64 + 96 + 64
    assert by["mixed6_1x1_192"].C == 384 + 96 + 288 == 4 * 192
    assert by["mixed7b_1x1_320"].C == 320 + 192 + 768 and by["mixed7c_1x1_320"].C == 320 + 2 * 384 + 2 * 384 + 192
    assert LS.out_extents(by["mixed7a_3x3"]) == (8, 8) and LS.out_extents(by["mixed6a_3x3"]) == (17, 17)
