"""GPU parity: Tucker-2-decomposed convolution (1x1 -> kxk core -> 1x1) forward/backward with
freezing, and the undecomposed convolution, through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity import check, code, dev, empty, f32, host, seen, workspace
from paper_2309_03824_amd import binding as lrd

pytestmark = pytest.mark.gpu

SENT = 4321.25


def run_tucker(N, Hh, Ww, C, S, r1, r2, k, stride, pad, dt, mask, seed, save=True, want_dx=True, factors=None):
    rng = np.random.Generator(np.random.PCG64(seed))
    X = si.gaussian((N, Hh, Ww, C), rng)
    P1, G, P2 = si.direct_tucker_factors(S, C, k, r1, r2, rng) if factors is None else factors
    g = lrd.conv_geom(N, Hh, Ww, C, S, r1, r2, k, stride, pad)
    Ho, Wo = g.out_hw()
    dY = si.gaussian((N, Ho, Wo, S), rng)

    X_, P1_, G_, P2_, dY_ = dev(X, dt), dev(P1, dt), dev(G, dt), dev(P2, dt), dev(dY, dt)
    Y_ = empty((N, Ho, Wo, S), dt)
    A_ = empty((N, Hh, Ww, r1), dt) if save else None
    B_ = empty((N, Ho, Wo, r2), dt) if save else None
    ws = workspace(lrd.tucker_conv_workspace_bytes(g, code(dt), mask))
    lrd.tucker_conv_fwd(X_, P1_, G_, P2_, Y_, A_, B_, g, ws)
    gX = empty((N, Hh, Ww, C), dt) if want_dx else None
    g1, gG, g2 = f32((r1, C), SENT), f32((r2, k, k, r1), SENT), f32((S, r2), SENT)
    lrd.tucker_conv_bwd(dY_, X_, A_, B_, P1_, G_, P2_, gX, g1, gG, g2, mask, g, ws)
    torch.cuda.synchronize()

    Xo, P1o, Go, P2o, dYo = (seen(a, dt) for a in (X, P1, G, P2, dY))
    Ao, Bo, Yo = oracle.tucker_fwd(Xo, P1o, Go, P2o, stride, pad)
    check(host(Y_), Yo, dt, "Y")
    if save:
        check(host(A_), Ao, dt, "A")
        check(host(B_), Bo, dt, "B")
    go = oracle.tucker_bwd(dYo, Xo, Ao, Bo, P1o, Go, P2o, mask, stride, pad, want_dX=want_dx)
    if want_dx:
        check(host(gX), go["dX"], dt, "dX")
    for bit, (name, t) in enumerate((("dP1", g1), ("dG", gG), ("dP2", g2))):
        if mask & (1 << bit):
            assert torch.all(t == SENT), f"frozen {name} was written"
        else:
            check(host(t), go[name], dt, name)
    return dict(Y=Y_, dX=gX, dP1=g1, dG=gG, dP2=g2)


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_small_tucker_all_masks(dt):
    for mask in range(8):
        run_tucker(2, 9, 7, 24, 40, 8, 16, 3, 1, 1, dt, mask, seed=mask)


@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("geo", [
    (1, 12, 12, 16, 16, 5, 7, 3, 2, 1),      # stride 2, raw ranks
    (3, 8, 10, 32, 24, 16, 8, 1, 1, 0),      # 1x1 core
    (2, 11, 9, 20, 12, 12, 12, 5, 1, 2),     # 5x5 core
    (1, 7, 7, 8, 8, 8, 8, 3, 1, 0),          # no padding, full ranks
    (1, 3, 3, 4, 4, 2, 2, 3, 1, 1),          # image as small as the kernel
    (2, 11, 9, 24, 16, 16, 8, 5, 1, 2),      # 5x5 core, channel counts on the 16-byte path
    (1, 16, 16, 8, 16, 8, 8, 7, 2, 3),       # 7x7 stride 2 pad 3 (stem geometry), 16-byte path
    (1, 20, 20, 3, 16, 3, 8, 7, 2, 3),       # the same with 3 input channels
    (2, 13, 11, 16, 24, 8, 16, 3, 2, 1),     # stride 2 on odd image sizes (parity classes of unequal size)
    (1, 14, 15, 16, 16, 8, 8, 3, 3, 1),      # stride 3: one tap per class
    (2, 9, 10, 16, 16, 8, 8, 5, 2, 2),       # 5x5 stride 2: 3 or 2 taps per class and direction
    (1, 6, 5, 16, 16, 8, 8, 3, 2, 0),        # stride 2 without padding
])
def test_tucker_geometries(dt, geo):
    run_tucker(*geo, dt, 0, seed=sum(geo))
    run_tucker(*geo, dt, lrd.freeze_mask(lrd.KIND_TUCKER, 1), seed=sum(geo) + 1)


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_tucker_nullable_arguments(dt):
    run_tucker(2, 8, 8, 16, 16, 8, 8, 3, 1, 1, dt, 0, seed=1, save=False)
    run_tucker(2, 8, 8, 16, 16, 8, 8, 3, 1, 1, dt, 0b101, seed=2, save=False, want_dx=False)
    run_tucker(2, 8, 8, 16, 16, 8, 8, 3, 1, 1, dt, 0b010, seed=3, want_dx=False)


def test_resnet_stage_shapes_bf16():
    """The four 3x3 stage shapes (C = 64/128/256/512 at 56/28/14/7 pixels, ranks C/2 quantized to
    multiples of 32, stride 1 pad 1), two images each, core frozen (odd epoch of Algorithm 2) and
    the 1x1 layers frozen (even epoch); Tucker factors from an HOSVD of W ~ N(0, 1/(9C))."""
    from paper_2309_03824_amd import factorize
    for stage, (C, hw) in enumerate(((64, 56), (128, 28), (256, 14), (512, 7))):
        r = lrd.quantize_rank(C // 2, 32)
        assert r == C // 2
        W = si.conv_weight(C, C, 3, si.rng_for(4, stage))
        factors = factorize.tucker2_factors(W, r, r)
        for epoch in (1, 0):
            run_tucker(2, hw, hw, C, C, r, r, 3, 1, 1, "bf16", lrd.freeze_mask(lrd.KIND_TUCKER, epoch),
                       seed=50 + stage, factors=factors)


def test_strided_stage_transitions_bf16():
    """3x3 stride-2 layers between stages (C -> 2C, unequal ranks r1 = C/2, r2 = C), two images."""
    for C, hw in ((64, 28), (128, 14)):
        run_tucker(2, hw, hw, C, 2 * C, C // 2, C, 3, 2, 1, "bf16", lrd.freeze_mask(lrd.KIND_TUCKER, 1), seed=70 + C)
        run_tucker(2, hw, hw, C, 2 * C, C // 2, C, 3, 2, 1, "bf16", 0, seed=71 + C)


@pytest.mark.parametrize("geo", [
    (2, 13, 37, 48, 40, 32, 32, 3, 1, 1),    # ragged in both directions, two column tiles
    (1, 9, 33, 40, 72, 32, 64, 3, 1, 0),     # no padding, unequal ranks, one pixel past a column tile
    (2, 17, 31, 64, 64, 64, 32, 3, 1, 2),    # padding 2 (output larger than input)
    (1, 8, 32, 64, 64, 64, 64, 3, 1, 1),     # exactly one tile
    (3, 5, 70, 32, 32, 30, 30, 3, 1, 1),     # ranks padded to 32, three column tiles
])
def test_small_rank_core_geometries_bf16(geo):
    """3 x 3 stride-1 cores with ranks 32 / 64 (the early ResNet stages) take the patch-staging
    convolution kernel in forward and data gradient: tile edges, paddings 0..2, rank mixes."""
    run_tucker(*geo, "bf16", 0, seed=sum(geo))
    run_tucker(*geo, "bf16", lrd.freeze_mask(lrd.KIND_TUCKER, 1), seed=sum(geo) + 1, save=False)


def test_tucker_rank_cliff_shapes_bf16():
    """Ranks one off a tile boundary (the 257 -> 256 situation of Section 2.1) must stay correct."""
    for r in (31, 33, 65, 127):
        run_tucker(1, 14, 14, 160, 136, r, r, 3, 1, 1, "bf16", 0, seed=r)


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_dense_conv(dt):
    for (N, Hh, Ww, C, S, k, stride, pad) in ((2, 9, 7, 24, 40, 3, 1, 1), (1, 12, 12, 16, 8, 3, 2, 1),
                                              (2, 14, 14, 64, 64, 3, 1, 1), (1, 6, 6, 5, 3, 5, 1, 2),
                                              (2, 11, 35, 32, 64, 3, 1, 1)):
        rng = np.random.Generator(np.random.PCG64(N * 1000 + C))
        X, W = si.gaussian((N, Hh, Ww, C), rng), si.conv_weight(S, C, k, rng)
        g = lrd.conv_geom(N, Hh, Ww, C, S, 1, 1, k, stride, pad)
        Ho, Wo = g.out_hw()
        dY = si.gaussian((N, Ho, Wo, S), rng)
        X_, W_, dY_ = dev(X, dt), dev(W, dt), dev(dY, dt)
        Y_ = empty((N, Ho, Wo, S), dt)
        ws = workspace(lrd.dense_conv_workspace_bytes(g, code(dt)))
        lrd.dense_conv_fwd(X_, W_, Y_, g, ws)
        gX, gW = empty((N, Hh, Ww, C), dt), f32((S, k, k, C))
        lrd.dense_conv_bwd(dY_, X_, W_, gX, gW, g, ws)
        torch.cuda.synchronize()
        Xo, Wo_, dYo = seen(X, dt), seen(W, dt), seen(dY, dt)
        check(host(Y_), oracle.conv_fwd(Xo, Wo_, stride, pad), dt, "Y")
        check(host(gX), oracle.conv_dgrad(dYo, Wo_, (Hh, Ww), stride, pad), dt, "dX")
        check(host(gW), oracle.conv_wgrad(dYo, Xo, k, stride, pad), dt, "dW")


@pytest.mark.parametrize("C,hw", [(32, 56), (64, 28)])
def test_core_layer_full_size_sampled_bf16(C, hw):
    """The 3 x 3 core of the first two ResNet stages at full size (128 images, ranks 32 at 56 x 56 and
    64 at 28 x 28), where every workgroup of the patch-staging kernels walks over several tiles.  The
    oracle evaluates sampled images: their outputs and input gradients, and the weight gradient of an
    output gradient that is zero on all other images."""
    N, k = 128, 3
    picks = [0, 1, 17, 42, 63, 64, 100, 127]
    rng = si.rng_for(4, 900 + C)
    X = si.gaussian((N, hw, hw, C), rng).astype(np.float32)
    W = si.conv_weight(C, C, k, rng)
    dY = np.zeros((N, hw, hw, C), dtype=np.float32)
    dY[picks] = si.gaussian((len(picks), hw, hw, C), rng)
    g = lrd.conv_geom(N, hw, hw, C, C, 1, 1, k, 1, 1)
    X_, W_, dY_ = dev(X, "bf16"), dev(W, "bf16"), dev(dY, "bf16")
    Y_ = empty((N, hw, hw, C), "bf16")
    ws = workspace(lrd.dense_conv_workspace_bytes(g, code("bf16")))
    lrd.dense_conv_fwd(X_, W_, Y_, g, ws)
    gX, gW = empty((N, hw, hw, C), "bf16"), f32((C, k, k, C))
    lrd.dense_conv_bwd(dY_, X_, W_, gX, gW, g, ws)
    torch.cuda.synchronize()
    Xo, Wo_, dYo = seen(X[picks], "bf16"), seen(W, "bf16"), seen(dY[picks], "bf16")
    check(host(Y_[picks]), oracle.conv_fwd(Xo, Wo_, 1, 1), "bf16", "Y")
    check(host(gX[picks]), oracle.conv_dgrad(dYo, Wo_, (hw, hw), 1, 1), "bf16", "dX")
    check(host(gW), oracle.conv_wgrad(dYo, Xo, k, 1, 1), "bf16", "dW")
    rest = [n for n in range(N) if n not in picks]
    assert torch.all(gX[rest] == 0), "input gradient of an image whose output gradient is zero"


@pytest.mark.parametrize("C,hw", [(64, 56), (128, 28)])
def test_tucker_stage_full_size_sampled_bf16(C, hw):
    """A whole Tucker layer of the first two ResNet stages at full size (128 images, ranks C / 2), forward
    and backward with nothing frozen, as the layer tables time it.  The oracle evaluates sampled
    images: Y, A, B and dX of those, and the three weight gradients of an output gradient that is
    zero on every other image."""
    N, k, r = 128, 3, C // 2
    picks = [0, 5, 31, 64, 90, 127]
    rng = si.rng_for(4, 950 + C)
    X = si.gaussian((N, hw, hw, C), rng).astype(np.float32)
    P1, G, P2 = si.direct_tucker_factors(C, C, k, r, r, rng)
    dY = np.zeros((N, hw, hw, C), dtype=np.float32)
    dY[picks] = si.gaussian((len(picks), hw, hw, C), rng)
    g = lrd.conv_geom(N, hw, hw, C, C, r, r, k, 1, 1)
    X_, P1_, G_, P2_, dY_ = dev(X, "bf16"), dev(P1, "bf16"), dev(G, "bf16"), dev(P2, "bf16"), dev(dY, "bf16")
    Y_, A_, B_ = empty((N, hw, hw, C), "bf16"), empty((N, hw, hw, r), "bf16"), empty((N, hw, hw, r), "bf16")
    ws = workspace(lrd.tucker_conv_workspace_bytes(g, code("bf16"), 0))
    lrd.tucker_conv_fwd(X_, P1_, G_, P2_, Y_, A_, B_, g, ws)
    gX = empty((N, hw, hw, C), "bf16")
    g1, gG, g2 = f32((r, C)), f32((r, k, k, r)), f32((C, r))
    lrd.tucker_conv_bwd(dY_, X_, A_, B_, P1_, G_, P2_, gX, g1, gG, g2, 0, g, ws)
    torch.cuda.synchronize()
    Xo, P1o, Go, P2o, dYo = (seen(a, "bf16") for a in (X[picks], P1, G, P2, dY[picks]))
    Ao, Bo, Yo = oracle.tucker_fwd(Xo, P1o, Go, P2o, 1, 1)
    check(host(Y_[picks]), Yo, "bf16", "Y")
    check(host(A_[picks]), Ao, "bf16", "A")
    check(host(B_[picks]), Bo, "bf16", "B")
    go = oracle.tucker_bwd(dYo, Xo, Ao, Bo, P1o, Go, P2o, 0, 1, 1)
    check(host(gX[picks]), go["dX"], "bf16", "dX")
    check(host(g1), go["dP1"], "bf16", "dP1")
    check(host(gG), go["dG"], "bf16", "dG")
    check(host(g2), go["dP2"], "bf16", "dP2")
    rest = [n for n in range(N) if n not in picks]
    assert torch.all(gX[rest] == 0), "input gradient of an image whose output gradient is zero"
