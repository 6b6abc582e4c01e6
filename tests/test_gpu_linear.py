"""GPU parity: SVD-decomposed linear layer forward/backward with freezing, through the C ABI,
against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from parity import TOL, check, code, dev, empty, f32, host, rel_err, seen, workspace
from paper_2309_03824_amd import binding as lrd

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["auto", "fused", "unfused"], autouse=True)
def fusion_mode(request):
    """Every test of this module runs with the library's default choice, with the rank-r
    intermediate kept in LDS wherever the fused kernel supports the shape, and with two
    separate products."""
    mode = {"auto": lrd.FUSION_AUTO, "fused": lrd.FUSION_ALWAYS, "unfused": lrd.FUSION_NEVER}[request.param]
    prev = lrd.set_fusion(mode)
    yield request.param
    lrd.set_fusion(prev)

SENT = -1234.5


def run_linear(T, n_in, n_out, r, dt, mask, seed, bias=False, save_h=True, want_dx=True, factors=None,
               X=None, dY=None, sample_rows=None):
    """Runs fwd+bwd on the GPU and on the oracle; returns dict of relative errors."""
    rng = np.random.Generator(np.random.PCG64(seed))
    X = si.gaussian((T, n_in), rng) if X is None else X
    U, V = si.direct_factors(n_out, n_in, r, rng) if factors is None else factors
    b = si.gaussian((n_out,), rng) if bias else None
    dYh = si.gaussian((T, n_out), rng) if dY is None else dY

    dX_, dV_, dU_ = dev(X, dt), dev(V, dt), dev(U, dt)
    db_ = None if b is None else dev(b, "f32")
    Y_ = empty((T, n_out), dt)
    H_ = empty((T, r), dt) if save_h else None
    ws = workspace(lrd.linear_workspace_bytes(T, n_in, n_out, r, code(dt), mask))
    lrd.linear_fwd(dX_, dV_, dU_, db_, Y_, H_, ws)

    dY_ = dev(dYh, dt)
    gX = empty((T, n_in), dt) if want_dx else None
    gV = f32((r, n_in), SENT)
    gU = f32((n_out, r), SENT)
    gb = f32((n_out,)) if bias else None
    lrd.linear_bwd(dY_, dX_, H_, dV_, dU_, gX, gV, gU, gb, mask, ws)
    torch.cuda.synchronize()

    Xo, Vo, Uo, dYo = seen(X, dt), seen(V, dt), seen(U, dt), seen(dYh, dt)
    bo = None if b is None else seen(b, "f32")
    rows = slice(None) if sample_rows is None else sample_rows
    Ho, Yo = oracle.linear_fwd(Xo[rows], Vo, Uo, bo)
    errs = {"Y": check(host(Y_)[rows], Yo, dt, "Y")}
    if save_h:
        errs["H"] = check(host(H_)[rows], Ho, dt, "H")
    if sample_rows is None:
        g = oracle.linear_bwd(dYo, Xo, Ho, Vo, Uo, mask, want_dX=want_dx, want_dbias=bias)
        if want_dx:
            errs["dX"] = check(host(gX), g["dX"], dt, "dX")
        if mask & 1:
            assert torch.all(gV == SENT), "frozen dV was written"
        else:
            errs["dV"] = check(host(gV), g["dV"], dt, "dV")
        if mask & 2:
            assert torch.all(gU == SENT), "frozen dU was written"
        else:
            errs["dU"] = check(host(gU), g["dU"], dt, "dU")
        if bias:
            errs["dbias"] = check(host(gb), g["dbias"], dt, "dbias")
    out = dict(errs=errs, Y=Y_, H=H_, dX=gX, dV=gV, dU=gU)
    return out


def test_config1_fp32_full_size():
    """256 x 768 tokens, W = Q1 diag(exp(-i/100)) Q2^T (768 x 768), rank 200 -> 208, V frozen,
    loss 0.5 ||Y||^2 (dY = Y), fp32 path, tolerance 1e-4."""
    W, _ = si.config1_weight()
    r = lrd.quantize_rank(200, 16)
    assert r == 208 == oracle.quantize_rank(200, 16)
    U, V, _ = oracle.svd_factors(W, r)
    X = si.gaussian((256, 768), si.rng_for(1, 1))
    _, Yo = oracle.linear_fwd(seen(X, "f32"), seen(V, "f32"), seen(U, "f32"))
    mask = lrd.freeze_mask(lrd.KIND_SVD, 0)
    assert mask == lrd.FREEZE_L0
    out = run_linear(256, 768, 768, r, "f32", mask, 0, factors=(U, V), X=X, dY=Yo)
    assert max(out["errs"].values()) <= TOL["f32"]


@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [
    (300, 200, 136, 64),     # several tiles, ragged token tail
    (257, 96, 520, 33),      # odd (raw) rank, nothing aligned
    (64, 48, 40, 40),        # rank = min(in,out)
    (1, 8, 8, 1),            # degenerate: one token, rank one
    (130, 264, 72, 16),
])
def test_small_shapes_all_masks(dt, shape):
    T, n_in, n_out, r = shape
    for mask in (0, 1, 2, 3):
        run_linear(T, n_in, n_out, r, dt, mask, seed=100 + mask, bias=(mask == 0))


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_nullable_arguments(dt):
    # no saved H (recomputed in the workspace), no dX (first layer)
    run_linear(200, 72, 88, 24, dt, 0, seed=7, save_h=False)
    run_linear(200, 72, 88, 24, dt, 1, seed=8, want_dx=False)
    run_linear(200, 72, 88, 24, dt, 2, seed=9, save_h=False, want_dx=False)


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_freezing_does_not_perturb_trainable_outputs(dt):
    T, n_in, n_out, r = 384, 256, 320, 64
    free = run_linear(T, n_in, n_out, r, dt, 0, seed=21)
    fv = run_linear(T, n_in, n_out, r, dt, 1, seed=21)
    fu = run_linear(T, n_in, n_out, r, dt, 2, seed=21)
    assert torch.equal(fv["dU"], free["dU"]) and torch.equal(fv["dX"], free["dX"])
    assert torch.equal(fu["dV"], free["dV"]) and torch.equal(fu["dX"], free["dX"])
    assert torch.equal(fv["Y"], free["Y"])


def test_rank_staircase_shapes_bf16():
    """Raw and quantized ranks around tile boundaries, at a width that spans several tiles."""
    for r in (255, 256, 257, 200, 208, 192, 1, 7, 8, 31, 32, 264, 320):
        run_linear(320, 512, 384, r, "bf16", 0, seed=300 + r)


def test_ffn_block_shapes_full_size_bf16():
    """One encoder FFN pair at full size: 8192 tokens, 768 -> 3072 -> 768, rank 192, bf16,
    alternating freeze masks; factors from an LAPACK SVD of W ~ N(0, 1/fan_in)."""
    from paper_2309_03824_amd import factorize
    rng = si.rng_for(2, 0)
    r = lrd.quantize_rank(int(0.25 * 768), 64)
    assert r == 192
    for step, (n_in, n_out) in enumerate(((768, 3072), (3072, 768))):
        W = si.linear_weight(n_out, n_in, rng)
        U, V, _ = factorize.svd_factors(W, r)
        run_linear(8192, n_in, n_out, r, "bf16", lrd.freeze_mask(lrd.KIND_SVD, step), seed=40 + step,
                   factors=(U, V))


def test_transformer_projection_shapes_bf16():
    """Encoder with hidden 1024 / FFN 4096 at rank 256: the Q/K/V/O shape (1024 -> 1024) at the full
    8192 tokens, the two FFN shapes on a 1024-token slice, masks cycling with the step."""
    r = lrd.quantize_rank(256, 64)
    for step, (T, n_in, n_out) in enumerate(((8192, 1024, 1024), (1024, 1024, 4096), (1024, 4096, 1024))):
        run_linear(T, n_in, n_out, r, "bf16", lrd.freeze_mask(lrd.KIND_SVD, step), seed=500 + step)


def test_large_layer_sampled_bf16():
    """4096 x 4096 layer, 16384 tokens, rank 256: the oracle evaluates sampled token rows of Y/H/dX
    and the weight gradients of a gradient that is non-zero on sampled tokens only."""
    T, d, r = 16384, 4096, 256
    rng = si.rng_for(3, 0)
    X = si.gaussian((T, d), rng)
    U, V = si.direct_factors(d, d, r, rng)
    rows = np.sort(rng.choice(T, size=192, replace=False))
    dY = np.zeros((T, d))
    dY[rows] = si.gaussian((rows.size, d), rng)
    dt = "bf16"
    X_, V_, U_, dY_ = dev(X, dt), dev(V, dt), dev(U, dt), dev(dY, dt)
    Y_, H_ = empty((T, d), dt), empty((T, r), dt)
    ws = workspace(lrd.linear_workspace_bytes(T, d, d, r, lrd.BF16, 0))
    lrd.linear_fwd(X_, V_, U_, None, Y_, H_, ws)
    gX, gV, gU = empty((T, d), dt), f32((r, d)), f32((d, r))
    lrd.linear_bwd(dY_, X_, H_, V_, U_, gX, gV, gU, None, 0, ws)
    torch.cuda.synchronize()
    Xo, Vo, Uo, dYo = seen(X[rows], dt), seen(V, dt), seen(U, dt), seen(dY[rows], dt)
    Ho, Yo = oracle.linear_fwd(Xo, Vo, Uo)
    check(host(Y_[torch.from_numpy(rows).cuda()]), Yo, dt, "Y rows")
    check(host(H_[torch.from_numpy(rows).cuda()]), Ho, dt, "H rows")
    g = oracle.linear_bwd(dYo, Xo, Ho, Vo, Uo, 0)
    check(host(gX[torch.from_numpy(rows).cuda()]), g["dX"], dt, "dX rows")
    check(host(gU), g["dU"], dt, "dU")
    check(host(gV), g["dV"], dt, "dV")
    others = np.setdiff1d(np.arange(0, T, 97), rows)
    assert torch.all(gX[torch.from_numpy(others).cuda()] == 0)       # zero gradient rows stay zero


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_dense_linear(dt):
    for (T, n_in, n_out) in ((300, 200, 136), (129, 520, 96), (1024, 768, 768)):
        rng = np.random.Generator(np.random.PCG64(T))
        X, W = si.gaussian((T, n_in), rng), si.linear_weight(n_out, n_in, rng)
        b, dY = si.gaussian((n_out,), rng), si.gaussian((T, n_out), rng)
        X_, W_, dY_, b_ = dev(X, dt), dev(W, dt), dev(dY, dt), dev(b, "f32")
        Y_ = empty((T, n_out), dt)
        ws = workspace(lrd.dense_linear_workspace_bytes(T, n_in, n_out, code(dt)))
        lrd.dense_linear_fwd(X_, W_, b_, Y_, ws)
        gX, gW = empty((T, n_in), dt), f32((n_out, n_in))
        lrd.dense_linear_bwd(dY_, X_, W_, gX, gW, ws)
        torch.cuda.synchronize()
        Xo, Wo, dYo = seen(X, dt), seen(W, dt), seen(dY, dt)
        check(host(Y_), oracle.dense_linear_fwd(Xo, Wo, seen(b, "f32")), dt, "Y")
        dXo, dWo = oracle.dense_linear_bwd(dYo, Xo, Wo)
        check(host(gX), dXo, dt, "dX")
        check(host(gW), dWo, dt, "dW")


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_gelu(dt):
    rng = np.random.Generator(np.random.PCG64(5))
    for n in (1, 7, 8, 1000, 65536 + 3):
        Z, dA = si.gaussian((n,), rng, 2.0), si.gaussian((n,), rng)
        Z_, dA_ = dev(Z, dt), dev(dA, dt)
        A_, dZ_ = empty((n,), dt), empty((n,), dt)
        lrd.gelu_fwd(Z_, A_)
        lrd.gelu_bwd(dA_, Z_, dZ_)
        torch.cuda.synchronize()
        check(host(A_), oracle.gelu_fwd(seen(Z, dt)), dt, "gelu")
        check(host(dZ_), oracle.gelu_bwd(seen(dA, dt), seen(Z, dt)), dt, "gelu bwd")


@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(384, 256, 512, 64), (130, 72, 88, 24), (257, 96, 520, 33)])
def test_activation_folded_into_the_pair(dt, shape):
    """lrd_linear_fwd_act / lrd_linear_bwd_act against the plain calls followed by the GELU kernels
    (bit-identical) and against the oracle: Z = pair(X), A = gelu(Z); dZ_in = (dH V) * gelu'(Z_in)."""
    T, n_in, n_out, r = shape
    rng = np.random.Generator(np.random.PCG64(sum(shape)))
    X, dY, Zin = si.gaussian((T, n_in), rng), si.gaussian((T, n_out), rng), si.gaussian((T, n_in), rng)
    U, V = si.direct_factors(n_out, n_in, r, rng)
    X_, V_, U_, dY_, Zin_ = (dev(a, dt) for a in (X, V, U, dY, Zin))
    ws = workspace(lrd.linear_workspace_bytes(T, n_in, n_out, r, code(dt), 0))
    Z1, A1, Z2, A2 = (empty((T, n_out), dt) for _ in range(4))
    H1, H2 = empty((T, r), dt), empty((T, r), dt)
    lrd.linear_fwd_act(X_, V_, U_, None, Z1, A1, H1, lrd.ACT_GELU, ws)
    lrd.linear_fwd(X_, V_, U_, None, Z2, H2, ws)
    lrd.gelu_fwd(Z2, A2)
    g1, g2, tmp = empty((T, n_in), dt), empty((T, n_in), dt), empty((T, n_in), dt)
    dU1, dU2, dV1, dV2 = f32((n_out, r)), f32((n_out, r)), f32((r, n_in)), f32((r, n_in))
    lrd.linear_bwd_act(dY_, X_, H1, V_, U_, g1, dV1, dU1, None, 0, Zin_, lrd.ACT_GELU, ws)
    lrd.linear_bwd(dY_, X_, H2, V_, U_, tmp, dV2, dU2, None, 0, ws)
    lrd.gelu_bwd(tmp, Zin_, g2)
    torch.cuda.synchronize()
    assert torch.equal(Z1, Z2) and torch.equal(A1, A2) and torch.equal(g1, g2)
    assert torch.equal(dU1, dU2) and torch.equal(dV1, dV2)
    Ho, Zo = oracle.linear_fwd(seen(X, dt), seen(V, dt), seen(U, dt))
    check(host(A1), oracle.gelu_fwd(Zo), dt, "act(Z)")
    go = oracle.linear_bwd(seen(dY, dt), seen(X, dt), Ho, seen(V, dt), seen(U, dt), 0)
    check(host(g1), oracle.gelu_bwd(go["dX"], seen(Zin, dt)), dt, "dZ_in")


def test_errors_reported_by_status():
    X = empty((8, 8), "f32", 1.0)
    dV, dU = f32((4, 8)), f32((8, 4))
    with pytest.raises(lrd.LrdError) as e:     # the backward needs workspace for dH; none is given
        lrd.linear_bwd(X, X, None, X[:4], X[:, :4].contiguous(), X.clone(), dV, dU, None, 0, None)
    assert e.value.status == lrd.ERR_WORKSPACE
    with pytest.raises(lrd.LrdError) as e:     # rank above min(in, out)
        lrd.linear_fwd(X, empty((9, 8), "f32"), empty((8, 9), "f32"), None, X.clone(), None, None)
    assert e.value.status == lrd.ERR_INVALID_ARG


# ---------------------------------------------------------------- grouped layers on one input (Q / K / V)
@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("case", [(3, 300, 128, 96, 32), (2, 257, 64, 160, 24), (1, 128, 64, 64, 16), (3, 200, 96, 80, 12)])
def test_grouped_linear_matches_separate_oracle_layers(dt, case):
    G, T, n_in, n_out, r = case
    rng = si.rng_for(5, sum(case))
    X = si.gaussian((T, n_in), rng)
    Us, Vs = zip(*[si.direct_factors(n_out, n_in, r, rng) for _ in range(G)])
    U, V_cat = np.stack(Us), np.concatenate(Vs, axis=0)
    bias = si.gaussian((G, n_out), rng).astype(np.float32)
    dY = si.gaussian((G, T, n_out), rng)
    ws = workspace(lrd.linear_group_workspace_bytes(T, n_in, n_out, r, G, code(dt), 0))
    Xd, Ud, Vd, dYd = dev(X, dt), dev(U, dt), dev(V_cat, dt), dev(dY, dt)
    bd = torch.from_numpy(bias).cuda()
    Y, H = empty((G, T, n_out), dt), empty((T, G * r), dt)
    lrd.linear_group_fwd(Xd, Vd, Ud, bd, Y, H, ws)
    Xo, Uo, Vo, dYo = seen(X, dt), seen(U, dt), seen(V_cat, dt), seen(dY, dt)
    for g in range(G):
        Ho, Yo = oracle.linear_fwd(Xo, Vo[g * r:(g + 1) * r], Uo[g], bias[g].astype(np.float64))
        check(host(Y[g]), Yo, dt, f"Y[{g}]")
        check(host(H)[:, g * r:(g + 1) * r], Ho, dt, f"H[{g}]")
    for mask in (0, 1, 2):
        dX, dV, dU, db = empty((T, n_in), dt), f32((G * r, n_in), 7.0), f32((G, n_out, r), 7.0), f32((G, n_out))
        lrd.linear_group_bwd(dYd, Xd, H if mask != 1 else None, Vd, Ud, dX, dV, dU, db, mask, ws)
        dXo = np.zeros((T, n_in))
        for g in range(G):
            Ho, _ = oracle.linear_fwd(Xo, Vo[g * r:(g + 1) * r], Uo[g])
            go = oracle.linear_bwd(dYo[g], Xo, Ho, Vo[g * r:(g + 1) * r], Uo[g], mask, want_dbias=True)
            dXo += go["dX"]
            if not mask & 2:
                check(host(dU[g]), go["dU"], dt, f"dU[{g}]")
            if not mask & 1:
                check(host(dV)[g * r:(g + 1) * r], go["dV"], dt, f"dV[{g}]")
            check(host(db[g]), go["dbias"], dt, f"dbias[{g}]")
        check(host(dX), dXo, dt, "dX")
        if mask & 2:
            assert torch.all(dU == 7.0)          # frozen factors are never written
        if mask & 1:
            assert torch.all(dV == 7.0)


# ---------------------------------------------------------------- backward + optimizer step in one call
@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [
    (384, 96, 160, 32),      # gradients stored whole: the step is a kernel of its own
    (1024, 192, 256, 64),    # 4 K-slices: the step runs in the sum over the slices
    (4096, 192, 256, 64),    # 16 slices, several threads per output in the sum
    (16384, 64, 64, 64),     # 64 slices
    (384, 96, 160, 30),      # rank padded to 32 inside: gradients cropped before the step
])
def test_backward_with_sgd_update(dt, shape):
    T, n_in, n_out, r = shape
    rng = si.rng_for(5, 900 + T + r)
    X, dY = si.gaussian((T, n_in), rng), si.gaussian((T, n_out), rng)
    U0, V0 = si.direct_factors(n_out, n_in, r, rng)
    opt = lrd.Sgd(0.05, 0.9, 1e-4)
    lr, mu, wd = float(opt.lr), float(opt.momentum), float(opt.weight_decay)
    Um, Vm = torch.from_numpy(U0.astype(np.float32)).cuda(), torch.from_numpy(V0.astype(np.float32)).cuda()
    Uc, Vc = dev(host(Um), dt), dev(host(Vm), dt)
    mU, mV = f32((n_out, r), 0.0), f32((r, n_in), 0.0)
    Xd, dYd = dev(X, dt), dev(dY, dt)
    H, Y, dX = empty((T, r), dt), empty((T, n_out), dt), empty((T, n_in), dt)
    ws = workspace(lrd.linear_sgd_workspace_bytes(T, n_in, n_out, r, code(dt), 0))
    Xo, dYo = seen(X, dt), seen(dY, dt)
    # oracle state: masters in fp64 (they hold fp32 values), momenta zero
    Uo, Vo, mUo, mVo = host(Um), host(Vm), np.zeros((n_out, r)), np.zeros((r, n_in))
    for step in range(4):
        mask = lrd.freeze_mask(lrd.KIND_SVD, step)
        lrd.linear_fwd(Xd, Vc, Uc, None, Y, H, ws)
        before = [t.clone() for t in (Um, Vm, mU, mV, Uc, Vc)]
        Uc_o, Vc_o = host(Uc), host(Vc)              # the values the layer multiplies with in this step
        lrd.linear_bwd_sgd(dYd, Xd, H, Vc, Uc, dX, Vm, Um, mV, mU, None, mask, None, lrd.ACT_NONE, opt, ws)
        Ho, _ = oracle.linear_fwd(Xo, Vc_o, Uc_o)
        go = oracle.linear_bwd(dYo, Xo, Ho, Vc_o, Uc_o, mask)
        check(host(dX), go["dX"], dt, "dX")
        if mask & lrd.FREEZE_L1:                                     # U frozen: nothing of U moves
            for a, b in ((Um, before[0]), (mU, before[2]), (Uc, before[4])):
                assert torch.equal(a, b)
        else:
            Uo, mUo = oracle.sgd_step(Uo, mUo, go["dU"], lr, mu, wd)
            check(host(mU), mUo, dt, "momentum U")
            assert rel_err((host(Um) - host(before[0])) / lr, (Uo - host(before[0])) / lr) <= TOL[dt]
            assert torch.equal(Uc, Um.to(Uc.dtype))                  # compute copy = rounded master
        if mask & lrd.FREEZE_L0:
            for a, b in ((Vm, before[1]), (mV, before[3]), (Vc, before[5])):
                assert torch.equal(a, b)
        else:
            Vo, mVo = oracle.sgd_step(Vo, mVo, go["dV"], lr, mu, wd)
            check(host(mV), mVo, dt, "momentum V")
            assert rel_err((host(Vm) - host(before[1])) / lr, (Vo - host(before[1])) / lr) <= TOL[dt]
            assert torch.equal(Vc, Vm.to(Vc.dtype))
        # keep the oracle's masters on the device's values so that steps stay comparable one by one
        Uo, Vo, mUo, mVo = host(Um), host(Vm), host(mU), host(mV)


def test_sgd_step_alone():
    n = 1000
    rng = si.rng_for(5, 901)
    w, g = si.gaussian((n,), rng).astype(np.float32), si.gaussian((n,), rng).astype(np.float32)
    wd_, md_, gd_ = torch.from_numpy(w.copy()).cuda(), f32((n,), 0.0), torch.from_numpy(g).cuda()
    copy = empty((n,), "bf16")
    opt = lrd.Sgd(0.01, 0.9, 1e-4)
    wo, mo = w.astype(np.float64), np.zeros(n)
    for _ in range(3):
        lrd.sgd_step(wd_, md_, gd_, copy, opt)
        wo, mo = oracle.sgd_step(wo, mo, g, float(opt.lr), float(opt.momentum), float(opt.weight_decay))
    assert np.max(np.abs(host(wd_) - wo)) <= 1e-6 * np.max(np.abs(wo))
    assert np.max(np.abs(host(md_) - mo)) <= 1e-6 * np.max(np.abs(mo))
    assert torch.equal(copy, wd_.to(torch.bfloat16))
