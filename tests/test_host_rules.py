"""Host-side checks that need no GPU: the library loads and exports every symbol include/lrd.h
declares, its integer rules agree bit for bit with the oracle, its one-time factorization agrees
with the oracle's (as products / spectra), and bad arguments are refused before any launch."""
import ctypes
import os
import re

import numpy as np

import oracle
import synth_inputs as si
from conftest import ROOT, read_golden
from paper_2309_03824_amd import binding as lrd
from paper_2309_03824_amd import factorize


def test_every_declared_symbol_is_exported():
    lib = ctypes.CDLL(lrd.LIB_PATH)
    for fname, exports in (("lrd.h", lrd.EXPORTS), ("lrd_measure.h", lrd.MEASURE_EXPORTS)):
        header = open(os.path.join(ROOT, "include", fname)).read()
        declared = set(re.findall(r"\b(lrd_[a-z0-9_]+)\s*\(", header))
        assert declared == set(exports), fname
        for name in declared:
            assert hasattr(lib, name), name


def test_integer_rules_match_oracle_bit_exact():
    for m in (1, 2, 3, 8, 16, 32, 64, 128, 100):
        for mode in (0, 1, 2):
            for r in range(1, 1100):
                assert lrd.quantize_rank(r, m, mode) == oracle.quantize_rank(r, m, mode)
                assert lrd.quantize_rank(r, m, mode, 100, 700) == oracle.quantize_rank(r, m, mode, 100, 700)
                assert lrd.quantize_rank(r, m, mode, 130, 140) == oracle.quantize_rank(r, m, mode, 130, 140)
    for kind in (0, 1):
        for e in list(range(64)) + [2**33, 2**33 + 1]:
            assert lrd.freeze_mask(kind, e) == oracle.freeze_mask(kind, e)
    for C in (3, 16, 64, 100, 256, 512, 2048):
        for S in (8, 64, 96, 512, 1024):
            for k in (1, 3, 5, 7):
                for alpha in (1.0, 1.5, 2.0, 3.0, 4.0, 10.0):
                    for beta in (0.5, 1.0, 2.0):
                        assert lrd.tucker_rank(C, S, k, alpha, beta) == oracle.tucker_rank(C, S, k, alpha, beta)
            for alpha in (0.5, 1.0, 2.0, 3.0, 7.5):
                assert lrd.svd_rank(C, S, alpha) == oracle.svd_rank(C, S, alpha)


def test_rank_search_matches_oracle_bit_exact():
    import random
    rng = random.Random(11)
    for _ in range(3000):
        n = rng.randint(1, 40)
        r_min = rng.randint(1, 300)
        r_max = r_min + n - 1
        # staircases with jitter, plateaus and exact ties: the cases where the scan order matters
        m = rng.choice((4, 8, 16, 32))
        times = [float(-(-r // m)) * rng.choice((1.0, 1.0, 1.25)) + rng.choice((0.0, 0.0, 0.01, 0.5)) for r in range(r_min, r_max + 1)]
        t_dense = rng.choice((0.5, 5.0, 50.0))
        noise = rng.choice((0.0, 0.05, 0.3, 2.0))
        for mode in (lrd.SELECT_FIRST_PEAK, lrd.SELECT_ARGMAX, lrd.SELECT_FIRST_PEAK | lrd.SELECT_REQUIRE_FASTER,
                     lrd.SELECT_ARGMAX | lrd.SELECT_REQUIRE_FASTER):
            assert lrd.select_rank(times, r_min, r_max, t_dense, noise, mode) == oracle.select_rank(
                times, r_min, r_max, t_dense, noise, mode), (times, r_min, noise, mode)
    for row in read_golden("alg1_rank_search.txt"):
        times = [float(x) for x in row[7:]]
        assert lrd.select_rank(times, int(row[1]), int(row[2]), float(row[4]), float(row[3]), int(row[0])) == (
            int(row[5]), bool(int(row[6])))
    for bad in (([1.0, 2.0], 0, 1, 1.0, 0.0, 0), ([1.0], 3, 3, 1.0, -1.0, 0), ([1.0, float("inf")], 3, 4, 1.0, 0.0, 0),
                ([1.0], 3, 3, 1.0, 0.0, 2), ([1.0], 3, 3, 1.0, 0.0, 8), ([1.0, 2.0], 3, 3, 1.0, 0.0, 0)):
        try:
            lrd.select_rank(*bad)
        except lrd.LrdError as e:
            assert e.status == lrd.ERR_INVALID_ARG
        else:
            raise AssertionError(bad)


def test_printed_examples_through_the_library():
    for row in read_golden("paper_rank_examples.txt"):
        if row[0] == "tucker_rank":
            assert lrd.tucker_rank(int(row[1]), int(row[2]), int(row[3]), float(row[4]), float(row[5])) == (
                int(row[6]), int(row[7]))
        elif row[0] == "quantize":
            assert lrd.quantize_rank(int(row[1]), 64) == int(row[2])
    for kind, parity, f0, f1, f2 in read_golden("alg2_truth_table.txt"):
        want = int(f0) + 2 * int(f1) + (0 if f2 == "-" else 4 * int(f2))
        assert lrd.freeze_mask(0 if kind == "svd" else 1, int(parity)) == want
    assert lrd.quantize_rank(200, 16) == 208


def test_integer_rules_reject_bad_arguments():
    for args in ((0, 16, 0, 1, 100), (10, 0, 0, 1, 100), (10, 16, 3, 1, 100), (10, 16, 0, 5, 4)):
        try:
            lrd.quantize_rank(*args)
        except lrd.LrdError as e:
            assert e.status == lrd.ERR_INVALID_ARG
        else:
            raise AssertionError(args)
    for args in ((0, 4, 3, 2.0, 1.0), (4, 4, 0, 2.0, 1.0), (4, 4, 3, 0.0, 1.0), (4, 4, 3, 2.0, -1.0)):
        try:
            lrd.tucker_rank(*args)
        except lrd.LrdError as e:
            assert e.status == lrd.ERR_INVALID_ARG
        else:
            raise AssertionError(args)


def test_device_entry_points_validate_before_launch():
    """Calls that must be refused on the host: no kernel is launched, so they run without a GPU."""
    lib = lrd._lib
    p = 4096  # a fake, 16-byte aligned, never dereferenced address
    ok_args = [p, p, p, None, p, None, 8, 8, 8, 4, lrd.BF16, None, 0, None]

    def fwd(**kw):
        a = list(ok_args)
        names = ["X", "V", "U", "bias", "Y", "H", "T", "n_in", "n_out", "r", "dt", "ws", "wsb", "st"]
        for k, v in kw.items():
            a[names.index(k)] = v
        return lib.lrd_linear_fwd(*a)

    assert fwd(X=None) == lrd.ERR_INVALID_ARG
    assert fwd(T=0) == lrd.ERR_INVALID_ARG
    assert fwd(r=9) == lrd.ERR_INVALID_ARG            # rank above min(in,out)
    assert fwd(dt=7) == lrd.ERR_INVALID_ARG
    assert fwd(X=p + 2) == lrd.ERR_ALIGNMENT
    assert fwd(H=p + 8) == lrd.ERR_ALIGNMENT
    # backward: trainable factor without a gradient buffer; unknown mask bit
    bwd = lib.lrd_linear_bwd
    base = [p, p, p, p, p, p, p, p, None, 0, 8, 8, 8, 4, lrd.BF16, None, 0, None]
    a = list(base); a[6] = None
    assert bwd(*a) == lrd.ERR_INVALID_ARG            # dV missing while V trains
    a = list(base); a[6] = None; a[9] = lrd.FREEZE_L0; a[15] = None
    assert bwd(*a) == lrd.ERR_WORKSPACE              # legal arguments, but no workspace given
    a = list(base); a[9] = 4
    assert bwd(*a) == lrd.ERR_INVALID_ARG
    g = lrd.conv_geom(1, 8, 8, 4, 4, 5, 2, 3, 1, 1)   # r1 > C
    assert lib.lrd_tucker_conv_fwd(p, p, p, p, p, None, None, ctypes.byref(g), lrd.BF16, None, 0, None) == lrd.ERR_INVALID_ARG
    assert lrd.tucker_conv_workspace_bytes(g, lrd.BF16) == 0
    g = lrd.conv_geom(1, 8, 8, 4, 4, 2, 2, 3, 1, 1)
    assert lib.lrd_tucker_conv_fwd(p, p, p, p, p, None, None, ctypes.byref(g), lrd.BF16, None, 0, None) == lrd.ERR_WORKSPACE
    assert lrd.tucker_conv_workspace_bytes(g, lrd.BF16) > 0
    assert lrd.linear_workspace_bytes(256, 768, 768, 208, lrd.F32) >= 256 * 208 * 4
    assert lrd.linear_workspace_bytes(256, 768, 768, 0, lrd.F32) == 0


def test_host_factorization_agrees_with_oracle():
    rng = np.random.Generator(np.random.PCG64(3))
    W = si.linear_weight(24, 40, rng)
    for r in (1, 7, 24):
        U, V, s = factorize.svd_factors(W, r)
        Uo, Vo, so = oracle.svd_factors(W, r)
        np.testing.assert_allclose(U @ V, Uo @ Vo, atol=1e-10)
        np.testing.assert_allclose(s, so, atol=1e-11)
    Wc = si.conv_weight(10, 8, 3, rng)
    P1, G, P2 = factorize.tucker2_factors(Wc, 5, 6)
    P1o, Go, P2o, _ = oracle.tucker2(Wc, 5, 6)
    rec = np.einsum("ob,buva,ac->ouvc", P2, G, P1)
    reco = np.einsum("ob,buva,ac->ouvc", P2o, Go, P1o)
    np.testing.assert_allclose(rec, reco, atol=1e-10)
