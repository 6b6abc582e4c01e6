"""Pins for the oracle's integer rules: rank quantization (Section 2.1), the rank formulas
(eq. 6 / eq. 7), the rank search of Algorithm 1 and the sequential-freezing schedule (Algorithm 2)."""
import math

import oracle
from conftest import read_golden


# ---------------------------------------------------------------- printed examples (golden)
def test_paper_examples():
    for row in read_golden("paper_rank_examples.txt"):
        kind = row[0]
        if kind == "tucker_rank":
            C, S, k = int(row[1]), int(row[2]), int(row[3])
            alpha, beta = float(row[4]), float(row[5])
            assert oracle.tucker_rank(C, S, k, alpha, beta) == (int(row[6]), int(row[7]))
        elif kind == "quantize":
            r, q = int(row[1]), int(row[2])
            # every power-of-two granularity from 4 to 256 sends 257 to 256, in NEAREST and DOWN mode
            for m in (4, 8, 16, 32, 64, 128, 256):
                assert oracle.quantize_rank(r, m, oracle.ROUND_NEAREST) == q
                assert oracle.quantize_rank(r, m, oracle.ROUND_DOWN) == q
        elif kind == "compression_change_below":
            ra, rb, C, S, k = (int(x) for x in row[1:6])
            bound = float(row[6])

            def ratio(r):
                return C * S * k * k / (C * r + k * k * r * r + r * S)

            assert abs(ratio(rb) / ratio(ra) - 1.0) < bound
        elif kind == "rmin_range":
            C, S, k = int(row[1]), int(row[2]), int(row[3])
            r1, _ = oracle.tucker_rank(C, S, k, float(row[4]), float(row[5]))
            assert int(row[6]) <= r1 <= int(row[7])
        else:
            raise AssertionError(kind)


def test_alg2_truth_table():
    for kind, parity, f0, f1, f2 in read_golden("alg2_truth_table.txt"):
        k = oracle.KIND_SVD if kind == "svd" else oracle.KIND_TUCKER
        want = int(f0) * 1 + int(f1) * 2 + (0 if f2 == "-" else int(f2) * 4)
        for e in (int(parity), int(parity) + 2, int(parity) + 100, int(parity) + 2**40):
            assert oracle.freeze_mask(k, e) == want


def test_freeze_mask_complements_and_period():
    for kind, bits in ((oracle.KIND_SVD, 0b11), (oracle.KIND_TUCKER, 0b111)):
        for e in range(20):
            a, b = oracle.freeze_mask(kind, e), oracle.freeze_mask(kind, e + 1)
            assert a ^ b == bits          # what was frozen is released, the rest is frozen
            assert a & b == 0
            assert oracle.freeze_mask(kind, e + 2) == a


# ---------------------------------------------------------------- eq. 6 / eq. 7
def _tucker_params(C, S, k, r1, r2):
    return C * r1 + k * k * r1 * r2 + r2 * S


def test_tucker_rank_is_parameter_count_root():
    """eq. 6 is the positive root of  C r1 + k^2 r1 r2 + r2 S = C S k^2 / alpha  with r2 = beta r1:
    the returned r1 meets the budget and r1 + 1 does not (beta = 1)."""
    for (C, S, k) in ((512, 512, 3), (64, 64, 3), (256, 512, 3), (128, 96, 5), (320, 64, 1), (48, 48, 7)):
        for alpha in (1.5, 2.0, 3.0, 4.0, 8.0):
            r1, r2 = oracle.tucker_rank(C, S, k, alpha, 1.0)
            assert r1 == r2 or r2 == min(r1, S) or r1 == min(r2, C)
            budget = C * S * k * k / alpha
            if 1 < r1 < min(C, S):
                assert _tucker_params(C, S, k, r1, r1) <= budget < _tucker_params(C, S, k, r1 + 1, r1 + 1)


def test_tucker_rank_worked_numbers():
    # closed form of the paper's example evaluates to 309.59... (alpha=2) and 244.1... (alpha+1=3)
    b = (512 + 512) / 9.0
    x2 = (-b + math.sqrt(b * b + 4 * 512 * 512 / 2.0)) / 2
    x3 = (-b + math.sqrt(b * b + 4 * 512 * 512 / 3.0)) / 2
    assert 309 < x2 < 310 and 244 < x3 < 245
    assert oracle.tucker_rank(512, 512, 3, 2.0)[0] == 309
    assert oracle.tucker_rank(512, 512, 3, 3.0)[0] == 244
    # the 2x example really is 2x: parameter ratio at 309 is 2.0066
    assert abs(512 * 512 * 9 / _tucker_params(512, 512, 3, 309, 309) - 2.0066) < 1e-4


def test_tucker_rank_beta():
    r1, r2 = oracle.tucker_rank(256, 512, 3, 2.0, 2.0)
    assert r2 == 2 * r1
    budget = 256 * 512 * 9 / 2.0
    assert _tucker_params(256, 512, 3, r1, 2 * r1) <= budget < _tucker_params(256, 512, 3, r1 + 1, 2 * (r1 + 1))


def test_svd_rank():
    for (n_in, n_out) in ((768, 768), (768, 3072), (4096, 4096), (1000, 10)):
        for alpha in (1.0, 2.0, 3.5):
            r = oracle.svd_rank(n_in, n_out, alpha)
            if 1 < r < min(n_in, n_out):
                assert r * (n_in + n_out) <= n_in * n_out / alpha < (r + 1) * (n_in + n_out)
    assert oracle.svd_rank(768, 768, 1.0) == 384
    assert oracle.svd_rank(4, 4, 1e-9) == 4          # clamped to min(in,out)
    assert oracle.svd_rank(4, 4, 1e9) == 1


# ---------------------------------------------------------------- quantization: brute force + properties
def _nearest_multiple_ties_up(r, m):
    """One-line definition: the multiple of m closest to r, the larger one on a tie."""
    cands = [(abs(q - r), -q, q) for q in range(0, r + 2 * m, m)]
    return min(cands)[2]


def test_quantize_brute_force():
    for m in (1, 3, 8, 16, 32, 64, 128):
        prev = {0: 0, 1: 0, 2: 0}
        for r in range(1, 2049):
            qn = oracle.quantize_rank(r, m, oracle.ROUND_NEAREST)
            qd = oracle.quantize_rank(r, m, oracle.ROUND_DOWN)
            qu = oracle.quantize_rank(r, m, oracle.ROUND_UP)
            want_n = max(_nearest_multiple_ties_up(r, m), m)   # confined to >= 1
            assert qn == want_n, (r, m, qn, want_n)
            assert qd == max((r // m) * m, m)
            assert qu == -(-r // m) * m
            for mode, q in ((0, qn), (1, qd), (2, qu)):
                assert q % m == 0
                assert oracle.quantize_rank(q, m, mode) == q      # idempotent
                assert q >= prev[mode]                             # monotone in r
                prev[mode] = q
            if r >= m:
                assert 2 * abs(qn - r) <= m and 0 <= r - qd < m and 0 <= qu - r < m
            if m == 1:
                assert qn == qd == qu == r


def test_quantize_examples_and_bounds():
    assert oracle.quantize_rank(200, 16) == 208        # exact tie between 192 and 208 goes up
    assert oracle.quantize_rank(200, 16, oracle.ROUND_DOWN) == 192
    assert oracle.quantize_rank(309, 16, oracle.ROUND_DOWN) == 304
    assert oracle.quantize_rank(309, 16, oracle.ROUND_UP) == 320
    assert oracle.quantize_rank(309, 64) == 320
    # bounds: stay inside [r_min, r_max] on multiples of m
    assert oracle.quantize_rank(250, 64, oracle.ROUND_NEAREST, 1, 200) == 192
    assert oracle.quantize_rank(250, 64, oracle.ROUND_DOWN, 257, 400) == 320
    assert oracle.quantize_rank(10, 64, oracle.ROUND_DOWN, 1, 1000) == 64
    # no multiple inside the bounds: the rank is returned as it came
    assert oracle.quantize_rank(250, 64, oracle.ROUND_NEAREST, 200, 250) == 250
    assert oracle.quantize_rank(5, 16, oracle.ROUND_NEAREST, 1, 10) == 5
    # paper's direction (Algorithm 1 only lowers the rank) with eq. 7 as the floor
    rmin = oracle.tucker_rank(512, 512, 3, 3.0)[0]
    assert oracle.quantize_rank(309, 64, oracle.ROUND_DOWN, rmin, 512) == 256
    # bad arguments
    for args in ((0, 16, 0, 1, 100), (10, 0, 0, 1, 100), (10, 16, 3, 1, 100), (10, 16, 0, 5, 4)):
        assert oracle.quantize_rank(*args) < 0


# ---------------------------------------------------------------- Algorithm 1: rank search from measured times
def test_alg1_worked_examples():
    for row in read_golden("alg1_rank_search.txt"):
        mode, r_min, r_max = int(row[0]), int(row[1]), int(row[2])
        noise, t_dense = float(row[3]), float(row[4])
        want_r, want_keep = int(row[5]), bool(int(row[6]))
        times = [float(x) for x in row[7:]]
        assert oracle.select_rank(times, r_min, r_max, t_dense, noise, mode) == (want_r, want_keep), row


def _staircase(r_min, r_max, m, slope=0.0):
    """Step time of a kernel that pads the rank up to a multiple of m (plus an optional small slope)."""
    return [float(-(-r // m)) + slope * r for r in range(r_min, r_max + 1)]


def test_alg1_staircase_agrees_with_rank_quantization():
    # On an ideal staircase the first drop below a misaligned estimated rank is the multiple of m just
    # below it: Algorithm 1 and rounding down to a multiple (two separate routines) must agree.
    for m in (8, 16, 32, 64):
        for R in (m + 1, 2 * m - 1, 3 * m + 5, 309, 257):
            if R % m == 0:
                continue
            for mode in (0, 1):
                # first-peak mode may see a second drop further down; arg max gets a range holding one drop only
                r_min = max(1, R - 2 * m) if mode == 0 else max(1, R - R % m - 3)
                times = _staircase(r_min, R, m, slope=1e-4)
                r_opt, keep = oracle.select_rank(times, r_min, R, 1e9, 0.01, mode)
                assert r_opt == oracle.quantize_rank(R, m, oracle.ROUND_DOWN), (m, R, mode)
                assert keep


def test_alg1_invariances():
    rng = __import__("random").Random(7)
    for _ in range(200):
        n = rng.randint(1, 12)
        r_min = rng.randint(1, 40)
        r_max = r_min + n - 1
        times = [rng.choice((1.0, 1.25, 1.5, 2.0)) for _ in range(n)]
        t_dense = rng.choice((0.5, 1.3, 3.0))
        noise = rng.choice((0.0, 0.1, 0.3))
        for mode in (0, 1, 4, 5):
            guarded, sel = bool(mode & 4), mode & 1
            base = oracle.select_rank(times, r_min, r_max, t_dense, noise, mode)
            # a constant offset on every time (dense included) and a common positive factor change nothing
            assert oracle.select_rank([t + 4.0 for t in times], r_min, r_max, t_dense + 4.0, noise, mode) == base
            assert oracle.select_rank([t * 8.0 for t in times], r_min, r_max, t_dense * 8.0, noise * 8.0, mode) == base
            r_opt, keep = base
            assert r_min <= r_opt <= r_max
            assert keep == (times[r_opt - r_min] < t_dense)
            d = {r: times[r - r_min] - times[r - 1 - r_min] for r in range(r_min + 1, r_max + 1)}
            big = [r for r in d if d[r] > noise]
            if r_opt == r_max:
                if not guarded:
                    # literal reading: nothing chosen means no difference exceeds the noise (the largest one
                    # that does is always a local maximum, so first-peak mode finds one whenever arg max does)
                    assert not big
                elif big:
                    # extension: the rank below the chosen drop is not faster than the estimated rank
                    r_star = max(big, key=lambda r: (d[r], r)) if sel == 1 else next(
                        r for r in sorted(big, reverse=True)
                        if d[r] >= d.get(r + 1, -math.inf) and d[r] >= d.get(r - 1, -math.inf))
                    assert not times[r_star - 1 - r_min] < times[-1]
            else:
                if guarded:
                    assert times[r_opt - r_min] < times[-1]
                r_star = r_opt + 1
                assert d[r_star] > noise
                if sel == 1:
                    assert d[r_star] == max(d.values()) and all(d[r] < d[r_star] for r in d if r > r_star)
                else:
                    assert d[r_star] >= d.get(r_star + 1, -math.inf) and d[r_star] >= d.get(r_star - 1, -math.inf)
                    for r in big:            # every higher candidate is beaten by a neighbour
                        if r > r_star:
                            assert d[r] < d.get(r + 1, -math.inf) or d[r] < d.get(r - 1, -math.inf)
            if guarded:
                # the flag only ever replaces a pick by r_max
                plain = oracle.select_rank(times, r_min, r_max, t_dense, noise, sel)
                assert base == plain or (r_opt == r_max and not times[plain[0] - r_min] < times[-1])


def test_alg1_rejects_bad_arguments():
    import pytest
    for bad in (dict(times=[1.0, 2.0], r_min=0, r_max=1), dict(times=[1.0], r_min=3, r_max=3, noise=-1.0),
                dict(times=[1.0, float("nan")], r_min=3, r_max=4), dict(times=[1.0], r_min=3, r_max=3, mode=2),
                dict(times=[1.0], r_min=3, r_max=3, mode=8), dict(times=[1.0], r_min=3, r_max=3, mode=6)):
        with pytest.raises(ValueError):
            oracle.select_rank(bad["times"], bad["r_min"], bad["r_max"], 1.0, bad.get("noise", 0.0), bad.get("mode", 0))


# ---------------------------------------------------------------- optimizer step (Section 3: SGD, momentum 0.9, weight decay 1e-4)
def test_sgd_step_matches_the_library_optimizer():
    """Five steps against torch.optim.SGD on the CPU in fp64, momentum buffers starting at zero."""
    import numpy as np
    import torch
    rng = np.random.default_rng(5)
    for lr, mu, wd in ((1e-3, 0.9, 1e-4), (0.1, 0.0, 0.0), (0.05, 0.5, 0.1)):
        w0 = rng.standard_normal((7, 5))
        p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
        opt = torch.optim.SGD([p], lr=lr, momentum=mu, weight_decay=wd)
        w, m = w0.copy(), np.zeros_like(w0)
        for step in range(5):
            g = rng.standard_normal(w0.shape)
            p.grad = torch.from_numpy(g.copy())
            opt.step()
            w, m = oracle.sgd_step(w, m, g, lr, mu, wd)
            assert np.max(np.abs(w - p.detach().numpy())) < 1e-14, (lr, mu, wd, step)


def test_sgd_step_closed_forms():
    import numpy as np
    # constant gradient, no decay: m_k = g (1 - mu^k) / (1 - mu), w_k = w_0 - lr * sum_j m_j
    g, mu, lr = np.array([2.0, -1.0]), 0.9, 0.01
    w, m = np.array([1.0, 1.0]), np.zeros(2)
    total = np.zeros(2)
    for k in range(1, 8):
        w, m = oracle.sgd_step(w, m, g, lr, mu, 0.0)
        want_m = g * (1 - mu ** k) / (1 - mu)
        total += want_m
        assert np.allclose(m, want_m, rtol=1e-13) and np.allclose(w, 1.0 - lr * total, rtol=1e-13)
    # zero gradient, no momentum: pure decay w_k = w_0 (1 - lr wd)^k
    w, m = np.array([3.0]), np.zeros(1)
    for k in range(1, 6):
        w, m = oracle.sgd_step(w, m, np.zeros(1), 0.1, 0.0, 0.5)
        assert np.allclose(w, 3.0 * (1 - 0.05) ** k, rtol=1e-13)
