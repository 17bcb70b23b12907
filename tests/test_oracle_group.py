"""Pins for the oracle's per-group steps (Sec. 3.2, 3.3; App. A, B): brute force,
special cases that reduce to textbook routines, and the paper's identities.
CPU only."""
import itertools

import numpy as np
import pytest

from oracle import bpdq_oracle as orc
from oracle import uniform_gptq as uni


def _local_factor(g, seed, corr=0.6):
    """A realistic local factor: diagonal block of chol((H + damping)^-1)."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((6 * g, g))
    X = X + corr * np.roll(X, 1, axis=1)
    X *= np.exp(0.5 * rng.standard_normal(g))
    U, _, info = orc.prepare(2 * X.T @ X, 0.01)
    assert info == 0
    return U


# ----------------------------------------------------------------- initialisation
@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_init_codes_all_256_values(k):
    # a row 0, 1, ..., 255 has lo = 0, hi = 255, scale 1: Z equals the entry
    T = np.arange(256, dtype=np.float64)[None, :].repeat(3, axis=0)
    T[1] = T[1] * 0.37 - 11.0            # affine images quantise to the same Z
    T[2] = T[2][::-1] * 2.0 + 5.0
    code = orc.init_codes(T, k, decision_dtype=None)
    Z = np.arange(256)
    assert np.array_equal(code[0], Z >> (8 - k))
    assert np.array_equal(code[1], Z >> (8 - k))
    assert np.array_equal(code[2], Z[::-1] >> (8 - k))
    # the kept planes are the k most significant planes of Z: B_i = P_{7-k+i}
    D = orc.design_matrix(code[:1], k)
    for i in range(1, k + 1):
        assert np.array_equal(D[0, :, i], (Z >> (7 - k + i)) & 1)
    assert np.all(D[0, :, 0] == 1.0)


def test_init_codes_rounding_and_flat_row():
    # lo = 0, hi = 255 -> scale 1; halves round to even
    T = np.zeros((2, 8))
    T[0] = [0.0, 255.0, 0.5, 1.5, 2.5, 127.5, 128.5, 254.5]
    T[1] = 3.25                                  # flat row
    code = orc.init_codes(T, 4, decision_dtype=None)
    Z = np.array([0, 255, 0, 2, 2, 128, 128, 254])
    assert np.array_equal(code[0], Z >> 4)
    assert np.array_equal(code[1], np.zeros(8))


# ----------------------------------------------------------------- coefficient fit
@pytest.mark.parametrize("k,g", [(2, 16), (3, 32), (4, 24)])
def test_fit_is_the_weighted_least_squares_optimum(k, g):
    rng = np.random.default_rng(k * 100 + g)
    UL = _local_factor(g, 5)
    rows = 7
    T = rng.standard_normal((rows, g))
    code = rng.integers(0, 1 << k, size=(rows, g)).astype(np.uint8)
    c = orc.fit_coefficients(code, T, UL, k, alpha=0.0)
    A_metric = np.linalg.inv(UL).T               # U_loc^-T
    for r in range(rows):
        B_r = np.column_stack([np.ones(g)] + [((code[r] >> i) & 1).astype(float) for i in range(k)])
        want, *_ = np.linalg.lstsq(A_metric @ B_r, A_metric @ T[r], rcond=None)
        assert np.allclose(c[r], want, rtol=1e-8, atol=1e-10)


def test_fit_ridge_is_relative_to_mean_diagonal():
    k, g, alpha = 2, 12, 1e-2
    rng = np.random.default_rng(3)
    UL = _local_factor(g, 9)
    T = rng.standard_normal((4, g))
    code = rng.integers(0, 4, size=(4, g)).astype(np.uint8)
    c = orc.fit_coefficients(code, T, UL, k, alpha=alpha)
    A_metric = np.linalg.inv(UL).T
    for r in range(4):
        B_r = np.column_stack([np.ones(g), code[r] & 1, (code[r] >> 1) & 1]).astype(float)
        Y = A_metric @ B_r
        mu = alpha * np.trace(Y.T @ Y) / (k + 1)
        # ridge regression = least squares on the system augmented with sqrt(mu) I
        Aug = np.vstack([Y, np.sqrt(mu) * np.eye(k + 1)])
        rhs = np.concatenate([A_metric @ T[r], np.zeros(k + 1)])
        want, *_ = np.linalg.lstsq(Aug, rhs, rcond=None)
        assert np.allclose(c[r], want, rtol=1e-9, atol=1e-12)


def test_fit_degenerate_planes_stay_finite():
    k, g = 2, 8
    UL = _local_factor(g, 2)
    T = np.linspace(-1, 1, g)[None, :]
    code = np.zeros((1, g), dtype=np.uint8)       # both planes empty
    c = orc.fit_coefficients(code, T, UL, k, alpha=1e-4)
    assert np.all(np.isfinite(c))
    assert abs(c[0, 1]) < 1e-12 and abs(c[0, 2]) < 1e-12


# ----------------------------------------------------------------- bit-plane update
@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_nearest_level_bruteforce(k):
    rng = np.random.default_rng(k)
    c = rng.standard_normal((50, k + 1))
    w = rng.standard_normal(50) * 2
    lv = orc.level_table(c, k)
    got = orc.nearest_level(w, lv)
    for r in range(50):
        best, bd = None, None
        for code in range(1 << k):
            v = c[r, 0] + sum(c[r, i] * ((code >> (i - 1)) & 1) for i in range(1, k + 1))
            assert np.isclose(lv[r, code], v, rtol=1e-14, atol=1e-15)
            d = (w[r] - lv[r, code]) ** 2
            if bd is None or d < bd:
                best, bd = code, d
        assert got[r] == best


def test_nearest_level_tie_takes_lowest_code():
    c = np.array([[0.0, 1.0, 1.0]])              # levels 0, 1, 1, 2
    lv = orc.level_table(c, 2)
    assert orc.nearest_level(np.array([1.0]), lv)[0] == 1
    assert orc.nearest_level(np.array([0.5]), lv)[0] == 0
    assert orc.nearest_level(np.array([1.5]), lv)[0] == 1


@pytest.mark.parametrize("k,g", [(2, 32), (3, 16), (4, 16)])
def test_frozen_uniform_coefficients_reproduce_gptq_bit_for_bit(k, g):
    # Prop. 1: with c = (lo, s, 2s, ...) the variable grid is the uniform grid,
    # so the sweep must equal a separately written uniform-grid GPTQ sweep.
    rng = np.random.default_rng(10 * k + g)
    UL = _local_factor(g, 7)
    T = rng.standard_normal((40, g)) * 0.02
    ref = uni.uniform_group(T, UL, k)
    code, What, E = orc.bitplane_sweep(T, UL, ref["coef"], k, decision_dtype=None)
    assert np.array_equal(code, ref["code"])
    assert np.allclose(What, ref["What"], rtol=1e-13, atol=1e-16)
    assert np.allclose(E, ref["E"], rtol=1e-9, atol=1e-13)


def test_sweep_propagation_invariant():
    # T - What_old = E @ UL  (App. B.2: W - What = E U, restricted to the group)
    k, g = 2, 24
    rng = np.random.default_rng(4)
    UL = _local_factor(g, 11)
    T = rng.standard_normal((9, g))
    c = rng.standard_normal((9, k + 1))
    code, What, E = orc.bitplane_sweep(T, UL, c, k)
    assert np.allclose(T - What, E @ UL, atol=1e-12)
    assert np.allclose(What, orc.reconstruct(code, c, k), atol=1e-14)


# ----------------------------------------------------------------- delta correction / selection
def test_delta_correction_identity_and_best_iterate():
    k, g, T_it = 2, 32, 6
    rng = np.random.default_rng(8)
    UL = _local_factor(g, 13)
    T = rng.standard_normal((20, g)) * 0.02
    trace = []
    res = orc.bpdq_group(T, UL, k, T_it, alpha=1e-4, trace=trace)
    assert len(trace) == T_it + 1
    for tr in trace[1:]:
        # App. B.3: after the correction, E' U_loc = T - What_new
        assert np.allclose(tr["E_corr"] @ UL, T - tr["What_new"], atol=1e-12)
        # and the uncorrected state belongs to the old block
        assert np.allclose(tr["E_sweep"] @ UL, T - tr["What_old"], atol=1e-12)
        # score is the local objective of App. B.1
        D = T - tr["What_new"]
        M = np.linalg.inv(UL.T @ UL)
        assert np.isclose(tr["score"], np.einsum("ri,ij,rj->", D, M, D), rtol=1e-9)
    scores = [tr["score"] for tr in trace]
    assert res["it"].max() == res["it"].min() == int(np.argmin(scores))
    assert np.isclose(res["score"], min(scores))
    assert np.allclose(res["E"] @ UL, T - res["What"], atol=1e-12)
    assert np.allclose(res["What"], orc.reconstruct(res["code"], res["coef"], k), atol=1e-14)


def test_per_row_selection_never_worse():
    k, g = 2, 32
    rng = np.random.default_rng(18)
    UL = _local_factor(g, 3)
    T = rng.standard_normal((30, g)) * 0.02
    a = orc.bpdq_group(T, UL, k, 5)
    b = orc.bpdq_group(T, UL, k, 5, select_per_row=True)
    assert b["score"].sum() <= a["score"] + 1e-15
    more = orc.bpdq_group(T, UL, k, 8)
    assert more["score"] <= a["score"] + 1e-15      # candidates are nested in T


# ----------------------------------------------------------------- brute force on tiny groups
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_bruteforce_global_optimum_tiny_group(seed):
    # enumerate all 4^g plane assignments, least-squares coefficients for each
    k, g = 2, 5
    rng = np.random.default_rng(seed)
    UL = _local_factor(g, 20 + seed)
    T = rng.standard_normal((3, g))
    A_metric = np.linalg.inv(UL).T
    res = orc.bpdq_group(T, UL, k, 10, alpha=0.0, select_per_row=True, decision_dtype=None)
    for r in range(3):
        y = A_metric @ T[r]
        best = np.inf
        for assign in itertools.product(range(4), repeat=g):
            a = np.array(assign)
            B_r = np.column_stack([np.ones(g), a & 1, (a >> 1) & 1]).astype(float)
            Y = A_metric @ B_r
            cc, *_ = np.linalg.lstsq(Y, y, rcond=None)
            best = min(best, float(np.sum((Y @ cc - y) ** 2)))
        assert res["score"][r] >= best - 1e-12      # a heuristic cannot beat the optimum
        # its coefficients are the least-squares optimum for its own planes
        a = res["code"][r]
        B_r = np.column_stack([np.ones(g), a & 1, (a >> 1) & 1]).astype(float)
        Y = A_metric @ B_r
        cc, *_ = np.linalg.lstsq(Y, y, rcond=None)
        assert np.isclose(res["score"][r], np.sum((Y @ cc - y) ** 2), rtol=1e-8, atol=1e-14)
        # and with 5 weights on 4 levels + 3 free coefficients the heuristic should
        # land within a small factor of the optimum
        assert res["score"][r] <= 50 * best + 1e-6


# ----------------------------------------------------------------- H = I special case
def _alternating_ls_euclid(t, k, iters):
    """Independent re-statement for the identity metric: MSB-plane start, then
    alternate nearest-level assignment and ordinary least squares; returns the
    per-iteration squared errors and final (code, coef)."""
    g = len(t)
    lo, hi = t.min(), t.max()
    Z = np.clip(np.rint((t - lo) / ((hi - lo) / 255.0)), 0, 255).astype(int)
    code = Z >> (8 - k)
    errs, states = [], []
    for it in range(iters + 1):
        if it > 0:
            lv = np.array([c[0] + sum(c[i] * ((cd >> (i - 1)) & 1) for i in range(1, k + 1))
                           for cd in range(1 << k)])
            code = np.array([int(np.argmin((x - lv) ** 2)) for x in t])
        A = np.column_stack([np.ones(g)] + [((code >> i) & 1).astype(float) for i in range(k)])
        c, *_ = np.linalg.lstsq(A, t, rcond=None)
        errs.append(float(np.sum((A @ c - t) ** 2)))
        states.append((code.copy(), c.copy()))
    return errs, states


@pytest.mark.parametrize("k", [2, 3])
def test_identity_hessian_reduces_to_plain_alternating_fit(k):
    g, iters = 32, 6
    rng = np.random.default_rng(30 + k)
    T = rng.standard_normal((12, g))
    UL = np.eye(g)
    trace = []
    res = orc.bpdq_group(T, UL, k, iters, alpha=0.0, select_per_row=True,
                         decision_dtype=None, trace=trace)
    for r in range(12):
        errs, states = _alternating_ls_euclid(T[r], k, iters)
        got = [tr["rowscore"][r] for tr in trace]
        assert np.allclose(got, errs, rtol=1e-9, atol=1e-14)
        # alternating minimisation cannot increase the error
        assert all(errs[i + 1] <= errs[i] + 1e-12 for i in range(iters))
        j = int(np.argmin(errs))
        assert res["it"][r] == j
        assert np.array_equal(res["code"][r], states[j][0])
        assert np.allclose(res["coef"][r], states[j][1], rtol=1e-8, atol=1e-12)
    # no propagation with a diagonal factor: E = T - What
    assert np.allclose(res["E"], T - res["What"], atol=1e-14)


# ----------------------------------------------------------------- variable grid <= uniform grid
@pytest.mark.parametrize("k,seed", [(2, 0), (2, 1), (3, 2)])
def test_variable_grid_not_worse_than_uniform_per_group(k, seed):
    # Prop. 1 (feasible-set inclusion): refitting the coefficients on the planes the
    # uniform sweep chose cannot increase the local objective.
    g = 32
    rng = np.random.default_rng(seed)
    UL = _local_factor(g, 40 + seed)
    T = rng.standard_t(4, size=(25, g)) * 0.02
    u = uni.uniform_group(T, UL, k)
    c = orc.fit_coefficients(u["code"], T, UL, k, alpha=0.0)
    E_var = orc.solve_right(T - orc.reconstruct(u["code"], c, k), UL)
    assert np.all(np.sum(E_var ** 2, axis=1) <= np.sum(u["E"] ** 2, axis=1) * (1 + 1e-12))


def test_uniform_frozen_group_is_the_uniform_grid_sweep():
    # the comparator entry point: same result as the plain uniform-grid GPTQ sweep
    k, g = 3, 32
    rng = np.random.default_rng(77)
    UL = _local_factor(g, 17)
    T = rng.standard_t(4, size=(30, g)) * 0.02
    T[7] = 0.125                                   # a flat row
    a = orc.uniform_frozen_group(T, UL, k, decision_dtype=None)
    b = uni.uniform_group(T, UL, k)
    assert np.array_equal(a["code"], b["code"])
    assert np.allclose(a["coef"], b["coef"], rtol=1e-15)
    assert np.allclose(a["What"], b["What"], rtol=1e-13, atol=1e-16)
    assert np.allclose(a["E"], b["E"], rtol=1e-9, atol=1e-13)
    assert np.all(a["code"][7] == 0)
