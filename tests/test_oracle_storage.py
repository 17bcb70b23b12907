"""Pins for the storage precision of the coefficients (fp16, the 16 bits per coefficient that
the BPW column of Table 1 counts).  The paper does not say when the rounding happens; the
oracle's reading (round right after every fit, so that everything downstream belongs to the
stored values) is pinned here to the identities that single it out.  CPU only."""
import numpy as np

from oracle import bpdq_oracle as orc
from tests.test_oracle_layer import _tiny_problem


def _fp16_exact(x):
    return np.array_equal(np.asarray(x, dtype=np.float64),
                          np.asarray(x).astype(np.float16).astype(np.float64))


def test_round_coefficients_is_round_to_nearest_even_fp16():
    # 1 + 2^-11 lies halfway between two fp16 neighbours: ties go to the even mantissa
    c = np.array([[1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 0.1, -65504.0, 1e-7]])
    r = orc.round_coefficients(c, np.float16)
    assert r[0, 0] == 1.0 and r[0, 1] == 1.0 + 2.0 ** -9
    assert abs(r[0, 2] - 0.1) <= 0.1 * 2.0 ** -11 and r[0, 3] == -65504.0
    assert r[0, 4] == 2 * 2.0 ** -24                      # subnormal grid of fp16: 2^-24
    assert orc.round_coefficients(c, None) is c


def test_stored_fp16_layer_is_self_consistent():
    # with fp16 storage the returned What, E and objective must all belong to the stored values:
    #   coefficients exactly representable; What = Eq. 1 of the stored format (bit for bit in
    #   fp64); W - What = E U; sum of group scores = tr((W-What) Ht (W-What)^T)  (App. B.2)
    wl, W, X, H, U, dead = _tiny_problem()
    res = orc.quantize_layer(W, U, dead, bits=3, group=32, block=64, refine_iters=3,
                             coef_dtype=np.float16)
    assert _fp16_exact(res["coef"])
    planes = orc.pack_planes(res["code"], 3)
    assert np.array_equal(orc.dequant(planes, res["coef"].astype(np.float16), 32), res["What"])
    Ht = H + wl.damp * np.mean(np.diag(H)) * np.eye(H.shape[0])
    assert np.allclose(W - res["What"], res["E"] @ U, atol=1e-10)
    assert np.isclose(res["objective"], orc.layer_objective(W, res["What"], Ht), rtol=1e-8)


def test_rounding_after_the_pass_breaks_the_identity_that_rounding_in_the_pass_keeps():
    # The alternative reading (quantize in full precision, round the stored coefficients
    # afterwards) returns scores that no longer describe the stored layer: its true objective
    # differs from the sum of its scores, and the compensation never saw the rounding.  The
    # reading taken pays for the rounding where it happens and stays close to full precision.
    wl, W, X, H, U, dead = _tiny_problem()
    Ht = H + wl.damp * np.mean(np.diag(H)) * np.eye(H.shape[0])
    full = orc.quantize_layer(W, U, dead, 2, 32, 64, 3)
    aware = orc.quantize_layer(W, U, dead, 2, 32, 64, 3, coef_dtype=np.float16)
    coef_post = orc.round_coefficients(full["coef"], np.float16)
    What_post = orc.dequant(orc.pack_planes(full["code"], 2), coef_post, 32)
    obj_post = orc.layer_objective(W, What_post, Ht)
    assert not np.isclose(obj_post, full["objective"], rtol=1e-9)        # identity broken
    assert np.isclose(aware["objective"], orc.layer_objective(W, aware["What"], Ht), rtol=1e-8)
    # fp16 keeps 11 significant bits: the objective moves by a small fraction either way
    assert abs(aware["objective"] / full["objective"] - 1) < 2e-2
    assert abs(obj_post / full["objective"] - 1) < 2e-2


def test_group_level_fp16_rounding_points():
    # one group: iterate 0 of the fp16 run has the planes of the full-precision run and exactly
    # its coefficients rounded; every later level table is built from rounded coefficients
    rng = np.random.default_rng(3)
    g, rows, k = 16, 6, 2
    A = rng.standard_normal((g, g))
    UL = np.triu(A @ A.T / g + np.eye(g))
    UL = np.triu(np.linalg.cholesky(np.linalg.inv(UL @ UL.T + np.eye(g))).T)
    T = rng.standard_normal((rows, g)) * 0.05
    tr_full, tr_h = [], []
    orc.bpdq_group(T, UL, k, 0, trace=tr_full)
    r0_full = orc.bpdq_group(T, UL, k, 0)
    r0_h = orc.bpdq_group(T, UL, k, 0, coef_dtype=np.float16)
    assert np.array_equal(r0_full["code"], r0_h["code"])
    assert np.array_equal(orc.round_coefficients(r0_full["coef"], np.float16), r0_h["coef"])
    assert np.allclose(T - orc.reconstruct(r0_h["code"], r0_h["coef"], k), r0_h["E"] @ UL, atol=1e-12)
    orc.bpdq_group(T, UL, k, 3, trace=tr_h, coef_dtype=np.float16)
    for rec in tr_h[1:]:
        assert _fp16_exact(rec["coef"])


def test_uniform_grid_with_fp16_storage_rounds_offset_and_step():
    rng = np.random.default_rng(4)
    g, rows, k = 16, 5, 3
    UL = np.triu(rng.standard_normal((g, g)) * 0.1) + np.eye(g)
    T = rng.standard_normal((rows, g))
    res = orc.uniform_frozen_group(T, UL, k, coef_dtype=np.float16)
    assert _fp16_exact(res["coef"])
    lo = T.min(axis=1)
    s = (T.max(axis=1) - lo) / 7.0
    expect = np.stack([lo, s, 2 * s, 4 * s], axis=1).astype(np.float32).astype(np.float16)
    assert np.array_equal(res["coef"], expect.astype(np.float64))
    assert np.allclose(T - res["What"], res["E"] @ UL, atol=1e-12)
