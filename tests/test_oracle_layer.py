"""Pins for the oracle's layer pass (GPTQ-order sweep, lazy block update, storage
format) and for the paper's layer-level claims on the tiny workload.  CPU only."""
import os

import numpy as np
import pytest

from oracle import bpdq_oracle as orc
from oracle import uniform_gptq as uni
from paper_2602_04163_amd import workloads as wk


def _tiny_problem(d_out=48, d_in=96, n_tok=400, seed=0):
    wl = wk.WORKLOADS["cfg1_tiny"].scaled(d_out=d_out, d_in=d_in, n_tok=n_tok, chunk=n_tok)
    W = wk.make_weight(wl).numpy()
    s = wk.channel_scales(wl)
    X = wk.make_activation_chunk(wl, 0, s).numpy()
    H = np.zeros((d_in, d_in))
    orc.hessian_accumulate(X, H)
    U, dead, info = orc.prepare(H, wl.damp)
    assert info == 0
    return wl, W, X, H, U, dead


def test_layer_objective_identity_and_propagation_invariant():
    # App. B.2: L = tr((W-What) Ht (W-What)^T) = ||E||_F^2 and W - What = E U
    wl, W, X, H, U, dead = _tiny_problem()
    res = orc.quantize_layer(W, U, dead, bits=2, group=32, block=64, refine_iters=3)
    Ht = H + wl.damp * np.mean(np.diag(H)) * np.eye(H.shape[0])
    assert np.allclose(W - res["What"], res["E"] @ U, atol=1e-10)
    assert np.isclose(res["objective"], orc.layer_objective(W, res["What"], Ht), rtol=1e-8)
    assert np.isclose(res["objective"], np.sum(res["E"] ** 2), rtol=1e-12)
    # the H-form of the objective equals the output-space form of Eq. 2
    X64 = X.astype(np.float64)
    out_err = 2.0 * np.sum(((W - res["What"]) @ X64.T) ** 2)
    assert np.isclose(orc.layer_objective(W, res["What"], H), out_err, rtol=1e-9)
    # Eq. 1: the returned block is REP(C_0) + sum REP(C_i) * B_i
    g = 32
    Wrep = np.repeat(res["coef"][0], g, axis=1)
    for i in (1, 2):
        Wrep += np.repeat(res["coef"][i], g, axis=1) * ((res["code"] >> (i - 1)) & 1)
    assert np.allclose(Wrep, res["What"], atol=1e-14)


def test_lazy_block_size_does_not_change_the_result():
    wl, W, X, H, U, dead = _tiny_problem()
    a = orc.quantize_layer(W, U, dead, 2, 16, 16, 2)
    b = orc.quantize_layer(W, U, dead, 2, 16, 48, 2)
    c = orc.quantize_layer(W, U, dead, 2, 16, 96, 2)
    for other in (b, c):
        assert np.mean(a["code"] != other["code"]) < 1e-3
        assert np.isclose(a["objective"], other["objective"], rtol=1e-6)
    # block smaller than the group is widened to the group
    d = orc.quantize_layer(W, U, dead, 2, 32, 8, 2)
    e = orc.quantize_layer(W, U, dead, 2, 32, 32, 2)
    assert np.array_equal(d["code"], e["code"])


def test_hessian_scale_invariance_exact_for_powers_of_two():
    # H -> 4H gives U -> U/2 exactly; planes and coefficients must not move,
    # E doubles, the objective scales by 4.
    wl, W, X, H, U, dead = _tiny_problem()
    U4, _, _ = orc.prepare(4.0 * H, wl.damp)
    assert np.allclose(U4, U / 2, rtol=1e-12)
    a = orc.quantize_layer(W, U, dead, 2, 32, 32, 3)
    b = orc.quantize_layer(W, U / 2, dead, 2, 32, 32, 3)
    assert np.array_equal(a["code"], b["code"])
    assert np.allclose(a["coef"], b["coef"], rtol=1e-12, atol=1e-18)
    assert np.allclose(b["E"], 2 * a["E"], rtol=1e-10, atol=1e-18)
    assert np.isclose(b["objective"], 4 * a["objective"], rtol=1e-10)


def test_identity_hessian_layer_has_no_cross_talk():
    # H = I: no propagation and a zero block update, so every group is
    # quantised from the original weights alone
    rng = np.random.default_rng(5)
    W = rng.standard_normal((10, 64))
    U, dead, _ = orc.prepare(np.eye(64), 0.0)
    assert np.allclose(U, np.eye(64))
    res = orc.quantize_layer(W, U, dead, 2, 16, 32, 4, alpha=0.0)
    for gi in range(4):
        sl = slice(16 * gi, 16 * gi + 16)
        alone = orc.bpdq_group(W[:, sl], np.eye(16), 2, 4, alpha=0.0)
        assert np.array_equal(res["code"][:, sl], alone["code"])
        assert np.allclose(res["What"][:, sl], alone["What"], atol=1e-14)
    assert np.allclose(res["E"], W - res["What"], atol=1e-13)


def test_dead_channel_column_is_zeroed():
    wl, W, X, H, U, dead = _tiny_problem()
    X2 = X.copy()
    X2[:, 5] = 0.0
    H2 = np.zeros_like(H)
    orc.hessian_accumulate(X2, H2)
    U2, dead2, info = orc.prepare(H2, wl.damp)
    assert info == 0 and dead2[5] and dead2.sum() == 1
    res = orc.quantize_layer(W, U2, dead2, 2, 32, 32, 2)
    Wz = W.astype(np.float64).copy()
    Wz[:, 5] = 0.0
    assert np.allclose(Wz - res["What"], res["E"] @ U2, atol=1e-10)


@pytest.mark.parametrize("bits,group", [(2, 32), (3, 32)])
def test_bpdq_layer_beats_fixed_uniform_grid(bits, group):
    # the paper's central claim at layer level (App. A; Table 1 shows it at model
    # level): statistical for two greedy runs, so checked on the tiny workload only
    wl, W, X, H, U, dead = _tiny_problem(64, 128, 600)
    v = orc.quantize_layer(W, U, dead, bits, group, group, 5)
    u = orc.quantize_layer(W, U, dead, bits, group, group, 0,
                           group_fn=lambda T, UL: uni.uniform_group(T, UL, bits))
    assert v["objective"] < u["objective"]
    # the comparator obeys the same invariants
    assert np.allclose(W - u["What"], u["E"] @ U, atol=1e-10)


def test_refinement_helps_on_average():
    wl, W, X, H, U, dead = _tiny_problem(64, 128, 600)
    o0 = orc.quantize_layer(W, U, dead, 2, 32, 32, 0)["objective"]
    o5 = orc.quantize_layer(W, U, dead, 2, 32, 32, 5)["objective"]
    assert o5 < o0


# ----------------------------------------------------------------- storage format
def test_pack_layout_and_roundtrip():
    rng = np.random.default_rng(0)
    code = rng.integers(0, 8, size=(5, 96)).astype(np.uint8)
    planes = orc.pack_planes(code, 3)
    assert planes.shape == (3, 5, 3) and planes.dtype == np.uint32
    for (i, r, c) in [(0, 0, 0), (1, 2, 31), (2, 4, 32), (0, 3, 95), (2, 1, 63)]:
        assert (int(planes[i, r, c // 32]) >> (c % 32)) & 1 == (int(code[r, c]) >> i) & 1
    assert np.array_equal(orc.unpack_planes(planes, 96), code)
    one = np.zeros((1, 64), dtype=np.uint8)
    one[0, 33] = 2                                  # plane B_2, column 33
    p = orc.pack_planes(one, 2)
    assert p[0].sum() == 0 and p[1, 0, 0] == 0 and p[1, 0, 1] == 2


def test_dequant_matches_layer_output():
    wl, W, X, H, U, dead = _tiny_problem()
    res = orc.quantize_layer(W, U, dead, 2, 32, 32, 2)
    planes = orc.pack_planes(res["code"], 2)
    assert np.allclose(orc.dequant(planes, res["coef"], 32), res["What"], atol=1e-15)


def test_bits_per_weight_matches_table1(golden_dir):
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "bpw_table1.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 6
    for k, g, bpw in rows:
        k, g, bpw = int(k), int(g), float(bpw)
        assert abs(orc.bits_per_weight(k, g) - bpw) < 0.006          # printed to 2 decimals
        # the same number from the actual buffers: packed planes + fp16 coefficients
        d_out, d_in = 4, 4 * g
        planes = orc.pack_planes(np.zeros((d_out, d_in), dtype=np.uint8), k)
        n_coef = (k + 1) * d_out * (d_in // g)
        assert abs((planes.nbytes * 8 + 16 * n_coef) / (d_out * d_in) - bpw) < 0.006


def test_gemv_is_dequant_then_matvec():
    # the serving-side product from the stored format equals Eq. 1's What times x, and the
    # regrouped form  sum_G (C_0 S(G) + sum_i C_i sum_{c in G} b_i x_c)  written out by hand
    rng = np.random.default_rng(9)
    d_out, d_in, g, k = 5, 64, 32, 3
    code = rng.integers(0, 8, size=(d_out, d_in)).astype(np.uint8)
    coef = rng.standard_normal((k + 1, d_out, d_in // g))
    x = rng.standard_normal(d_in)
    planes = orc.pack_planes(code, k)
    y = orc.gemv(planes, coef, g, x)
    want = np.zeros(d_out)
    for r in range(d_out):
        for G in range(d_in // g):
            xs = x[G * g:(G + 1) * g]
            want[r] += coef[0, r, G] * xs.sum()
            for i in range(1, k + 1):
                b = (code[r, G * g:(G + 1) * g] >> (i - 1)) & 1
                want[r] += coef[i, r, G] * np.dot(b, xs)
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)
