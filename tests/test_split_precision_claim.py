"""The arithmetic claim behind the split-precision Hessian kernel, checked on the CPU with numpy
(no GPU, none of the library's code): an fp32 value is the exact sum of three bf16 pieces up to
2^-24 of its magnitude, and the six piece products of weight >= 2^-16 reproduce an fp32 product
to within a few 2^-24 of it -- the rounding an fp32 multiply-add commits anyway."""
import numpy as np


def _bf16_rne(x):
    """float32 -> nearest bfloat16 (ties to even), returned as float32."""
    u = x.astype(np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def _pieces(x):
    h = _bf16_rne(x)
    r = (x - h).astype(np.float32)
    m = _bf16_rne(r)
    r2 = (r - m).astype(np.float32)
    l = _bf16_rne(r2)
    return h, m, l, r, r2


def test_three_bf16_pieces_reconstruct_an_fp32_value():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * np.exp(3.0 * rng.standard_normal(200000))).astype(np.float32)
    h, m, l, r, r2 = _pieces(x)
    x64 = x.astype(np.float64)
    # both residuals are exact in fp32
    assert np.array_equal(r.astype(np.float64), x64 - h.astype(np.float64))
    assert np.array_equal(r2.astype(np.float64), x64 - h.astype(np.float64) - m.astype(np.float64))
    err = np.abs(x64 - (h.astype(np.float64) + m.astype(np.float64) + l.astype(np.float64)))
    assert np.max(err / np.abs(x64)) <= 2.0 ** -24
    # values with at most 8 significant bits are their own first piece
    s = np.float32([1.0, -3.5, 255.0, 0.0078125, 1.9921875])
    hs, ms, ls, _, _ = _pieces(s)
    assert np.array_equal(hs, s) and not ms.any() and not ls.any()


def test_six_piece_products_match_the_fp32_product():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(200000) * np.exp(2.0 * rng.standard_normal(200000))).astype(np.float32)
    y = (rng.standard_normal(200000) * np.exp(2.0 * rng.standard_normal(200000))).astype(np.float32)
    hx, mx, lx, _, _ = (a.astype(np.float64) for a in _pieces(x))
    hy, my, ly, _, _ = (a.astype(np.float64) for a in _pieces(y))
    six = hx * hy + (hx * my + mx * hy) + (mx * my + hx * ly + lx * hy)
    exact = x.astype(np.float64) * y.astype(np.float64)
    rel = np.abs(six - exact) / np.abs(exact)
    assert np.max(rel) <= 3.0 * 2.0 ** -24
    # dropping the three terms of weight 2^-16 is visibly worse: they are needed
    three = hx * hy + (hx * my + mx * hy)
    assert np.max(np.abs(three - exact) / np.abs(exact)) > 2.0 ** -18
