"""Pins for oracle steps 1-2 (Hessian, damping, U = chol(H^-1)) against closed forms,
brute force and an independent factorisation route.  CPU only."""
import numpy as np
import pytest

from oracle import bpdq_oracle as orc


def test_hessian_bruteforce_tiny():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((7, 5)).astype(np.float32)      # tokens x d_in
    H = np.zeros((5, 5))
    orc.hessian_accumulate(X, H)
    ref = [[2.0 * sum(float(X[t, i]) * float(X[t, j]) for t in range(7)) for j in range(5)]
           for i in range(5)]
    assert np.allclose(H, np.array(ref), rtol=1e-14, atol=1e-14)


def test_hessian_one_hot_closed_form():
    # each token activates one channel with amplitude a: H = 2 * diag(sum a^2)
    d = 6
    ch = np.array([0, 0, 3, 5, 5, 5, 1])
    amp = np.array([1.0, 2.0, 3.0, 0.5, 0.5, 1.0, 4.0])
    X = np.zeros((len(ch), d), dtype=np.float32)
    X[np.arange(len(ch)), ch] = amp
    H = np.zeros((d, d))
    orc.hessian_accumulate(X, H)
    want = np.zeros(d)
    np.add.at(want, ch, 2.0 * amp ** 2)
    assert np.array_equal(H, np.diag(want))


def test_hessian_chunks_add_and_scale():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((40, 9)).astype(np.float32)
    H1 = np.zeros((9, 9))
    orc.hessian_accumulate(X, H1, scale=1.0)
    H2 = np.zeros((9, 9))
    for c in range(4):
        orc.hessian_accumulate(X[10 * c:10 * c + 10], H2, scale=1.0)
    assert np.allclose(H1, H2, rtol=1e-13)
    assert np.allclose(H1, H1.T)
    # X X^T with X = d_in x N is the paper's form
    Xp = X.T.astype(np.float64)
    assert np.allclose(H1, Xp @ Xp.T, rtol=1e-13)
    H3 = np.zeros((9, 9))
    orc.hessian_accumulate(X, H3)            # default scale 2
    assert np.allclose(H3, 2 * H1)
    assert np.all(np.linalg.eigvalsh(H1) > -1e-9)


def _rand_spd(d, seed, cond_scale=1.0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((4 * d, d)) * np.exp(cond_scale * rng.standard_normal(d))
    return 2 * X.T @ X


def test_prepare_2x2_closed_form():
    a, b, c = 3.0, 1.0, 2.0
    H = np.array([[a, b], [b, c]])
    U, dead, info = orc.prepare(H, damp=0.0)
    det = a * c - b * b
    want = np.array([[np.sqrt(c / det), -b / np.sqrt(c * det)], [0.0, 1.0 / np.sqrt(c)]])
    assert info == 0 and not dead.any()
    assert np.allclose(U, want, rtol=1e-14)


def test_prepare_diagonal_closed_form():
    h = np.array([4.0, 1.0, 9.0, 16.0])
    damp = 0.01
    U, dead, info = orc.prepare(np.diag(h), damp)
    lam = damp * h.mean()
    assert np.allclose(U, np.diag(1.0 / np.sqrt(h + lam)), rtol=1e-14)


@pytest.mark.parametrize("d,seed", [(8, 0), (33, 1), (96, 2)])
def test_prepare_defining_properties(d, seed):
    H = _rand_spd(d, seed)
    damp = 0.01
    U, dead, info = orc.prepare(H, damp)
    assert info == 0
    Ht = H + damp * np.mean(np.diag(H)) * np.eye(d)
    assert np.allclose(U, np.triu(U))
    assert np.all(np.diag(U) > 0)
    assert np.allclose(U.T @ U @ Ht, np.eye(d), atol=1e-9)
    # independent route: Ht = R R^T with R upper (Cholesky of the index-reversed
    # matrix) gives U = R^-1
    J = np.eye(d)[::-1]
    Lf = np.linalg.cholesky(J @ Ht @ J)
    R = J @ Lf @ J
    assert np.allclose(R, np.triu(R))
    assert np.allclose(U, np.linalg.inv(R), rtol=1e-8, atol=1e-12)
    # trailing property: the factor of a trailing principal block is the
    # trailing block of the factor
    s = d // 3
    Us, _, _ = orc.prepare(Ht[s:, s:], 0.0)
    assert np.allclose(U[s:, s:], Us, rtol=1e-8, atol=1e-12)


def test_prepare_dead_channel_and_failure():
    H = _rand_spd(6, 3)
    H[2, :] = 0.0
    H[:, 2] = 0.0
    U, dead, info = orc.prepare(H, 0.01)
    assert info == 0
    assert dead.tolist() == [False, False, True, False, False, False]
    Hfix = H.copy()
    Hfix[2, 2] = 1.0
    Ht = Hfix + 0.01 * np.mean(np.diag(Hfix)) * np.eye(6)
    assert np.allclose(U.T @ U @ Ht, np.eye(6), atol=1e-10)
    # an indefinite matrix is reported, not factored
    Hbad = np.array([[1.0, 2.0], [2.0, 1.0]])
    _, _, info = orc.prepare(Hbad, 0.0)
    assert info != 0
