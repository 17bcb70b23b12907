"""Pins for the channel ordering around the pass (Sec. 4.1: channels sorted in descending order of
the Hessian diagonal; a group-preserving variant).  CPU only."""
import numpy as np

from oracle import bpdq_oracle as orc
from tests.test_oracle_layer import _tiny_problem


def test_descending_order_with_stable_ties():
    H = np.diag([3.0, 7.0, 3.0, 9.0, 7.0, 0.0])
    assert orc.channel_order(H).tolist() == [3, 1, 4, 0, 2, 5]
    rng = np.random.default_rng(0)
    d = rng.random(200)
    perm = orc.channel_order(np.diag(d))
    assert sorted(perm.tolist()) == list(range(200))            # a permutation
    assert np.all(np.diff(d[perm]) <= 0)                         # descending


def test_group_preserving_order_keeps_blocks_together():
    d = np.array([1.0, 1.0, 5.0, 0.5, 2.0, 2.0, 9.0, 0.0])      # block sums (g = 2): 2, 5.5, 4, 9
    perm = orc.channel_order(np.diag(d), group_size=2)
    assert perm.tolist() == [6, 7, 2, 3, 4, 5, 0, 1]
    # brute force: among all block orders this is the one with non-increasing sums, ties by index
    sums = d.reshape(4, 2).sum(axis=1)
    blocks = perm.reshape(4, 2)[:, 0] // 2
    assert np.all(np.diff(sums[blocks]) <= 0)
    assert orc.channel_order(np.diag(d), group_size=8).tolist() == list(range(8))


def test_pass_in_permuted_order_is_the_same_problem():
    # tr((W - What) Ht (W - What)^T) does not depend on the order of the channels: quantizing the
    # permuted problem and scattering What back gives a layer whose objective under the ORIGINAL
    # Ht equals the permuted pass's own sum of scores (App. B.2), and the sorted order puts the
    # largest diagonal first
    wl, W, X, H, U, dead = _tiny_problem()
    perm = orc.channel_order(H)
    assert np.all(np.diff(np.diag(H)[perm]) <= 0)
    Hp = H[np.ix_(perm, perm)]
    Up, deadp, info = orc.prepare(Hp, wl.damp)
    assert info == 0
    res = orc.quantize_layer(W[:, perm], Up, deadp, bits=2, group=32, block=64, refine_iters=3)
    What = np.empty_like(res["What"])
    What[:, perm] = res["What"]
    Ht = H + wl.damp * np.mean(np.diag(H)) * np.eye(H.shape[0])
    assert np.isclose(res["objective"], orc.layer_objective(W, What, Ht), rtol=1e-8)
    # identity permutation reproduces the plain pass bit for bit
    ident = np.arange(H.shape[0])
    a = orc.quantize_layer(W[:, ident], U, dead, 2, 32, 64, 3)
    b = orc.quantize_layer(W, U, dead, 2, 32, 64, 3)
    assert np.array_equal(a["code"], b["code"]) and np.array_equal(a["coef"], b["coef"])
