"""CPU checks of the teacher-forced comparison (tests/parity_tools.py) and of the oracle's
instrumentation it relies on (decision margins, forced iterate): the tool must find nothing on
the oracle's own output, must find a planted flip, and its near-tie classification must cover
the only flips that a change of the decision precision can cause."""
import numpy as np

from oracle import bpdq_oracle as orc
from tests import parity_tools as pt


def _layer(seed, d_out=48, d_in=256, n_tok=1024):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((d_out, d_in)) * 0.02).astype(np.float32)
    X = (rng.standard_normal((n_tok, d_in)) * np.exp(rng.standard_normal(d_in))).astype(np.float32)
    H = np.zeros((d_in, d_in))
    orc.hessian_accumulate(X, H)
    U, dead, info = orc.prepare(H, 0.01)
    return W, U.astype(np.float32).astype(np.float64)


def test_margins_and_forced_iterate_leave_results_alone():
    W, U = _layer(1)
    T, UL = W[:, :64].astype(np.float64), U[:64, :64]
    a = orc.bpdq_group(T, UL, 2, 4)
    m = np.full(T.shape[0], np.inf)
    b = orc.bpdq_group(T, UL, 2, 4, margins=m)
    for key in ("code", "coef", "What", "E"):
        assert np.array_equal(a[key], b[key])
    assert np.all(m >= 0) and np.all(np.isfinite(m))
    assert len(b["scores"]) == 5 and np.argmin(b["scores"]) == int(np.max(b["it"]))
    # forcing iterate t returns exactly what the trace recorded for t
    trace = []
    orc.bpdq_group(T, UL, 2, 4, trace=trace)
    for t in (1, 3):
        f = orc.bpdq_group(T, UL, 2, 4, forced_iter=t)
        assert np.array_equal(f["code"], trace[t]["code"]) and np.all(f["it"] == t)
        assert np.allclose(f["E"], trace[t]["E_corr"], rtol=0, atol=0)


def test_sweep_margin_is_the_brute_force_gap():
    # one column, U_loc = 1: the margin is the gap between the two smallest |w - level|
    rng = np.random.default_rng(3)
    w = rng.standard_normal((200, 1))
    c = np.tile(np.array([[-1.0, 0.7, 1.6]]), (200, 1))
    m = np.full(200, np.inf)
    code, _, _ = orc.bitplane_sweep(w, np.ones((1, 1)), c, 2, None, m)
    levels = np.array([-1.0, -0.3, 0.6, 1.3])
    gaps = np.sort(np.abs(w - levels[None, :]), axis=1)
    assert np.allclose(m, gaps[:, 1] - gaps[:, 0], rtol=1e-12, atol=1e-15)
    assert np.array_equal(code[:, 0], np.argmin(np.abs(w - levels[None, :]), axis=1))
    # init: a weight exactly between two kept codes has margin zero
    t = np.array([[0.0, 255.0, 63.5, 10.0]])
    m = np.full(1, np.inf)
    orc.init_codes(t, 2, None, m)
    assert m[0] == 0.0


def test_tool_finds_nothing_on_the_oracles_own_output_and_finds_a_planted_flip():
    W, U = _layer(2)
    ref = orc.quantize_layer(W, U, None, 2, 64, 128, 3)
    Wd = W.astype(np.float64)
    E = pt.propagation_coordinates(Wd, ref["What"], U)
    assert np.allclose(E, ref["E"], rtol=0, atol=1e-9 * np.abs(ref["E"]).max())
    st = pt.teacher_forced(Wd, U, ref["code"], ref["coef"], ref["grp_iter"], 2, 64, 3, 1e-4,
                           What=ref["What"])
    assert st["groups"] == 4 and st["rows"] == 4 * 48
    assert st["mismatch_rows"] == 0 and st["selection_differs"] == 0
    assert st["coef_dev"] < 1e-9 and st["clear_score_rel"] < 1e-9
    # plant one flipped plane bit in group 2 (What kept: the group-start blocks stay the oracle's)
    code = ref["code"].copy()
    code[5, 130] ^= 1
    st = pt.teacher_forced(Wd, U, code, ref["coef"], ref["grp_iter"], 2, 64, 3, 1e-4, What=ref["What"])
    assert st["mismatch_rows"] == 1
    # a wrong kept iterate is reported as a selection difference with a visible score gap
    it = ref["grp_iter"].copy()
    it[1] = (it[1] + 1) % 4
    st = pt.teacher_forced(Wd, U, ref["code"], ref["coef"], it, 2, 64, 3, 1e-4, What=ref["What"])
    assert st["selection_differs"] == 1 and st["selection_gap"] > 1e-6


def test_near_tie_rows_cover_the_flips_of_a_decision_precision_change():
    """fp32 and fp64 decisions differ only where a decision is closer to a tie than fp32 rounding:
    every row whose planes differ between the two must be classified near-tie."""
    W, U = _layer(4, d_out=400, d_in=128)
    Wd = W.astype(np.float64)
    ref64 = orc.quantize_layer(W, U, None, 3, 128, 128, 5, decision_dtype=None)
    st = pt.teacher_forced(Wd, U, ref64["code"], ref64["coef"], ref64["grp_iter"], 3, 128, 5, 1e-4,
                           What=ref64["What"], decision_dtype=np.float32)
    assert st["mismatch_clear_rows"] == 0
    assert st["near_tie_rows"] < 0.1 * st["rows"]
