"""Teacher-forced comparison of a quantized layer against the oracle (test helper, no test in it).

End to end, one flipped near-tie in an early group changes the working weights of every later
group of that row, so two correct implementations drift apart row by row.  The teacher-forced
check removes that cascade: for every checked group the oracle starts from the *other side's own*
group-start working block and solves just that group, so a difference can only come from a
decision taken inside the group.

The group-start block is not an output of the pass, but it follows from the outputs: the pass
keeps W - What = E U for the columns done so far (App. B.2 of the paper), hence
    E = (W - What) U^-1            (one triangular solve, fp64)
    T_s = W[:, s:s+g] - E[:, :s] U[:s, s:s+g]       (Eq. 4 applied to everything before s)
Both are evaluated here with scipy / numpy in fp64 -- neither side's code.

Rows are sorted into two classes by the oracle's own margins (bpdq_oracle.init_codes,
bitplane_sweep): a row is a "near-tie row" of a group when some decision of the oracle for it
was closer to a tie than `tie_tol` times the largest magnitude of the row's group-start
weights.  The fp32 state of the GPU differs from the exact state by rounding of the block
updates (a few 2^-24 per update, random sign, tens to hundreds of updates: about 1e-6 of the
row's magnitude), so with tie_tol = 1e-5 a row that is not a near-tie row has no decision the
GPU may legitimately take differently: its planes must be identical and its coefficients agree
to rounding.  Near-tie rows are counted and reported separately.  With 16-bit coefficient storage
the rounding of a fitted coefficient to a half is one more decision: a row is also a near-tie row
when a coefficient lay within `COEF_TIE_TOL` (relative to the row's largest coefficient; the
GPU's fitted coefficients deviate from the exact ones by about that) of the boundary between two
halves -- the other half would move every level of the next bit-plane update by 2^-11.  The
GPU's fitted coefficients are less exact than its weights (fp32 solves over the whole group feed
the normal equations), so a flip of that rounding can also hit a row outside the flagged ones; such
a row is accepted only if it is a valid result in its own right: its stored coefficients are the
oracle's fit on the row's OWN planes, each within one half-precision step, and its error is close
to the oracle row's.  These rows are counted (`rounding_flip_rows`).
"""
import numpy as np
from scipy.linalg import solve_triangular

from oracle import bpdq_oracle as orc

TIE_TOL = 1e-5
COEF_TIE_TOL = 1e-5


def propagation_coordinates(W, What, U):
    """E with W - What = E U (U upper triangular), fp64."""
    D = np.asarray(W, dtype=np.float64) - np.asarray(What, dtype=np.float64)
    return solve_triangular(np.asarray(U, dtype=np.float64).T, D.T, lower=True).T


def group_start_block(W, E, U, s, g):
    """Working weights of columns [s, s+g) after the compensation of all columns before s."""
    return np.asarray(W[:, s:s + g], dtype=np.float64) - E[:, :s] @ np.asarray(U[:s, s:s + g], dtype=np.float64)


def teacher_forced(W, U, code, coef, grp_iter, bits, group, iters, alpha, What=None, groups=None,
                   force_selection=False, coef_dtype=None, uniform=False, tie_tol=TIE_TOL,
                   decision_dtype=np.float32):
    """Compare the layer (code uint8 d_out x d_in, coef (k+1, d_out, d_in/g), grp_iter (d_in/g))
    with the oracle group by group, each group started from the layer's own group-start block.

    W must already have its dead columns zeroed.  `groups` restricts the comparison to some
    groups.  With `force_selection` the kept iterate of every group is taken from grp_iter: for
    rows sampled from a larger layer, which cannot reproduce the group-wise choice on their own.
    Returns a dict of counts and the largest deviations."""
    W = np.asarray(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    d_out, d_in = W.shape
    k, g = bits, group
    if What is None:
        What = np.repeat(coef[0].astype(np.float64), g, axis=1)
        for i in range(1, k + 1):
            What = What + np.repeat(coef[i].astype(np.float64), g, axis=1) * ((code >> (i - 1)) & 1)
    E = propagation_coordinates(W, What, U)
    ridx = np.arange(d_out)
    glist = range(d_in // g) if groups is None else groups
    st = dict(groups=0, rows=0, near_tie_rows=0, mismatch_rows=0, mismatch_clear_rows=0,
              selection_differs=0, selection_gap=0.0, coef_dev=0.0, clear_score_rel=0.0,
              bits_differing_clear=0, bits_total_clear=0,
              rounding_flip_rows=0,
              near_tie_row_set=np.zeros(d_out, dtype=bool), mismatch_row_set=np.zeros(d_out, dtype=bool))
    for gi in glist:
        s = gi * g
        T = group_start_block(W[ridx], E[ridx], U, s, g)
        UL = U[s:s + g, s:s + g]
        margins = np.full(len(ridx), np.inf)
        cmarg = np.full(len(ridx), np.inf)
        if uniform:
            res = orc.uniform_frozen_group(T, UL, k, decision_dtype, coef_dtype, margins, cmarg)
            it_o = 0
        else:
            forced = int(grp_iter[gi]) if force_selection else None
            res = orc.bpdq_group(T, UL, k, iters, alpha, False, decision_dtype, coef_dtype=coef_dtype,
                                 margins=margins, forced_iter=forced, coef_margins=cmarg)
            it_o = int(np.max(res["it"]))
            if it_o != int(grp_iter[gi]):
                # the other side kept another iterate: legitimate only if the two scores tie
                sc = res["scores"]
                st["selection_differs"] += 1
                st["selection_gap"] = max(st["selection_gap"],
                                          abs(sc[it_o] - sc[int(grp_iter[gi])]) / sc[it_o])
                margins = np.full(len(ridx), np.inf)
                cmarg = np.full(len(ridx), np.inf)
                res = orc.bpdq_group(T, UL, k, iters, alpha, False, decision_dtype,
                                     coef_dtype=coef_dtype, margins=margins,
                                     forced_iter=int(grp_iter[gi]), coef_margins=cmarg)
        scale = np.abs(T).max(axis=1)
        near = (margins <= tie_tol * scale) | (cmarg <= COEF_TIE_TOL)
        cg = code[ridx, s:s + g]
        differ = (cg != res["code"]).any(axis=1)
        clear = ~near
        odd = differ & clear
        if coef_dtype is not None and odd.any() and not uniform:
            # 16-bit storage: is the row the consistent result of another rounding of a coefficient?
            c_fit = orc.round_coefficients(orc.fit_coefficients(cg[odd], T[odd], UL, k, alpha), coef_dtype)
            c_g = coef[:, ridx, gi].T.astype(np.float64)[odd]
            r16 = c_fit.astype(coef_dtype)
            step = np.maximum(np.abs(np.nextafter(r16, coef_dtype(np.inf)).astype(np.float64) - c_fit),
                              np.abs(np.nextafter(r16, coef_dtype(-np.inf)).astype(np.float64) - c_fit))
            coef_ok = (np.abs(c_g - c_fit) <= step).all(axis=1)
            Eg = orc.solve_right(T[odd] - What[ridx][odd][:, s:s + g], UL)
            eg, eo = np.sum(Eg * Eg, axis=1), np.sum(res["E"][odd] ** 2, axis=1)
            err_ok = np.abs(eg - eo) <= 0.1 * eo
            valid = np.zeros(len(ridx), dtype=bool)
            valid[np.flatnonzero(odd)] = coef_ok & err_ok
            st["rounding_flip_rows"] += int(valid.sum())
            near = near | valid
            clear = ~near
        st["near_tie_row_set"] |= near
        st["mismatch_row_set"] |= differ
        st["groups"] += 1
        st["rows"] += len(ridx)
        st["near_tie_rows"] += int(near.sum())
        st["mismatch_rows"] += int(differ.sum())
        st["mismatch_clear_rows"] += int((differ & clear).sum())
        st["bits_differing_clear"] += sum(int(np.sum((((cg >> i) & 1) != ((res["code"] >> i) & 1))[clear]))
                                          for i in range(k))
        st["bits_total_clear"] += k * g * int(clear.sum())
        same = clear & ~differ
        if same.any():
            c_g = coef[:, ridx, gi].T.astype(np.float64)[same]
            c_o = np.asarray(res["coef"])[same]
            dev = np.abs(c_g - c_o) / (np.abs(c_o).max(axis=1, keepdims=True) + 1e-300)
            st["coef_dev"] = max(st["coef_dev"], float(dev.max()))
            # the group's error over the rows that must agree, from each side's own What
            Eg = orc.solve_right(T[same] - What[ridx][same][:, s:s + g], UL)
            sg, so = float(np.sum(Eg * Eg)), float(np.sum(res["E"][same] ** 2))
            if so > 0:
                st["clear_score_rel"] = max(st["clear_score_rel"], abs(sg - so) / so)
    return st


def end_to_end_rows(W, U, code, What, ref, st, obj_tol=1e-3):
    """End-to-end comparison of a layer with the oracle's free-running result `ref`, stated so that
    it holds for layers of any size: a row may differ from the oracle's only if teacher forcing
    (`st`, over ALL groups) found a near-tie in it -- its first differing decision is one -- or
    if the kept iterate of some group differs (scores tie); every other row has identical planes
    and the same error in the metric of U to `obj_tol`.  Returns (rows differing, rows allowed to)."""
    differ = (code != ref["code"]).any(axis=1)
    allowed = st["near_tie_row_set"].copy()
    if st["selection_differs"]:
        allowed[:] = True
    assert not np.any(differ & ~allowed), "rows differ from the oracle without a near-tie decision"
    same = ~differ
    if same.any():
        Eg = propagation_coordinates(np.asarray(W, dtype=np.float64)[same], np.asarray(What, dtype=np.float64)[same], U)
        Er = ref["E"][same]
        og, orf = float(np.sum(Eg * Eg)), float(np.sum(Er * Er))
        assert abs(og - orf) <= obj_tol * orf, (og, orf)
    return int(differ.sum()), int(allowed.sum())


def describe(st):
    return (f"teacher-forced: {st['groups']} groups, {st['rows']} (row, group) pairs; "
            f"near-tie {st['near_tie_rows']} ({st['near_tie_rows'] / max(st['rows'], 1):.2%}); "
            f"planes differ in {st['mismatch_rows']}, of which outside near-ties "
            f"{st['mismatch_clear_rows']} (+{st['rounding_flip_rows']} valid after another coefficient rounding); kept iterate differs in {st['selection_differs']} groups "
            f"(score gap {st['selection_gap']:.1e}); coefficient deviation {st['coef_dev']:.1e}; "
            f"score over agreeing rows rel {st['clear_score_rel']:.1e}")
