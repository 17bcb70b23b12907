"""CPU oracle for the BPDQ per-layer quantization pass.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the pass computes, written from the
paper (BPDQ: Bit-Plane Decomposition Quantization on a Variable Grid) so that a
reader can check it against the text by eye.  It shares no code with the GPU
library and must never be imported by it; only the tests, the smoke check and
the benchmark's `cpu_baseline` leg call it.

Every function names the passage it follows.  Library primitives used as steps:
matrix product, matrix inverse, Cholesky factorisation, triangular solve, small
dense solve.  There is no blocking or fusion beyond what the text states; loops
over rows are written as numpy batch operations because every formula of the
method is row-wise (App. B.1, B.2).

Precision.  State is fp64.  The two places where floating point decides an
integer -- the 8-bit round-to-nearest code of the initialisation and the
nearest-level choice of the bit-plane update -- are evaluated in `decision_dtype`
(default float32, the arithmetic type of the GPU path; the paper fixes none) on
operands rounded to that type, in the operation order written in `init_codes`
and `nearest_level`.  `decision_dtype=None` keeps them in fp64.

Readings of points the paper leaves open (all listed again in the design notes):
  * H = scale * X X^T with scale = 2 by default; no 1/N.  (Sec. 3.1 writes X X^T;
    the factor cancels in every output except the absolute objective.)
  * Hessian damping lambda = damp * mean(diag H) is added before inversion; the
    paper inherits it from GPTQ without writing it.             [parity unpinned]
  * Dead input channels (H_ii == 0): H_ii <- 1 and the weight column is zeroed.
  * The group's affine RTN (Sec. 3.2) sees the *working* block at group start,
    uses plain per-(row, group) min/max, round-half-even, hi == lo -> code 0.
                                                                [parity unpinned]
  * Kept planes: code = Z >> (8 - k); B_1 is the least significant kept bit,
    B_k the MSB (B_i = P_{7-k+i}).
  * The fit / refit target (Eq. 6) is the frozen group-start working block.
  * Ridge alpha acts on the (k+1)x(k+1) normal matrix, relative to its mean
    diagonal: G += alpha * tr(G)/(k+1) * I.                     [parity unpinned]
  * Every iteration restarts the sweep from the group-start block.
  * The initial state (iteration 0) is a candidate for the retained iterate;
    the score is ||E'||_F^2 after delta correction, summed over all rows; the
    earliest iterate wins ties.                                 [parity unpinned]
  * Nearest-level ties: the lowest code wins.
  * Effective lazy block = max(block, group).
"""
from __future__ import annotations

import numpy as np
from scipy.linalg import solve_triangular

__all__ = [
    "hessian_accumulate", "prepare", "init_codes", "design_matrix", "fit_coefficients",
    "level_table", "nearest_level", "bitplane_sweep", "reconstruct", "solve_right",
    "round_coefficients", "bpdq_group", "uniform_frozen_group", "quantize_layer", "pack_planes", "unpack_planes", "dequant",
    "layer_objective", "bits_per_weight", "channel_order", "gemv",
]


# --------------------------------------------------------------------------- #
# Step 1: Hessian  (Sec. 3.1, text under Eq. 2: H = X X^T)
# --------------------------------------------------------------------------- #
def hessian_accumulate(Xc, H, scale=2.0):
    """H += scale * Xc^T Xc for one chunk of tokens.

    Xc is (tokens x d_in): the paper's X (d_in x N) holds one token per column,
    so X X^T = sum over tokens of x x^T = Xc^T Xc.  H is fp64 (d_in x d_in) and is
    updated in place.
    """
    X64 = np.asarray(Xc, dtype=np.float64)
    H += scale * (X64.T @ X64)
    return H


# --------------------------------------------------------------------------- #
# Step 2: damping and U = chol(H^-1)  (Sec. 3.1, "Quantization Error Compensation")
# --------------------------------------------------------------------------- #
def prepare(H, damp=0.01):
    """Return (U, dead, info): U upper triangular with positive diagonal and
    (H + lambda I)^-1 = U^T U, written as its definition: invert, then factor.

    info = 0 on success, 1 if the damped matrix is not positive definite.
    """
    Ht = np.array(H, dtype=np.float64)
    d = Ht.shape[0]
    idx = np.arange(d)
    dead = Ht[idx, idx] == 0.0
    Ht[idx[dead], idx[dead]] = 1.0
    lam = damp * np.mean(Ht[idx, idx])
    Ht[idx, idx] += lam
    try:
        Hinv = np.linalg.inv(Ht)
        Hinv = 0.5 * (Hinv + Hinv.T)            # inverse of a symmetric matrix is symmetric
        L = np.linalg.cholesky(Hinv)            # Hinv = L L^T, L lower
    except np.linalg.LinAlgError:
        return np.zeros_like(Ht), dead, 1
    return np.ascontiguousarray(L.T), dead, 0   # U = L^T:  U^T U = L L^T = Hinv


# --------------------------------------------------------------------------- #
# Step 3a: bit-plane initialisation  (Sec. 3.2 "Bit-Plane Selection", Eq. 5)
# --------------------------------------------------------------------------- #
def init_codes(T, k, decision_dtype=np.float32, margins=None):
    """Per row: affine round-to-nearest of the group to Z in 0..255, keep the k
    most significant planes.  Returns code = Z >> (8-k) as uint8 (rows x g); bit
    (i-1) of code is plane B_i.
    Operation order (in decision_dtype): sc = (hi - lo) / 255; q = (t - lo) / sc;
    Z = clamp(round_half_even(q), 0, 255).
    `margins` (rows,), if given, is lowered to the smallest distance (in weight units) of any
    weight of the row from a rounding boundary that separates two kept codes (instrumentation
    for the parity tests: how close a decision came to a tie; the result does not depend on it)."""
    dt = np.float64 if decision_dtype is None else decision_dtype
    t = np.asarray(T).astype(dt)
    lo = t.min(axis=1, keepdims=True)
    hi = t.max(axis=1, keepdims=True)
    sc = (hi - lo) / dt(255.0)
    flat = (hi == lo)
    sc_safe = np.where(flat, dt(1.0), sc)
    q = (t - lo) / sc_safe
    Z = np.clip(np.rint(q), 0, 255).astype(np.int64)
    Z = np.where(flat, 0, Z)
    if margins is not None:
        step = 1 << (8 - k)                       # Z values per kept code
        bounds = np.arange(1, 1 << k) * step - 0.5
        dist = np.abs(q.astype(np.float64)[:, :, None] - bounds[None, None, :]).min(axis=(1, 2))
        dist = np.where(flat[:, 0], np.inf, dist * sc_safe[:, 0].astype(np.float64))
        np.minimum(margins, dist, out=margins)
    return (Z >> (8 - k)).astype(np.uint8)


def design_matrix(code, k):
    """B_r = [1, b_1, ..., b_k] for every row: (rows x g x (k+1)), fp64 (Sec. 3.2)."""
    rows, g = code.shape
    D = np.empty((rows, g, k + 1), dtype=np.float64)
    D[:, :, 0] = 1.0
    for i in range(1, k + 1):
        D[:, :, i] = (code >> (i - 1)) & 1
    return D


# --------------------------------------------------------------------------- #
# Step 3b/3d: coefficient fit  (Sec. 3.2 "Scalar Coefficient Fitting", Eq. 6; App. B.1)
# --------------------------------------------------------------------------- #
def fit_coefficients(code, T, UL, k, alpha=1e-4):
    """c_r = argmin_c || UL^-T (B_r c - t_r) ||^2 per row, with the ridge
    alpha * tr(G)/(k+1) on the diagonal of the normal matrix G = Y^T Y,
    Y = UL^-T B_r.  Returns (rows x (k+1)) fp64."""
    rows, g = code.shape
    D = design_matrix(code, k)                                   # rows x g x (k+1)
    # Y_r = UL^-T D_r : one triangular solve with all rows' columns side by side
    rhs = D.transpose(1, 0, 2).reshape(g, rows * (k + 1))
    Y = solve_triangular(UL.T, rhs, lower=True).reshape(g, rows, k + 1).transpose(1, 0, 2)
    y = solve_triangular(UL.T, np.asarray(T, dtype=np.float64).T, lower=True).T   # rows x g
    G = np.einsum("rgi,rgj->rij", Y, Y)
    b = np.einsum("rgi,rg->ri", Y, y)
    tr = np.einsum("rii->r", G)
    G = G + (alpha * tr / (k + 1))[:, None, None] * np.eye(k + 1)[None]
    return np.linalg.solve(G, b[:, :, None])[:, :, 0]


def round_coefficients(c, coef_dtype=None, margins=None):
    """Storage precision of the coefficients.  Table 1 counts 16 bits per coefficient; the
    paper does not say when the rounding happens.  Reading taken: with `coef_dtype=np.float16`
    every fitted coefficient is rounded (fp64 -> fp32 -> fp16, round to nearest even) right
    after the fit, so that the levels of the next bit-plane update, What, the propagation
    coordinates E and the score all belong to the values that are stored.  None = no rounding.
    `margins` (rows,), if given, is lowered to the smallest distance of any coefficient of the
    row from the boundary between two neighbouring storage values, relative to the row's largest
    coefficient magnitude (instrumentation for the parity tests: the rounding is a decision too)."""
    if coef_dtype is None:
        return c
    r = np.asarray(c).astype(np.float32).astype(coef_dtype)
    if margins is not None:
        c64 = np.asarray(c, dtype=np.float64)
        up = np.nextafter(r, coef_dtype(np.inf)).astype(np.float64)
        dn = np.nextafter(r, coef_dtype(-np.inf)).astype(np.float64)
        r64 = r.astype(np.float64)
        dist = np.minimum(np.abs(0.5 * (r64 + up) - c64), np.abs(0.5 * (r64 + dn) - c64))
        rel = dist.min(axis=1) / (np.abs(c64).max(axis=1) + 1e-300)
        np.minimum(margins, rel, out=margins)
    return r.astype(np.float64)


# --------------------------------------------------------------------------- #
# Step 3c: bit-plane update  (Sec. 3.3 "Bit-plane Update", Eq. 7-8; Eq. 3-4)
# --------------------------------------------------------------------------- #
def level_table(c, k, dtype=np.float64):
    """v_r(b) for all 2^k bit vectors (Eq. 7): (rows x 2^k).  Evaluated as
    ((c0 + b1 c1) + b2 c2) + ...  in `dtype` on coefficients rounded to it."""
    cc = np.asarray(c).astype(dtype)
    rows = cc.shape[0]
    lv = np.empty((rows, 1 << k), dtype=dtype)
    for code in range(1 << k):
        v = cc[:, 0].copy()
        for i in range(1, k + 1):
            if (code >> (i - 1)) & 1:
                v = v + cc[:, i]
        lv[:, code] = v
    return lv


def nearest_level(w, lv):
    """argmin over codes of (w - v(code))^2 (Eq. 8), lowest code on ties.
    w: (rows,), lv: (rows x 2^k), same dtype; the squared distance is formed in
    that dtype as diff = w - v; dist = diff * diff."""
    diff = w[:, None] - lv
    dist = diff * diff
    return np.argmin(dist, axis=1)          # first minimum = lowest code


def bitplane_sweep(T, UL, c, k, decision_dtype=np.float32, margins=None):
    """One column-by-column pass over a group with fixed coefficients c.
    Starts from the group-start working block T; at each column picks the
    nearest level per row, forms the error coordinate (Eq. 3) and compensates
    the remaining columns of the group (Eq. 4).
    Returns (code, What_old, E), each rows x g.
    `margins` (rows,), if given, is lowered to the smallest gap between the distances of the
    working weight to its nearest and to its second nearest *distinct* level value met in this
    pass (instrumentation for the parity tests; the result does not depend on it)."""
    T = np.asarray(T, dtype=np.float64)
    rows, g = T.shape
    Wg = T.copy()
    lv64 = level_table(c, k, np.float64)
    dt = np.float64 if decision_dtype is None else decision_dtype
    lvd = level_table(c, k, dt)
    code = np.zeros((rows, g), dtype=np.uint8)
    What = np.zeros((rows, g))
    E = np.zeros((rows, g))
    ar = np.arange(rows)
    for l in range(g):
        sel = nearest_level(Wg[:, l].astype(dt), lvd)
        code[:, l] = sel
        if margins is not None:
            gap = np.abs(Wg[:, l][:, None] - lv64)
            best = gap[ar, sel][:, None]
            other = np.where(lv64 != lv64[ar, sel][:, None], gap, np.inf).min(axis=1)
            np.minimum(margins, other - best[:, 0], out=margins)
        What[:, l] = lv64[ar, sel]
        E[:, l] = (Wg[:, l] - What[:, l]) / UL[l, l]
        Wg[:, l + 1:] -= np.outer(E[:, l], UL[l, l + 1:])
    return code, What, E


def reconstruct(code, c, k):
    """Group block of Eq. 1: What[r, j] = c_r0 + sum_i c_ri * b_i[r, j]."""
    return np.einsum("rgi,ri->rg", design_matrix(code, k), np.asarray(c, dtype=np.float64))


def solve_right(R, UL):
    """X with X @ UL = R (UL upper triangular), e.g. Eq. 9."""
    return solve_triangular(UL.T, np.asarray(R, dtype=np.float64).T, lower=True).T


# --------------------------------------------------------------------------- #
# Step 3 for one group: init, fit, iterate, keep the best iterate (Sec. 3.2, 3.3)
# --------------------------------------------------------------------------- #
def bpdq_group(T, UL, k, refine_iters, alpha=1e-4, select_per_row=False,
               decision_dtype=np.float32, trace=None, coef_dtype=None, margins=None,
               forced_iter=None, coef_margins=None):
    """Quantize one group given its group-start working block T (rows x g) and
    the local factor UL.  Returns dict(code, coef, What, E, score, it):
    E is the propagation coordinate block consistent with the returned What
    (T - What = E @ UL), score = ||E||_F^2 (scalar, or per row when
    select_per_row), it = index of the retained iterate (0 = initialisation).
    Test instrumentation: `margins` (rows,) collects the closest call of any decision of the
    row (see init_codes, bitplane_sweep), `coef_margins` (rows,) that of the coefficient
    roundings (see round_coefficients); `forced_iter` = t returns iterate t instead of the
    one with the smallest score (used when rows are sampled from a larger layer whose
    group-wise choice they cannot reproduce on their own); the scores of all iterates are
    returned as `scores`."""
    T = np.asarray(T, dtype=np.float64)
    rows, g = T.shape
    code = init_codes(T, k, decision_dtype, margins)
    c = round_coefficients(fit_coefficients(code, T, UL, k, alpha), coef_dtype, coef_margins)
    What = reconstruct(code, c, k)
    E = solve_right(T - What, UL)
    rs = np.sum(E * E, axis=1)
    best = dict(code=code, coef=c, What=What, E=E, rowscore=rs,
                it=np.zeros(rows, dtype=np.int32))
    scores = [float(rs.sum())]
    if trace is not None:
        trace.append(dict(it=0, score=float(rs.sum()), rowscore=rs.copy()))
    for t in range(1, refine_iters + 1):
        code_t, What_old, E_t = bitplane_sweep(T, UL, c, k, decision_dtype, margins)
        c = round_coefficients(fit_coefficients(code_t, T, UL, k, alpha), coef_dtype, coef_margins)  # refit, Sec. 3.3
        What_new = reconstruct(code_t, c, k)
        dE = solve_right(What_old - What_new, UL)                     # Eq. 9
        Ep = E_t + dE
        rs = np.sum(Ep * Ep, axis=1)
        if trace is not None:
            trace.append(dict(it=t, score=float(rs.sum()), rowscore=rs.copy(),
                              code=code_t.copy(), What_old=What_old, What_new=What_new,
                              E_sweep=E_t, E_corr=Ep, coef=c.copy()))
        scores.append(float(rs.sum()))
        if forced_iter is not None:
            take = np.full(rows, t == int(forced_iter))
        elif select_per_row:
            take = rs < best["rowscore"]
        else:
            take = np.full(rows, rs.sum() < best["rowscore"].sum())
        if take.any():
            for key, val in (("code", code_t), ("coef", c), ("What", What_new), ("E", Ep),
                             ("rowscore", rs)):
                best[key] = np.where(take.reshape((-1,) + (1,) * (val.ndim - 1)), val, best[key])
            best["it"] = np.where(take, t, best["it"]).astype(np.int32)
    best["score"] = best["rowscore"] if select_per_row else float(best["rowscore"].sum())
    best["scores"] = np.asarray(scores)
    return best


def uniform_frozen_group(T, UL, k, decision_dtype=np.float32, coef_dtype=None, margins=None,
                         coef_margins=None):
    """The fixed uniform grid written as a variable grid (App. A, Prop. 1): coefficients frozen
    to (lo, s, 2s, 4s, ...), s = (hi - lo) / (2^k - 1) from the group-start block's per-row
    min / max (a flat row gets s = 1), one bit-plane update pass, no fit, no iteration.  This is
    GPTQ on the asymmetric min/max grid; `uniform_gptq.uniform_group` states the same thing with
    round-to-nearest on the integer grid and the two are pinned to each other."""
    T = np.asarray(T, dtype=np.float64)
    lo = T.min(axis=1)
    hi = T.max(axis=1)
    s = (hi - lo) / float((1 << k) - 1)
    s = np.where(s == 0.0, 1.0, s)
    c = np.stack([lo] + [s * (1 << i) for i in range(k)], axis=1)
    c = round_coefficients(c, coef_dtype, coef_margins)
    code, What, E = bitplane_sweep(T, UL, c, k, decision_dtype, margins)
    return dict(code=code, coef=c, What=What, E=E, it=np.zeros(T.shape[0], dtype=np.int32))


# --------------------------------------------------------------------------- #
# Steps 3-4 for a layer: groups in GPTQ order with lazy block updates
# --------------------------------------------------------------------------- #
def quantize_layer(W, U, dead, bits, group, block, refine_iters, alpha=1e-4,
                   select_per_row=False, decision_dtype=np.float32, group_fn=None, progress=None,
                   coef_dtype=None, forced_iter=None):
    """Sweep the columns of W block by block (Sec. 3.1 compensation; App. B.3 tail
    form).  Returns dict with
      code   uint8  (d_out x d_in)     plane bits, bit (i-1) = B_i
      coef   fp64   (k+1, d_out, d_in/g)   C_0..C_k of Eq. 1
      What   fp64   (d_out x d_in)
      E      fp64   (d_out x d_in)     committed propagation coordinates
      grp_err fp64  (d_in/g)           ||E_group||_F^2 of the retained iterate
      grp_iter int32 (d_in/g) or (d_out, d_in/g) when select_per_row
      objective = sum grp_err  (= tr((W-What) Ht (W-What)^T), App. B.2)
    `group_fn(T, UL)` may replace the BPDQ group solver (used for the
    fixed-uniform-grid comparison of App. A).  `progress(b1, d_in)`, if given, is called after
    every block (long runs report where they are).  `forced_iter` (d_in/g ints), if given, fixes
    the retained iterate of every group (see bpdq_group)."""
    Wp = np.array(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    d_out, d_in = Wp.shape
    k, g = bits, group
    if d_in % g:
        raise ValueError("group must divide d_in")
    B = max(block, g)
    if B % g:
        raise ValueError("group must divide the block")
    if dead is not None:
        Wp[:, np.asarray(dead, dtype=bool)] = 0.0
    ngrp = d_in // g
    code = np.zeros((d_out, d_in), dtype=np.uint8)
    coef = np.zeros((k + 1, d_out, ngrp))
    What = np.zeros((d_out, d_in))
    Eall = np.zeros((d_out, d_in))
    grp_err = np.zeros(ngrp)
    grp_iter = np.zeros((d_out, ngrp) if select_per_row else ngrp, dtype=np.int32)
    forced = [None]
    if group_fn is None:
        def group_fn(T, UL):
            return bpdq_group(T, UL, k, refine_iters, alpha, select_per_row, decision_dtype,
                              coef_dtype=coef_dtype, forced_iter=forced[0])
    for b0 in range(0, d_in, B):
        b1 = min(b0 + B, d_in)
        for s in range(b0, b1, g):
            gi = s // g
            T = Wp[:, s:s + g].copy()
            UL = U[s:s + g, s:s + g]
            forced[0] = None if forced_iter is None else int(forced_iter[gi])
            res = group_fn(T, UL)
            code[:, s:s + g] = res["code"]
            coef[:, :, gi] = np.asarray(res["coef"]).T
            What[:, s:s + g] = res["What"]
            Eall[:, s:s + g] = res["E"]
            grp_err[gi] = np.sum(res["E"] ** 2)
            if select_per_row:
                grp_iter[:, gi] = res["it"]
            else:
                grp_iter[gi] = int(np.max(res["it"]))
            # rest of this block (only when g < B)
            Wp[:, s + g:b1] -= res["E"] @ U[s:s + g, s + g:b1]
        # lazy block update of everything to the right
        Wp[:, b1:] -= Eall[:, b0:b1] @ U[b0:b1, b1:]
        if progress is not None:
            progress(b1, d_in)
    return dict(code=code, coef=coef, What=What, E=Eall, grp_err=grp_err, grp_iter=grp_iter,
                objective=float(grp_err.sum()))


# --------------------------------------------------------------------------- #
# Storage format (Eq. 1; BPW column of Table 1)
# --------------------------------------------------------------------------- #
def pack_planes(code, bits):
    """planes[i-1, r, w] bit (c % 32) = B_i[r, c] for c = 32 w + (c % 32), LSB first."""
    d_out, d_in = code.shape
    if d_in % 32:
        raise ValueError("d_in must be a multiple of 32")
    out = np.zeros((bits, d_out, d_in // 32), dtype=np.uint32)
    for i in range(bits):
        b = ((code >> i) & 1).astype(np.uint32).reshape(d_out, d_in // 32, 32)
        for j in range(32):
            out[i] |= b[:, :, j] << np.uint32(j)
    return out


def unpack_planes(planes, d_in):
    bits, d_out, nw = planes.shape
    code = np.zeros((d_out, d_in), dtype=np.uint8)
    for i in range(bits):
        for j in range(32):
            code.reshape(d_out, nw, 32)[:, :, j] |= (((planes[i] >> np.uint32(j)) & 1) << i).astype(np.uint8)
    return code


def dequant(planes, coef, group):
    """What = REP(C_0) + sum_i REP(C_i) * B_i (Eq. 1) from the packed format, fp64."""
    bits, d_out, nw = planes.shape
    d_in = nw * 32
    code = unpack_planes(planes, d_in)
    What = np.repeat(np.asarray(coef[0], dtype=np.float64), group, axis=1)
    for i in range(1, bits + 1):
        What = What + np.repeat(np.asarray(coef[i], dtype=np.float64), group, axis=1) * ((code >> (i - 1)) & 1)
    return What


# --------------------------------------------------------------------------- #
# Channel ordering around the pass (Sec. 4.1)
# --------------------------------------------------------------------------- #
def channel_order(H, group_size=1):
    """Order in which the input channels are quantized.  Sec. 4.1: GPTQ's `desc_act` sorts the
    channels in descending order of the (approximate) Hessian values, i.e. of diag(H)
    (group_size = 1; equal values keep their index order).  The paper's own experiments use a
    group-preserving reordering that another paper defines; the stand-in offered here
    (group_size = g) keeps every block of g consecutive channels together and in order, and sorts
    the blocks by the descending sum of their diagonal entries (summed in fp64 in index order).
    Returns perm with perm[i] = original index of the channel at position i."""
    diag = np.asarray(np.diag(np.asarray(H)), dtype=np.float64)
    d = diag.shape[0]
    if d % group_size:
        raise ValueError("group_size must divide d_in")
    blocks = diag.reshape(d // group_size, group_size)
    key = np.zeros(d // group_size)
    for m in range(group_size):
        key = key + blocks[:, m]
    order = np.argsort(-key, kind="stable")
    return (order[:, None] * group_size + np.arange(group_size)[None, :]).reshape(-1).astype(np.int32)


def gemv(planes, coef, group, x):
    """y = What x for one token, from the stored format (Eq. 1, then a matrix-vector product),
    fp64: the serving-side use of a quantized layer (Sec. 5)."""
    return dequant(planes, coef, group) @ np.asarray(x, dtype=np.float64)


def bits_per_weight(bits, group, coef_bits=16):
    """k plane bits per weight plus (k+1) coefficients of coef_bits per group
    (BPW column of Table 1 with 16-bit coefficients)."""
    return bits + coef_bits * (bits + 1) / group


def layer_objective(W, What, H):
    """tr((W - What) H (W - What)^T) (Eq. 2) in fp64."""
    D = np.asarray(W, dtype=np.float64) - np.asarray(What, dtype=np.float64)
    return float(np.einsum("ij,ij->", D @ np.asarray(H, dtype=np.float64), D))
