"""GPU parity on the five workloads of the benchmark definition, all at FULL size.

* The benchmark workload (Qwen2.5-7B-shaped attention projection, 3584 x 3584, 262144
  tokens) runs in the launch configuration bench.py times (one Hessian call over all
  tokens), against the full oracle, with the oracle's decisions in fp32 (the kernel's type) and,
  as an independent figure, in fp64; a teacher-forced comparison of sampled groups follows.
* The 7B up/gate projection (18944 x 3584) and the 72B attention projection (8192 x 8192) run
  the whole pass on both sides as well.
* The two widest layers (3584 x 18944 and 8192 x 29568) would need ten minutes of host fp64
  work for a full oracle pass; they are compared stage by stage instead, every stage at full
  size on the GPU: the Hessian over all 262144 tokens on sampled sub-matrices the oracle
  computes exactly; U through its defining property on sampled columns and against the oracle
  on the trailing corner (which depends only on the trailing block of H); the sweep of the FULL
  layer against the oracle on sampled rows, both sides using the GPU's U, plus the identities
  that tie the outputs of all rows together (per-group errors, stored format).
* Scaled-down versions of the four (1/8 linear size) stay as quick cases with ragged tiles.
"""
import os
import time

import numpy as np
import pytest
import torch

from oracle import bpdq_oracle as orc
from paper_2602_04163_amd import binding as bq
from paper_2602_04163_amd import workloads as wk
from tests import parity_tools as pt

pytestmark = pytest.mark.gpu

H_TOL = 1e-5
OBJ_TOL = 1e-3
PLANE_TOL = 1e-3
FULL_ORACLE = os.environ.get("BPDQ_FULL_ORACLE", "0") == "1"   # whole-oracle runs of the two widest layers


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    bq.load()
    return torch.device("cuda:0")


def _log(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)


def _plane_bits_differing(code, ref_code, bits):
    nd = sum(int(np.sum(((code >> i) & 1) != ((ref_code >> i) & 1))) for i in range(bits))
    return nd / (bits * code.size)


def _teacher_forced_sample(wl, Wn, U64, code, coefs, grp_iter, rows, groups):
    """Sampled rows and groups of a finished layer against the oracle started from the layer's
    own group-start blocks (tests/parity_tools.py); the kept iterate is the layer's."""
    st = pt.teacher_forced(Wn[rows], U64, code[rows], coefs[:, rows], grp_iter, wl.bits, wl.group,
                           wl.refine_iters, float(np.float32(wl.alpha)), groups=groups,
                           force_selection=True)
    _log(f"{wl.name}: {pt.describe(st)}")
    assert st["mismatch_clear_rows"] == 0
    assert st["near_tie_rows"] <= 0.05 * st["rows"]
    assert st["coef_dev"] < 1e-3 and st["clear_score_rel"] < OBJ_TOL
    return st


def _end_to_end(dev, wl, tokens_per_call=0, hess=None, fp64_decisions=False, teacher=False):
    """Whole pass on both sides from the same seeded inputs; returns the parity numbers."""
    d_in = wl.d_in
    W = wk.make_weight(wl, device=dev)
    scales = wk.channel_scales(wl, device=dev)
    X = torch.empty((wl.n_tok, d_in), device=dev)
    for c in range(wk.n_chunks(wl)):
        wk.make_activation_chunk(wl, c, scales, device=dev, out=X[c * wl.chunk:(c + 1) * wl.chunk])
    # ---- GPU: every step inside the library
    H = torch.zeros((d_in, d_in), device=dev)
    per = tokens_per_call or wl.n_tok
    hess = hess or bq.bpdq_hessian_accumulate
    for a in range(0, wl.n_tok, per):
        b = min(a + per, wl.n_tok)
        hess(X[a:b], H, symmetrize=(b == wl.n_tok))
    U, dead, info = bq.bpdq_prepare(H, wl.damp)
    p = bq.make_params(wl.bits, wl.group, wl.block, wl.refine_iters, wl.alpha)
    out = bq.bpdq_quantize_layer(W, U, dead, p)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    _log(f"{wl.name}: gpu pass done")
    # ---- oracle on the same buffers
    Href = np.zeros((d_in, d_in))
    last = [time.time()]
    for c in range(wk.n_chunks(wl)):
        orc.hessian_accumulate(X[c * wl.chunk:(c + 1) * wl.chunk].cpu().numpy(), Href)
        if time.time() - last[0] > 45:
            last[0] = time.time()
            _log(f"{wl.name}: oracle H at chunk {c + 1} of {wk.n_chunks(wl)}")
    _log(f"{wl.name}: oracle H done")
    Hg = H.cpu().numpy().astype(np.float64)
    h_err = float(np.linalg.norm(Hg - Href) / np.linalg.norm(Href))
    del Hg
    Uref, dead_ref, info_ref = orc.prepare(Href, wl.damp)
    assert info_ref == 0
    _log(f"{wl.name}: oracle prepare done")
    u_err = float(np.linalg.norm(U.cpu().numpy() - Uref) / np.linalg.norm(Uref))
    Wn = W.cpu().numpy()
    def progress(done, total):
        if time.time() - last[0] > 45:
            last[0] = time.time()
            _log(f"{wl.name}: oracle sweep at column {done} of {total}")

    ref = orc.quantize_layer(Wn, Uref, dead_ref, wl.bits, wl.group, wl.block, wl.refine_iters,
                             alpha=float(np.float32(wl.alpha)), progress=progress)
    _log(f"{wl.name}: oracle sweep done")
    code = orc.unpack_planes(out["planes"].cpu().numpy().view(np.uint32), d_in)
    plane_frac = _plane_bits_differing(code, ref["code"], wl.bits)
    # the paper's layer objective ||WX - What X||^2 / ||WX||^2, via the undamped oracle H,
    # same scorer for both sides
    Wn64 = Wn.astype(np.float64)
    den = orc.layer_objective(Wn64, np.zeros_like(Wn64), Href)
    o_g = orc.layer_objective(Wn64, out["W_hat"].cpu().numpy(), Href) / den
    o_r = orc.layer_objective(Wn64, ref["What"], Href) / den
    it_same = float(np.mean(out["grp_iter"].cpu().numpy() == ref["grp_iter"]))
    err_sum_rel = abs(float(out["grp_err"].sum().item()) - ref["objective"]) / ref["objective"]
    _log(f"{wl.name}: H relFro {h_err:.2e} | U relFro {u_err:.2e} | plane bits differing "
         f"{plane_frac:.2e} | objective gpu {o_g:.6e} oracle {o_r:.6e} (rel {abs(o_g - o_r) / o_r:.2e}) "
         f"| sum grp_err rel {err_sum_rel:.2e} | kept-iterate agreement {it_same:.3f}")
    assert h_err < H_TOL
    assert plane_frac <= PLANE_TOL
    assert abs(o_g - o_r) / o_r <= OBJ_TOL
    assert err_sum_rel <= OBJ_TOL
    if fp64_decisions:
        # the independent figure: the oracle with every decision (8-bit code, nearest level)
        # taken in fp64, against the GPU, which takes them in fp32 -- same bars
        ref64 = orc.quantize_layer(Wn, Uref, dead_ref, wl.bits, wl.group, wl.block, wl.refine_iters,
                                   alpha=float(np.float32(wl.alpha)), decision_dtype=None,
                                   progress=progress)
        frac64 = _plane_bits_differing(code, ref64["code"], wl.bits)
        o_r64 = orc.layer_objective(Wn64, ref64["What"], Href) / den
        _log(f"{wl.name}: against fp64-decision oracle: plane bits differing {frac64:.2e} | objective "
             f"oracle {o_r64:.6e} (rel {abs(o_g - o_r64) / o_r64:.2e}) | oracle fp32 vs fp64 decisions: "
             f"plane bits {_plane_bits_differing(ref['code'], ref64['code'], wl.bits):.2e}")
        assert frac64 <= PLANE_TOL
        assert abs(o_g - o_r64) / o_r64 <= OBJ_TOL
    if teacher:
        n_grp = d_in // wl.group
        rows = np.arange(0, wl.d_out, max(1, wl.d_out // 448))[:448]
        groups = sorted({0, 1, n_grp // 3, (2 * n_grp) // 3, n_grp - 1})
        _teacher_forced_sample(wl, Wn64, U.cpu().numpy().astype(np.float64), code,
                               out["coefs"].cpu().numpy(), out["grp_iter"].cpu().numpy(), rows, groups)
    return dict(h_err=h_err, plane_frac=plane_frac, obj_gpu=o_g, obj_oracle=o_r)


HESSIANS = {"f16x2": bq.bpdq_hessian_accumulate, "bf16x3": bq.bpdq_hessian_accumulate_bf16x3,
            "f32": bq.bpdq_hessian_accumulate_f32}


@pytest.mark.parametrize("hess", ["f16x2", "bf16x3", "f32"])
def test_benchmark_workload_full_size(dev, hess):
    """configs[1]: 3584 x 3584, 262144 tokens, 2-bit, g = B = 128, 5 iterations; one Hessian
    call over all tokens, exactly as bench.py launches it (bench.py times bpdq_hessian_accumulate,
    the fp16-halves kernel; the bf16-pieces and fp32 matrix-core entries are the alternatives)."""
    fn = HESSIANS[hess]
    first = hess == "f16x2"
    _end_to_end(dev, wk.WORKLOADS["cfg2_qwen7b_attn"], hess=fn, fp64_decisions=first, teacher=first)


def test_benchmark_workload_chunked_hessian(dev):
    """Same layer shape with the Hessian streamed in 4096-token calls (fewer tokens so the
    oracle stays short)."""
    wl = wk.WORKLOADS["cfg2_qwen7b_attn"].scaled(n_tok=16384)
    for fn in HESSIANS.values():
        _end_to_end(dev, wl, tokens_per_call=4096, hess=fn)


SCALED = {
    # about 1/8 linear size (widths rounded to a multiple of the group), same distributions / bits / group / block / iterations
    "cfg3a_qwen7b_up": dict(d_out=2368, d_in=512, n_tok=8192),
    "cfg3b_qwen7b_down": dict(d_out=456, d_in=2432, n_tok=8192),
    "cfg4_qwen72b_attn": dict(d_out=1024, d_in=1024, n_tok=8192),
    "cfg5_qwen72b_down": dict(d_out=1024, d_in=3712, n_tok=8192),
}


@pytest.mark.parametrize("name", sorted(SCALED))
def test_other_workloads_scaled(dev, name):
    wl = wk.WORKLOADS[name].scaled(**SCALED[name])
    _end_to_end(dev, wl, tokens_per_call=4096)


@pytest.mark.parametrize("name", ["cfg3a_qwen7b_up", "cfg4_qwen72b_attn"])
def test_whole_pass_full_size(dev, name):
    """configs[2] (up/gate, 18944 x 3584, 3-bit) and configs[3] (8192 x 8192): the whole pass on
    both sides at full shape and token count, the Hessian streamed in 4096-token calls."""
    _end_to_end(dev, wk.WORKLOADS[name], tokens_per_call=4096, teacher=True)


if FULL_ORACLE:
    # ten minutes of host fp64 work per case: defined only on request (BPDQ_FULL_ORACLE=1); the
    # default run covers these two layers stage by stage (test_widest_layers_stage_by_stage)
    @pytest.mark.parametrize("name", ["cfg3b_qwen7b_down", "cfg5_qwen72b_down"])
    def test_widest_layers_whole_oracle(dev, name):
        _end_to_end(dev, wk.WORKLOADS[name], tokens_per_call=4096)


N_SAMPLED_CH = 96          # channels of the sampled sub-matrix of H
N_CORNER = 1024            # trailing corner of U compared with the oracle
N_SAMPLED_ROWS = 256       # rows of W the oracle sweeps


@pytest.mark.parametrize("name", ["cfg3b_qwen7b_down", "cfg5_qwen72b_down"])
def test_widest_layers_stage_by_stage(dev, name):
    """configs[2] (down, 3584 x 18944, 3-bit) and configs[4] (8192 x 29568, g = 64, T = 8) at full
    shape and token count on the GPU; every stage against what the oracle can compute of it."""
    wl = wk.WORKLOADS[name]
    d_in, d_out, g = wl.d_in, wl.d_out, wl.group
    scales = wk.channel_scales(wl, device=dev)
    gen = torch.Generator().manual_seed(5)
    idx = torch.randperm(d_in - N_CORNER, generator=gen)[:N_SAMPLED_CH].sort().values
    idx_d = idx.to(dev)
    corner = torch.arange(d_in - N_CORNER, d_in, device=dev)

    # ---- stage 1: H over all tokens, 4096-token calls (how the workload is stated)
    H = torch.zeros((d_in, d_in), device=dev)
    Hsub = np.zeros((N_SAMPLED_CH, N_SAMPLED_CH))
    Hcorner = np.zeros((N_CORNER, N_CORNER))
    diag = np.zeros(d_in)
    buf = torch.empty((wl.chunk, d_in), device=dev)
    nc = wk.n_chunks(wl)
    for c in range(nc):
        Xc = wk.make_activation_chunk(wl, c, scales, device=dev, out=buf)
        bq.bpdq_hessian_accumulate(Xc, H, symmetrize=(c == nc - 1))
        orc.hessian_accumulate(Xc[:, idx_d].cpu().numpy(), Hsub)
        orc.hessian_accumulate(Xc[:, corner].cpu().numpy(), Hcorner)
        x64 = Xc.double()
        diag += 2.0 * (x64 * x64).sum(dim=0).cpu().numpy()      # scorer-side fp64 diagonal (lambda)
        if c % 16 == 15:
            _log(f"{name}: Hessian chunk {c + 1} of {nc}")
    torch.cuda.synchronize()
    del buf
    Hg = H[idx_d][:, idx_d].cpu().numpy().astype(np.float64)
    h_sub = float(np.linalg.norm(Hg - Hsub) / np.linalg.norm(Hsub))
    Hgc = H[d_in - N_CORNER:, d_in - N_CORNER:].cpu().numpy().astype(np.float64)
    h_cor = float(np.linalg.norm(Hgc - Hcorner) / np.linalg.norm(Hcorner))
    d_err = float(np.linalg.norm(H.diagonal().cpu().numpy() - diag) / np.linalg.norm(diag))
    _log(f"{name}: H over {wl.n_tok} tokens: sampled {N_SAMPLED_CH}x{N_SAMPLED_CH} relFro {h_sub:.2e}, "
         f"trailing {N_CORNER}x{N_CORNER} relFro {h_cor:.2e}, diagonal rel {d_err:.2e}")
    assert h_sub < H_TOL and h_cor < H_TOL and d_err < H_TOL
    assert torch.equal(H[idx_d][:, corner], H[corner][:, idx_d].T)          # symmetrized

    # ---- stage 2: U at full width
    U, dead, info = bq.bpdq_prepare(H, wl.damp)
    torch.cuda.synchronize()
    assert int(info.item()) == 0 and not bool(dead.any())
    lam = wl.damp * float(H.diagonal().double().mean())
    # defining property (U^T U)(H + lambda I) = I on sampled columns, torch fp64 as the scorer
    cols = torch.cat([idx_d[::2], corner[::64]])
    Hc = H[:, cols].double()
    Hc[cols, torch.arange(len(cols), device=dev)] += lam
    U64d = U.double()
    R = U64d.T @ (U64d @ Hc)
    R[cols, torch.arange(len(cols), device=dev)] -= 1.0
    prop = float(R.abs().max())
    del Hc, R
    assert bool((U.tril(-1) == 0).all()) and bool((U.diagonal() > 0).all())
    # trailing corner: U[s:, s:] = chol_upper((Ht[s:, s:])^-1) depends only on that block of H; the
    # oracle gets its own fp64 block and the same lambda (damp rescaled to the block's mean diagonal)
    damp_c = wl.damp * float(np.mean(diag)) / float(np.mean(np.diag(Hcorner)))
    Uc_ref, _, info_c = orc.prepare(Hcorner, damp_c)
    assert info_c == 0
    Uc = U[d_in - N_CORNER:, d_in - N_CORNER:].cpu().numpy().astype(np.float64)
    u_cor = float(np.linalg.norm(Uc - Uc_ref) / np.linalg.norm(Uc_ref))
    _log(f"{name}: U: max |U^T U Ht - I| on {len(cols)} columns {prop:.2e}; trailing corner vs oracle "
         f"relFro {u_cor:.2e}")
    assert prop < 1e-5 and u_cor < 1e-5

    # ---- stages 3-4: the sweep of the full layer, as bench.py launches it
    W = wk.make_weight(wl, device=dev)
    p = bq.make_params(wl.bits, wl.group, wl.block, wl.refine_iters, wl.alpha)
    out = bq.bpdq_quantize_layer(W, U, dead, p)
    torch.cuda.synchronize()
    _log(f"{name}: gpu sweep done")
    # all rows: the stored format reproduces W_hat; per-group errors equal ||E_grp||_F^2 with
    # E = (W - What) U^-1 (App. B.2), evaluated in fp64 by torch -- 1 relative bar per group
    assert torch.equal(bq.bpdq_dequant(out["planes"], out["coefs"], g), out["W_hat"])
    D = (W.double() - out["W_hat"].double())
    E = torch.linalg.solve_triangular(U64d, D, upper=True, left=False)
    del D
    ge = (E * E).sum(dim=0).view(d_in // g, g).sum(dim=1)
    ge_rel = float(((out["grp_err"] - ge).abs() / ge).max())
    tot_rel = abs(float(out["grp_err"].sum()) - float(ge.sum())) / float(ge.sum())
    _log(f"{name}: per-group error identity: worst group rel {ge_rel:.2e}, layer rel {tot_rel:.2e}")
    assert ge_rel < OBJ_TOL and tot_rel < 1e-4
    del E, U64d
    it = out["grp_iter"].cpu().numpy()
    assert np.all(it >= 0) and np.all(it <= wl.refine_iters)
    # sampled rows: the oracle sweeps them over the FULL width with the GPU's U and the layer's kept
    # iterates (the group-wise choice needs all rows); end-to-end figures, then teacher-forced
    rows = np.arange(0, d_out, d_out // N_SAMPLED_ROWS)[:N_SAMPLED_ROWS]
    rows_d = torch.from_numpy(rows).to(dev)
    Wn = W[rows_d].cpu().numpy()
    Un = U.cpu().numpy().astype(np.float64)
    last = [time.time()]

    def progress(done, total):
        if time.time() - last[0] > 45:
            last[0] = time.time()
            _log(f"{name}: oracle sweep at column {done} of {total}")

    ref = orc.quantize_layer(Wn, Un, None, wl.bits, g, wl.block, wl.refine_iters,
                             alpha=float(np.float32(wl.alpha)), forced_iter=it, progress=progress)
    _log(f"{name}: oracle sweep of {len(rows)} sampled rows done")
    code = orc.unpack_planes(out["planes"][:, rows_d].cpu().numpy().view(np.uint32), d_in)
    frac = _plane_bits_differing(code, ref["code"], wl.bits)
    What_g = out["W_hat"][rows_d].cpu().numpy().astype(np.float64)
    # objective of the sampled rows in the damped metric (= sum of E^2, App. B.2), both sides
    Eg = pt.propagation_coordinates(Wn, What_g, Un)
    o_g, o_r = float(np.sum(Eg * Eg)), ref["objective"]
    same_rows = float(np.mean((code == ref["code"]).all(axis=1)))
    _log(f"{name}: sampled rows end to end: plane bits differing {frac:.2e} | objective gpu {o_g:.6e} "
         f"oracle {o_r:.6e} (rel {abs(o_g - o_r) / o_r:.2e}) | rows identical over the full width {same_rows:.3f}")
    assert frac <= PLANE_TOL
    assert abs(o_g - o_r) / o_r <= OBJ_TOL
    n_grp = d_in // g
    groups = sorted({0, 1, 2, n_grp // 4, n_grp // 2, (3 * n_grp) // 4, n_grp - 2, n_grp - 1})
    _teacher_forced_sample(wl, Wn.astype(np.float64), Un, code, out["coefs"][:, rows_d].cpu().numpy(),
                           it, np.arange(len(rows)), groups)
