"""Thin ctypes binding of libbpdq.so: same names as the C ABI (include/bpdq.h).

Only argument marshalling happens here: torch tensors supply device memory and the
current HIP stream; every step of the pass runs inside the library's kernels.  There is
no CPU fallback -- a missing library raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbpdq.so")
_lib = None

EXPORTS = [
    "bpdq_version",
    "bpdq_hessian_workspace_bytes", "bpdq_hessian_accumulate_f32", "bpdq_hessian_accumulate",
    "bpdq_hessian_accumulate_bf16x3", "bpdq_hessian_accumulate_timed",
    "bpdq_prepare_workspace_bytes", "bpdq_prepare",
    "bpdq_quantize_workspace_bytes", "bpdq_quantize_layer", "bpdq_quantize_layers", "bpdq_block_update",
    "bpdq_pack_planes", "bpdq_dequant", "bpdq_coefs_to_fp16", "bpdq_dequant_fp16",
    "bpdq_channel_order_workspace_bytes", "bpdq_channel_order", "bpdq_channel_order_noalloc",
    "bpdq_gather_columns",
    "bpdq_scatter_columns", "bpdq_gather_symmetric", "bpdq_gemv",
    "bpdq_probe_mfma", "bpdq_probe_copy",
]


class BpdqParams(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_int), ("group", ctypes.c_int), ("block", ctypes.c_int),
                ("refine_iters", ctypes.c_int), ("alpha", ctypes.c_float),
                ("grid", ctypes.c_int), ("coef_fp16", ctypes.c_int)]


class BpdqError(RuntimeError):
    pass


def load():
    """Load libbpdq.so (built by `python -m paper_2602_04163_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise BpdqError(f"{LIB_PATH} is missing: build it with "
                        "`python -m paper_2602_04163_amd.build` (there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    pp = ctypes.POINTER(BpdqParams)
    lib.bpdq_version.restype = ci
    lib.bpdq_version.argtypes = []
    lib.bpdq_hessian_workspace_bytes.restype = sz
    lib.bpdq_hessian_workspace_bytes.argtypes = [ci, ci]
    lib.bpdq_hessian_accumulate_f32.restype = ci
    lib.bpdq_hessian_accumulate_f32.argtypes = [vp, ci, ci, ci, cf, vp, ci, vp, sz, vp]
    for name in ("bpdq_hessian_accumulate", "bpdq_hessian_accumulate_bf16x3"):
        getattr(lib, name).restype = ci
        getattr(lib, name).argtypes = [vp, ci, ci, ci, cf, vp, ci, vp, sz, vp]
    lib.bpdq_hessian_accumulate_timed.restype = ci
    lib.bpdq_hessian_accumulate_timed.argtypes = [ci, vp, ci, ci, ci, cf, vp, ci, vp, sz, vp, vp, vp]
    lib.bpdq_prepare_workspace_bytes.restype = sz
    lib.bpdq_prepare_workspace_bytes.argtypes = [ci]
    lib.bpdq_prepare.restype = ci
    lib.bpdq_prepare.argtypes = [vp, ci, cf, vp, vp, vp, vp, sz, vp]
    lib.bpdq_quantize_workspace_bytes.restype = sz
    lib.bpdq_quantize_workspace_bytes.argtypes = [ci, ci, pp]
    lib.bpdq_quantize_layer.restype = ci
    lib.bpdq_quantize_layer.argtypes = [vp, ci, ci, vp, vp, pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.bpdq_quantize_layers.restype = ci
    lib.bpdq_quantize_layers.argtypes = [vp, ci, ci, vp, vp, pp, ci, ctypes.POINTER(ci), vp, vp, vp,
                                         vp, vp, vp, sz, vp]
    lib.bpdq_block_update.restype = ci
    lib.bpdq_block_update.argtypes = [vp, ci, ci, vp, ci, ci, vp, ci, ci, ci, ci, vp]
    lib.bpdq_pack_planes.restype = ci
    lib.bpdq_pack_planes.argtypes = [vp, ci, ci, ci, vp, vp]
    lib.bpdq_dequant.restype = ci
    lib.bpdq_dequant.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp]
    lib.bpdq_dequant_fp16.restype = ci
    lib.bpdq_dequant_fp16.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp]
    lib.bpdq_coefs_to_fp16.restype = ci
    lib.bpdq_coefs_to_fp16.argtypes = [vp, ctypes.c_long, vp, vp]
    lib.bpdq_gemv.restype = ci
    lib.bpdq_gemv.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, vp]
    lib.bpdq_channel_order_workspace_bytes.restype = sz
    lib.bpdq_channel_order_workspace_bytes.argtypes = [ci]
    lib.bpdq_channel_order.restype = ci
    lib.bpdq_channel_order.argtypes = [vp, ci, ci, vp, vp, sz, vp]
    lib.bpdq_channel_order_noalloc.restype = ci
    lib.bpdq_channel_order_noalloc.argtypes = [vp, ci, ci, vp, vp]
    lib.bpdq_gather_columns.restype = ci
    lib.bpdq_gather_columns.argtypes = [vp, ci, ci, vp, vp, vp]
    lib.bpdq_scatter_columns.restype = ci
    lib.bpdq_scatter_columns.argtypes = [vp, ci, ci, vp, vp, vp]
    lib.bpdq_gather_symmetric.restype = ci
    lib.bpdq_gather_symmetric.argtypes = [vp, ci, vp, vp, vp]
    lib.bpdq_probe_mfma.restype = ci
    lib.bpdq_probe_mfma.argtypes = [ci, ci, ci, ci, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.bpdq_probe_copy.restype = ci
    lib.bpdq_probe_copy.argtypes = [vp, vp, ctypes.c_long, vp]
    _lib = lib
    return lib


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _check(rc, name):
    if rc != 0:
        raise BpdqError(f"{name} returned {rc}" + (f" (argument {-rc} invalid)" if -99 < rc < 0 else ""))


def _dev(t, dtype, name):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise BpdqError(f"{name}: expected a contiguous {dtype} tensor on the GPU")


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def bpdq_version() -> int:
    return load().bpdq_version()


def bpdq_hessian_workspace_bytes(n_tok: int, d_in: int) -> int:
    return load().bpdq_hessian_workspace_bytes(n_tok, d_in)


def bpdq_hessian_accumulate(Xc, H, scale=2.0, symmetrize=False, ws=None, _entry="bpdq_hessian_accumulate"):
    """H += scale * Xc^T Xc (upper triangle; mirrored when symmetrize), on the fp16 matrix cores
    with two fp16 halves per channel-scaled value."""
    lib = load()
    _dev(H, torch.float32, "H")
    if not (Xc.is_cuda and Xc.dtype == torch.float32 and Xc.dim() == 2 and Xc.stride(1) == 1):
        raise BpdqError("Xc: expected a float32 GPU matrix with unit column stride")
    n_tok, d_in = Xc.shape
    if H.shape != (d_in, d_in):
        raise BpdqError("H: expected d_in x d_in")
    need = lib.bpdq_hessian_workspace_bytes(n_tok, d_in)
    if ws is None:
        ws = _workspace(need, H.device)
    rc = getattr(lib, _entry)(_ptr(Xc), n_tok, d_in, Xc.stride(0) if n_tok > 1 else d_in,
                              scale, _ptr(H), int(bool(symmetrize)), _ptr(ws), ws.numel(),
                              _stream())
    _check(rc, _entry)
    return H


def bpdq_hessian_accumulate_f32(Xc, H, scale=2.0, symmetrize=False, ws=None):
    """bpdq_hessian_accumulate on the fp32 matrix cores."""
    return bpdq_hessian_accumulate(Xc, H, scale, symmetrize, ws, _entry="bpdq_hessian_accumulate_f32")


def bpdq_hessian_accumulate_bf16x3(Xc, H, scale=2.0, symmetrize=False, ws=None):
    """bpdq_hessian_accumulate on the bf16 matrix cores, three bf16 pieces per value."""
    return bpdq_hessian_accumulate(Xc, H, scale, symmetrize, ws, _entry="bpdq_hessian_accumulate_bf16x3")


HESSIAN_KERNELS = {"f16x2": 0, "bf16x3": 1, "f32": 2}


def bpdq_hessian_accumulate_timed(kernel, Xc, H, scale=2.0, symmetrize=False, ws=None, ev_begin=None,
                                  ev_end=None):
    """bpdq_hessian_accumulate with the kernel chosen by name; ev_begin / ev_end are torch.cuda.Event
    objects (timing enabled, recorded at least once before so that they exist) that the library
    records right around the tile-product kernel."""
    lib = load()
    _dev(H, torch.float32, "H")
    n_tok, d_in = Xc.shape
    if ws is None:
        ws = _workspace(lib.bpdq_hessian_workspace_bytes(n_tok, d_in), H.device)
    ev = [ctypes.c_void_p(0 if e is None else e.cuda_event) for e in (ev_begin, ev_end)]
    rc = lib.bpdq_hessian_accumulate_timed(HESSIAN_KERNELS[kernel], _ptr(Xc), n_tok, d_in,
                                           Xc.stride(0) if n_tok > 1 else d_in, scale, _ptr(H),
                                           int(bool(symmetrize)), _ptr(ws), ws.numel(), _stream(), ev[0], ev[1])
    _check(rc, "bpdq_hessian_accumulate_timed")
    return H


def bpdq_prepare_workspace_bytes(d_in: int) -> int:
    return load().bpdq_prepare_workspace_bytes(d_in)


def bpdq_prepare(H, damp=0.01, U=None, ws=None):
    """Returns (U, dead, info): U = chol_upper((H + damp*mean(diag H) I)^-1)."""
    lib = load()
    _dev(H, torch.float32, "H")
    d_in = H.shape[0]
    if U is None:
        U = torch.empty_like(H)
    _dev(U, torch.float32, "U")
    dead = torch.empty(d_in, dtype=torch.uint8, device=H.device)
    info = torch.empty(1, dtype=torch.int32, device=H.device)
    if ws is None:
        ws = _workspace(lib.bpdq_prepare_workspace_bytes(d_in), H.device)
    rc = lib.bpdq_prepare(_ptr(H), d_in, damp, _ptr(U), _ptr(dead), _ptr(info), _ptr(ws),
                          ws.numel(), _stream())
    _check(rc, "bpdq_prepare")
    return U, dead, info


GRID_VARIABLE, GRID_UNIFORM = 0, 1


def make_params(bits, group, block, refine_iters, alpha=1e-4, grid=GRID_VARIABLE,
                coef_fp16=False) -> BpdqParams:
    return BpdqParams(bits, group, block, refine_iters, alpha, grid, int(bool(coef_fp16)))


def bpdq_quantize_workspace_bytes(d_out, d_in, params: BpdqParams) -> int:
    return load().bpdq_quantize_workspace_bytes(d_out, d_in, ctypes.byref(params))


def bpdq_quantize_layer(W, U, dead, params: BpdqParams, want_w_hat=True, ws=None, out=None):
    """Returns dict(planes, coefs, W_hat, grp_err, grp_iter) of device tensors."""
    lib = load()
    _dev(W, torch.float32, "W")
    _dev(U, torch.float32, "U")
    d_out, d_in = W.shape
    k, g = params.bits, params.group
    dev = W.device
    if out is None:
        out = dict(
            planes=torch.empty((k, d_out, d_in // 32), dtype=torch.int32, device=dev),
            coefs=torch.empty((k + 1, d_out, d_in // g), dtype=torch.float32, device=dev),
            W_hat=torch.empty((d_out, d_in), dtype=torch.float32, device=dev) if want_w_hat else None,
            grp_err=torch.empty(d_in // g, dtype=torch.float64, device=dev),
            grp_iter=torch.empty(d_in // g, dtype=torch.int32, device=dev),
        )
    if ws is None:
        need = lib.bpdq_quantize_workspace_bytes(d_out, d_in, ctypes.byref(params))
        if need == 0:
            raise BpdqError("bpdq_quantize_workspace_bytes: invalid parameters")
        ws = _workspace(need, dev)
    rc = lib.bpdq_quantize_layer(_ptr(W), d_out, d_in, _ptr(U), _ptr(dead), ctypes.byref(params),
                                 _ptr(out["planes"]), _ptr(out["coefs"]), _ptr(out["W_hat"]),
                                 _ptr(out["grp_err"]), _ptr(out["grp_iter"]), _ptr(ws), ws.numel(),
                                 _stream())
    _check(rc, "bpdq_quantize_layer")
    return out


def bpdq_quantize_layers(W, seg_end, U, dead, params: BpdqParams, want_w_hat=True, ws=None):
    """Layers sharing one U, stacked by rows (seg_end = ascending row boundaries).  Returns the
    same dict as bpdq_quantize_layer with grp_err / grp_iter of shape (n_seg, d_in/g)."""
    lib = load()
    _dev(W, torch.float32, "W")
    _dev(U, torch.float32, "U")
    d_out, d_in = W.shape
    k, g = params.bits, params.group
    dev = W.device
    n_seg = len(seg_end)
    out = dict(
        planes=torch.empty((k, d_out, d_in // 32), dtype=torch.int32, device=dev),
        coefs=torch.empty((k + 1, d_out, d_in // g), dtype=torch.float32, device=dev),
        W_hat=torch.empty((d_out, d_in), dtype=torch.float32, device=dev) if want_w_hat else None,
        grp_err=torch.empty((n_seg, d_in // g), dtype=torch.float64, device=dev),
        grp_iter=torch.empty((n_seg, d_in // g), dtype=torch.int32, device=dev),
    )
    if ws is None:
        need = lib.bpdq_quantize_workspace_bytes(d_out, d_in, ctypes.byref(params))
        if need == 0:
            raise BpdqError("bpdq_quantize_workspace_bytes: invalid parameters")
        ws = _workspace(need, dev)
    seg = (ctypes.c_int * n_seg)(*[int(e) for e in seg_end])
    rc = lib.bpdq_quantize_layers(_ptr(W), d_out, d_in, _ptr(U), _ptr(dead), ctypes.byref(params),
                                  n_seg, seg, _ptr(out["planes"]), _ptr(out["coefs"]),
                                  _ptr(out["W_hat"]), _ptr(out["grp_err"]), _ptr(out["grp_iter"]),
                                  _ptr(ws), ws.numel(), _stream())
    _check(rc, "bpdq_quantize_layers")
    return out


def bpdq_block_update(Et, U, k0, Wp, c_begin, c_end, d_out=None):
    """Wp[:, c_begin:c_end] -= Et^T U[k0:k0+Kd, c_begin:c_end] in place (Et: Kd x lde, K-major)."""
    lib = load()
    _dev(Et, torch.float32, "Et")
    _dev(U, torch.float32, "U")
    _dev(Wp, torch.float32, "Wp")
    Kd, lde = Et.shape
    d_out = Wp.shape[0] if d_out is None else d_out
    _check(lib.bpdq_block_update(_ptr(Et), lde, Kd, _ptr(U), U.shape[1], k0, _ptr(Wp), Wp.shape[1], d_out,
                                 c_begin, c_end, _stream()), "bpdq_block_update")
    return Wp


def bpdq_pack_planes(codes, bits):
    lib = load()
    _dev(codes, torch.uint8, "codes")
    d_out, d_in = codes.shape
    planes = torch.empty((bits, d_out, d_in // 32), dtype=torch.int32, device=codes.device)
    _check(lib.bpdq_pack_planes(_ptr(codes), d_out, d_in, bits, _ptr(planes), _stream()),
           "bpdq_pack_planes")
    return planes


def bpdq_dequant(planes, coefs, group):
    lib = load()
    _dev(planes, torch.int32, "planes")
    _dev(coefs, torch.float32, "coefs")
    bits, d_out, nw = planes.shape
    d_in = nw * 32
    W_hat = torch.empty((d_out, d_in), dtype=torch.float32, device=planes.device)
    _check(lib.bpdq_dequant(_ptr(planes), _ptr(coefs), d_out, d_in, bits, group, _ptr(W_hat),
                            _stream()), "bpdq_dequant")
    return W_hat


def bpdq_coefs_to_fp16(coefs):
    """Half-precision copy of the coefficients (same shape, torch.float16)."""
    lib = load()
    _dev(coefs, torch.float32, "coefs")
    out = torch.empty(coefs.shape, dtype=torch.float16, device=coefs.device)
    _check(lib.bpdq_coefs_to_fp16(_ptr(coefs), coefs.numel(), _ptr(out), _stream()),
           "bpdq_coefs_to_fp16")
    return out


def bpdq_dequant_fp16(planes, coefs_h, group):
    lib = load()
    _dev(planes, torch.int32, "planes")
    _dev(coefs_h, torch.float16, "coefs_h")
    bits, d_out, nw = planes.shape
    d_in = nw * 32
    W_hat = torch.empty((d_out, d_in), dtype=torch.float32, device=planes.device)
    _check(lib.bpdq_dequant_fp16(_ptr(planes), _ptr(coefs_h), d_out, d_in, bits, group, _ptr(W_hat),
                                 _stream()), "bpdq_dequant_fp16")
    return W_hat


def bpdq_channel_order(H, group_size=1):
    """perm (int32, d_in): channels by descending H_jj, or blocks of group_size channels by
    descending block sum."""
    lib = load()
    _dev(H, torch.float32, "H")
    d_in = H.shape[0]
    perm = torch.empty(d_in, dtype=torch.int32, device=H.device)
    ws = _workspace(lib.bpdq_channel_order_workspace_bytes(d_in), H.device)
    _check(lib.bpdq_channel_order(_ptr(H), d_in, group_size, _ptr(perm), _ptr(ws), ws.numel(),
                                  _stream()), "bpdq_channel_order")
    return perm


def bpdq_channel_order_noalloc(H, group_size=1, perm=None):
    """bpdq_channel_order without a workspace: the library's built-in scratch holds the keys.
    `perm` may be passed in, so that the call allocates nothing at all."""
    lib = load()
    _dev(H, torch.float32, "H")
    d_in = H.shape[0]
    if perm is None:
        perm = torch.empty(d_in, dtype=torch.int32, device=H.device)
    _dev(perm, torch.int32, "perm")
    _check(lib.bpdq_channel_order_noalloc(_ptr(H), d_in, group_size, _ptr(perm), _stream()),
           "bpdq_channel_order_noalloc")
    return perm


def bpdq_gather_columns(W, perm):
    lib = load()
    _dev(W, torch.float32, "W")
    _dev(perm, torch.int32, "perm")
    out = torch.empty_like(W)
    _check(lib.bpdq_gather_columns(_ptr(W), W.shape[0], W.shape[1], _ptr(perm), _ptr(out), _stream()),
           "bpdq_gather_columns")
    return out


def bpdq_scatter_columns(Wp, perm):
    lib = load()
    _dev(Wp, torch.float32, "Wp")
    _dev(perm, torch.int32, "perm")
    out = torch.empty_like(Wp)
    _check(lib.bpdq_scatter_columns(_ptr(Wp), Wp.shape[0], Wp.shape[1], _ptr(perm), _ptr(out),
                                    _stream()), "bpdq_scatter_columns")
    return out


def bpdq_gather_symmetric(H, perm):
    lib = load()
    _dev(H, torch.float32, "H")
    _dev(perm, torch.int32, "perm")
    out = torch.empty_like(H)
    _check(lib.bpdq_gather_symmetric(_ptr(H), H.shape[0], _ptr(perm), _ptr(out), _stream()),
           "bpdq_gather_symmetric")
    return out


def bpdq_gemv(planes, coefs_h, group, x, y=None):
    """y = What x for one token from the stored format (planes int32, coefficients float16)."""
    lib = load()
    _dev(planes, torch.int32, "planes")
    _dev(coefs_h, torch.float16, "coefs_h")
    _dev(x, torch.float32, "x")
    bits, d_out, nw = planes.shape
    d_in = nw * 32
    if x.numel() != d_in:
        raise BpdqError("x: expected d_in values")
    if y is None:
        y = torch.empty(d_out, dtype=torch.float32, device=planes.device)
    _check(lib.bpdq_gemv(_ptr(planes), _ptr(coefs_h), d_out, d_in, bits, group, _ptr(x), _ptr(y),
                         _stream()), "bpdq_gemv")
    return y


PROBE_KINDS = {"f32": 0, "bf16": 1, "f16": 2, "f64": 3, "i8": 4}
PROBE_DATA = {"zeros": 0, "ones": 1, "normal": 2}


def bpdq_probe_mfma(kind, data, waves_per_simd, groups, iters, out):
    """Enqueue one register-only matrix-core loop; returns the flops it performs."""
    lib = load()
    _dev(out, torch.float32, "out")
    if out.numel() < groups * 256 * waves_per_simd:
        raise BpdqError("out: too small")
    flops = ctypes.c_double(0.0)
    _check(lib.bpdq_probe_mfma(PROBE_KINDS[kind], PROBE_DATA[data], waves_per_simd, groups, iters,
                               _ptr(out), ctypes.byref(flops), _stream()), "bpdq_probe_mfma")
    return flops.value


def bpdq_probe_copy(src, dst):
    lib = load()
    _dev(src, torch.float32, "src")
    _dev(dst, torch.float32, "dst")
    _check(lib.bpdq_probe_copy(_ptr(src), _ptr(dst), min(src.numel(), dst.numel()), _stream()),
           "bpdq_probe_copy")
    return dst
