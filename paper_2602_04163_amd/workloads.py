"""Seeded synthetic inputs for the BPDQ per-layer quantization pass.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic.  Both the CPU oracle's tests and the GPU path's tests
consume the buffers made here, so the two sides always see identical inputs.

The five workloads stand in for the Qwen2.5-7B / Qwen2.5-72B linear layers and
the calibration activations the paper quantizes (Sec. 4.1): only shapes and
value distributions are imitated (heavy-tailed weights, a few very loud input
channels), no real weights or text are involved.

Values depend on the device the generator runs on (torch's CPU and GPU
generators are different streams); a test always generates once and hands the
same tensors to both sides.
"""
from __future__ import annotations

import dataclasses
import math

import torch

_BASE_SEED = 26020416


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int            # used in the seed
    d_out: int
    d_in: int
    n_tok: int
    chunk: int            # tokens per Hessian chunk
    bits: int
    group: int
    block: int
    refine_iters: int
    damp: float = 0.01
    alpha: float = 1e-4
    # weights
    w_kind: str = "student_t"   # "normal" | "student_t"
    w_nu: int = 4
    w_std: float = 0.02
    w_outlier_p: float = 0.0    # iid Bernoulli(p) mask ...
    w_outlier_x: float = 1.0    # ... entries multiplied by this
    # activations
    x_kind: str = "loud_channels"   # "loud_channels" | "lognormal"
    x_loud_frac: float = 0.01
    x_loud_x: float = 20.0
    x_sigma: float = 1.0

    @property
    def params(self) -> int:
        return self.d_out * self.d_in

    def seed(self, what: int) -> int:
        return _BASE_SEED + 1000 * self.index + what

    def scaled(self, **kw) -> "Workload":
        """Same distributions at another size (for parity cases between the
        tiny and the full configuration)."""
        return dataclasses.replace(self, **kw)


WORKLOADS = {
    "cfg1_tiny": Workload("cfg1_tiny", 1, 256, 256, 512, 512, 2, 64, 128, 3,
                          w_kind="normal", w_outlier_p=0.01, w_outlier_x=10.0,
                          x_kind="lognormal", x_sigma=1.0),
    "cfg2_qwen7b_attn": Workload("cfg2_qwen7b_attn", 2, 3584, 3584, 128 * 2048, 4096,
                                 2, 128, 128, 5),
    "cfg3a_qwen7b_up": Workload("cfg3a_qwen7b_up", 3, 18944, 3584, 262144, 4096,
                                3, 128, 128, 5, x_kind="lognormal", x_sigma=1.0),
    "cfg3b_qwen7b_down": Workload("cfg3b_qwen7b_down", 3, 3584, 18944, 262144, 4096,
                                  3, 128, 128, 5, x_kind="lognormal", x_sigma=1.0),
    "cfg4_qwen72b_attn": Workload("cfg4_qwen72b_attn", 4, 8192, 8192, 262144, 4096,
                                  2, 128, 128, 5, w_std=0.015),
    "cfg5_qwen72b_down": Workload("cfg5_qwen72b_down", 5, 8192, 29568, 262144, 4096,
                                  2, 64, 128, 8, w_nu=3, w_std=0.015,
                                  w_outlier_p=0.005, w_outlier_x=15.0,
                                  x_kind="lognormal", x_sigma=1.5),
}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_weight(wl: Workload, device="cpu") -> torch.Tensor:
    """W (d_out x d_in, fp32, row-major)."""
    g = _gen(wl.seed(1), device)
    shape = (wl.d_out, wl.d_in)
    z = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if wl.w_kind == "student_t":
        nu = wl.w_nu
        chi2 = torch.zeros(shape, device=device, dtype=torch.float32)
        for _ in range(nu):
            chi2 += torch.randn(shape, generator=g, device=device, dtype=torch.float32) ** 2
        z = z / torch.sqrt(chi2 / nu)
        # Student-t(nu) has variance nu/(nu-2): normalise with the theoretical value
        z = z * (wl.w_std * math.sqrt((nu - 2) / nu))
    elif wl.w_kind == "normal":
        z = z * wl.w_std
    else:
        raise ValueError(wl.w_kind)
    if wl.w_outlier_p > 0:
        g2 = _gen(wl.seed(2), device)
        mask = torch.rand(shape, generator=g2, device=device) < wl.w_outlier_p
        z = torch.where(mask, z * wl.w_outlier_x, z)
    return z.contiguous()


def channel_scales(wl: Workload, device="cpu") -> torch.Tensor:
    """Per-input-channel multipliers of the activations (d_in, fp32)."""
    g = _gen(wl.seed(3), device)
    if wl.x_kind == "lognormal":
        return torch.exp(wl.x_sigma * torch.randn(wl.d_in, generator=g, device=device,
                                                  dtype=torch.float32))
    if wl.x_kind == "loud_channels":
        n_loud = int(round(wl.x_loud_frac * wl.d_in))
        perm = torch.randperm(wl.d_in, generator=g, device=device)
        s = torch.ones(wl.d_in, device=device, dtype=torch.float32)
        s[perm[:n_loud]] = wl.x_loud_x
        return s
    raise ValueError(wl.x_kind)


def n_chunks(wl: Workload) -> int:
    return (wl.n_tok + wl.chunk - 1) // wl.chunk


def make_activation_chunk(wl: Workload, c: int, scales: torch.Tensor, device="cpu",
                          out: torch.Tensor | None = None) -> torch.Tensor:
    """Chunk c of the calibration activations, token-major: (tokens x d_in) fp32.
    This is the paper's X (d_in x N) stored column-major, one token per row."""
    n = min(wl.chunk, wl.n_tok - c * wl.chunk)
    g = _gen(wl.seed(100 + c), device)
    if out is None:
        out = torch.empty((n, wl.d_in), device=device, dtype=torch.float32)
    out = out[:n]
    out.normal_(generator=g)
    out.mul_(scales.to(device))
    return out
