"""Seeded synthetic inputs shaped like Visual-Mamba (Vim) linear-layer workloads.

This module only *draws inputs*: activations, weights, biases, and the
calibration-time parameters (smoothing vector ``m`` and per-token static steps
``s_tok``) that a quantized linear layer receives from the offline calibration
stage.  It contains none of the hot path's arithmetic (no rounding to integer
codes, no integer GEMM, no dequantization) and is the only code shared by the
CPU oracle's tests and the HIP path's tests/bench.

The distributions follow the paper's qualitative observations of Visual Mamba
activations (Sec. 4, Observations 1-3): a token-wise variance pattern that is the
same for every input, a fixed small set of outlier channels, and a long-tailed
value distribution.  They stand in for ImageNet-1K activations of pretrained
checkpoints, which are not available offline.

Calibration recipe (closed-form initialisers only; the learned JLSS stages of
Sec. 5.2 are out of scope):
  * smoothing vector, Eq. (smooth_scale) with alpha = 0.5 read per input channel:
    m[k] = sqrt(max|X[:, k]| / max|W[:, k]|) over the calibration set;
  * per-token static step (Sec. 5.1, min-max initialiser of Sec. 2.3):
    s_tok[t] = max over calibration samples and channels of |X[., t, k] / m[k]| / 127.
The evaluation batch is a fresh draw, so a small fraction of it exceeds the
calibrated range and exercises the clamp.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Tuple

import torch

# (name, K = D_in, N = D_out) per linear of one Vim block, in execution order.
_VIM = {
    "ti": dict(dim=192, d_inner=384, d_state=16, dt_rank=12),
    "s": dict(dim=384, d_inner=768, d_state=16, dt_rank=24),
    "b": dict(dim=768, d_inner=1536, d_state=16, dt_rank=48),
}


def _block_linears(size: str) -> List[Tuple[str, int, int]]:
    g = _VIM[size]
    return [
        ("in_proj", g["dim"], 2 * g["d_inner"]),
        ("x_proj", g["d_inner"], g["dt_rank"] + 2 * g["d_state"]),
        ("dt_proj", g["dt_rank"], g["d_inner"]),
        ("out_proj", g["d_inner"], g["dim"]),
    ]


@dataclasses.dataclass(frozen=True)
class WorkloadConfig:
    index: int
    name: str
    B: int
    L: int
    layers: int
    linears: Tuple[Tuple[str, int, int], ...]
    base: str            # "normal" | "laplace"
    outlier_frac: Optional[float]
    outlier_count: Optional[int]
    outlier_gain: float

    @property
    def M(self) -> int:
        return self.B * self.L


CONFIGS: Dict[int, WorkloadConfig] = {
    0: WorkloadConfig(0, "vim_ti_out_proj_single", 1, 197, 1, (("out_proj", 384, 192),),
                      "normal", None, 4, 20.0),
    1: WorkloadConfig(1, "vim_ti_stack_b64", 64, 197, 24, tuple(_block_linears("ti")),
                      "laplace", 0.01, None, 20.0),
    2: WorkloadConfig(2, "vim_s_stack_b128", 128, 197, 24, tuple(_block_linears("s")),
                      "laplace", 0.01, None, 20.0),
    3: WorkloadConfig(3, "vim_b_stack_b256", 256, 197, 24, tuple(_block_linears("b")),
                      "laplace", 0.01, None, 20.0),
    4: WorkloadConfig(4, "vim_s_long_l785_b64", 64, 785, 24, tuple(_block_linears("s")),
                      "laplace", 0.02, None, 50.0),
}

CALIB_BATCHES = 8
CALIB_BATCH_SIZE = 32
CLASS_TOKEN_GAIN = 8.0


def case_seed(cfg: int, layer: int, linear: int) -> int:
    return 20386 * 10_000 + cfg * 1000 + layer * 10 + linear


@dataclasses.dataclass
class LinearCase:
    """Everything one quantized linear receives. Tensors live on `device`."""
    cfg: int
    layer: int
    linear: int
    name: str
    B: int
    L: int
    K: int
    N: int
    x: torch.Tensor       # [B*L, K] fp16, evaluation batch
    w: torch.Tensor       # [N, K]   fp16, unsmoothed weight
    bias: torch.Tensor    # [N]      fp16
    m: torch.Tensor       # [K]      fp32 smoothing vector (> 0)
    s_tok: torch.Tensor   # [L]      fp32 per-token static step (> 0), calibrated on X / m
    clipped: int          # evaluation elements beyond the calibrated range


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _draw_base(shape, base: str, g: torch.Generator, device) -> torch.Tensor:
    if base == "normal":
        return torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    # Laplace(0, b=1) by inverse CDF of a uniform on (-1/2, 1/2)
    u = torch.rand(shape, generator=g, device=device, dtype=torch.float32) - 0.5
    return -torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp_(max=0.5 - 1e-7))


def _static_structure(c: WorkloadConfig, K: int, N: int, seed: int, device):
    """Per-(config, layer, linear) quantities that are the same for every input."""
    g = _gen(device, seed)
    sigma = torch.exp(0.5 * torch.randn(c.L, generator=g, device=device, dtype=torch.float32))
    sigma[0] *= CLASS_TOKEN_GAIN
    n_out = c.outlier_count if c.outlier_count is not None else max(1, round(c.outlier_frac * K))
    n_out = min(n_out, K)
    perm = torch.randperm(K, generator=g, device=device)
    gain = torch.ones(K, device=device, dtype=torch.float32)
    gain[perm[:n_out]] = c.outlier_gain
    w = (0.02 * torch.randn((N, K), generator=g, device=device, dtype=torch.float32)).to(torch.float16)
    bias = (0.01 * torch.randn(N, generator=g, device=device, dtype=torch.float32)).to(torch.float16)
    return sigma, gain, w, bias


def _draw_x(c: WorkloadConfig, nb: int, K: int, sigma, gain, seed: int, device) -> torch.Tensor:
    g = _gen(device, seed)
    z = _draw_base((nb, c.L, K), c.base, g, device)
    z *= sigma.view(1, c.L, 1)
    z *= gain.view(1, 1, K)
    return z.to(torch.float16)


def make_linear_case(cfg: int, layer: int = 0, linear: int = 0, device="cpu",
                     batch: Optional[int] = None) -> LinearCase:
    """Draw one linear's evaluation batch and its calibrated parameters.

    `batch` overrides the config's batch size for the evaluation draw (the
    calibration set is always CALIB_BATCHES x CALIB_BATCH_SIZE samples).
    """
    c = CONFIGS[cfg]
    name, K, N = c.linears[linear]
    B = c.B if batch is None else batch
    seed = case_seed(cfg, layer, linear)
    sigma, gain, w, bias = _static_structure(c, K, N, seed, device)

    xmax = torch.zeros(K, device=device, dtype=torch.float32)
    calib = []
    for j in range(CALIB_BATCHES):
        xc = _draw_x(c, CALIB_BATCH_SIZE, K, sigma, gain, seed + 1_000_000 * (j + 1), device)
        xmax = torch.maximum(xmax, xc.abs().amax(dim=(0, 1)).float())
        calib.append(xc if K * c.L * CALIB_BATCH_SIZE <= (1 << 26) else None)
    wmax = w.abs().amax(dim=0).float()
    m = torch.sqrt(xmax / wmax).clamp_(1e-5, 1e5)
    m = torch.where(torch.isfinite(m), m, torch.ones_like(m)).contiguous()

    tmax = torch.zeros(c.L, device=device, dtype=torch.float32)
    for j in range(CALIB_BATCHES):
        xc = calib[j]
        if xc is None:
            xc = _draw_x(c, CALIB_BATCH_SIZE, K, sigma, gain, seed + 1_000_000 * (j + 1), device)
        tmax = torch.maximum(tmax, (xc.float() / m.view(1, 1, K)).abs().amax(dim=(0, 2)))
    s_tok = (tmax / 127.0).clamp_(min=1e-30).contiguous()

    x3 = _draw_x(c, B, K, sigma, gain, seed + 9_000_000, device)
    clipped = int(((x3.float() / m.view(1, 1, K)).abs() > (127.5 * s_tok).view(1, c.L, 1)).sum().item())
    x = x3.reshape(B * c.L, K).contiguous()
    return LinearCase(cfg, layer, linear, name, B, c.L, K, N, x, w.contiguous(), bias.contiguous(),
                      m, s_tok, clipped)


def random_problem(seed: int, B: int, L: int, K: int, N: int, device="cpu",
                   base: str = "laplace") -> LinearCase:
    """An ad-hoc shape (ragged / adversarial sizes) with the same recipe as config 1."""
    c = WorkloadConfig(-1, "adhoc", B, L, 1, (("adhoc", K, N),), base, 0.01, None, 20.0)
    sigma, gain, w, bias = _static_structure(c, K, N, seed, device)
    xc = _draw_x(c, 16, K, sigma, gain, seed + 1_000_000, device)
    xmax = xc.abs().amax(dim=(0, 1)).float()
    wmax = w.abs().amax(dim=0).float()
    m = torch.sqrt(xmax / wmax).clamp_(1e-5, 1e5)
    m = torch.where(torch.isfinite(m), m, torch.ones_like(m)).contiguous()
    tmax = (xc.float() / m.view(1, 1, K)).abs().amax(dim=(0, 2))
    s_tok = (tmax / 127.0).clamp_(min=1e-30).contiguous()
    x3 = _draw_x(c, B, K, sigma, gain, seed + 9_000_000, device)
    clipped = int(((x3.float() / m.view(1, 1, K)).abs() > (127.5 * s_tok).view(1, L, 1)).sum().item())
    return LinearCase(-1, 0, 0, "adhoc", B, L, K, N, x3.reshape(B * L, K).contiguous(),
                      w.contiguous(), bias.contiguous(), m, s_tok, clipped)


# ---------------------------------------------------------------------------------- per-token zero offset
def token_shift(L: int, seed: int, device="cpu", scale: float = 2.0) -> torch.Tensor:
    """A fixed per-token-position offset (fp16 [L]) to add to activations: makes each token's
    distribution asymmetric about zero, the situation a per-token zero offset is for."""
    g = _gen(device, seed + 77_000_000)
    return (scale * torch.randn(L, generator=g, device=device, dtype=torch.float32)).to(torch.float16)


def calibrate_offset(x_cal: torch.Tensor, m: torch.Tensor, L: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """Min-max initialiser of the asymmetric quantizer (Sec. 2.3) applied per token position on
    smoothed calibration activations x_cal [n*L, K]: step (max - min) / 255 and the offset
    round(-min / step), shifted by 128 so that codes are int8.  Returns (s_tok fp32 [L], z_tok int32 [L])."""
    K = x_cal.shape[1]
    v = (x_cal.float() / m.view(1, K)).view(-1, L, K)
    lo = v.amin(dim=(0, 2)).clamp(max=0.0)
    hi = v.amax(dim=(0, 2)).clamp(min=0.0)
    s = ((hi - lo) / 255.0).clamp_(min=1e-30)
    z = (torch.round(-lo / s) - 128.0).clamp_(-128.0, 127.0).to(torch.int32)
    return s.contiguous(), z.contiguous()
