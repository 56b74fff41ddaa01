"""Shared comparison helpers for the GPU-vs-oracle parity tests (no arithmetic of the method)."""
import numpy as np


def f16_ordered(a: np.ndarray) -> np.ndarray:
    """Map fp16 bit patterns to integers that are monotone in the value (+-0 -> 0)."""
    bits = a.view(np.uint16).astype(np.int32)
    mag = bits & 0x7FFF
    return np.where(bits & 0x8000, -mag, mag)


def check_dequantized_output(y_gpu: np.ndarray, y_ref: np.ndarray, y64: np.ndarray, prod_abs: np.ndarray,
                             bias_abs: np.ndarray, what: str = "") -> dict:
    """fp16 output bar: the GPU value is the oracle's fp16 value or one of its two neighbours
    (<= 1 fp16 ulp), i.e. relative error <= 1e-3, except where the fp32 epilogue's own rounding
    (4 roundings of 2^-24 on the product term and the bias) exceeds that because the product
    and the bias cancel; there the error is bounded by 2^-21 (|acc s_t s_w| + |bias|) + 2^-24.

    prod_abs = |acc * s_tok * s_w| in double, bias_abs = |bias| broadcast to the same shape.
    """
    assert y_gpu.shape == y_ref.shape == y64.shape
    g64 = y_gpu.astype(np.float64)
    finite = np.isfinite(y_ref.astype(np.float64))
    # overflow: both sides must agree on +-Inf, unless the value sits within fp32 rounding of
    # the fp16 overflow threshold 65520
    edge = np.abs(np.abs(y64) - 65520.0) <= 2.0 ** -21 * (prod_abs + bias_abs)
    inf_ok = (g64 == y_ref.astype(np.float64)) | edge
    assert np.all(inf_ok[~finite]), f"{what}: Inf mismatch"
    assert not np.any(np.isnan(g64[finite & ~edge])), f"{what}: NaN in output"
    floor = 2.0 ** -21 * (prod_abs + bias_abs) + 2.0 ** -24
    err = np.abs(g64 - y64)
    dist = np.abs(f16_ordered(y_gpu) - f16_ordered(y_ref))
    sel = finite & ~edge
    ok_ulp = (dist <= 1) | (err <= floor)
    assert np.all(ok_ulp[sel]), (
        f"{what}: {np.count_nonzero(~ok_ulp & sel)} outputs differ from the oracle by more than 1 fp16 ulp; "
        f"worst distance {dist[sel].max()}")
    ok_rel = err <= 1e-3 * np.abs(y64) + floor
    assert np.all(ok_rel[sel]), f"{what}: relative error above 1e-3"
    mismatch = np.count_nonzero((dist != 0) & sel) / max(1, np.count_nonzero(sel))
    assert mismatch < 0.01, f"{what}: {mismatch:.3%} of outputs are not the oracle's fp16 value"
    return {"mismatch_fraction": mismatch, "max_ulp": int(dist[sel].max()) if sel.any() else 0}
