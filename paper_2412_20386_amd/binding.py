"""Thin ctypes binding of libptq4vm.so: argument marshalling only.

Every function takes torch CUDA tensors (used purely as device buffers), passes raw device
pointers, sizes and the current HIP stream to the C ABI declared in include/ptq4vm.h, and
returns the output tensors.  No arithmetic happens here and there is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# PTQ4VM_LIB: another build of the same sources (the sanitized host build of the test suite)
LIB_PATH = os.environ.get("PTQ4VM_LIB") or os.path.join(_HERE, "libptq4vm.so")

EXPORTS = (
    "ptq4vm_fold_smoothing",
    "ptq4vm_quantize_pts",
    "ptq4vm_quantize_dynamic",
    "ptq4vm_quantize_pts_offset",
    "ptq4vm_weight_rowsum",
    "ptq4vm_w8a8_linear_offset",
    "ptq4vm_fold_smoothing_w4",
    "ptq4vm_quantize_pts_a4",
    "ptq4vm_w4a4_linear",
    "ptq4vm_fold_smoothing_w4_e2m3",
    "ptq4vm_quantize_pts_a4_e2m3",
    "ptq4vm_w4a4_linear_e2m3",
    "ptq4vm_w4a4_linear_fused",
    "ptq4vm_w8a8_linear_offset_fused",
    "ptq4vm_w8a8_linear",
    "ptq4vm_w8a8_linear_fused",
    "ptq4vm_f16_linear",
    "ptq4vm_validate_scales",
    "ptq4vm_validate_scales_static",
    "ptq4vm_status_string",
    "ptq4vm_last_hip_error",
    "ptq4vm_version",
)

_lib = None


class Ptq4vmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"ptq4vm status {status}: {text}")
        self.status = status


def load() -> ctypes.CDLL:
    """Load libptq4vm.so (built by paper_2412_20386_amd.build). Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2412_20386_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.ptq4vm_fold_smoothing.restype = ci
    lib.ptq4vm_fold_smoothing.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, vp]
    lib.ptq4vm_quantize_pts.restype = ci
    lib.ptq4vm_quantize_pts.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_quantize_dynamic.restype = ci
    lib.ptq4vm_quantize_dynamic.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp]
    lib.ptq4vm_quantize_pts_offset.restype = ci
    lib.ptq4vm_quantize_pts_offset.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_weight_rowsum.restype = ci
    lib.ptq4vm_weight_rowsum.argtypes = [vp, vp, i64, i64, i64, vp]
    lib.ptq4vm_w8a8_linear_offset.restype = ci
    lib.ptq4vm_w8a8_linear_offset.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_fold_smoothing_w4.restype = ci
    lib.ptq4vm_fold_smoothing_w4.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, vp]
    lib.ptq4vm_quantize_pts_a4.restype = ci
    lib.ptq4vm_quantize_pts_a4.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_w4a4_linear.restype = ci
    lib.ptq4vm_w4a4_linear.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_fold_smoothing_w4_e2m3.restype = ci
    lib.ptq4vm_fold_smoothing_w4_e2m3.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, vp]
    lib.ptq4vm_quantize_pts_a4_e2m3.restype = ci
    lib.ptq4vm_quantize_pts_a4_e2m3.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_w4a4_linear_e2m3.restype = ci
    lib.ptq4vm_w4a4_linear_e2m3.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_w8a8_linear_offset_fused.restype = ci
    lib.ptq4vm_w8a8_linear_offset_fused.argtypes = [vp] * 11 + [i64] * 8 + [vp]
    lib.ptq4vm_w4a4_linear_fused.restype = ci
    lib.ptq4vm_w4a4_linear_fused.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_w8a8_linear.restype = ci
    lib.ptq4vm_w8a8_linear.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_w8a8_linear_fused.restype = ci
    lib.ptq4vm_w8a8_linear_fused.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64,
                                             i64, vp]
    lib.ptq4vm_f16_linear.restype = ci
    lib.ptq4vm_f16_linear.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, vp]
    lib.ptq4vm_validate_scales.restype = ci
    lib.ptq4vm_validate_scales.argtypes = [vp, i64, vp, i64, vp, i64, vp, vp, i64, vp]
    lib.ptq4vm_validate_scales_static.restype = ci
    lib.ptq4vm_validate_scales_static.argtypes = [vp, i64, vp, i64, vp, i64, vp, vp]
    lib.ptq4vm_status_string.restype = ctypes.c_char_p
    lib.ptq4vm_status_string.argtypes = [ci]
    lib.ptq4vm_last_hip_error.restype = ctypes.c_char_p
    lib.ptq4vm_last_hip_error.argtypes = []
    lib.ptq4vm_version.restype = ci
    lib.ptq4vm_version.argtypes = []
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().ptq4vm_status_string(int(status)).decode()


def check(status: int) -> None:
    if status != 0:
        text = status_string(status)
        if status == -5:
            text += ": " + load().ptq4vm_last_hip_error().decode()
        raise Ptq4vmError(status, text)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()  # plain ints: the declared argtypes convert them


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _matrix(t: torch.Tensor, dtype, name: str) -> Tuple[int, int, int]:
    if not t.is_cuda or t.dtype != dtype or t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise TypeError(f"{name}: expected a 2-D CUDA tensor of {dtype} with unit inner stride")
    return t.shape[0], t.shape[1], (t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1]))


def _vector(t: Optional[torch.Tensor], dtype, n: int, name: str, optional=False):
    if t is None:
        if optional:
            return
        raise TypeError(f"{name} is required")
    if not t.is_cuda or t.dtype != dtype or t.dim() != 1 or t.shape[0] != n or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous CUDA vector of {n} x {dtype}")


def fold_smoothing(w: torch.Tensor, m: torch.Tensor, wq: Optional[torch.Tensor] = None):
    """ptq4vm_fold_smoothing: (wq int8 [N,K], s_w f32 [N], inv_m f32 [K])."""
    N, K, ldw = _matrix(w, torch.float16, "w")
    _vector(m, torch.float32, K, "m")
    if wq is None:
        wq = torch.empty((N, K), dtype=torch.int8, device=w.device)
    _, _, ldwq = _matrix(wq, torch.int8, "wq")
    s_w = torch.empty(N, dtype=torch.float32, device=w.device)
    inv_m = torch.empty(K, dtype=torch.float32, device=w.device)
    check(load().ptq4vm_fold_smoothing(_ptr(w), _ptr(m), _ptr(wq), _ptr(s_w), _ptr(inv_m), N, K, ldw, ldwq,
                                       _stream()))
    return wq, s_w, inv_m


def quantize_pts(x: torch.Tensor, inv_m: Optional[torch.Tensor], s_tok: torch.Tensor, B: int, L: int,
                 xq: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_quantize_pts: xq int8 [B*L, K]."""
    M, K, ldx = _matrix(x, torch.float16, "x")
    if M != B * L:
        raise ValueError("x must have B*L rows")
    _vector(inv_m, torch.float32, K, "inv_m", optional=True)
    _vector(s_tok, torch.float32, L, "s_tok")
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    _, _, ldxq = _matrix(xq, torch.int8, "xq")
    check(load().ptq4vm_quantize_pts(_ptr(x), _ptr(inv_m), _ptr(s_tok), _ptr(xq), B, L, K, ldx, ldxq, _stream()))
    return xq


def quantize_dynamic(x: torch.Tensor, inv_m: Optional[torch.Tensor], xq: Optional[torch.Tensor] = None,
                     s_row: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """ptq4vm_quantize_dynamic: (xq int8 [M, K], s_row f32 [M])."""
    M, K, ldx = _matrix(x, torch.float16, "x")
    _vector(inv_m, torch.float32, K, "inv_m", optional=True)
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    _, _, ldxq = _matrix(xq, torch.int8, "xq")
    if s_row is None:
        s_row = torch.empty(M, dtype=torch.float32, device=x.device)
    _vector(s_row, torch.float32, M, "s_row")
    check(load().ptq4vm_quantize_dynamic(_ptr(x), _ptr(inv_m), _ptr(xq), _ptr(s_row), M, K, ldx, ldxq, _stream()))
    return xq, s_row


def w8a8_linear(xq: torch.Tensor, wq: torch.Tensor, s_tok: torch.Tensor, s_w: torch.Tensor,
                bias: Optional[torch.Tensor], B: int, L: int, y: Optional[torch.Tensor] = None,
                acc_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_w8a8_linear: y fp16 [B*L, N]; acc_out (int32 [B*L, N], dense) is filled if given."""
    M, K, ldxq = _matrix(xq, torch.int8, "xq")
    N, K2, ldwq = _matrix(wq, torch.int8, "wq")
    if K != K2 or M != B * L:
        raise ValueError("shape mismatch")
    _vector(s_tok, torch.float32, L, "s_tok")
    _vector(s_w, torch.float32, N, "s_w")
    _vector(bias, torch.float16, N, "bias", optional=True)
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _, _, ldy = _matrix(y, torch.float16, "y")
    if acc_out is not None and (acc_out.dtype != torch.int32 or tuple(acc_out.shape) != (M, N)
                                or not acc_out.is_contiguous() or not acc_out.is_cuda):
        raise TypeError("acc_out: expected a dense CUDA int32 [M, N] tensor")
    check(load().ptq4vm_w8a8_linear(_ptr(xq), _ptr(wq), _ptr(s_tok), _ptr(s_w), _ptr(bias), _ptr(y),
                                    _ptr(acc_out), B, L, K, N, ldxq, ldwq, ldy, _stream()))
    return y


def quantize_pts_offset(x: torch.Tensor, inv_m: Optional[torch.Tensor], s_tok: torch.Tensor, z_tok: torch.Tensor,
                        B: int, L: int, xq: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_quantize_pts_offset: xq int8 [B*L, K] with the per-token zero offset z_tok (int32 [L])."""
    M, K, ldx = _matrix(x, torch.float16, "x")
    if M != B * L:
        raise ValueError("x must have B*L rows")
    _vector(inv_m, torch.float32, K, "inv_m", optional=True)
    _vector(s_tok, torch.float32, L, "s_tok")
    _vector(z_tok, torch.int32, L, "z_tok")
    if xq is None:
        xq = torch.empty((M, K), dtype=torch.int8, device=x.device)
    _, _, ldxq = _matrix(xq, torch.int8, "xq")
    check(load().ptq4vm_quantize_pts_offset(_ptr(x), _ptr(inv_m), _ptr(s_tok), _ptr(z_tok), _ptr(xq), B, L, K, ldx,
                                            ldxq, _stream()))
    return xq


def weight_rowsum(wq: torch.Tensor) -> torch.Tensor:
    """ptq4vm_weight_rowsum: int32 [N] = sum_k wq[o, k]."""
    N, K, ldwq = _matrix(wq, torch.int8, "wq")
    out = torch.empty(N, dtype=torch.int32, device=wq.device)
    check(load().ptq4vm_weight_rowsum(_ptr(wq), _ptr(out), N, K, ldwq, _stream()))
    return out


def w8a8_linear_offset(xq: torch.Tensor, wq: torch.Tensor, s_tok: torch.Tensor, z_tok: torch.Tensor,
                       rowsum: torch.Tensor, s_w: torch.Tensor, bias: Optional[torch.Tensor], B: int, L: int,
                       y: Optional[torch.Tensor] = None, acc_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_w8a8_linear_offset: y fp16 [B*L, N] with the zero-offset correction in the epilogue."""
    M, K, ldxq = _matrix(xq, torch.int8, "xq")
    N, K2, ldwq = _matrix(wq, torch.int8, "wq")
    if K != K2 or M != B * L:
        raise ValueError("shape mismatch")
    _vector(s_tok, torch.float32, L, "s_tok")
    _vector(z_tok, torch.int32, L, "z_tok")
    _vector(rowsum, torch.int32, N, "rowsum")
    _vector(s_w, torch.float32, N, "s_w")
    _vector(bias, torch.float16, N, "bias", optional=True)
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=xq.device)
    _, _, ldy = _matrix(y, torch.float16, "y")
    if acc_out is not None and (acc_out.dtype != torch.int32 or tuple(acc_out.shape) != (M, N)
                                or not acc_out.is_contiguous() or not acc_out.is_cuda):
        raise TypeError("acc_out: expected a dense CUDA int32 [M, N] tensor")
    check(load().ptq4vm_w8a8_linear_offset(_ptr(xq), _ptr(wq), _ptr(s_tok), _ptr(z_tok), _ptr(rowsum), _ptr(s_w),
                                           _ptr(bias), _ptr(y), _ptr(acc_out), B, L, K, N, ldxq, ldwq, ldy, _stream()))
    return y


def fold_smoothing_w4(w: torch.Tensor, m: torch.Tensor, wq4: Optional[torch.Tensor] = None):
    """ptq4vm_fold_smoothing_w4: (wq4 uint8 [N, K/2] packed, s_w f32 [N], inv_m f32 [K])."""
    N, K, ldw = _matrix(w, torch.float16, "w")
    _vector(m, torch.float32, K, "m")
    if wq4 is None:
        wq4 = torch.empty((N, K // 2), dtype=torch.uint8, device=w.device)
    _, _, ldwq = _matrix(wq4, torch.uint8, "wq4")
    s_w = torch.empty(N, dtype=torch.float32, device=w.device)
    inv_m = torch.empty(K, dtype=torch.float32, device=w.device)
    check(load().ptq4vm_fold_smoothing_w4(_ptr(w), _ptr(m), _ptr(wq4), _ptr(s_w), _ptr(inv_m), N, K, ldw, ldwq,
                                          _stream()))
    return wq4, s_w, inv_m


def quantize_pts_a4(x: torch.Tensor, inv_m: Optional[torch.Tensor], s_tok: torch.Tensor, B: int, L: int,
                    xq4: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_quantize_pts_a4: xq4 uint8 [B*L, K/2], two 4-bit codes per byte."""
    M, K, ldx = _matrix(x, torch.float16, "x")
    if M != B * L:
        raise ValueError("x must have B*L rows")
    _vector(inv_m, torch.float32, K, "inv_m", optional=True)
    _vector(s_tok, torch.float32, L, "s_tok")
    if xq4 is None:
        xq4 = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
    _, _, ldxq = _matrix(xq4, torch.uint8, "xq4")
    check(load().ptq4vm_quantize_pts_a4(_ptr(x), _ptr(inv_m), _ptr(s_tok), _ptr(xq4), B, L, K, ldx, ldxq, _stream()))
    return xq4


def w4a4_linear(xq4: torch.Tensor, wq4: torch.Tensor, s_tok: torch.Tensor, s_w: torch.Tensor,
                bias: Optional[torch.Tensor], B: int, L: int, y: Optional[torch.Tensor] = None,
                acc_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_w4a4_linear: y fp16 [B*L, N] from packed 4-bit operands."""
    M, K2, ldxq = _matrix(xq4, torch.uint8, "xq4")
    N, K2w, ldwq = _matrix(wq4, torch.uint8, "wq4")
    if K2 != K2w or M != B * L:
        raise ValueError("shape mismatch")
    _vector(s_tok, torch.float32, L, "s_tok")
    _vector(s_w, torch.float32, N, "s_w")
    _vector(bias, torch.float16, N, "bias", optional=True)
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=xq4.device)
    _, _, ldy = _matrix(y, torch.float16, "y")
    if acc_out is not None and (acc_out.dtype != torch.int32 or tuple(acc_out.shape) != (M, N)
                                or not acc_out.is_contiguous() or not acc_out.is_cuda):
        raise TypeError("acc_out: expected a dense CUDA int32 [M, N] tensor")
    check(load().ptq4vm_w4a4_linear(_ptr(xq4), _ptr(wq4), _ptr(s_tok), _ptr(s_w), _ptr(bias), _ptr(y), _ptr(acc_out),
                                    B, L, 2 * K2, N, ldxq, ldwq, ldy, _stream()))
    return y


def e2m3_blocks(K: int) -> int:
    """PTQ4VM_E2M3_BLOCKS: 96-byte blocks of 128 codes that a row of K codes takes in the E2M3 container."""
    return (K + 127) // 128


def _e2m3_container(t: torch.Tensor, rows: int, K: int, what: str) -> int:
    """Checks a block-major container [e2m3_blocks(K), rows, 96] uint8 and returns its plane pitch in bytes."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.uint8 or t.dim() != 3:
        raise TypeError(f"{what}: expected a CUDA uint8 tensor [blocks, rows, 96]")
    if tuple(t.shape) != (e2m3_blocks(K), rows, 96) or t.stride(2) != 1 or (rows > 1 and t.stride(1) != 96):
        raise ValueError(f"{what}: expected shape {(e2m3_blocks(K), rows, 96)} with dense 96-byte blocks")
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), 96 * rows)


def fold_smoothing_w4_e2m3(w: torch.Tensor, m: torch.Tensor, wq6: Optional[torch.Tensor] = None):
    """ptq4vm_fold_smoothing_w4_e2m3: (wq6 uint8 [e2m3_blocks(K), N, 96] block-major, s_w f32 [N], inv_m f32 [K])."""
    N, K, ldw = _matrix(w, torch.float16, "w")
    _vector(m, torch.float32, K, "m")
    if wq6 is None:
        wq6 = torch.empty((e2m3_blocks(K), N, 96), dtype=torch.uint8, device=w.device)
    ldwq = _e2m3_container(wq6, N, K, "wq6")
    s_w = torch.empty(N, dtype=torch.float32, device=w.device)
    inv_m = torch.empty(K, dtype=torch.float32, device=w.device)
    check(load().ptq4vm_fold_smoothing_w4_e2m3(_ptr(w), _ptr(m), _ptr(wq6), _ptr(s_w), _ptr(inv_m), N, K, ldw, ldwq,
                                               _stream()))
    return wq6, s_w, inv_m


def quantize_pts_a4_e2m3(x: torch.Tensor, inv_m: Optional[torch.Tensor], s_tok: torch.Tensor, B: int, L: int,
                         xq6: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_quantize_pts_a4_e2m3: xq6 uint8 [e2m3_blocks(K), B*L, 96], 4-bit codes as E2M3 patterns, block-major."""
    M, K, ldx = _matrix(x, torch.float16, "x")
    if M != B * L:
        raise ValueError("x must have B*L rows")
    _vector(inv_m, torch.float32, K, "inv_m", optional=True)
    _vector(s_tok, torch.float32, L, "s_tok")
    if xq6 is None:
        xq6 = torch.empty((e2m3_blocks(K), M, 96), dtype=torch.uint8, device=x.device)
    ldxq = _e2m3_container(xq6, M, K, "xq6")
    check(load().ptq4vm_quantize_pts_a4_e2m3(_ptr(x), _ptr(inv_m), _ptr(s_tok), _ptr(xq6), B, L, K, ldx, ldxq,
                                             _stream()))
    return xq6


def w4a4_linear_e2m3(xq6: torch.Tensor, wq6: torch.Tensor, s_tok: torch.Tensor, s_w: torch.Tensor,
                     bias: Optional[torch.Tensor], B: int, L: int, K: int, y: Optional[torch.Tensor] = None,
                     acc_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_w4a4_linear_e2m3: y fp16 [B*L, N] from operands in the block-major E2M3 container (K codes per row)."""
    M = B * L
    ldxq = _e2m3_container(xq6, M, K, "xq6")
    if not isinstance(wq6, torch.Tensor) or wq6.dim() != 3:
        raise TypeError("wq6: expected a CUDA uint8 tensor [blocks, N, 96]")
    N = wq6.shape[1]
    ldwq = _e2m3_container(wq6, N, K, "wq6")
    _vector(s_tok, torch.float32, L, "s_tok")
    _vector(s_w, torch.float32, N, "s_w")
    _vector(bias, torch.float16, N, "bias", optional=True)
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=xq6.device)
    _, _, ldy = _matrix(y, torch.float16, "y")
    if acc_out is not None and (acc_out.dtype != torch.int32 or tuple(acc_out.shape) != (M, N)
                                or not acc_out.is_contiguous() or not acc_out.is_cuda):
        raise TypeError("acc_out: expected a dense CUDA int32 [M, N] tensor")
    check(load().ptq4vm_w4a4_linear_e2m3(_ptr(xq6), _ptr(wq6), _ptr(s_tok), _ptr(s_w), _ptr(bias), _ptr(y),
                                         _ptr(acc_out), B, L, K, N, ldxq, ldwq, ldy, _stream()))
    return y


def w8a8_linear_fused(x: torch.Tensor, inv_m: Optional[torch.Tensor], s_tok: torch.Tensor, wq: torch.Tensor,
                      s_w: torch.Tensor, bias: Optional[torch.Tensor], B: int, L: int,
                      y: Optional[torch.Tensor] = None, acc_out: Optional[torch.Tensor] = None,
                      xq_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_w8a8_linear_fused: y fp16 [B*L, N] from fp16 activations; acc_out / xq_out are filled if given."""
    M, K, ldx = _matrix(x, torch.float16, "x")
    N, K2, ldwq = _matrix(wq, torch.int8, "wq")
    if K != K2 or M != B * L:
        raise ValueError("shape mismatch")
    _vector(inv_m, torch.float32, K, "inv_m", optional=True)
    _vector(s_tok, torch.float32, L, "s_tok")
    _vector(s_w, torch.float32, N, "s_w")
    _vector(bias, torch.float16, N, "bias", optional=True)
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _, _, ldy = _matrix(y, torch.float16, "y")
    if acc_out is not None and (acc_out.dtype != torch.int32 or tuple(acc_out.shape) != (M, N)
                                or not acc_out.is_contiguous() or not acc_out.is_cuda):
        raise TypeError("acc_out: expected a dense CUDA int32 [M, N] tensor")
    ldxq = 0
    if xq_out is not None:
        Mq, Kq, ldxq = _matrix(xq_out, torch.int8, "xq_out")
        if (Mq, Kq) != (M, K):
            raise ValueError("xq_out must be [B*L, K]")
    check(load().ptq4vm_w8a8_linear_fused(_ptr(x), _ptr(inv_m), _ptr(s_tok), _ptr(wq), _ptr(s_w), _ptr(bias), _ptr(y),
                                          _ptr(acc_out), _ptr(xq_out), B, L, K, N, ldx, ldwq, ldy, ldxq, _stream()))
    return y


def w8a8_linear_offset_fused(x: torch.Tensor, inv_m: Optional[torch.Tensor], s_tok: torch.Tensor, z_tok: torch.Tensor,
                             wq: torch.Tensor, rowsum: torch.Tensor, s_w: torch.Tensor, bias: Optional[torch.Tensor],
                             B: int, L: int, y: Optional[torch.Tensor] = None, acc_out: Optional[torch.Tensor] = None,
                             xq_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_w8a8_linear_offset_fused: y fp16 [B*L, N] from fp16 activations, per-token steps and zero offsets;
    acc_out (raw accumulators) / xq_out (codes with the offset in them) are filled if given."""
    M, K, ldx = _matrix(x, torch.float16, "x")
    N, K2, ldwq = _matrix(wq, torch.int8, "wq")
    if K != K2 or M != B * L:
        raise ValueError("shape mismatch")
    _vector(inv_m, torch.float32, K, "inv_m", optional=True)
    _vector(s_tok, torch.float32, L, "s_tok")
    _vector(z_tok, torch.int32, L, "z_tok")
    _vector(rowsum, torch.int32, N, "rowsum")
    _vector(s_w, torch.float32, N, "s_w")
    _vector(bias, torch.float16, N, "bias", optional=True)
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _, _, ldy = _matrix(y, torch.float16, "y")
    if acc_out is not None and (acc_out.dtype != torch.int32 or tuple(acc_out.shape) != (M, N)
                                or not acc_out.is_contiguous() or not acc_out.is_cuda):
        raise TypeError("acc_out: expected a dense CUDA int32 [M, N] tensor")
    ldxq = 0
    if xq_out is not None:
        Mq, Kq, ldxq = _matrix(xq_out, torch.int8, "xq_out")
        if (Mq, Kq) != (M, K):
            raise ValueError("xq_out must be [B*L, K]")
    check(load().ptq4vm_w8a8_linear_offset_fused(_ptr(x), _ptr(inv_m), _ptr(s_tok), _ptr(z_tok), _ptr(wq), _ptr(rowsum),
                                                 _ptr(s_w), _ptr(bias), _ptr(y), _ptr(acc_out), _ptr(xq_out), B, L, K, N,
                                                 ldx, ldwq, ldy, ldxq, _stream()))
    return y


def w4a4_linear_fused(x: torch.Tensor, inv_m: Optional[torch.Tensor], s_tok: torch.Tensor, wq4: torch.Tensor,
                      s_w: torch.Tensor, bias: Optional[torch.Tensor], B: int, L: int,
                      y: Optional[torch.Tensor] = None, acc_out: Optional[torch.Tensor] = None,
                      xq_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_w4a4_linear_fused: y fp16 [B*L, N] from fp16 activations and a packed 4-bit weight [N, K/2];
    acc_out / xq_out (int8, one 4-bit code per byte) are filled if given."""
    M, K, ldx = _matrix(x, torch.float16, "x")
    N, K2, ldwq = _matrix(wq4, torch.uint8, "wq4")
    if K != 2 * K2 or M != B * L:
        raise ValueError("shape mismatch")
    _vector(inv_m, torch.float32, K, "inv_m", optional=True)
    _vector(s_tok, torch.float32, L, "s_tok")
    _vector(s_w, torch.float32, N, "s_w")
    _vector(bias, torch.float16, N, "bias", optional=True)
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _, _, ldy = _matrix(y, torch.float16, "y")
    if acc_out is not None and (acc_out.dtype != torch.int32 or tuple(acc_out.shape) != (M, N)
                                or not acc_out.is_contiguous() or not acc_out.is_cuda):
        raise TypeError("acc_out: expected a dense CUDA int32 [M, N] tensor")
    ldxq = 0
    if xq_out is not None:
        Mq, Kq, ldxq = _matrix(xq_out, torch.int8, "xq_out")
        if (Mq, Kq) != (M, K):
            raise ValueError("xq_out must be [B*L, K]")
    check(load().ptq4vm_w4a4_linear_fused(_ptr(x), _ptr(inv_m), _ptr(s_tok), _ptr(wq4), _ptr(s_w), _ptr(bias), _ptr(y),
                                          _ptr(acc_out), _ptr(xq_out), B, L, K, N, ldx, ldwq, ldy, ldxq, _stream()))
    return y

def f16_linear(x: torch.Tensor, w: torch.Tensor, bias: Optional[torch.Tensor],
               y: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ptq4vm_f16_linear: y fp16 [M, N]."""
    M, K, ldx = _matrix(x, torch.float16, "x")
    N, K2, ldw = _matrix(w, torch.float16, "w")
    if K != K2:
        raise ValueError("shape mismatch")
    _vector(bias, torch.float16, N, "bias", optional=True)
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    _, _, ldy = _matrix(y, torch.float16, "y")
    check(load().ptq4vm_f16_linear(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), M, K, N, ldx, ldw, ldy, _stream()))
    return y


VALIDATE_BLOCK = 4096  # PTQ4VM_VALIDATE_BLOCK


def validate_scales(s_tok: Optional[torch.Tensor], m: Optional[torch.Tensor], s_w: Optional[torch.Tensor],
                    workspace: Optional[torch.Tensor] = None) -> Tuple[int, torch.Tensor]:
    """ptq4vm_validate_scales: (status, bad_counts int32 [3] on the device).  status is 0 or
    PTQ4VM_ERR_VALUE (-6, some entry is not a finite number > 0); other errors raise.  Synchronises."""
    vecs = [v for v in (s_tok, m, s_w) if v is not None]
    if not vecs:
        raise TypeError("at least one vector is required")
    dev = vecs[0].device
    sizes = []
    for v, name in ((s_tok, "s_tok"), (m, "m"), (s_w, "s_w")):
        if v is not None:
            _vector(v, torch.float32, v.shape[0], name)
        sizes.append(0 if v is None else v.shape[0])
    need = 16 * ((sum(sizes) + VALIDATE_BLOCK - 1) // VALIDATE_BLOCK + 1)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    counts = torch.empty(3, dtype=torch.int32, device=dev)
    rc = load().ptq4vm_validate_scales(_ptr(s_tok), sizes[0], _ptr(m), sizes[1], _ptr(s_w), sizes[2], _ptr(counts),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    if rc not in (0, -6):
        check(rc)
    return rc, counts


def validate_scales_static(s_tok: Optional[torch.Tensor], m: Optional[torch.Tensor], s_w: Optional[torch.Tensor],
                           counts: torch.Tensor) -> None:
    """ptq4vm_validate_scales_static: enqueue only; `counts` (int32 [3], device, the caller's) holds the bad-entry
    counts once the current stream has run the two kernels.  Allocates nothing and does not synchronise."""
    sizes = []
    for v, name in ((s_tok, "s_tok"), (m, "m"), (s_w, "s_w")):
        if v is not None:
            _vector(v, torch.float32, v.shape[0], name)
        sizes.append(0 if v is None else v.shape[0])
    _vector(counts, torch.int32, 3, "counts")
    check(load().ptq4vm_validate_scales_static(_ptr(s_tok), sizes[0], _ptr(m), sizes[1], _ptr(s_w), sizes[2],
                                               _ptr(counts), _stream()))
