"""ctypes front-end of the plain-C CPU oracle (test infrastructure only).

Argument marshalling only: every function takes and returns dense NumPy arrays
(fp16 as np.float16) and forwards to oracle/ptq4vm_oracle.c, which holds all of
the arithmetic.  Nothing here imports the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ptq4vm_oracle.c")
_LIB = os.path.join(_HERE, "libptq4vm_oracle.so")
_lib = None

# No fast-math, no FMA contraction: the fp32 decision order in the C file is law.
_CFLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-std=c11"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (always when force=True, else only if stale)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *_CFLAGS, _SRC, "-o", tmp, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized() -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (-O1), next to the normal library.
    To run the pins under it: PTQ4VM_ORACLE_LIB=<this path>, with gcc's libasan.so preloaded."""
    out = os.path.join(_HERE, "libptq4vm_oracle_asan.so")
    flags = [f for f in _CFLAGS if f != "-O2"] + ["-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"]
    subprocess.run(["gcc", *flags, _SRC, "-o", out, "-lm"], check=True)
    return out


def _load():
    global _lib
    if _lib is None:
        override = os.environ.get("PTQ4VM_ORACLE_LIB")  # a sanitized build of the same source
        if not override:
            build()
        lib = ctypes.CDLL(override or _LIB)
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_half_to_float.restype = ctypes.c_float
        lib.oracle_half_to_float.argtypes = [ctypes.c_uint16]
        lib.oracle_double_to_half.restype = ctypes.c_uint16
        lib.oracle_double_to_half.argtypes = [ctypes.c_double]
        lib.oracle_threads.restype = ctypes.c_int
        lib.oracle_fold_smoothing.restype = None
        lib.oracle_fold_smoothing.argtypes = [vp, vp, vp, vp, vp, i64, i64]
        lib.oracle_quantize_pts.restype = None
        lib.oracle_quantize_pts.argtypes = [vp, vp, vp, vp, i64, i64, i64]
        lib.oracle_int8_gemm.restype = i64
        lib.oracle_int8_gemm.argtypes = [vp, vp, vp, i64, i64, i64]
        lib.oracle_dequant.restype = None
        lib.oracle_dequant.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64]
        lib.oracle_f16_linear.restype = None
        lib.oracle_f16_linear.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64]
        lib.oracle_quantize_dynamic.restype = None
        lib.oracle_quantize_dynamic.argtypes = [vp, vp, vp, vp, i64, i64]
        lib.oracle_fold_smoothing_bits.restype = None
        lib.oracle_fold_smoothing_bits.argtypes = [vp, vp, vp, vp, vp, i64, i64, ctypes.c_int]
        lib.oracle_quantize_pts_bits.restype = None
        lib.oracle_quantize_pts_bits.argtypes = [vp, vp, vp, vp, i64, i64, i64, ctypes.c_int]
        lib.oracle_pack_int4.restype = None
        lib.oracle_pack_int4.argtypes = [vp, vp, i64, i64]
        lib.oracle_unpack_int4.restype = None
        lib.oracle_unpack_int4.argtypes = [vp, vp, i64, i64]
        lib.oracle_e2m3_blocks.restype = i64
        lib.oracle_e2m3_blocks.argtypes = [i64]
        lib.oracle_pack_e2m3.restype = ctypes.c_int
        lib.oracle_pack_e2m3.argtypes = [vp, vp, i64, i64]
        lib.oracle_unpack_e2m3.restype = ctypes.c_int
        lib.oracle_unpack_e2m3.argtypes = [vp, vp, i64, i64]
        lib.oracle_quantize_pts_offset.restype = None
        lib.oracle_quantize_pts_offset.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64]
        lib.oracle_weight_rowsum.restype = None
        lib.oracle_weight_rowsum.argtypes = [vp, vp, i64, i64]
        lib.oracle_dequant_offset.restype = None
        lib.oracle_dequant_offset.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64]
        _lib = lib
    return _lib


def _arr(a, dtype, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(_load().oracle_threads())


def half_to_float(bits: int) -> float:
    return float(_load().oracle_half_to_float(int(bits) & 0xFFFF))


def double_to_half(x: float) -> int:
    return int(_load().oracle_double_to_half(float(x)))


def fold_smoothing(w: np.ndarray, m: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(Wq int8 [N,K], s_w fp32 [N], inv_m fp32 [K]) from W fp16 [N,K] and m fp32 [K]."""
    w = _arr(w, np.float16)
    N, K = w.shape
    m = _arr(m, np.float32, (K,))
    wq = np.empty((N, K), np.int8)
    s_w = np.empty(N, np.float32)
    inv_m = np.empty(K, np.float32)
    _load().oracle_fold_smoothing(_p(w), _p(m), _p(wq), _p(s_w), _p(inv_m), N, K)
    return wq, s_w, inv_m


def quantize_pts(x: np.ndarray, inv_m: Optional[np.ndarray], s_tok: np.ndarray, B: int,
                 L: int) -> np.ndarray:
    """Xq int8 [B*L,K] from X fp16 [B*L,K], inv_m fp32 [K] (or None), s_tok fp32 [L]."""
    x = _arr(x, np.float16)
    M, K = x.shape
    if M != B * L:
        raise ValueError("x must have B*L rows")
    inv_m = None if inv_m is None else _arr(inv_m, np.float32, (K,))
    s_tok = _arr(s_tok, np.float32, (L,))
    xq = np.empty((M, K), np.int8)
    _load().oracle_quantize_pts(_p(x), _p(inv_m), _p(s_tok), _p(xq), B, L, K)
    return xq


def int8_gemm(xq: np.ndarray, wq: np.ndarray) -> np.ndarray:
    """acc int32 [M,N] = Xq [M,K] . Wq[N,K]^T; raises if any exact sum overflows int32."""
    xq = _arr(xq, np.int8)
    wq = _arr(wq, np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    if K != K2:
        raise ValueError("K mismatch")
    acc = np.empty((M, N), np.int32)
    bad = _load().oracle_int8_gemm(_p(xq), _p(wq), _p(acc), M, K, N)
    if bad:
        raise OverflowError(f"{bad} accumulators exceed int32")
    return acc


def dequant(acc: np.ndarray, s_tok: np.ndarray, s_w: np.ndarray, bias: Optional[np.ndarray],
            B: int, L: int) -> Tuple[np.ndarray, np.ndarray]:
    """(Y fp16 [M,N], y64 double [M,N]) from int32 accumulators and the two step vectors."""
    acc = _arr(acc, np.int32)
    M, N = acc.shape
    if M != B * L:
        raise ValueError("acc must have B*L rows")
    s_tok = _arr(s_tok, np.float32, (L,))
    s_w = _arr(s_w, np.float32, (N,))
    bias = None if bias is None else _arr(bias, np.float16, (N,))
    y = np.empty((M, N), np.float16)
    y64 = np.empty((M, N), np.float64)
    _load().oracle_dequant(_p(acc), _p(s_tok), _p(s_w), _p(bias), _p(y), _p(y64), B, L, N)
    return y, y64


def w8a8_linear(xq, wq, s_tok, s_w, bias, B: int, L: int):
    """Integer GEMM followed by dequantization: (Y fp16, y64, acc int32)."""
    acc = int8_gemm(xq, wq)
    y, y64 = dequant(acc, s_tok, s_w, bias, B, L)
    return y, y64, acc


def f16_linear(x: np.ndarray, w: np.ndarray, bias: Optional[np.ndarray]):
    """(Y fp16, y64, sum|terms|) of the unquantized linear, double accumulation."""
    x = _arr(x, np.float16)
    w = _arr(w, np.float16)
    M, K = x.shape
    N, K2 = w.shape
    if K != K2:
        raise ValueError("K mismatch")
    bias = None if bias is None else _arr(bias, np.float16, (N,))
    y = np.empty((M, N), np.float16)
    y64 = np.empty((M, N), np.float64)
    asum = np.empty((M, N), np.float64)
    _load().oracle_f16_linear(_p(x), _p(w), _p(bias), _p(y), _p(y64), _p(asum), M, K, N)
    return y, y64, asum


# ---------------------------------------------------------------------------------- widened rows
def quantize_dynamic(x: np.ndarray, inv_m: Optional[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """Per-token dynamic quantizer: (Xq int8 [M,K], s_row fp32 [M]) from X fp16 [M,K]."""
    x = _arr(x, np.float16)
    M, K = x.shape
    inv_m = None if inv_m is None else _arr(inv_m, np.float32, (K,))
    xq = np.empty((M, K), np.int8)
    s_row = np.empty(M, np.float32)
    _load().oracle_quantize_dynamic(_p(x), _p(inv_m), _p(xq), _p(s_row), M, K)
    return xq, s_row


def fold_smoothing_bits(w: np.ndarray, m: np.ndarray, bits: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """b-bit weight fold: codes (one per int8) in [-(2^(b-1)-1), 2^(b-1)-1], s_w, inv_m."""
    w = _arr(w, np.float16)
    N, K = w.shape
    m = _arr(m, np.float32, (K,))
    wq = np.empty((N, K), np.int8)
    s_w = np.empty(N, np.float32)
    inv_m = np.empty(K, np.float32)
    _load().oracle_fold_smoothing_bits(_p(w), _p(m), _p(wq), _p(s_w), _p(inv_m), N, K, (1 << (bits - 1)) - 1)
    return wq, s_w, inv_m


def quantize_pts_bits(x: np.ndarray, inv_m: Optional[np.ndarray], s_tok: np.ndarray, B: int, L: int,
                      bits: int) -> np.ndarray:
    """b-bit PTS codes, one per int8."""
    x = _arr(x, np.float16)
    M, K = x.shape
    if M != B * L:
        raise ValueError("x must have B*L rows")
    inv_m = None if inv_m is None else _arr(inv_m, np.float32, (K,))
    s_tok = _arr(s_tok, np.float32, (L,))
    xq = np.empty((M, K), np.int8)
    _load().oracle_quantize_pts_bits(_p(x), _p(inv_m), _p(s_tok), _p(xq), B, L, K, (1 << (bits - 1)) - 1)
    return xq


def pack_int4(codes: np.ndarray) -> np.ndarray:
    """[rows, K] int8 codes in [-8, 7] -> [rows, K/2] bytes, even index in the low nibble."""
    codes = _arr(codes, np.int8)
    rows, K = codes.shape
    if K % 2:
        raise ValueError("K must be even")
    packed = np.empty((rows, K // 2), np.uint8)
    _load().oracle_pack_int4(_p(codes), _p(packed), rows, K)
    return packed


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    packed = _arr(packed, np.uint8)
    rows, half = packed.shape
    codes = np.empty((rows, 2 * half), np.int8)
    _load().oracle_unpack_int4(_p(packed), _p(codes), rows, 2 * half)
    return codes


def e2m3_blocks(K: int) -> int:
    """Blocks of 128 codes (96 bytes each) that a row of K codes takes in the E2M3 container."""
    return int(_load().oracle_e2m3_blocks(K))


def pack_e2m3(codes: np.ndarray) -> np.ndarray:
    """[rows, K] int8 codes in [-7, 7] -> [e2m3_blocks(K), rows, 96] bytes: 6-bit E2M3 patterns, rows zero padded
    to whole blocks, block-major (plane b holds block b of every row)."""
    codes = _arr(codes, np.int8)
    rows, K = codes.shape
    packed = np.empty((e2m3_blocks(K), rows, 96), np.uint8)
    if _load().oracle_pack_e2m3(_p(codes), _p(packed), rows, K) != 0:
        raise ValueError("codes outside [-7, 7] have no E2M3 pattern")
    return packed


def unpack_e2m3(packed: np.ndarray, K: int) -> np.ndarray:
    packed = _arr(packed, np.uint8)
    blocks, rows, width = packed.shape
    if blocks != e2m3_blocks(K) or width != 96:
        raise ValueError("container shape does not match K")
    codes = np.empty((rows, K), np.int8)
    if _load().oracle_unpack_e2m3(_p(packed), _p(codes), rows, K) != 0:
        raise ValueError("a pattern does not stand for an integer")
    return codes


def quantize_pts_offset(x: np.ndarray, inv_m: Optional[np.ndarray], s_tok: np.ndarray, z_tok: np.ndarray,
                        B: int, L: int) -> np.ndarray:
    """PTS codes with a per-token zero offset z_tok int32 [L] (int8 range): clip(rint(v) + z, -128, 127)."""
    x = _arr(x, np.float16)
    M, K = x.shape
    if M != B * L:
        raise ValueError("x must have B*L rows")
    inv_m = None if inv_m is None else _arr(inv_m, np.float32, (K,))
    s_tok = _arr(s_tok, np.float32, (L,))
    z_tok = _arr(z_tok, np.int32, (L,))
    xq = np.empty((M, K), np.int8)
    _load().oracle_quantize_pts_offset(_p(x), _p(inv_m), _p(s_tok), _p(z_tok), _p(xq), B, L, K)
    return xq


def weight_rowsum(wq: np.ndarray) -> np.ndarray:
    wq = _arr(wq, np.int8)
    N, K = wq.shape
    out = np.empty(N, np.int32)
    _load().oracle_weight_rowsum(_p(wq), _p(out), N, K)
    return out


def dequant_offset(acc: np.ndarray, s_tok: np.ndarray, z_tok: np.ndarray, rowsum: np.ndarray, s_w: np.ndarray,
                   bias: Optional[np.ndarray], B: int, L: int) -> Tuple[np.ndarray, np.ndarray]:
    """(Y fp16, y64) = (acc - z_tok[r mod L] * rowsum[o]) * s_tok[r mod L] * s_w[o] + bias[o]."""
    acc = _arr(acc, np.int32)
    M, N = acc.shape
    if M != B * L:
        raise ValueError("acc must have B*L rows")
    s_tok = _arr(s_tok, np.float32, (L,))
    z_tok = _arr(z_tok, np.int32, (L,))
    rowsum = _arr(rowsum, np.int32, (N,))
    s_w = _arr(s_w, np.float32, (N,))
    bias = None if bias is None else _arr(bias, np.float16, (N,))
    y = np.empty((M, N), np.float16)
    y64 = np.empty((M, N), np.float64)
    _load().oracle_dequant_offset(_p(acc), _p(s_tok), _p(z_tok), _p(rowsum), _p(s_w), _p(bias), _p(y), _p(y64), B, L, N)
    return y, y64
