"""GPU parity: every entry point of libptq4vm.so, called through the C ABI, against the CPU
oracle on the same seeded inputs.  int8 codes and int32 accumulators bit-exact; fp16 outputs
within 1 fp16 ulp (see parity_util.check_dequantized_output for the exact bar)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2412_20386_amd as ptq
from paper_2412_20386_amd import synth

from parity_util import check_dequantized_output

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _np(t):
    return t.detach().cpu().numpy()


def _padded(rows, cols, ld, dtype, fill):
    """A [rows, cols] view with row pitch ld inside a sentinel-filled buffer."""
    buf = torch.full((rows, ld), fill, dtype=dtype, device=DEV)
    return buf, buf[:, :cols]


# ---------------------------------------------------------------------------------- quantizer
QUANT_SHAPES = [  # B, L, K
    (1, 197, 384),    # config 0
    (3, 197, 768),
    (2, 7, 12),       # dt_proj input: 24-byte rows -> 4-wide path
    (5, 33, 44),
    (4, 9, 13),       # odd K -> element path
    (3, 5, 8),        # one chunk per row
    (1, 3, 2056),     # more than 256 chunks per row
    (257, 1, 48),     # L = 1: per-tensor static
    (2, 785, 24),
    (1, 1, 1536),
    (1, 20000, 16),   # token table too long for LDS: per-row division path
    (2, 3, 776),      # 97 chunks per row: grid rounded to a multiple of 97
]


@pytest.mark.parametrize("B,L,K", QUANT_SHAPES)
@pytest.mark.parametrize("use_m", [True, False])
def test_quantize_pts_bit_exact(B, L, K, use_m):
    print(f"quantize B={B} L={L} K={K} use_m={use_m}", flush=True)
    c = synth.random_problem(1000 + B * 7 + K, B, L, K, 8, device=DEV)
    _, _, inv_m = oracle.fold_smoothing(_np(c.w), _np(c.m))
    inv_m_t = torch.from_numpy(inv_m).to(DEV) if use_m else None
    xq = ptq.quantize_pts(c.x, inv_m_t, c.s_tok, B, L)
    torch.cuda.synchronize()
    want = oracle.quantize_pts(_np(c.x), inv_m if use_m else None, _np(c.s_tok), B, L)
    assert np.array_equal(_np(xq), want)
    assert np.abs(want.astype(np.int32)).max() > 16  # the case is not degenerate


def test_quantize_pts_special_values_and_ties():
    K = 16
    row = [0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.5, 128.0, 1000.0, float("inf"), float("-inf"),
           float("nan"), -127.49, -127.5, -60000.0]
    x = torch.tensor([row, row[::-1]], dtype=torch.float16, device=DEV)
    s_tok = torch.tensor([1.0, 0.5], dtype=torch.float32, device=DEV)
    for inv_m in (None, torch.full((K,), 1.0, device=DEV), torch.full((K,), 0.25, device=DEV)):
        xq = ptq.quantize_pts(x, inv_m, s_tok, 1, 2)
        torch.cuda.synchronize()
        want = oracle.quantize_pts(_np(x), None if inv_m is None else _np(inv_m), _np(s_tok), 1, 2)
        assert np.array_equal(_np(xq), want)
    assert _np(ptq.quantize_pts(x, None, s_tok, 1, 2))[0].tolist() == \
        [0, 2, 2, 0, -2, -2, 126, 127, 127, 127, 127, -127, 0, -127, -127, -127]


def test_quantize_pts_every_fp16_value():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = torch.from_numpy(bits.view(np.float16).reshape(64, 1024).copy()).to(DEV)
    rng = np.random.default_rng(3)
    inv_m = rng.uniform(0.01, 30, 1024).astype(np.float32)
    s_tok = rng.uniform(0.001, 50, 8).astype(np.float32)
    xq = ptq.quantize_pts(x, torch.from_numpy(inv_m).to(DEV), torch.from_numpy(s_tok).to(DEV), 8, 8)
    torch.cuda.synchronize()
    assert np.array_equal(_np(xq), oracle.quantize_pts(_np(x), inv_m, s_tok, 8, 8))


@pytest.mark.parametrize("K,ldx,ldxq", [(384, 400, 416), (12, 20, 16), (13, 17, 19)])
def test_quantize_pts_padded_rows_leave_padding_untouched(K, ldx, ldxq):
    B, L = 3, 11
    c = synth.random_problem(77 + K, B, L, K, 8, device=DEV)
    xbuf, xv = _padded(B * L, K, ldx, torch.float16, 777.0)
    xv.copy_(c.x)
    qbuf, qv = _padded(B * L, K, ldxq, torch.int8, 0x55)
    inv_m = (1.0 / c.m).contiguous()
    ptq.quantize_pts(xv, inv_m, c.s_tok, B, L, xq=qv)
    torch.cuda.synchronize()
    want = oracle.quantize_pts(_np(c.x), _np(inv_m), _np(c.s_tok), B, L)
    assert np.array_equal(_np(qv), want)
    assert np.all(_np(qbuf[:, K:]) == 0x55)


# ---------------------------------------------------------------------------------- fold
@pytest.mark.parametrize("N,K,ldw,ldwq", [(192, 384, 384, 384), (44, 384, 384, 384), (384, 12, 12, 12),
                                           (17, 1000, 1008, 1024), (3, 5, 8, 16), (3072, 768, 768, 768)])
def test_fold_smoothing_bit_exact(N, K, ldw, ldwq):
    print(f"fold N={N} K={K}", flush=True)
    c = synth.random_problem(500 + N + K, 2, 5, K, N, device=DEV)
    w = c.w.clone()
    if N > 2:
        w[1].zero_()  # dead output channel
    wbuf, wv = _padded(N, K, ldw, torch.float16, 9.0)
    wv.copy_(w)
    qbuf, qv = _padded(N, K, ldwq, torch.int8, 0x55)
    wq, s_w, inv_m = ptq.fold_smoothing(wv, c.m, wq=qv)
    torch.cuda.synchronize()
    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing(_np(w), _np(c.m))
    assert np.array_equal(_np(s_w).view(np.uint32), s_w_o.view(np.uint32))
    assert np.array_equal(_np(inv_m).view(np.uint32), inv_m_o.view(np.uint32))
    assert np.array_equal(_np(qv), wq_o)
    if ldwq > K:
        assert np.all(_np(qbuf[:, K:]) == 0x55)


# ---------------------------------------------------------------------------------- W8A8 linear
def _run_w8a8_case(c, use_bias=True, ldy=None, what=""):
    """Full path on the GPU vs the oracle chain on the CPU, each from the same fp16 inputs."""
    print(f"w8a8 {what} B={c.B} L={c.L} K={c.K} N={c.N} bias={use_bias} ldy={ldy}", flush=True)
    M = c.B * c.L
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    xq = ptq.quantize_pts(c.x, inv_m, c.s_tok, c.B, c.L)
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    bias = c.bias if use_bias else None
    if ldy is None:
        y = ptq.w8a8_linear(xq, wq, c.s_tok, s_w, bias, c.B, c.L, acc_out=acc)
        ybuf = None
    else:
        ybuf, yv = _padded(M, c.N, ldy, torch.float16, 12345.0)
        y = ptq.w8a8_linear(xq, wq, c.s_tok, s_w, bias, c.B, c.L, y=yv, acc_out=acc)
    y2 = ptq.w8a8_linear(xq, wq, c.s_tok, s_w, bias, c.B, c.L)  # timed configuration: no acc_out
    torch.cuda.synchronize()

    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing(_np(c.w), _np(c.m))
    xq_o = oracle.quantize_pts(_np(c.x), inv_m_o, _np(c.s_tok), c.B, c.L)
    b_o = _np(c.bias) if use_bias else None
    y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, _np(c.s_tok), s_w_o, b_o, c.B, c.L)

    assert np.array_equal(_np(wq), wq_o) and np.array_equal(_np(xq), xq_o)
    assert np.array_equal(_np(acc), acc_o), "int32 accumulators differ"
    st = np.tile(_np(c.s_tok).astype(np.float64), c.B)[:, None]
    prod_abs = np.abs(acc_o.astype(np.float64) * st * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(b_o.astype(np.float64))[None, :] if use_bias else 0.0, prod_abs.shape)
    stats = check_dequantized_output(_np(y), y_o, y64, prod_abs, bias_abs, what)
    assert np.array_equal(_np(y).view(np.uint16), _np(y2).view(np.uint16)), "acc_out changes the result"
    if ybuf is not None:
        assert np.all(_np(ybuf[:, c.N:]) == np.float16(12345.0))
    return stats


def test_w8a8_linear_config0():
    c = synth.make_linear_case(0, device=DEV)
    assert c.clipped > 0
    _run_w8a8_case(c, what="config0")


W8A8_SHAPES = [  # B, L, K, N
    (3, 197, 384, 192),
    (2, 197, 192, 768),
    (2, 197, 384, 44),    # x_proj (Vim-Ti): 88-byte output rows
    (3, 197, 12, 384),    # dt_proj (Vim-Ti): 12-byte activation rows
    (2, 65, 24, 768),
    (2, 50, 768, 56),
    (1, 300, 1536, 80),
    (1, 1, 64, 32),       # a single row
    (1, 257, 100, 130),   # K, N multiples of 4 only
    (2, 33, 13, 5),       # nothing aligned
    (1, 129, 1000, 257),
    (5, 7, 16, 1),
]


@pytest.mark.parametrize("B,L,K,N", W8A8_SHAPES)
def test_w8a8_linear_shapes(B, L, K, N):
    c = synth.random_problem(31 * K + N, B, L, K, N, device=DEV)
    _run_w8a8_case(c, what="adhoc")


def test_w8a8_linear_without_bias_and_padded_output():
    c = synth.random_problem(5, 2, 197, 384, 192, device=DEV)
    _run_w8a8_case(c, use_bias=False, what="nobias")
    _run_w8a8_case(c, ldy=200, what="ldy200")
    c = synth.random_problem(6, 2, 31, 384, 44, device=DEV)
    _run_w8a8_case(c, ldy=45, what="ldy45")


def test_w8a8_linear_extreme_codes():
    """All codes at +-127 with the largest K of the workloads: |acc| = 1536 * 127^2."""
    B, L, K, N = 1, 40, 1536, 96
    xq = torch.full((B * L, K), 127, dtype=torch.int8, device=DEV)
    xq[1::2] = -127
    wq = torch.full((N, K), 127, dtype=torch.int8, device=DEV)
    wq[::3] = -127
    s_tok = torch.full((L,), 2.0 ** -12, device=DEV)
    s_w = torch.full((N,), 2.0 ** -10, device=DEV)
    acc = torch.empty((B * L, N), dtype=torch.int32, device=DEV)
    y = ptq.w8a8_linear(xq, wq, s_tok, s_w, None, B, L, acc_out=acc)
    torch.cuda.synchronize()
    y_o, y64, acc_o = oracle.w8a8_linear(_np(xq), _np(wq), _np(s_tok), _np(s_w), None, B, L)
    assert np.abs(acc_o).max() == 1536 * 16129
    assert np.array_equal(_np(acc), acc_o)
    assert np.array_equal(_np(y).view(np.uint16), y_o.view(np.uint16))  # exact: power-of-two steps


@pytest.mark.parametrize("K", [133143, 133120])
def test_w8a8_linear_longest_reduction_fills_int32(K):
    """The largest accepted K (odd: element-wise loads; and the largest multiple of 128: slab kernels) with
    every code at +-127: the accumulators come within 0.02 % of the int32 range and must not wrap."""
    B, L, N = 1, 37, 24
    xq = torch.full((B * L, K), 127, dtype=torch.int8, device=DEV)
    xq[1::2] = -127
    wq = torch.full((N, K), 127, dtype=torch.int8, device=DEV)
    wq[::3] = -127
    wq[5, ::2] = -127                                   # a row that cancels to (almost) zero
    s_tok = torch.full((L,), 2.0 ** -20, device=DEV)
    s_w = torch.full((N,), 2.0 ** -12, device=DEV)
    acc = torch.empty((B * L, N), dtype=torch.int32, device=DEV)
    y = ptq.w8a8_linear(xq, wq, s_tok, s_w, None, B, L, acc_out=acc)
    torch.cuda.synchronize()
    y_o, y64, acc_o = oracle.w8a8_linear(_np(xq), _np(wq), _np(s_tok), _np(s_w), None, B, L)
    assert np.abs(acc_o.astype(np.int64)).max() == K * 16129 > 2 ** 31 - 2 ** 19
    assert np.array_equal(_np(acc), acc_o)
    prod_abs = np.abs(acc_o.astype(np.float64)) * 2.0 ** -32
    check_dequantized_output(_np(y), y_o, y64, prod_abs, np.zeros_like(prod_abs), "longest reduction")


def test_zero_offset_longest_reduction_24_bit_product():
    """K = 65536 with every weight code at -128: rowsum = -2^23, the most negative 24-bit value, times the
    largest offsets; acc - z * rowsum reaches 2^30 + 127 * 2^23 and must be exact."""
    B, L, K, N = 1, 35, 65536, 24
    xq = torch.full((B * L, K), -128, dtype=torch.int8, device=DEV)
    xq[1::2] = 127
    wq = torch.full((N, K), -128, dtype=torch.int8, device=DEV)
    wq[::4] = 127
    s_tok = torch.full((L,), 2.0 ** -20, device=DEV)
    z_tok = torch.full((L,), -128, dtype=torch.int32, device=DEV)
    z_tok[::2] = 127                                    # opposite to the row's codes: x - z = -+255
    s_w = torch.full((N,), 2.0 ** -12, device=DEV)
    rowsum = ptq.weight_rowsum(wq)
    acc = torch.empty((B * L, N), dtype=torch.int32, device=DEV)
    y = ptq.w8a8_linear_offset(xq, wq, s_tok, z_tok, rowsum, s_w, None, B, L, acc_out=acc)
    torch.cuda.synchronize()
    rowsum_o = oracle.weight_rowsum(_np(wq))
    assert rowsum_o.min() == -(2 ** 23) and np.array_equal(_np(rowsum), rowsum_o)
    acc_o = oracle.int8_gemm(_np(xq), _np(wq))
    assert np.array_equal(_np(acc), acc_o)
    y_o, y64 = oracle.dequant_offset(acc_o, _np(s_tok), _np(z_tok), rowsum_o, _np(s_w), None, B, L)
    corrected = acc_o.astype(np.int64) - np.tile(_np(z_tok).astype(np.int64), B)[:, None] * rowsum_o.astype(np.int64)[None, :]
    assert np.abs(corrected).max() == 2 ** 30 + 127 * 2 ** 23
    prod_abs = np.abs(corrected.astype(np.float64)) * 2.0 ** -32
    check_dequantized_output(_np(y), y_o, y64, prod_abs, np.zeros_like(prod_abs), "offset longest reduction")


DETERMINISM_SHAPES = [  # B, L, K, N, which kernels the library picks at this shape
    (4, 197, 768, 384, "tiled 4-wavefront kernel"),
    (64, 197, 768, 3072, "persistent 256 x 256 kernel, whole rounds plus a round of half tiles"),
    (64, 197, 1536, 80, "weight-resident kernels (two-launch and fused)"),
    (110, 197, 48, 1536, "row-streaming short-reduction kernel (two-launch and fused)"),
]


@pytest.mark.parametrize("B,L,K,N,kernels", DETERMINISM_SHAPES)
def test_w8a8_linear_is_deterministic(B, L, K, N, kernels):
    """20 runs of quantizer + linear and of the fused launch on the same inputs: identical bytes every
    time (integer sums do not depend on order, so any difference is a race or an uninitialised read)."""
    print(f"determinism B={B} L={L} K={K} N={N}: {kernels}", flush=True)
    c = synth.random_problem(9, B, L, K, N, device=DEV)
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    first_q = first_y = None
    for rep in range(20):
        xq = ptq.quantize_pts(c.x, inv_m, c.s_tok, c.B, c.L)
        y = ptq.w8a8_linear(xq, wq, c.s_tok, s_w, c.bias, c.B, c.L)
        y_fused = ptq.w8a8_linear_fused(c.x, inv_m, c.s_tok, wq, s_w, c.bias, c.B, c.L)
        torch.cuda.synchronize()
        if first_q is None:
            first_q, first_y = xq.clone(), y.clone()
        assert torch.equal(xq, first_q), f"codes changed in repeat {rep}"
        assert torch.equal(y.view(torch.int16), first_y.view(torch.int16)), f"output changed in repeat {rep}"
        assert torch.equal(y_fused.view(torch.int16), first_y.view(torch.int16)), f"fused output changed in repeat {rep}"


# ---------------------------------------------------------------------------------- FP16 linear
@pytest.mark.parametrize("M,K,N", [(197, 384, 192), (500, 768, 3072), (300, 1536, 80), (100, 12, 384),
                                    (77, 50, 33), (64, 13, 7)])
def test_f16_linear_within_accumulation_bound(M, K, N):
    print(f"f16 M={M} K={K} N={N}", flush=True)
    c = synth.random_problem(3 * M + K, 1, M, K, N, device=DEV)
    y = ptq.f16_linear(c.x, c.w, c.bias)
    torch.cuda.synchronize()
    y_o, y64, asum = oracle.f16_linear(_np(c.x), _np(c.w), _np(c.bias))
    g = _np(y).astype(np.float64)
    # fp32 accumulation in any order: |err| <= (K+1) 2^-24 sum|terms|, then one fp16 rounding
    tol = (K + 2) * 2.0 ** -24 * asum + 2.0 ** -11 * np.abs(y64) + 2.0 ** -24
    assert np.all(np.abs(g - y64) <= tol)


# ---------------------------------------------------------------------------------- full-size workloads
def _sampled_rows(M, step, L):
    rows = np.unique(np.concatenate([np.arange(0, M, step), [0, 1, L - 1, L, M - 1, M - 2], np.arange(M - 300, M, 7)]))
    return rows[(rows >= 0) & (rows < M)]


ROW_CHUNK = 8192  # rows handed to the oracle at a time (bounds the host memory of a whole-tensor comparison)


def _compare_rows_with_oracle(c, rows, x, xq, acc, y, what, use_bias=True):
    """The oracle recomputes the given rows (all of them when rows = arange(M)) from the fp16 inputs, in
    chunks: int8 codes and int32 accumulators must be equal, fp16 outputs within the bar of parity_util."""
    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing(_np(c.w), _np(c.m))
    b_o = _np(c.bias) if use_bias else None
    s_tok = _np(c.s_tok)
    worst = {"mismatch_fraction": 0.0, "max_ulp": 0}
    for lo in range(0, len(rows), ROW_CHUNK):
        part = rows[lo:lo + ROW_CHUNK]
        n = len(part)
        contiguous = n > 1 and int(part[-1]) - int(part[0]) == n - 1
        sel = slice(int(part[0]), int(part[-1]) + 1) if contiguous else torch.from_numpy(part).to(DEV)
        st_rows = s_tok[part % c.L]                               # token position of each row
        xq_o = oracle.quantize_pts(_np(x[sel]), inv_m_o, st_rows, 1, n)  # B=1, L=n: one step per row
        assert np.array_equal(_np(xq[sel]), xq_o), f"{what}: int8 codes differ in rows {part[0]}..{part[-1]}"
        y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, st_rows, s_w_o, b_o, 1, n)
        assert np.array_equal(_np(acc[sel]), acc_o), f"{what}: int32 accumulators differ in rows {part[0]}..{part[-1]}"
        prod_abs = np.abs(acc_o.astype(np.float64) * st_rows.astype(np.float64)[:, None] * s_w_o.astype(np.float64)[None, :])
        bias_abs = np.broadcast_to(np.abs(b_o.astype(np.float64))[None, :] if use_bias else 0.0, prod_abs.shape)
        stats = check_dequantized_output(_np(y[sel]), y_o, y64, prod_abs, bias_abs, what)
        worst = {k: max(worst[k], stats[k]) for k in worst}
    return worst


def _check_case_on_sampled_rows(c, rows, what, ldy=None, use_bias=True):
    """Whole problem on the GPU in the benchmark's launch configuration (no accumulator dump),
    plus one launch with the dump; the oracle recomputes the given rows from the fp16 inputs."""
    print(f"full-size {what}: M={c.B * c.L} K={c.K} N={c.N} ldy={ldy} bias={use_bias}, {len(rows)} rows compared",
          flush=True)
    M = c.B * c.L
    bias = c.bias if use_bias else None
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    xq = ptq.quantize_pts(c.x, inv_m, c.s_tok, c.B, c.L)
    ybuf = None
    if ldy is None:
        y = ptq.w8a8_linear(xq, wq, c.s_tok, s_w, bias, c.B, c.L)
    else:
        ybuf, yv = _padded(M, c.N, ldy, torch.float16, 12345.0)
        y = ptq.w8a8_linear(xq, wq, c.s_tok, s_w, bias, c.B, c.L, y=yv)
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    y_dump = ptq.w8a8_linear(xq, wq, c.s_tok, s_w, bias, c.B, c.L, acc_out=acc)
    torch.cuda.synchronize()
    assert torch.equal(y.contiguous().view(torch.int16), y_dump.view(torch.int16))
    if ybuf is not None:
        assert bool((ybuf[:, c.N:] == 12345.0).all())
    wq_o, s_w_o, _ = oracle.fold_smoothing(_np(c.w), _np(c.m))
    assert np.array_equal(_np(wq), wq_o) and np.array_equal(_np(s_w), s_w_o)
    return _compare_rows_with_oracle(c, rows, c.x, xq, acc, y, what, use_bias)


ALL_LINEARS_OF_THE_STACKS = [(cfg, linear) for cfg in (1, 2, 3, 4) for linear in (0, 1, 2, 3)]


@pytest.mark.parametrize("cfg,linear", ALL_LINEARS_OF_THE_STACKS)
def test_stack_configs_layer0_whole_tensors_both_launch_forms(cfg, linear):
    """BASELINE configs[1..4], layer 0, every linear at the config's size: EVERY int8 code, int32
    accumulator and fp16 output against the oracle, in the two-launch form (quantizer, then linear) and in
    the one-launch fused form, each in the launch configuration bench.py times (no dumps) and with the
    parity dumps.  The four GPU results must agree bit for bit; the oracle then checks all M rows."""
    c = synth.make_linear_case(cfg, 0, linear, device=DEV)
    assert c.clipped > 0
    M = c.B * c.L
    print(f"whole tensors cfg{cfg} {c.name}: M={M} K={c.K} N={c.N}", flush=True)
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    xq = ptq.quantize_pts(c.x, inv_m, c.s_tok, c.B, c.L)
    y = ptq.w8a8_linear(xq, wq, c.s_tok, s_w, c.bias, c.B, c.L)
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    y_dump = ptq.w8a8_linear(xq, wq, c.s_tok, s_w, c.bias, c.B, c.L, acc_out=acc)
    y_fused = ptq.w8a8_linear_fused(c.x, inv_m, c.s_tok, wq, s_w, c.bias, c.B, c.L)
    acc_f = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    xq_f = torch.full((M, c.K), 0x55, dtype=torch.int8, device=DEV)
    y_fused_dump = ptq.w8a8_linear_fused(c.x, inv_m, c.s_tok, wq, s_w, c.bias, c.B, c.L, acc_out=acc_f, xq_out=xq_f)
    torch.cuda.synchronize()
    for other, name in ((y_dump, "two-launch with dump"), (y_fused, "fused"), (y_fused_dump, "fused with dumps")):
        assert torch.equal(y.view(torch.int16), other.view(torch.int16)), f"{name} differs from the two-launch output"
    assert torch.equal(acc, acc_f), "fused accumulators differ from the two-launch ones"
    assert torch.equal(xq, xq_f), "fused codes differ from the quantizer's"
    del y_dump, y_fused, y_fused_dump, acc_f, xq_f
    wq_o, s_w_o, _ = oracle.fold_smoothing(_np(c.w), _np(c.m))
    assert np.array_equal(_np(wq), wq_o) and np.array_equal(_np(s_w), s_w_o)
    stats = _compare_rows_with_oracle(c, np.arange(M), c.x, xq, acc, y, f"cfg{cfg} {c.name}")
    print(f"  {stats}", flush=True)


@pytest.mark.parametrize("layer", [11, 23])
@pytest.mark.parametrize("linear", [0, 1, 2, 3])
def test_vim_b_other_layers_sampled(layer, linear):
    """Two further layers of BASELINE configs[3] (their own seeded weights and activations): every 97th
    row plus the edges, all columns."""
    c = synth.make_linear_case(3, layer, linear, device=DEV)
    assert c.clipped > 0
    _check_case_on_sampled_rows(c, _sampled_rows(c.B * c.L, 97, c.L), f"vim_b layer {layer} {c.name}")


@pytest.mark.parametrize("B,L,K,N", [(41, 251, 192, 1544), (33, 300, 64, 2056), (20, 517, 128, 6400),
                                     (41, 251, 256, 1544), (20, 517, 384, 3400), (45, 229, 640, 1800),
                                     (41, 251, 768, 1280), (67, 193, 768, 256), (53, 211, 384, 768), (20, 517, 384, 3328),
                                     (129, 199, 512, 376), (105, 251, 256, 264)])
def test_large_ragged_shapes_sampled(B, L, K, N):
    """Many 256 x 256 tiles with ragged last tiles in both directions; shapes 4 and 6 have a reduction
    length the persistent kernel takes (2 and 5 slabs of 128 bytes), with and without a partial last
    round of tiles that is cut into half tiles.  K = 384 and K = 768 with at least 8192 rows and N a
    multiple of 256 run on the weights-in-registers kernel: ragged last row tile, a single strip, more
    workgroups than units in an XCD's last band.  The last two (fewer than 256 tiles of 256 x 256, 256 < N <= 384)
    run on 256 x 128 tiles of the persistent kernel: ragged rows and a ragged third / nearly empty third column tile."""
    c = synth.random_problem(4242 + N, B, L, K, N, device=DEV)
    _check_case_on_sampled_rows(c, _sampled_rows(B * L, 61, L), "ragged")


SKINNY_SHAPES = [  # B, L, K, N, ldy, bias: few output channels over many rows (weight-resident kernel)
    (83, 199, 192, 44, None, True),     # 3 k-steps; 88-byte dense rows; M mod 32 = 5
    (64, 257, 320, 80, None, False),    # 5 k-steps, fewer than the fragments kept in flight
    (70, 241, 1024, 128, None, True),   # exactly two register groups of k-steps; 8 channel blocks; M mod 32 = 6
    (83, 199, 704, 50, None, True),     # 11 k-steps; N not a multiple of 4: 2-byte stores
    (83, 199, 1536, 72, 80, True),      # padded output rows
    (66, 250, 1600, 16, None, True),    # 25 k-steps; one channel block; M mod 32 = 20
    (65, 253, 448, 97, 100, False),     # odd N with padded rows
]


@pytest.mark.parametrize("B,L,K,N,ldy,bias", SKINNY_SHAPES)
def test_skinny_output_shapes_sampled(B, L, K, N, ldy, bias):
    c = synth.random_problem(777 + K + N, B, L, K, N, device=DEV)
    _check_case_on_sampled_rows(c, _sampled_rows(B * L, 37, L), "skinny", ldy=ldy, use_bias=bias)


@pytest.mark.parametrize("B,L,K,N,bias", [(43, 197, 768, 512, True), (65, 131, 384, 256, False)])
def test_weights_in_registers_kernel_whole_result(B, L, K, N, bias):
    """Every code, accumulator and output of a launch of the weights-in-registers kernel (K = 768 / 384,
    at least 8192 rows), ragged in rows and channels."""
    c = synth.random_problem(4100 + K + N, B, L, K, N, device=DEV)
    _run_w8a8_case(c, use_bias=bias, what="wreg-whole")


def test_skinny_output_whole_result():
    """Every element of a weight-resident launch, not a sample: 83 * 199 rows, 192 -> 44."""
    c = synth.random_problem(99, 83, 199, 192, 44, device=DEV)
    _run_w8a8_case(c, what="skinny-whole")


@pytest.mark.parametrize("M,K,N", [(16517, 192, 44), (16400, 512, 80)])
def test_f16_linear_skinny_output(M, K, N):
    test_f16_linear_within_accumulation_bound(M, K, N)


# ---------------------------------------------------------------------------------- fused quantizer + linear
def _run_fused_case(c, use_bias=True, use_m=True, ldy=None, what=""):
    """ptq4vm_w8a8_linear_fused on the GPU vs the oracle's quantizer -> GEMM -> dequantization chain."""
    print(f"fused {what} B={c.B} L={c.L} K={c.K} N={c.N} bias={use_bias} m={use_m} ldy={ldy}", flush=True)
    M = c.B * c.L
    m = c.m if use_m else torch.ones_like(c.m)
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, m)
    bias = c.bias if use_bias else None
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    xq = torch.full((M, c.K), 0x55, dtype=torch.int8, device=DEV)
    ybuf = None
    if ldy is None:
        y = ptq.w8a8_linear_fused(c.x, inv_m if use_m else None, c.s_tok, wq, s_w, bias, c.B, c.L, acc_out=acc, xq_out=xq)
    else:
        ybuf, yv = _padded(M, c.N, ldy, torch.float16, 12345.0)
        y = ptq.w8a8_linear_fused(c.x, inv_m if use_m else None, c.s_tok, wq, s_w, bias, c.B, c.L, y=yv, acc_out=acc,
                                  xq_out=xq)
    y2 = ptq.w8a8_linear_fused(c.x, inv_m if use_m else None, c.s_tok, wq, s_w, bias, c.B, c.L)  # timed configuration
    torch.cuda.synchronize()

    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing(_np(c.w), _np(m))
    xq_o = oracle.quantize_pts(_np(c.x), inv_m_o if use_m else None, _np(c.s_tok), c.B, c.L)
    b_o = _np(c.bias) if use_bias else None
    y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, _np(c.s_tok), s_w_o, b_o, c.B, c.L)
    assert np.array_equal(_np(wq), wq_o)
    assert np.array_equal(_np(xq), xq_o), "int8 codes differ"
    assert np.array_equal(_np(acc), acc_o), "int32 accumulators differ"
    st = np.tile(_np(c.s_tok).astype(np.float64), c.B)[:, None]
    prod_abs = np.abs(acc_o.astype(np.float64) * st * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(b_o.astype(np.float64))[None, :] if use_bias else 0.0, prod_abs.shape)
    stats = check_dequantized_output(_np(y), y_o, y64, prod_abs, bias_abs, what)
    assert np.array_equal(_np(y).view(np.uint16), _np(y2).view(np.uint16)), "the parity outputs change the result"
    if ybuf is not None:
        assert np.all(_np(ybuf[:, c.N:]) == np.float16(12345.0))
    return stats


FUSED_SHAPES = [  # B, L, K, N: the tiled kernel with the quantizer in its loader
    (3, 197, 384, 192),
    (2, 197, 384, 44),
    (3, 197, 12, 384),    # dt_proj (Vim-Ti): 24-byte fp16 rows
    (2, 50, 768, 56),
    (1, 1, 64, 32),
    (1, 257, 100, 130),   # K a multiple of 4 only
    (2, 33, 13, 5),       # nothing aligned
    (1, 129, 1000, 257),
    (5, 7, 16, 1),
]


@pytest.mark.parametrize("B,L,K,N", FUSED_SHAPES)
def test_fused_linear_shapes(B, L, K, N):
    c = synth.random_problem(57 * K + N, B, L, K, N, device=DEV)
    _run_fused_case(c, what="fused-adhoc")


def test_fused_linear_config0_and_options():
    c = synth.make_linear_case(0, device=DEV)
    assert c.clipped > 0
    _run_fused_case(c, what="fused-config0")
    _run_fused_case(c, use_bias=False, use_m=False, what="fused-plain")
    _run_fused_case(c, ldy=c.N + 8, what="fused-ldy")


FUSED_SKINNY = [  # B, L, K, N, ldy, bias, m: weight-resident fused kernel (N <= 128, >= 2048 rows)
    (83, 199, 128, 44, None, True, True),     # 2 k-steps (depth 2); 88-byte dense rows; M mod 32 = 5
    (64, 257, 320, 80, None, False, True),    # 5 k-steps (depth 1)
    (70, 241, 1024, 128, None, True, True),   # 16 k-steps, 8 channel blocks (depth 2); M mod 32 = 6
    (83, 199, 768, 50, None, True, False),    # 12 k-steps (depth 4); N not a multiple of 4; no smoothing
    (83, 199, 1536, 72, 80, True, True),      # padded output rows
    (66, 250, 1600, 16, None, True, True),    # 25 k-steps (depth 1); one channel block; M mod 32 = 20
    (330, 199, 128, 44, None, True, True),    # 65670 rows: one full pass of 16-row units, then a tail of 17 groups of 8 rows
    (11, 191, 256, 80, None, True, True),     # 2101 rows: a grid of 9 workgroups, 29 or 30 groups each (wavefronts with 2 and 1)
    (13, 163, 192, 33, None, False, True),    # 2119 rows, M mod 8 = 7: the last group is ragged
]


@pytest.mark.parametrize("B,L,K,N,ldy,bias,use_m", FUSED_SKINNY)
def test_fused_linear_skinny_whole_result(B, L, K, N, ldy, bias, use_m):
    """Every code, accumulator and output of a weight-resident fused launch against the oracle."""
    c = synth.random_problem(1234 + K + N, B, L, K, N, device=DEV)
    _run_fused_case(c, use_bias=bias, use_m=use_m, ldy=ldy, what="fused-skinny")


# ---------------------------------------------------------------------------------- per-token dynamic quantizer
DYNAMIC_SHAPES = [  # M, K
    (197, 384), (591, 768), (300, 1536), (257, 48), (100, 2048),   # register-resident rows: 1..4 chunks per lane
    (64, 8), (33, 24), (130, 1000), (50, 776),                      # ragged chunk counts
    (40, 12), (9, 13), (21, 2056), (7, 4100),                       # element-wise kernel
    (1, 64), (3, 1),
]


@pytest.mark.parametrize("M,K", DYNAMIC_SHAPES)
@pytest.mark.parametrize("use_m", [True, False])
def test_quantize_dynamic_bit_exact(M, K, use_m):
    print(f"dynamic M={M} K={K} m={use_m}", flush=True)
    c = synth.random_problem(91 * K + M, 1, M, K, 8, device=DEV)
    x = c.x.clone()
    if M > 2:
        x[1] = 0                                              # an all-zero row: step 1
    inv_m = (1.0 / c.m) if use_m else None
    xq, s_row = ptq.quantize_dynamic(x, inv_m)
    torch.cuda.synchronize()
    xq_o, s_o = oracle.quantize_dynamic(_np(x), None if inv_m is None else _np(inv_m))
    assert np.array_equal(_np(s_row).view(np.uint32), s_o.view(np.uint32))
    assert np.array_equal(_np(xq), xq_o)


def test_quantize_dynamic_specials_and_padded_rows():
    M, K, ldx, ldxq = 70, 384, 400, 416
    c = synth.random_problem(17, 1, M, K, 8, device=DEV)
    xbuf, xv = _padded(M, K, ldx, torch.float16, 3.0)
    xv.copy_(c.x)
    xv[0, 5] = float("nan")
    xv[2, 7] = float("inf")
    xv[3, :] = 65504.0
    xv[4, 9] = -65504.0
    qbuf, qv = _padded(M, K, ldxq, torch.int8, 0x55)
    xq, s_row = ptq.quantize_dynamic(xv, 1.0 / c.m, xq=qv)
    torch.cuda.synchronize()
    xq_o, s_o = oracle.quantize_dynamic(_np(xv), _np(1.0 / c.m))
    assert np.array_equal(_np(s_row).view(np.uint32), s_o.view(np.uint32))
    assert np.array_equal(_np(qv), xq_o)
    assert np.all(_np(qbuf[:, K:]) == 0x55)


@pytest.mark.parametrize("cfg,linear", [(3, 0), (3, 1), (3, 2)])
def test_dynamic_path_full_size(cfg, linear):
    """Dynamic quantizer + W8A8 linear (one step per row) at the benchmark's size, sampled rows vs the oracle."""
    c = synth.make_linear_case(cfg, 0, linear, device=DEV)
    M = c.B * c.L
    print(f"dynamic full-size cfg{cfg} {c.name}: M={M} K={c.K} N={c.N}", flush=True)
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    xq, s_row = ptq.quantize_dynamic(c.x, inv_m)
    y = ptq.w8a8_linear(xq, wq, s_row, s_w, c.bias, 1, M)
    torch.cuda.synchronize()
    rows = _sampled_rows(M, 97, c.L)
    ridx = torch.from_numpy(rows).to(DEV)
    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing(_np(c.w), _np(c.m))
    xq_o, s_o = oracle.quantize_dynamic(_np(c.x[ridx]), inv_m_o)
    assert np.array_equal(_np(xq[ridx]), xq_o) and np.array_equal(_np(s_row[ridx]), s_o)
    y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, s_o, s_w_o, _np(c.bias), 1, len(rows))
    prod_abs = np.abs(acc_o.astype(np.float64) * s_o.astype(np.float64)[:, None] * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(_np(c.bias).astype(np.float64))[None, :], prod_abs.shape)
    check_dequantized_output(_np(y[ridx]), y_o, y64, prod_abs, bias_abs, f"dynamic cfg{cfg} {c.name}")


# ---------------------------------------------------------------------------------- per-token zero offset
def _offset_case(seed, B, L, K, N):
    """Activations shifted per token position (asymmetric about zero); offsets calibrated on the first
    half of the images, so the second half exercises the clip at both ends."""
    c = synth.random_problem(seed, B, L, K, N, device=DEV)
    shift = synth.token_shift(L, seed, device=DEV)
    x = (c.x.view(B, L, K) + shift.view(1, L, 1)).reshape(B * L, K).contiguous()
    s_off, z_off = synth.calibrate_offset(x[: max(1, B // 2) * L], c.m, L)
    return c, x, s_off, z_off


OFFSET_SHAPES = [  # B, L, K, N
    (4, 197, 384, 192), (4, 197, 384, 44), (4, 50, 768, 56), (2, 300, 1536, 80), (4, 65, 24, 768),
    (2, 257, 100, 130), (4, 33, 13, 5), (2, 129, 1000, 257), (6, 7, 16, 1),
]


@pytest.mark.parametrize("B,L,K,N", OFFSET_SHAPES)
def test_zero_offset_path_against_oracle(B, L, K, N):
    print(f"offset B={B} L={L} K={K} N={N}", flush=True)
    c, x, s_off, z_off = _offset_case(400 + K + N, B, L, K, N)
    M = B * L
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    rowsum = ptq.weight_rowsum(wq)
    xq = ptq.quantize_pts_offset(x, inv_m, s_off, z_off, B, L)
    acc = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
    y = ptq.w8a8_linear_offset(xq, wq, s_off, z_off, rowsum, s_w, c.bias, B, L, acc_out=acc)
    y2 = ptq.w8a8_linear_offset(xq, wq, s_off, z_off, rowsum, s_w, c.bias, B, L)
    torch.cuda.synchronize()

    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing(_np(c.w), _np(c.m))
    rowsum_o = oracle.weight_rowsum(wq_o)
    xq_o = oracle.quantize_pts_offset(_np(x), inv_m_o, _np(s_off), _np(z_off), B, L)
    acc_o = oracle.int8_gemm(xq_o, wq_o)
    y_o, y64 = oracle.dequant_offset(acc_o, _np(s_off), _np(z_off), rowsum_o, s_w_o, _np(c.bias), B, L)
    assert np.array_equal(_np(rowsum), rowsum_o)
    assert np.array_equal(_np(xq), xq_o), "int8 codes differ"
    assert xq_o.min() == -128 or xq_o.max() == 127                    # the clip is exercised
    assert np.array_equal(_np(acc), acc_o), "int32 accumulators differ"
    st = np.tile(_np(s_off).astype(np.float64), B)[:, None]
    zt = np.tile(_np(z_off).astype(np.float64), B)[:, None]
    corrected = acc_o.astype(np.float64) - zt * rowsum_o.astype(np.float64)[None, :]
    prod_abs = np.abs(corrected * st * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(_np(c.bias).astype(np.float64))[None, :], prod_abs.shape)
    check_dequantized_output(_np(y), y_o, y64, prod_abs, bias_abs, "offset")
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))


def _check_offset_on_sampled_rows(c, x, s_off, z_off, rows, what):
    """Whole problem on the GPU (with and without the accumulator dump); the oracle recomputes sampled rows."""
    print(f"offset full-size {what}: M={c.B * c.L} K={c.K} N={c.N}, {len(rows)} sampled rows", flush=True)
    M = c.B * c.L
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    rowsum = ptq.weight_rowsum(wq)
    xq = ptq.quantize_pts_offset(x, inv_m, s_off, z_off, c.B, c.L)
    y = ptq.w8a8_linear_offset(xq, wq, s_off, z_off, rowsum, s_w, c.bias, c.B, c.L)
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    y_dump = ptq.w8a8_linear_offset(xq, wq, s_off, z_off, rowsum, s_w, c.bias, c.B, c.L, acc_out=acc)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y_dump.view(torch.int16))
    ridx = torch.from_numpy(rows).to(DEV)
    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing(_np(c.w), _np(c.m))
    rowsum_o = oracle.weight_rowsum(wq_o)
    assert np.array_equal(_np(rowsum), rowsum_o)
    st_rows, z_rows = _np(s_off)[rows % c.L], _np(z_off)[rows % c.L]
    n = len(rows)
    xq_o = oracle.quantize_pts_offset(_np(x[ridx]), inv_m_o, st_rows, z_rows, 1, n)
    assert np.array_equal(_np(xq[ridx]), xq_o), "int8 codes differ"
    acc_o = oracle.int8_gemm(xq_o, wq_o)
    assert np.array_equal(_np(acc[ridx]), acc_o), "int32 accumulators differ"
    y_o, y64 = oracle.dequant_offset(acc_o, st_rows, z_rows, rowsum_o, s_w_o, _np(c.bias), 1, n)
    corrected = acc_o.astype(np.float64) - z_rows.astype(np.float64)[:, None] * rowsum_o.astype(np.float64)[None, :]
    prod_abs = np.abs(corrected * st_rows.astype(np.float64)[:, None] * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(_np(c.bias).astype(np.float64))[None, :], prod_abs.shape)
    check_dequantized_output(_np(y[ridx]), y_o, y64, prod_abs, bias_abs, f"offset {what}")


@pytest.mark.parametrize("linear", [0, 1, 2, 3])
def test_zero_offset_vim_b_full_size_sampled(linear):
    c = synth.make_linear_case(3, 0, linear, device=DEV)
    shift = synth.token_shift(c.L, 77 + linear, device=DEV)
    x = (c.x.view(c.B, c.L, c.K) + shift.view(1, c.L, 1).to(c.x.dtype)).reshape(c.B * c.L, c.K).contiguous()
    s_off, z_off = synth.calibrate_offset(x[: 16 * c.L], c.m, c.L)
    _check_offset_on_sampled_rows(c, x, s_off, z_off, _sampled_rows(c.B * c.L, 97, c.L), f"vim_b {c.name}")


@pytest.mark.parametrize("B,L,K,N", [(41, 251, 256, 1544), (20, 517, 384, 3400), (300, 65, 24, 776), (250, 33, 100, 520),
                                     (110, 197, 24, 776), (105, 197, 100, 520), (107, 199, 48, 1536),
                                     (83, 199, 256, 80), (64, 257, 1536, 44), (70, 241, 704, 121)])
def test_zero_offset_large_ragged_shapes_sampled(B, L, K, N):
    """Ragged last tiles in the persistent kernel (first two), the short-reduction kernel (next two), the
    row-streaming kernel (from 20 480 rows: one and two k-steps, ragged rows and channels) and the weight-resident
    kernel (N <= 128: 5, 3 and 8 channel blocks, ragged rows and channels)."""
    c, x, s_off, z_off = _offset_case(5000 + K + N, B, L, K, N)
    _check_offset_on_sampled_rows(c, x, s_off, z_off, _sampled_rows(B * L, 61, L), "ragged")


def test_zero_offset_quantizer_long_sequence_and_plain_kernels():
    """L beyond the LDS table (per-row division), K a multiple of 4 only, K odd."""
    for B, L, K in [(1, 9000, 64), (3, 41, 20), (2, 19, 7)]:
        c, x, s_off, z_off = _offset_case(900 + L + K, B, L, K, 8)
        xq = ptq.quantize_pts_offset(x, 1.0 / c.m, s_off, z_off, B, L)
        torch.cuda.synchronize()
        xq_o = oracle.quantize_pts_offset(_np(x), _np(1.0 / c.m), _np(s_off), _np(z_off), B, L)
        assert np.array_equal(_np(xq), xq_o), (B, L, K)


FUSED_OFFSET_SHAPES = [  # B, L, K, N, ldy, bias
    # weight-resident kernel (N <= 128, K a multiple of 64, >= 2048 rows)
    (83, 199, 128, 44, None, True),      # 2 k-steps; M mod 32 = 5
    (64, 257, 320, 80, None, False),     # 5 k-steps (depth 1)
    (70, 241, 1024, 96, None, True),     # 16 k-steps, 6 channel blocks
    (70, 241, 512, 128, None, True),     # 8 channel blocks
    (83, 199, 1536, 72, 80, True),       # x_proj-like, padded output rows
    (13, 163, 192, 33, None, False),     # 2119 rows, M mod 8 = 7: the last group is ragged
    # row-streaming kernel (K <= 128, >= 1024 rows)
    (105, 197, 40, 100, 104, True),      # padded output rows
    (21, 199, 12, 130, None, True),      # 24-byte fp16 rows
    (35, 120, 128, 200, None, True),     # two k-steps (N > 128: not the weight-resident kernel)
    (33, 127, 100, 33, 40, True),        # odd N with padding; M mod 16 = 15
    (30, 197, 48, 1536, None, True),     # dt_proj (Vim-B) shape on fewer rows
    (11, 100, 13, 5, None, True),        # nothing aligned
]


@pytest.mark.parametrize("B,L,K,N,ldy,bias", FUSED_OFFSET_SHAPES)
def test_fused_zero_offset_whole_result(B, L, K, N, ldy, bias):
    """Every code, accumulator and output of the one-launch zero-offset form against the oracle and the two launches."""
    print(f"fused offset B={B} L={L} K={K} N={N} ldy={ldy} bias={bias}", flush=True)
    c, x, s_off, z_off = _offset_case(8100 + K + N, B, L, K, N)
    M = B * L
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    rowsum = ptq.weight_rowsum(wq)
    b = c.bias if bias else None
    acc = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
    xq = torch.full((M, K), 0x55, dtype=torch.int8, device=DEV)
    ybuf = None
    if ldy is None:
        y = ptq.w8a8_linear_offset_fused(x, inv_m, s_off, z_off, wq, rowsum, s_w, b, B, L, acc_out=acc, xq_out=xq)
    else:
        ybuf, yv = _padded(M, N, ldy, torch.float16, 12345.0)
        y = ptq.w8a8_linear_offset_fused(x, inv_m, s_off, z_off, wq, rowsum, s_w, b, B, L, y=yv, acc_out=acc, xq_out=xq)
    y2 = ptq.w8a8_linear_offset_fused(x, inv_m, s_off, z_off, wq, rowsum, s_w, b, B, L)  # timed configuration
    xq_two = ptq.quantize_pts_offset(x, inv_m, s_off, z_off, B, L)
    y_two = ptq.w8a8_linear_offset(xq_two, wq, s_off, z_off, rowsum, s_w, b, B, L)
    torch.cuda.synchronize()

    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing(_np(c.w), _np(c.m))
    rowsum_o = oracle.weight_rowsum(wq_o)
    xq_o = oracle.quantize_pts_offset(_np(x), inv_m_o, _np(s_off), _np(z_off), B, L)
    acc_o = oracle.int8_gemm(xq_o, wq_o)
    b_o = _np(c.bias) if bias else None
    y_o, y64 = oracle.dequant_offset(acc_o, _np(s_off), _np(z_off), rowsum_o, s_w_o, b_o, B, L)
    assert np.array_equal(_np(xq), xq_o), "int8 codes differ"
    assert xq_o.min() == -128 or xq_o.max() == 127                    # the clip is exercised
    assert np.array_equal(_np(acc), acc_o), "int32 accumulators differ"
    st = np.tile(_np(s_off).astype(np.float64), B)[:, None]
    zt = np.tile(_np(z_off).astype(np.float64), B)[:, None]
    corrected = acc_o.astype(np.float64) - zt * rowsum_o.astype(np.float64)[None, :]
    prod_abs = np.abs(corrected * st * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(b_o.astype(np.float64))[None, :] if bias else 0.0, prod_abs.shape)
    check_dequantized_output(_np(y), y_o, y64, prod_abs, bias_abs, "fused offset")
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16)), "the parity outputs change the result"
    assert torch.equal(y.view(torch.int16), y_two.view(torch.int16)), "fused and two-launch forms differ"
    if ybuf is not None:
        assert np.all(_np(ybuf[:, N:]) == np.float16(12345.0))


@pytest.mark.parametrize("linear", [1, 2])
def test_fused_zero_offset_vim_b_full_size_sampled(linear):
    """x_proj and dt_proj of Vim-B at the timed size: the one-launch zero-offset form on sampled rows."""
    c = synth.make_linear_case(3, 0, linear, device=DEV)
    M = c.B * c.L
    print(f"fused offset full-size {c.name}: M={M} K={c.K} N={c.N}", flush=True)
    shift = synth.token_shift(c.L, 77 + linear, device=DEV)
    x = (c.x.view(c.B, c.L, c.K) + shift.view(1, c.L, 1).to(c.x.dtype)).reshape(M, c.K).contiguous()
    s_off, z_off = synth.calibrate_offset(x[: 16 * c.L], c.m, c.L)
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    rowsum = ptq.weight_rowsum(wq)
    y = ptq.w8a8_linear_offset_fused(x, inv_m, s_off, z_off, wq, rowsum, s_w, c.bias, c.B, c.L)
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    xq = torch.full((M, c.K), 0x55, dtype=torch.int8, device=DEV)
    y_dump = ptq.w8a8_linear_offset_fused(x, inv_m, s_off, z_off, wq, rowsum, s_w, c.bias, c.B, c.L, acc_out=acc, xq_out=xq)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y_dump.view(torch.int16))
    rows = _sampled_rows(M, 97, c.L)
    ridx = torch.from_numpy(rows).to(DEV)
    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing(_np(c.w), _np(c.m))
    rowsum_o = oracle.weight_rowsum(wq_o)
    st_rows, z_rows = _np(s_off)[rows % c.L], _np(z_off)[rows % c.L]
    n = len(rows)
    xq_o = oracle.quantize_pts_offset(_np(x[ridx]), inv_m_o, st_rows, z_rows, 1, n)
    assert np.array_equal(_np(xq[ridx]), xq_o), "int8 codes differ"
    acc_o = oracle.int8_gemm(xq_o, wq_o)
    assert np.array_equal(_np(acc[ridx]), acc_o), "int32 accumulators differ"
    y_o, y64 = oracle.dequant_offset(acc_o, st_rows, z_rows, rowsum_o, s_w_o, _np(c.bias), 1, n)
    corrected = acc_o.astype(np.float64) - z_rows.astype(np.float64)[:, None] * rowsum_o.astype(np.float64)[None, :]
    prod_abs = np.abs(corrected * st_rows.astype(np.float64)[:, None] * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(_np(c.bias).astype(np.float64))[None, :], prod_abs.shape)
    check_dequantized_output(_np(y[ridx]), y_o, y64, prod_abs, bias_abs, f"fused offset {c.name}")


def test_fused_zero_offset_specials_and_refused_shapes():
    """Infinities and NaN with offsets at both ends of the int8 range (the saturated conversion must not wrap when the
    offset is added); shapes outside the two kernels return PTQ4VM_ERR_SHAPE."""
    B, L, K, N = 8, 256, 64, 32
    c = synth.random_problem(31, B, L, K, N, device=DEV)
    x = c.x.clone()
    x[::3, 0] = float("inf")
    x[1::3, 1] = float("-inf")
    x[2::3, 2] = float("nan")
    x[::5, 3] = 65504.0
    z = torch.randint(-128, 128, (L,), dtype=torch.int32, device=DEV)
    z[0], z[1] = 127, -128
    wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
    rowsum = ptq.weight_rowsum(wq)
    xq = torch.empty((B * L, K), dtype=torch.int8, device=DEV)
    ptq.w8a8_linear_offset_fused(x, inv_m, c.s_tok, z, wq, rowsum, s_w, c.bias, B, L, xq_out=xq)
    torch.cuda.synchronize()
    xq_o = oracle.quantize_pts_offset(_np(x), _np(inv_m), _np(c.s_tok), _np(z), B, L)
    assert np.array_equal(_np(xq), xq_o)
    for Bs, Ls, Ks, Ns in [(1, 50, 64, 32), (20, 197, 768, 3072)]:
        cs = synth.random_problem(78, Bs, Ls, Ks, Ns, device=DEV)
        wq, s_w, inv_m = ptq.fold_smoothing(cs.w, cs.m)
        zz = torch.zeros(Ls, dtype=torch.int32, device=DEV)
        with pytest.raises(ptq.Ptq4vmError) as e:
            ptq.w8a8_linear_offset_fused(cs.x, inv_m, cs.s_tok, zz, wq, ptq.weight_rowsum(wq), s_w, cs.bias, Bs, Ls)
        assert e.value.status == -2  # PTQ4VM_ERR_SHAPE


# ---------------------------------------------------------------------------------- W4A4 (packed 4-bit codes)
def _steps_4bit(c):
    """The calibrated +-127 steps rescaled to the +-7 range (input preparation, fp32)."""
    return (c.s_tok * (127.0 / 7.0)).contiguous()


W4A4_SHAPES = [  # B, L, K, N
    (3, 197, 384, 192), (2, 197, 192, 768), (2, 197, 384, 44), (3, 197, 12, 384), (2, 65, 24, 768), (2, 50, 768, 56),
    (1, 300, 1536, 80), (1, 1, 64, 32), (1, 257, 100, 130), (2, 33, 14, 5), (1, 129, 1000, 257), (5, 7, 16, 1),
    (2, 140, 128, 300),
]


@pytest.mark.parametrize("B,L,K,N", W4A4_SHAPES)
def test_w4a4_path_against_oracle(B, L, K, N):
    print(f"w4a4 B={B} L={L} K={K} N={N}", flush=True)
    c = synth.random_problem(53 * K + N, B, L, K, N, device=DEV)
    s4 = _steps_4bit(c)
    M = B * L
    wq4, s_w, inv_m = ptq.fold_smoothing_w4(c.w, c.m)
    xq4 = ptq.quantize_pts_a4(c.x, inv_m, s4, B, L)
    acc = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
    y = ptq.w4a4_linear(xq4, wq4, s4, s_w, c.bias, B, L, acc_out=acc)
    y2 = ptq.w4a4_linear(xq4, wq4, s4, s_w, c.bias, B, L)
    torch.cuda.synchronize()

    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing_bits(_np(c.w), _np(c.m), 4)
    xq_o = oracle.quantize_pts_bits(_np(c.x), inv_m_o, _np(s4), B, L, 4)
    assert np.array_equal(_np(s_w).view(np.uint32), s_w_o.view(np.uint32))
    assert np.array_equal(_np(inv_m).view(np.uint32), inv_m_o.view(np.uint32))
    assert np.array_equal(_np(wq4), oracle.pack_int4(wq_o)), "packed weight codes differ"
    assert np.array_equal(_np(xq4), oracle.pack_int4(xq_o)), "packed activation codes differ"
    y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, _np(s4), s_w_o, _np(c.bias), B, L)
    assert np.array_equal(_np(acc), acc_o), "int32 accumulators differ"
    st = np.tile(_np(s4).astype(np.float64), B)[:, None]
    prod_abs = np.abs(acc_o.astype(np.float64) * st * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(_np(c.bias).astype(np.float64))[None, :], prod_abs.shape)
    check_dequantized_output(_np(y), y_o, y64, prod_abs, bias_abs, "w4a4")
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))


def test_w4a4_all_nibble_pairs_through_the_linear():
    """Every (activation code, weight code) pair in [-8, 7]^2, including the -8 the quantizers never emit."""
    codes = np.arange(-8, 8, dtype=np.int8)
    xq = np.repeat(codes, 16)[None, :].repeat(3, axis=0)             # [3, 256]
    wq = np.tile(codes, 16)[None, :].repeat(2, axis=0)
    wq[1] = wq[1, ::-1]
    xq4 = torch.from_numpy(oracle.pack_int4(xq)).to(DEV)
    wq4 = torch.from_numpy(oracle.pack_int4(wq)).to(DEV)
    s_tok = torch.full((3,), 2.0 ** -6, device=DEV)
    s_w = torch.full((2,), 2.0 ** -5, device=DEV)
    acc = torch.empty((3, 2), dtype=torch.int32, device=DEV)
    y = ptq.w4a4_linear(xq4, wq4, s_tok, s_w, None, 1, 3, acc_out=acc)
    torch.cuda.synchronize()
    y_o, y64, acc_o = oracle.w8a8_linear(xq, wq, _np(s_tok), _np(s_w), None, 1, 3)
    assert np.array_equal(_np(acc), acc_o)
    assert np.array_equal(_np(y).view(np.uint16), y_o.view(np.uint16))


def _check_w4a4_on_sampled_rows(c, what):
    M = c.B * c.L
    print(f"w4a4 full-size {what}: M={M} K={c.K} N={c.N}", flush=True)
    s4 = _steps_4bit(c)
    wq4, s_w, inv_m = ptq.fold_smoothing_w4(c.w, c.m)
    xq4 = ptq.quantize_pts_a4(c.x, inv_m, s4, c.B, c.L)
    y = ptq.w4a4_linear(xq4, wq4, s4, s_w, c.bias, c.B, c.L)
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    y_dump = ptq.w4a4_linear(xq4, wq4, s4, s_w, c.bias, c.B, c.L, acc_out=acc)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y_dump.view(torch.int16))
    rows = _sampled_rows(M, 97, c.L)
    ridx = torch.from_numpy(rows).to(DEV)
    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing_bits(_np(c.w), _np(c.m), 4)
    st_rows = _np(s4)[rows % c.L]
    xq_o = oracle.quantize_pts_bits(_np(c.x[ridx]), inv_m_o, st_rows, 1, len(rows), 4)
    assert np.array_equal(_np(xq4[ridx]), oracle.pack_int4(xq_o))
    y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, st_rows, s_w_o, _np(c.bias), 1, len(rows))
    assert np.array_equal(_np(acc[ridx]), acc_o), "int32 accumulators differ"
    prod_abs = np.abs(acc_o.astype(np.float64) * st_rows.astype(np.float64)[:, None] * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(_np(c.bias).astype(np.float64))[None, :], prod_abs.shape)
    check_dequantized_output(_np(y[ridx]), y_o, y64, prod_abs, bias_abs, f"w4a4 {what}")


@pytest.mark.parametrize("cfg,linear", [(3, 0), (3, 1), (3, 2), (3, 3), (1, 2)])
def test_w4a4_full_size_sampled(cfg, linear):
    c = synth.make_linear_case(cfg, 0, linear, device=DEV)
    _check_w4a4_on_sampled_rows(c, f"cfg{cfg} {c.name}")


@pytest.mark.parametrize("B,L,K,N", [(41, 251, 512, 1544), (20, 517, 768, 3400), (300, 65, 24, 776), (250, 33, 100, 520),
                                     (110, 197, 24, 776), (105, 197, 100, 520), (107, 199, 48, 1536), (104, 197, 128, 130)])
def test_w4a4_large_ragged_shapes_sampled(B, L, K, N):
    """Ragged last tiles in the persistent kernel (128-row tiles; 2 and 3 slabs of packed bytes), in
    the short-reduction kernel (12 and 50 packed bytes per row) and, from 20 480 rows, in the row-streaming
    kernel (12, 50, 24 and 64 packed bytes per row: one and two k-steps once expanded, ragged rows and channels)."""
    c = synth.random_problem(6000 + K + N, B, L, K, N, device=DEV)
    _check_w4a4_on_sampled_rows(c, "ragged")


def _run_fused_w4a4_case(c, use_bias=True, use_m=True, ldy=None, what=""):
    """ptq4vm_w4a4_linear_fused on the GPU vs the oracle's 4-bit quantizer -> GEMM -> dequantization chain."""
    print(f"fused w4a4 {what} B={c.B} L={c.L} K={c.K} N={c.N} bias={use_bias} m={use_m} ldy={ldy}", flush=True)
    M = c.B * c.L
    s4 = _steps_4bit(c)
    m = c.m if use_m else torch.ones_like(c.m)
    wq4, s_w, inv_m = ptq.fold_smoothing_w4(c.w, m)
    bias = c.bias if use_bias else None
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    xq = torch.full((M, c.K), 0x55, dtype=torch.int8, device=DEV)
    ybuf = None
    if ldy is None:
        y = ptq.w4a4_linear_fused(c.x, inv_m if use_m else None, s4, wq4, s_w, bias, c.B, c.L, acc_out=acc, xq_out=xq)
    else:
        ybuf, yv = _padded(M, c.N, ldy, torch.float16, 12345.0)
        y = ptq.w4a4_linear_fused(c.x, inv_m if use_m else None, s4, wq4, s_w, bias, c.B, c.L, y=yv, acc_out=acc, xq_out=xq)
    y2 = ptq.w4a4_linear_fused(c.x, inv_m if use_m else None, s4, wq4, s_w, bias, c.B, c.L)  # timed configuration
    torch.cuda.synchronize()

    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing_bits(_np(c.w), _np(m), 4)
    xq_o = oracle.quantize_pts_bits(_np(c.x), inv_m_o if use_m else None, _np(s4), c.B, c.L, 4)
    b_o = _np(c.bias) if use_bias else None
    y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, _np(s4), s_w_o, b_o, c.B, c.L)
    assert np.array_equal(_np(wq4), oracle.pack_int4(wq_o))
    assert np.array_equal(_np(xq), xq_o), "4-bit codes differ"
    assert np.array_equal(_np(acc), acc_o), "int32 accumulators differ"
    st = np.tile(_np(s4).astype(np.float64), c.B)[:, None]
    prod_abs = np.abs(acc_o.astype(np.float64) * st * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(b_o.astype(np.float64))[None, :] if use_bias else 0.0, prod_abs.shape)
    check_dequantized_output(_np(y), y_o, y64, prod_abs, bias_abs, what)
    assert np.array_equal(_np(y).view(np.uint16), _np(y2).view(np.uint16)), "the parity outputs change the result"
    if ybuf is not None:
        assert np.all(_np(ybuf[:, c.N:]) == np.float16(12345.0))
    # the two-launch form gives the same bits
    xq4 = ptq.quantize_pts_a4(c.x, inv_m if use_m else None, s4, c.B, c.L)
    y_two = ptq.w4a4_linear(xq4, wq4, s4, s_w, bias, c.B, c.L)
    torch.cuda.synchronize()
    assert np.array_equal(_np(y).view(np.uint16), _np(y_two).view(np.uint16)), "fused and two-launch forms differ"


FUSED_W4A4_SHAPES = [  # B, L, K, N, ldy, bias, m
    # weight-resident kernel (N <= 128, K a multiple of 64, >= 2048 rows)
    (83, 199, 128, 44, None, True, True),     # 2 k-steps; M mod 32 = 5
    (64, 257, 320, 80, None, False, True),    # 5 k-steps (depth 1)
    (70, 241, 1024, 96, None, True, True),    # 16 k-steps, 6 channel blocks
    (70, 241, 512, 128, None, True, True),    # 8 channel blocks
    (83, 199, 768, 50, None, True, False),    # N not a multiple of 4; no smoothing
    (83, 199, 1536, 72, 80, True, True),      # x_proj-like, padded output rows
    (66, 250, 1600, 16, None, True, True),    # 25 k-steps; one channel block
    (13, 163, 192, 33, None, False, True),    # 2119 rows, M mod 8 = 7: the last group is ragged
    # row-streaming kernel (K <= 128, >= 1024 rows)
    (105, 197, 40, 100, 104, True, True),     # 20-byte packed weight rows, padded output rows
    (21, 199, 12, 130, None, True, True),     # 6 packed bytes per weight row: element-wise weight loads
    (35, 120, 128, 200, None, True, True),    # two k-steps (N > 128: not the weight-resident kernel)
    (33, 127, 100, 33, 40, True, False),      # odd N with padding; M mod 16 = 15; K a multiple of 4 only
    (30, 197, 48, 1536, None, True, True),    # dt_proj (Vim-B) shape on fewer rows
    (30, 197, 24, 576, None, False, True),    # 9 channel groups in 4 parts of 3: the last part is empty
    (11, 100, 14, 5, None, True, True),       # K even only
]


@pytest.mark.parametrize("B,L,K,N,ldy,bias,use_m", FUSED_W4A4_SHAPES)
def test_fused_w4a4_whole_result(B, L, K, N, ldy, bias, use_m):
    """Every code, accumulator and output of the one-launch W4A4 form against the oracle, and against the two launches."""
    c = synth.random_problem(4321 + K + N, B, L, K, N, device=DEV)
    _run_fused_w4a4_case(c, use_bias=bias, use_m=use_m, ldy=ldy, what="fused-w4a4")


@pytest.mark.parametrize("linear", [1, 2])
def test_fused_w4a4_vim_b_full_size_sampled(linear):
    """x_proj and dt_proj of Vim-B at the timed size: the one-launch W4A4 form on sampled rows against the oracle."""
    c = synth.make_linear_case(3, 0, linear, device=DEV)
    M = c.B * c.L
    print(f"fused w4a4 full-size {c.name}: M={M} K={c.K} N={c.N}", flush=True)
    s4 = _steps_4bit(c)
    wq4, s_w, inv_m = ptq.fold_smoothing_w4(c.w, c.m)
    y = ptq.w4a4_linear_fused(c.x, inv_m, s4, wq4, s_w, c.bias, c.B, c.L)
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    xq = torch.full((M, c.K), 0x55, dtype=torch.int8, device=DEV)
    y_dump = ptq.w4a4_linear_fused(c.x, inv_m, s4, wq4, s_w, c.bias, c.B, c.L, acc_out=acc, xq_out=xq)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y_dump.view(torch.int16))
    rows = _sampled_rows(M, 97, c.L)
    ridx = torch.from_numpy(rows).to(DEV)
    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing_bits(_np(c.w), _np(c.m), 4)
    st_rows = _np(s4)[rows % c.L]
    xq_o = oracle.quantize_pts_bits(_np(c.x[ridx]), inv_m_o, st_rows, 1, len(rows), 4)
    assert np.array_equal(_np(xq[ridx]), xq_o)
    y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, st_rows, s_w_o, _np(c.bias), 1, len(rows))
    assert np.array_equal(_np(acc[ridx]), acc_o), "int32 accumulators differ"
    prod_abs = np.abs(acc_o.astype(np.float64) * st_rows.astype(np.float64)[:, None] * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(_np(c.bias).astype(np.float64))[None, :], prod_abs.shape)
    check_dequantized_output(_np(y[ridx]), y_o, y64, prod_abs, bias_abs, f"fused w4a4 {c.name}")


def test_fused_w4a4_shapes_outside_its_kernels_are_refused():
    """Fewer rows than either kernel takes, or a long reduction with many channels: PTQ4VM_ERR_SHAPE, nothing written."""
    for B, L, K, N in [(1, 50, 64, 32), (20, 197, 768, 3072), (70, 241, 1024, 128)]:  # the last: tables beyond the LDS
        c = synth.random_problem(77, B, L, K, N, device=DEV)
        s4 = _steps_4bit(c)
        wq4, s_w, inv_m = ptq.fold_smoothing_w4(c.w, c.m)
        y = torch.full((B * L, N), 3.0, dtype=torch.float16, device=DEV)
        with pytest.raises(ptq.Ptq4vmError) as e:
            ptq.w4a4_linear_fused(c.x, inv_m, s4, wq4, s_w, c.bias, B, L, y=y)
        assert e.value.status == -2  # PTQ4VM_ERR_SHAPE
        torch.cuda.synchronize()
        assert bool((y == 3.0).all())


def test_fused_linear_every_fp16_value():
    """All 65 536 fp16 bit patterns (subnormals, infinities, NaNs) through the fused weight-resident kernel's
    quantizer, with steps from 1e-8 to 10 so that subnormal inputs reach non-zero codes: the codes it feeds
    to the MFMA must equal the oracle's."""
    B, L, K, N = 64, 256, 64, 16
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    x = bits.repeat(B * L * K // 65536).view(torch.float16).reshape(B * L, K).to(DEV).contiguous()
    g = torch.Generator().manual_seed(5)
    s_tok = (10.0 ** (torch.rand(L, generator=g) * 9.0 - 8.0)).to(DEV)
    inv_m = (0.5 + torch.rand(K, generator=g)).to(DEV)
    wq = torch.randint(-127, 128, (N, K), generator=g, dtype=torch.int8).to(DEV)
    s_w = torch.full((N,), 2.0 ** -10, device=DEV)
    xq = torch.full((B * L, K), 0x55, dtype=torch.int8, device=DEV)
    ptq.w8a8_linear_fused(x, inv_m, s_tok, wq, s_w, None, B, L, xq_out=xq)
    xq_two = ptq.quantize_pts(x, inv_m, s_tok, B, L)
    torch.cuda.synchronize()
    xq_o = oracle.quantize_pts(_np(x), _np(inv_m), _np(s_tok), B, L)
    assert np.array_equal(_np(xq), xq_o)
    assert np.array_equal(_np(xq_two), xq_o)


STREAM_SHAPES = [  # B, L, K, N, ldy, bias: short reductions, ragged channel counts.  The row-streaming kernel takes the
    # fused form from 1024 rows and the two-launch form from 20480 rows (the channel-strip kernel below that).
    (105, 197, 40, 100, 104, True),    # 20685 rows: both forms on the row-streaming kernel; padded rows (8-byte stores)
    (104, 199, 12, 130, None, True),   # 20696 rows; 12-byte int8 rows / 24-byte fp16 rows
    (172, 120, 128, 64, None, False),  # 20640 rows; two k-steps
    (22, 197, 40, 100, 104, True),     # N not a multiple of 64, padded rows (8-byte stores)
    (22, 197, 48, 70, None, False),    # 140-byte rows: 4-byte aligned only
    (21, 199, 12, 130, None, True),    # 12-byte int8 rows / 24-byte fp16 rows
    (35, 120, 128, 64, None, True),    # two k-steps
    (33, 127, 100, 33, 40, True),      # odd N with padding; M mod 16 = 15
    (106, 197, 48, 320, None, True),   # 5 channel groups in 4 parts of 2: the last part is half empty
    (30, 197, 24, 576, None, False),   # 9 channel groups in 4 parts of 3: the last part is empty
]


@pytest.mark.parametrize("B,L,K,N,ldy,bias", STREAM_SHAPES)
def test_short_reduction_many_rows_two_launch_and_fused(B, L, K, N, ldy, bias):
    c = synth.random_problem(3100 + K + N, B, L, K, N, device=DEV)
    _run_w8a8_case(c, use_bias=bias, ldy=ldy, what="stream")
    _run_fused_case(c, use_bias=bias, ldy=ldy, what="stream-fused")


# ---------------------------------------------------------------------------------- scale validator
def test_validate_scales_counts_bad_entries():
    """Not part of the method's arithmetic: the expected counts are plain numpy predicates on the inputs."""
    g = torch.Generator().manual_seed(11)
    for L, K, N in [(197, 768, 3072), (785, 24, 56), (1, 1, 1), (5000, 4096, 9000)]:
        vecs = [torch.rand(n, generator=g) + 0.01 for n in (L, K, N)]
        rc, counts = ptq.validate_scales(*[v.to(DEV) for v in vecs])
        assert rc == 0 and _np(counts).tolist() == [0, 0, 0], (L, K, N)
        bad_values = [0.0, -1.0, float("nan"), float("inf"), float("-inf"), -0.0]
        for vi, v in enumerate(vecs):
            for j, b in enumerate(bad_values):
                if j < v.numel():
                    v[(j * 977 + vi) % v.numel()] = b
        want = [int(np.count_nonzero(~((_v > 0) & np.isfinite(_v)))) for _v in (v.numpy() for v in vecs)]
        rc, counts = ptq.validate_scales(*[v.to(DEV) for v in vecs])
        assert rc == -6 and _np(counts).tolist() == want, (L, K, N, want)
    # a vector may be absent; denormal steps are valid
    rc, counts = ptq.validate_scales(torch.full((3,), 1e-40, device=DEV), None, None)
    assert rc == 0 and _np(counts).tolist() == [0, 0, 0]
