"""GPU parity of the W4A4 entry points that keep the 4-bit codes in the FP6 (E2M3) container
(ptq4vm_fold_smoothing_w4_e2m3, ptq4vm_quantize_pts_a4_e2m3, ptq4vm_w4a4_linear_e2m3), called through the C ABI,
against the CPU oracle on the same seeded inputs: container bytes and int32 accumulators bit-exact, fp16
outputs within 1 fp16 ulp (parity_util.check_dequantized_output)."""
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


def _steps_4bit(c):
    """The calibrated +-127 steps rescaled to the +-7 range (input preparation, fp32)."""
    return (c.s_tok * (127.0 / 7.0)).contiguous()


def _sampled_rows(M, step, L):
    rows = np.unique(np.concatenate([np.arange(0, M, step), [0, 1, L - 1, L, M - 1, M - 2], np.arange(M - 300, M, 7)]))
    return rows[(rows >= 0) & (rows < M)]


E2M3_SHAPES = [  # B, L, K, N: small tiled kernel (few tiles, odd shapes) and persistent kernel (>= 128 tiles of 256 x 256)
    (3, 197, 384, 192), (2, 197, 192, 768), (2, 197, 384, 44), (3, 197, 12, 384), (2, 50, 768, 56),
    (1, 300, 1536, 80), (1, 1, 64, 32), (1, 257, 100, 130), (2, 33, 14, 5), (1, 129, 1000, 257), (5, 7, 16, 1),
    (2, 140, 128, 300), (1, 70, 33, 9),
    (33, 197, 256, 1288),   # persistent: 26 x 6 tiles, 2 blocks, ragged last row and channel tiles
    (40, 211, 384, 776),    # persistent: 33 x 4 tiles, 3 blocks, N = 8 (mod 256)
]


@pytest.mark.parametrize("B,L,K,N", E2M3_SHAPES)
def test_e2m3_path_against_oracle(B, L, K, N):
    print(f"w4a4 e2m3 B={B} L={L} K={K} N={N}", flush=True)
    c = synth.random_problem(59 * K + N, B, L, K, N, device=DEV)
    s4 = _steps_4bit(c)
    M = B * L
    wq6, s_w, inv_m = ptq.fold_smoothing_w4_e2m3(c.w, c.m)
    xq6 = ptq.quantize_pts_a4_e2m3(c.x, inv_m, s4, B, L)
    acc = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
    y = ptq.w4a4_linear_e2m3(xq6, wq6, s4, s_w, c.bias, B, L, K, acc_out=acc)
    y2 = ptq.w4a4_linear_e2m3(xq6, wq6, s4, s_w, c.bias, B, L, K)
    y3 = ptq.w4a4_linear_e2m3(xq6, wq6, s4, s_w, None, B, L, K)
    torch.cuda.synchronize()

    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing_bits(_np(c.w), _np(c.m), 4)
    xq_o = oracle.quantize_pts_bits(_np(c.x), inv_m_o, _np(s4), B, L, 4)
    assert np.array_equal(_np(s_w).view(np.uint32), s_w_o.view(np.uint32))
    assert np.array_equal(_np(inv_m).view(np.uint32), inv_m_o.view(np.uint32))
    assert np.array_equal(_np(wq6), oracle.pack_e2m3(wq_o)), "weight containers differ"
    assert np.array_equal(_np(xq6), oracle.pack_e2m3(xq_o)), "activation containers differ"
    assert np.abs(xq_o.astype(np.int32)).max() >= 2  # the case is not degenerate
    y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, _np(s4), s_w_o, _np(c.bias), B, L)
    assert np.array_equal(_np(acc), acc_o), "int32 accumulators differ"
    st = np.tile(_np(s4).astype(np.float64), B)[:, None]
    prod_abs = np.abs(acc_o.astype(np.float64) * st * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(_np(c.bias).astype(np.float64))[None, :], prod_abs.shape)
    check_dequantized_output(_np(y), y_o, y64, prod_abs, bias_abs, "w4a4 e2m3")
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    y_nb, y64_nb, _ = oracle.w8a8_linear(xq_o, wq_o, _np(s4), s_w_o, None, B, L)
    check_dequantized_output(_np(y3), y_nb, y64_nb, prod_abs, np.zeros_like(prod_abs), "w4a4 e2m3, no bias")


def test_e2m3_codes_and_accumulators_equal_the_nibble_path():
    """Same codes, two containers: the two W4A4 paths hold the same codes and produce the same accumulators."""
    B, L, K, N = 3, 197, 384, 200
    c = synth.random_problem(77, B, L, K, N, device=DEV)
    s4 = _steps_4bit(c)
    wq6, s_w, inv_m = ptq.fold_smoothing_w4_e2m3(c.w, c.m)
    wq4, s_w4, _ = ptq.fold_smoothing_w4(c.w, c.m)
    xq6 = ptq.quantize_pts_a4_e2m3(c.x, inv_m, s4, B, L)
    xq4 = ptq.quantize_pts_a4(c.x, inv_m, s4, B, L)
    acc6 = torch.empty((B * L, N), dtype=torch.int32, device=DEV)
    acc4 = torch.empty_like(acc6)
    ptq.w4a4_linear_e2m3(xq6, wq6, s4, s_w, c.bias, B, L, K, acc_out=acc6)
    ptq.w4a4_linear(xq4, wq4, s4, s_w4, c.bias, B, L, acc_out=acc4)
    torch.cuda.synchronize()
    assert torch.equal(s_w, s_w4) and torch.equal(acc6, acc4)
    assert np.array_equal(oracle.unpack_e2m3(_np(xq6), K), oracle.unpack_int4(_np(xq4)))
    assert np.array_equal(oracle.unpack_e2m3(_np(wq6), K), oracle.unpack_int4(_np(wq4)))


def test_e2m3_extreme_codes_and_every_code_pair():
    """All 15 x 15 code pairs, and rows of +-7 only over a long reduction (|acc| = 49 K: the largest sums)."""
    codes = np.arange(-7, 8, dtype=np.int8)
    xq = np.repeat(codes, 15)[None, :].repeat(3, axis=0)             # [3, 225]
    wq = np.tile(codes, 15)[None, :].repeat(2, axis=0)
    wq[1] = wq[1, ::-1]
    K = 1536
    big_x = np.full((3, K), 7, np.int8)
    big_x[1] = -7
    big_x[2, ::2] = -7
    big_w = np.full((2, K), 7, np.int8)
    big_w[1, ::3] = -7
    for xq_c, wq_c in ((xq, wq), (big_x, big_w)):
        Kc = xq_c.shape[1]
        xq6 = torch.from_numpy(oracle.pack_e2m3(xq_c)).to(DEV)
        wq6 = torch.from_numpy(oracle.pack_e2m3(wq_c)).to(DEV)
        s_tok = torch.full((3,), 2.0 ** -6, device=DEV)
        s_w = torch.full((2,), 2.0 ** -5, device=DEV)
        acc = torch.empty((3, 2), dtype=torch.int32, device=DEV)
        y = ptq.w4a4_linear_e2m3(xq6, wq6, s_tok, s_w, None, 1, 3, Kc, acc_out=acc)
        torch.cuda.synchronize()
        y_o, y64, acc_o = oracle.w8a8_linear(xq_c, wq_c, _np(s_tok), _np(s_w), None, 1, 3)
        assert np.array_equal(_np(acc), acc_o)
        assert np.array_equal(_np(y).view(np.uint16), y_o.view(np.uint16))


def test_e2m3_quantizer_special_values_padding_and_pitch():
    """NaN -> 0, +-Inf -> +-7, ties to even, negative values that round to zero (no "-0" pattern), a plane pitch
    wider than the rows need (bytes beyond them stay untouched), K that is no multiple of 32 (element path)."""
    for K in (64, 50):
        B, L = 2, 5
        M = B * L
        x = torch.zeros((M, K), dtype=torch.float16, device=DEV)
        vals = [float("nan"), float("inf"), float("-inf"), 0.5, 1.5, 2.5, -0.5, -1.5, -0.25, 0.25, -0.0, 6.5, 7.5, -7.5, 100.0, -100.0]
        x[:, :len(vals)] = torch.tensor(vals, dtype=torch.float16, device=DEV)
        x[:, len(vals):] = torch.linspace(-9, 9, K - len(vals), device=DEV).half()
        s_tok = torch.ones(L, device=DEV)
        buf = torch.full((ptq.e2m3_blocks(K), M + 3, 96), 0xAB, dtype=torch.uint8, device=DEV)  # planes 3 rows longer
        ptq.quantize_pts_a4_e2m3(x, None, s_tok, B, L, xq6=buf[:, :M, :])
        torch.cuda.synchronize()
        want = oracle.pack_e2m3(oracle.quantize_pts_bits(_np(x), None, _np(s_tok), B, L, 4))
        assert np.array_equal(_np(buf[:, :M, :]), want)
        assert (_np(buf[:, M:, :]) == 0xAB).all()


@pytest.mark.parametrize("B,L,K", [(40, 7, 128), (3, 5, 256), (1, 5000, 128), (1, 20000, 128), (7, 33, 96), (2, 9, 1000), (5, 197, 640)])
@pytest.mark.parametrize("use_m", [True, False])
def test_e2m3_quantizer_kernels(B, L, K, use_m):
    """Block-column kernel (K a multiple of 128; token periods shorter than a 16-row unit), the column-stationary
    kernel (longer token tables, K a multiple of 32 only; per-row division beyond the LDS table) and the element path."""
    print(f"quantize e2m3 B={B} L={L} K={K} use_m={use_m}", flush=True)
    c = synth.random_problem(4000 + 3 * L + K, B, L, K, 8, device=DEV)
    s4 = _steps_4bit(c)
    inv_m = (1.0 / c.m).contiguous() if use_m else None
    xq6 = ptq.quantize_pts_a4_e2m3(c.x, inv_m, s4, B, L)
    torch.cuda.synchronize()
    want = oracle.quantize_pts_bits(_np(c.x), _np(inv_m) if use_m else None, _np(s4), B, L, 4)
    assert np.array_equal(_np(xq6), oracle.pack_e2m3(want))


def _check_e2m3_on_sampled_rows(c, what):
    M = c.B * c.L
    print(f"w4a4 e2m3 full-size {what}: M={M} K={c.K} N={c.N}", flush=True)
    s4 = _steps_4bit(c)
    wq6, s_w, inv_m = ptq.fold_smoothing_w4_e2m3(c.w, c.m)
    xq6 = ptq.quantize_pts_a4_e2m3(c.x, inv_m, s4, c.B, c.L)
    y = ptq.w4a4_linear_e2m3(xq6, wq6, s4, s_w, c.bias, c.B, c.L, c.K)
    acc = torch.full((M, c.N), -1, dtype=torch.int32, device=DEV)
    y_dump = ptq.w4a4_linear_e2m3(xq6, wq6, s4, s_w, c.bias, c.B, c.L, c.K, acc_out=acc)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y_dump.view(torch.int16))
    rows = _sampled_rows(M, 97, c.L)
    ridx = torch.from_numpy(rows).to(DEV)
    wq_o, s_w_o, inv_m_o = oracle.fold_smoothing_bits(_np(c.w), _np(c.m), 4)
    assert np.array_equal(_np(wq6), oracle.pack_e2m3(wq_o))
    st_rows = _np(s4)[rows % c.L]
    xq_o = oracle.quantize_pts_bits(_np(c.x[ridx]), inv_m_o, st_rows, 1, len(rows), 4)
    assert np.array_equal(_np(xq6[:, ridx]), oracle.pack_e2m3(xq_o))
    y_o, y64, acc_o = oracle.w8a8_linear(xq_o, wq_o, st_rows, s_w_o, _np(c.bias), 1, len(rows))
    assert np.array_equal(_np(acc[ridx]), acc_o), "int32 accumulators differ"
    prod_abs = np.abs(acc_o.astype(np.float64) * st_rows.astype(np.float64)[:, None] * s_w_o.astype(np.float64)[None, :])
    bias_abs = np.broadcast_to(np.abs(_np(c.bias).astype(np.float64))[None, :], prod_abs.shape)
    check_dequantized_output(_np(y[ridx]), y_o, y64, prod_abs, bias_abs, f"w4a4 e2m3 {what}")
    # every row once more, cheaply: the accumulators of all rows against the nibble path's (already checked kernels)
    wq4, s_w4, _ = ptq.fold_smoothing_w4(c.w, c.m)
    xq4 = ptq.quantize_pts_a4(c.x, inv_m, s4, c.B, c.L)
    acc4 = torch.empty_like(acc)
    y4 = ptq.w4a4_linear(xq4, wq4, s4, s_w4, c.bias, c.B, c.L, acc_out=acc4)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc4), "accumulators differ from the nibble path's somewhere in the tensor"
    differing = (y.view(torch.int16) != y4.view(torch.int16)).sum().item()
    assert differing <= 1e-4 * y.numel(), f"{differing} outputs differ from the nibble path's"


@pytest.mark.parametrize("cfg,linear", [(3, 0), (3, 1), (3, 2), (3, 3), (2, 0), (1, 3)])
def test_e2m3_full_size_sampled(cfg, linear):
    c = synth.make_linear_case(cfg, 0, linear, device=DEV)
    _check_e2m3_on_sampled_rows(c, f"cfg{cfg} {c.name}")


@pytest.mark.parametrize("B,L,K,N", [(41, 251, 512, 1544), (20, 517, 768, 3400), (300, 65, 24, 776)])
def test_e2m3_large_ragged_shapes_sampled(B, L, K, N):
    c = synth.random_problem(6100 + K + N, B, L, K, N, device=DEV)
    _check_e2m3_on_sampled_rows(c, "ragged")


def test_e2m3_linear_is_deterministic():
    c = synth.make_linear_case(3, 0, 0, device=DEV)
    s4 = _steps_4bit(c)
    wq6, s_w, inv_m = ptq.fold_smoothing_w4_e2m3(c.w, c.m)
    xq6 = ptq.quantize_pts_a4_e2m3(c.x, inv_m, s4, c.B, c.L)
    first = ptq.w4a4_linear_e2m3(xq6, wq6, s4, s_w, c.bias, c.B, c.L, c.K).clone()
    for rep in range(10):
        again = ptq.w4a4_linear_e2m3(xq6, wq6, s4, s_w, c.bias, c.B, c.L, c.K)
        assert torch.equal(first.view(torch.int16), again.view(torch.int16)), f"repeat {rep} differs"
