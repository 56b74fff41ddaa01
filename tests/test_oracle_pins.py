"""Pins for the CPU oracle: it is checked against what the paper's equations and plain
mathematics fix, never against itself and never against the HIP path.

Each test names the passage it pins and the mistake it is meant to catch.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle

F16_ALL = np.arange(65536, dtype=np.uint32).astype(np.uint16)


def _rne_exact(v: np.ndarray) -> np.ndarray:
    """Round-half-to-even of float64 values (np.rint is RNE; values are far from 2^52)."""
    return np.rint(v)


# --------------------------------------------------------------------------------------
# fp16 conversions used by every oracle function
# --------------------------------------------------------------------------------------
def test_half_to_float_all_bit_patterns():
    want = F16_ALL.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in F16_ALL], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_double_to_half_exact_midpoints_and_random():
    halves = F16_ALL[(F16_ALL & 0x7C00) != 0x7C00].view(np.float16).astype(np.float64)
    pos = np.sort(np.unique(np.abs(halves)))
    mids = 0.5 * (pos[:-1] + pos[1:])                     # exact ties between neighbours
    nudged = np.concatenate([np.nextafter(mids, np.inf), np.nextafter(mids, -np.inf)])
    rng = np.random.default_rng(7)
    rnd = np.concatenate([
        rng.normal(size=4000) * 10.0 ** rng.integers(-9, 6, size=4000),
        [65504.0, 65519.999, 65520.0, 65536.0, 1e30, 2.0 ** -24, 2.0 ** -25,
         np.nextafter(2.0 ** -25, 1), 2.0 ** -26, 1e-300, 5e-324, 0.0, np.inf],
    ])
    vals = np.concatenate([halves, mids, nudged, rnd, -mids, -nudged, -rnd])
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)    # NumPy converts double->half directly
    got = np.array([oracle.double_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, want)
    assert np.isnan(np.array([oracle.double_to_half(float("nan"))], np.uint16).view(np.float16))[0]


# --------------------------------------------------------------------------------------
# a1: per-token static quantizer (Sec. 5.1; round/clip of Sec. 2.3)
# --------------------------------------------------------------------------------------
def test_quantizer_ties_saturation_and_specials():
    # step 1, no smoothing: codes are the rounded inputs. Catches half-away-from-zero
    # rounding, a -128 code, a missing clamp, NaN/Inf mishandling.
    x = np.array([[0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.5, 128.0, 1000.0,
                   np.inf, -np.inf, np.nan, -127.49, -127.5, -60000.0]], np.float16)
    want = np.array([[0, 2, 2, 0, -2, -2, 126, 127, 127, 127, 127, -127, 0, -127, -127, -127]],
                    np.int8)
    got = oracle.quantize_pts(x, None, np.ones(1, np.float32), 1, 1)
    assert np.array_equal(got, want)
    got = oracle.quantize_pts(x, np.ones(16, np.float32), np.ones(1, np.float32), 1, 1)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("m,s", [(1.0, 1.0), (3.7, 0.0131), (0.0123, 9.5), (250.0, 0.3),
                                 (1.0 / 3.0, 1.0 / 7.0)])
def test_quantizer_every_fp16_value_against_exact_division(m, s):
    """Definition: q = clip(rne(x / (m*s)), -127, 127).  The oracle evaluates the quotient with
    two fp32 multiplies by correctly rounded reciprocals (<= 4 roundings of 2^-24), so it must
    equal the exactly computed code except within 4e-5 of a rounding tie, where it may take
    either neighbour.  Catches a dropped or doubled factor, a wrong clamp, use of m for 1/m."""
    m32, s32 = np.float32(m), np.float32(s)
    inv_m = np.float32(1.0) / m32
    finite = F16_ALL[(F16_ALL & 0x7C00) != 0x7C00]
    x = finite.view(np.float16).reshape(1, -1)
    K = x.shape[1]
    q = oracle.quantize_pts(x, np.full(K, inv_m, np.float32), np.array([s32]), 1, 1).astype(np.int64)
    v = x.astype(np.float64) / (float(m32) * float(s32))
    exact = np.clip(_rne_exact(v), -127, 127).astype(np.int64)
    frac = np.abs(v - np.floor(v) - 0.5)                 # distance to the nearest tie
    near_tie = frac <= 4e-5 * np.maximum(1.0, np.abs(v) / 128.0)
    strict = ~near_tie
    assert np.array_equal(q[strict], exact[strict])
    lo = np.clip(np.floor(v), -127, 127)
    hi = np.clip(np.ceil(v), -127, 127)
    assert np.all((q[near_tie] == lo[near_tie]) | (q[near_tie] == hi[near_tie]))
    assert q.min() >= -127 and q.max() <= 127


def test_quantizer_half_step_bound_and_token_indexing():
    """|q*s_t - x/m_k| <= s_t/2 inside the clip range and codes saturate at +-127 outside it,
    with the step taken from the row's token position r mod L (not r div L, not the channel)."""
    rng = np.random.default_rng(11)
    B, L, K = 3, 5, 37
    x = (rng.laplace(size=(B * L, K)) * 4).astype(np.float16)
    m = rng.uniform(0.2, 5.0, K).astype(np.float32)
    s_tok = rng.uniform(0.005, 0.08, L).astype(np.float32)
    inv_m = (np.float32(1) / m).astype(np.float32)
    q = oracle.quantize_pts(x, inv_m, s_tok, B, L).astype(np.float64)
    xs = x.astype(np.float64) / m.astype(np.float64)[None, :]
    st = np.tile(s_tok.astype(np.float64), B)[:, None]
    inside = np.abs(xs) <= 127.0 * st
    err = np.abs(q * st - xs)
    assert inside.sum() > 100 and (~inside).sum() > 10
    assert np.all(err[inside] <= st.repeat(K, 1)[inside] * (0.5 + 2.0 ** -14))
    sat = np.abs(xs) >= 127.5 * st
    assert np.array_equal(q[sat], 127.0 * np.sign(xs[sat]))


def test_quantizer_constant_step_is_per_tensor_static():
    """With one step for every token PTS reduces to the per-tensor static symmetric quantizer
    (Sec. 4, Fig. 'overall').  A power-of-two step makes x/s exact in every precision, so the
    textbook clip(round(x/s)) must be reproduced bit for bit."""
    rng = np.random.default_rng(5)
    B, L, K = 4, 7, 33
    x = (rng.normal(size=(B * L, K)) * 3).astype(np.float16)
    s = np.float32(2.0 ** -5)
    q = oracle.quantize_pts(x, None, np.full(L, s, np.float32), B, L)
    textbook = np.clip(np.rint(x.astype(np.float64) / float(s)), -127, 127).astype(np.int8)
    assert np.array_equal(q, textbook)
    # L = 1: the same through the degenerate token vector
    q1 = oracle.quantize_pts(x, None, np.array([s], np.float32), B * L, 1)
    assert np.array_equal(q1, textbook)


def test_quantizer_error_statistics():
    """Uniform inputs inside the clip range: dequantization error is uniform on (-s/2, s/2),
    variance s^2/12."""
    rng = np.random.default_rng(3)
    s = np.float32(0.0371)
    x = rng.uniform(-120 * s, 120 * s, size=(1, 400_000)).astype(np.float16)
    q = oracle.quantize_pts(x, None, np.array([s], np.float32), 1, 1).astype(np.float64)
    err = q * float(s) - x.astype(np.float64)
    assert abs(err.var() / (float(s) ** 2 / 12.0) - 1.0) < 0.02
    assert abs(err.mean()) < 1e-3 * float(s)


# --------------------------------------------------------------------------------------
# a0: smoothing fold + per-output-channel symmetric weight quantizer (Eq. smooth; Sec. 2.3)
# --------------------------------------------------------------------------------------
def test_fold_generic_properties():
    rng = np.random.default_rng(21)
    N, K = 19, 53
    w = (rng.normal(size=(N, K)) * 0.02).astype(np.float16)
    w[7, :] = 0                                            # dead output channel
    m = rng.uniform(0.05, 30.0, K).astype(np.float32)
    wq, s_w, inv_m = oracle.fold_smoothing(w, m)
    wf = w.astype(np.float64) * m.astype(np.float64)[None, :]
    amax = np.abs(wf).max(axis=1)
    live = amax > 0
    # Delta_W = max|W'| / (2^(b-1) - 1), per output channel (row), after the fold
    assert np.allclose(s_w[live], amax[live] / 127.0, rtol=3e-7, atol=0)
    assert s_w[7] == 1.0 and np.all(wq[7] == 0)
    # each live row reaches +-127 exactly where its maximum sits; -128 never appears
    assert np.all(np.abs(wq.astype(np.int32)).max(axis=1)[live] == 127)
    assert wq.min() >= -127
    assert np.array_equal(np.abs(wq.astype(np.int32)).argmax(axis=1)[live], np.abs(wf).argmax(axis=1)[live])
    # round-to-nearest: reconstruction error at most half a step
    rec = wq.astype(np.float64) * s_w.astype(np.float64)[:, None]
    assert np.all(np.abs(rec - wf) <= s_w.astype(np.float64)[:, None] * (0.5 + 1e-4))
    # codes equal the exactly computed ones away from ties
    v = wf / s_w.astype(np.float64)[:, None]
    away = np.abs(v - np.floor(v) - 0.5) > 1e-4
    assert np.array_equal(wq[away], np.rint(v)[away].astype(np.int8))
    # inverse smoothing vector: correctly rounded reciprocal
    assert np.array_equal(inv_m, (np.float32(1) / m).astype(np.float32))
    exact = np.array([float(Fraction(1) / Fraction(float(mk))) for mk in m])
    assert np.all(np.abs(inv_m.astype(np.float64) - exact) <= 2.0 ** -24 * exact)


def test_smoothing_identity_exact_with_power_of_two_scales():
    """Eq. (smooth): (X diag(m)^-1)(W diag(m))^T = X W^T.  With power-of-two m and values placed
    on the quantization grids nothing is rounded anywhere, so fold -> quantize -> integer GEMM
    -> dequantize must reproduce X W^T + b exactly.  Catches transposed operands, s_w/s_tok
    swapped or indexed by the wrong axis, r div L used for r mod L, m used for 1/m, a dropped
    bias, sign errors."""
    rng = np.random.default_rng(2)
    B, L, K, N = 3, 4, 10, 6
    M = B * L
    A = rng.integers(-127, 128, size=(M, K))               # intended activation codes
    C = rng.integers(-126, 127, size=(N, K))               # intended weight codes
    C[np.arange(N), rng.integers(0, K, N)] = rng.choice([-127, 127], N)  # row max = 127
    e_m = rng.integers(-3, 4, K)
    e_t = rng.integers(-6, 0, L)
    e_w = rng.integers(-9, -4, N)
    m = (2.0 ** e_m).astype(np.float32)
    s_tok = (2.0 ** e_t).astype(np.float32)
    t_of_r = np.arange(M) % L
    x64 = A * (2.0 ** e_m)[None, :] * (2.0 ** e_t)[t_of_r][:, None]
    w64 = C * (2.0 ** e_w)[:, None] / (2.0 ** e_m)[None, :]
    x = x64.astype(np.float16)
    w = w64.astype(np.float16)
    assert np.array_equal(x.astype(np.float64), x64) and np.array_equal(w.astype(np.float64), w64)
    bias = (rng.integers(-64, 64, N) * 2.0 ** -10).astype(np.float16)

    wq, s_w, inv_m = oracle.fold_smoothing(w, m)
    assert np.array_equal(wq, C.astype(np.int8))
    assert np.array_equal(s_w, (2.0 ** e_w).astype(np.float32))
    assert np.array_equal(inv_m, (2.0 ** -e_m).astype(np.float32))
    xq = oracle.quantize_pts(x, inv_m, s_tok, B, L)
    assert np.array_equal(xq, A.astype(np.int8))
    y, y64, acc = oracle.w8a8_linear(xq, wq, s_tok, s_w, bias, B, L)
    want = np.array([[sum(Fraction(float(x64[r, k])) * Fraction(float(w64[o, k])) for k in range(K))
                      + Fraction(float(bias[o])) for o in range(N)] for r in range(M)], dtype=object)
    assert all(Fraction(float(y64[r, o])) == want[r, o] for r in range(M) for o in range(N))
    assert np.array_equal(acc, A @ C.T)
    with np.errstate(over="ignore"):
        assert np.array_equal(y.view(np.uint16), y64.astype(np.float16).view(np.uint16))
    # and without the bias
    y0, y064, _ = oracle.w8a8_linear(xq, wq, s_tok, s_w, None, B, L)
    assert all(Fraction(float(y064[r, o])) == want[r, o] - Fraction(float(bias[o]))
               for r in range(M) for o in range(N))


def test_smoothing_identity_random_scales_float64():
    """Eq. (smooth) with arbitrary m: the folded weight times the smoothed activation equals
    the original product up to fp32 rounding of W*m and 1/m (relative 2^-23 per term)."""
    rng = np.random.default_rng(9)
    N, K, M = 8, 40, 6
    w = (rng.normal(size=(N, K)) * 0.05).astype(np.float16)
    x = rng.normal(size=(M, K)).astype(np.float16)
    m = rng.uniform(0.1, 10, K).astype(np.float32)
    wq, s_w, inv_m = oracle.fold_smoothing(w, m)
    # dequantized folded weight is within half a step of W*m; undo the fold with inv_m
    w_fold = wq.astype(np.float64) * s_w.astype(np.float64)[:, None]
    y_smooth = (x.astype(np.float64) * inv_m.astype(np.float64)[None, :]) @ w_fold.T
    y_plain = x.astype(np.float64) @ w.astype(np.float64).T
    bound = (np.abs(x.astype(np.float64)) * inv_m.astype(np.float64)[None, :]).sum(axis=1)[:, None] \
        * (0.5 * s_w.astype(np.float64))[None, :] * 1.001 + 1e-6 * np.abs(y_plain)
    assert np.all(np.abs(y_smooth - y_plain) <= bound)


# --------------------------------------------------------------------------------------
# a2: integer GEMM (W-bar . X-bar of the PTS equation)
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (5, 12, 44), (33, 100, 17), (64, 1536, 9), (7, 384, 192)])
def test_int_gemm_equals_float64_matmul(M, K, N):
    """float64 matmul of int8 values is exact (K*127^2 << 2^53); catches wrong strides,
    transposition, sign-extension mistakes (values below -64 and above 63 are present)."""
    rng = np.random.default_rng(M * 1000 + K)
    xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    wq = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    acc = oracle.int8_gemm(xq, wq)
    want = (xq.astype(np.float64) @ wq.astype(np.float64).T)
    assert np.array_equal(acc.astype(np.float64), want)
    if K * 127 * 127 <= 2 ** 24:                           # fp32 sgemm is exact too
        want32 = xq.astype(np.float32) @ wq.astype(np.float32).T
        assert np.array_equal(acc.astype(np.float32), want32)


def test_int_gemm_closed_forms():
    K = 1536
    xq = np.full((3, K), 127, np.int8)
    wq = np.full((2, K), 127, np.int8)
    assert np.all(oracle.int8_gemm(xq, wq) == K * 16129)   # 24 774 144 at K = 1536
    assert np.all(oracle.int8_gemm(-xq, wq) == -K * 16129)
    eye = np.eye(16, dtype=np.int8)
    rng = np.random.default_rng(1)
    wq = rng.integers(-127, 128, size=(9, 16)).astype(np.int8)
    assert np.array_equal(oracle.int8_gemm(eye, wq), wq.T.astype(np.int32))
    assert np.array_equal(oracle.int8_gemm(wq, eye), wq.astype(np.int32))


def test_int_gemm_reports_int32_overflow():
    K = 140_000                                            # > 2^31 / 127^2 = 133 143
    with pytest.raises(OverflowError):
        oracle.int8_gemm(np.full((1, K), 127, np.int8), np.full((1, K), 127, np.int8))


# --------------------------------------------------------------------------------------
# a3: dequantization (diag-factoring identity of the PTS equation, Sec. 5.1)
# --------------------------------------------------------------------------------------
def test_dequant_matches_dequantize_then_matmul():
    """diag(D_X) (Xq Wq^T) diag(D_W)  ==  (diag(D_X) Xq)(diag(D_W) Wq)^T in float64."""
    rng = np.random.default_rng(4)
    B, L, K, N = 3, 5, 64, 11
    xq = rng.integers(-127, 128, size=(B * L, K)).astype(np.int8)
    wq = rng.integers(-127, 128, size=(N, K)).astype(np.int8)
    s_tok = rng.uniform(1e-3, 1e-1, L).astype(np.float32)
    s_w = rng.uniform(1e-4, 1e-2, N).astype(np.float32)
    bias = rng.normal(size=N).astype(np.float16)
    y, y64, acc = oracle.w8a8_linear(xq, wq, s_tok, s_w, bias, B, L)
    xd = xq.astype(np.float64) * np.tile(s_tok.astype(np.float64), B)[:, None]
    wd = wq.astype(np.float64) * s_w.astype(np.float64)[:, None]
    want = xd @ wd.T + bias.astype(np.float64)[None, :]
    assert np.allclose(y64, want, rtol=1e-12, atol=1e-12)
    assert np.array_equal(y.view(np.uint16), y64.astype(np.float16).view(np.uint16))


def test_dequant_overflow_goes_to_infinity():
    acc = np.array([[2_000_000, -2_000_000, 1]], np.int32)
    y, y64 = oracle.dequant(acc, np.array([1.0], np.float32), np.array([1.0, 1.0, 1.0], np.float32),
                            None, 1, 1)
    assert np.isposinf(y[0, 0]) and np.isneginf(y[0, 1]) and y[0, 2] == 1.0


def test_hand_worked_example():
    """B=1, L=2, K=3, N=2, every number derived by hand.

    m = (2, 1/2, 1)            -> inv_m = (1/2, 2, 1)
    W = [[1, -4, 2], [0.5, 8, -3]] -> W*m = [[2, -2, 2], [1, 4, -3]]
      row 0: max 2 -> s_w = 2/127;  codes = (127, -127, 127)
      row 1: max 4 -> s_w = 4/127;  W*m/s_w = (31.75, 127, -95.25) -> codes (32, 127, -95)
    s_tok = (1/4, 1)
    X = [[1, 0.25, -0.75], [3, -1.25, 200]]
      row 0 (t=0): X*inv_m = (0.5, 0.5, -0.75), /0.25 = (2, 2, -3)       -> codes (2, 2, -3)
      row 1 (t=1): X*inv_m = (1.5, -2.5, 200),  /1    = (1.5, -2.5, 200) -> codes (2, -2, 127)
    acc[0] = (2*127 - 2*127 - 3*127, 2*32 + 2*127 + 3*95)      = (-381, 603)
    acc[1] = (2*127 + 2*127 + 127*127, 2*32 - 2*127 - 127*95)  = (16637, -12255)
    Y = acc * s_tok[t] * s_w[o] + bias,  bias = (0.5, -1)
      Y[0] = (-381*0.25*2/127 + 0.5, 603*0.25*4/127 - 1)  = (-1.0, 3.748031...)
      Y[1] = (16637*2/127 + 0.5,   -12255*4/127 - 1)      = (262.5, -386.984251...)
    """
    m = np.array([2, 0.5, 1], np.float32)
    w = np.array([[1, -4, 2], [0.5, 8, -3]], np.float16)
    x = np.array([[1, 0.25, -0.75], [3, -1.25, 200]], np.float16)
    s_tok = np.array([0.25, 1], np.float32)
    bias = np.array([0.5, -1], np.float16)
    wq, s_w, inv_m = oracle.fold_smoothing(w, m)
    assert wq.tolist() == [[127, -127, 127], [32, 127, -95]]
    assert np.allclose(s_w, [2 / 127, 4 / 127], rtol=2e-7)
    assert inv_m.tolist() == [0.5, 2.0, 1.0]
    xq = oracle.quantize_pts(x, inv_m, s_tok, 1, 2)
    assert xq.tolist() == [[2, 2, -3], [2, -2, 127]]
    y, y64, acc = oracle.w8a8_linear(xq, wq, s_tok, s_w, bias, 1, 2)
    assert acc.tolist() == [[-381, 603], [16637, -12255]]
    want = np.array([[-381 * 0.25 * 2 / 127 + 0.5, 603 * 0.25 * 4 / 127 - 1],
                     [16637 * 2 / 127 + 0.5, -12255 * 4 / 127 - 1]])
    assert np.allclose(y64, want, rtol=1e-6)
    assert np.array_equal(y, want.astype(np.float16))


# --------------------------------------------------------------------------------------
# a4: unquantized comparison linear
# --------------------------------------------------------------------------------------
def test_f16_linear_vs_float64_matmul():
    rng = np.random.default_rng(8)
    M, K, N = 9, 77, 13
    x = rng.normal(size=(M, K)).astype(np.float16)
    w = (rng.normal(size=(N, K)) * 0.1).astype(np.float16)
    b = rng.normal(size=N).astype(np.float16)
    y, y64, asum = oracle.f16_linear(x, w, b)
    want = x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    assert np.allclose(y64, want, rtol=1e-12, atol=1e-12)
    assert np.array_equal(y.view(np.uint16), y64.astype(np.float16).view(np.uint16))
    assert np.all(asum >= np.abs(y64) - 1e-12)


# --------------------------------------------------------------------------------------
# the quantized path approximates the unquantized one (end-to-end sanity on synthetic data)
# --------------------------------------------------------------------------------------
def test_quantized_linear_tracks_fp16_linear_on_vim_shaped_data():
    """Y ~= diag(D_W)(W-bar X-bar)diag(D_X) (Sec. 5.1): at 8 bits, with smoothing, the quantized
    output must sit close to the FP16 linear on the synthetic Vim-Ti out_proj workload."""
    from paper_2412_20386_amd import synth

    c = synth.make_linear_case(0)
    assert c.clipped > 0                                   # evaluation draw exceeds calibration
    x, w, b = c.x.numpy(), c.w.numpy(), c.bias.numpy()
    wq, s_w, inv_m = oracle.fold_smoothing(w, c.m.numpy())
    xq = oracle.quantize_pts(x, inv_m, c.s_tok.numpy(), c.B, c.L)
    _, y64, _ = oracle.w8a8_linear(xq, wq, c.s_tok.numpy(), s_w, b, c.B, c.L)
    _, ref64, _ = oracle.f16_linear(x, w, b)
    rel = np.linalg.norm(y64 - ref64) / np.linalg.norm(ref64)
    assert rel < 0.03, rel
    assert np.abs(xq.astype(np.int32)).max() == 127
