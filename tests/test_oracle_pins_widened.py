"""Pins for the oracle functions of the widened rows (per-token dynamic quantizer, 4-bit codes and
their packing, per-token zero offset).  As in test_oracle_pins.py nothing here retypes the oracle's
formula: values come from closed forms, exact rational arithmetic, the paper's packing expression
evaluated by hand, or reductions to an already pinned function."""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _f16(a):
    return np.asarray(a, np.float16)


# --------------------------------------------------------------------------------------
# per-token dynamic quantizer (Sec. 4; latency table of Sec. 6.4)
# --------------------------------------------------------------------------------------
def test_dynamic_closed_form_grid_rows():
    # A row holding j * c for j = -127..127 has max |v| = 127 c, so its step is exactly c and the
    # codes are exactly j, whatever c.  Catches: wrong divisor (128, 255), max over the wrong axis,
    # max of signed values instead of magnitudes, a step shared between rows.
    j = np.arange(-127, 128, dtype=np.float64)
    rows = np.stack([j * 0.5, j * 2.0, j * 0.03125, (j * 0.25)[::-1]])
    xq, s_row = oracle.quantize_dynamic(_f16(rows), None)
    assert np.array_equal(s_row, np.array([0.5, 2.0, 0.03125, 0.25], np.float32))
    assert np.array_equal(xq[0], j.astype(np.int8)) and np.array_equal(xq[1], j.astype(np.int8))
    assert np.array_equal(xq[3], j[::-1].astype(np.int8))


def test_dynamic_step_and_codes_against_exact_rational_arithmetic():
    # s_r = max|x inv_m| / 127 with every operation rounded to fp32 as stated; codes are the exact
    # quotient rounded half to even wherever the exact quotient is not within 1e-4 of a tie
    # (fp32 rounding of the reciprocal step can only matter there).
    rng = np.random.default_rng(11)
    M, K = 37, 96
    x = _f16(rng.standard_normal((M, K)) * np.exp(rng.normal(0, 1.0, (M, 1))))
    inv_m = (0.5 + rng.random(K)).astype(np.float32)
    xq, s_row = oracle.quantize_dynamic(x, inv_m)
    v32 = x.astype(np.float32) * inv_m[None, :]                       # one fp32 rounding per product
    amax = np.abs(v32).max(axis=1)
    want_step = (amax / np.float32(127.0)).astype(np.float32)
    assert np.array_equal(s_row.view(np.uint32), want_step.view(np.uint32))
    for r in range(M):
        s = Fraction(float(s_row[r]))
        for k in range(K):
            exact = Fraction(float(v32[r, k])) / s
            lo = exact.numerator // exact.denominator
            frac = exact - lo
            if abs(frac - Fraction(1, 2)) < Fraction(1, 10000):
                assert int(xq[r, k]) in (lo, lo + 1)
            else:
                want = lo + (1 if frac > Fraction(1, 2) else 0)
                assert int(xq[r, k]) == max(-127, min(127, want)), (r, k)
    assert np.all(np.abs(xq).max(axis=1) == 127)                      # every row uses its full range


def test_dynamic_equals_static_quantizer_given_the_same_steps():
    # With the dynamic steps handed to the (separately pinned) PTS quantizer as one "token position"
    # per row, the codes must coincide: the two differ only in where the step comes from.
    rng = np.random.default_rng(12)
    M, K = 64, 80
    x = _f16(rng.laplace(0, 1, (M, K)) * 3)
    inv_m = (0.25 + rng.random(K)).astype(np.float32)
    xq, s_row = oracle.quantize_dynamic(x, inv_m)
    assert np.array_equal(xq, oracle.quantize_pts(x, inv_m, s_row, 1, M))


def test_dynamic_scale_invariance_zero_rows_and_specials():
    rng = np.random.default_rng(13)
    x = _f16(rng.standard_normal((8, 40)))
    x[3] = 0.0                                                          # all-zero row: step 1, codes 0
    xq, s = oracle.quantize_dynamic(x, None)
    xq4, s4 = oracle.quantize_dynamic(_f16(x.astype(np.float32) * 4.0), None)   # power of two: exact
    assert np.array_equal(xq, xq4) and np.array_equal(s4, s * np.float32(4.0) * (s != 1.0) + (s == 1.0))
    assert s[3] == 1.0 and not xq[3].any()
    y = _f16([[1.0, np.nan, -2.0, 0.5], [np.inf, 1.0, -1.0, 0.0]])
    q, st = oracle.quantize_dynamic(y, None)
    assert st[0] == np.float32(2.0) / np.float32(127.0) and list(q[0]) == [64, 0, -127, 32]   # NaN ignored by the max
    assert np.isinf(st[1]) and list(q[1]) == [0, 0, 0, 0]                # Inf step: Inf * 0 = NaN -> 0, finite * 0 = 0


# --------------------------------------------------------------------------------------
# 4-bit codes and their packing (Sec. 2.3 clip range; App. B.1 packing expression)
# --------------------------------------------------------------------------------------
def test_int4_packing_matches_the_papers_expression_by_hand():
    # App. B.1 packing: element 2i in the low nibble of byte i, element 2i+1 in its high nibble, two's
    # complement nibbles; values worked by hand.
    codes = np.array([[1, 2, -1, 3, 7, -7, -8, 0, 0, -1]], np.int8)
    want = np.array([[0x21, 0x3F, 0x97, 0x08, 0xF0]], np.uint8)
    assert np.array_equal(oracle.pack_int4(codes), want)
    assert np.array_equal(oracle.unpack_int4(want), codes)


def test_int4_pack_unpack_is_a_bijection_on_all_bytes():
    allb = np.arange(256, dtype=np.uint8).reshape(1, 256)
    codes = oracle.unpack_int4(allb)
    assert codes.min() == -8 and codes.max() == 7
    lo, hi = codes[0, 0::2].astype(int), codes[0, 1::2].astype(int)
    assert np.array_equal((lo & 15) | ((hi & 15) << 4), np.arange(256))  # numeric identity, not the oracle's code
    assert np.array_equal(oracle.pack_int4(codes), allb)


# The E2M3 container of the 4-bit codes (a storage format of the boundary: 6-bit floating-point patterns with
# 1 sign, 2 exponent and 3 mantissa bits, exponent bias 1, which hold the integers -7..7 exactly).
def _e2m3_value(pattern):
    s, e, m = (pattern >> 5) & 1, (pattern >> 3) & 3, pattern & 7
    mag = Fraction(m, 8) if e == 0 else Fraction(2) ** (e - 1) * (1 + Fraction(m, 8))
    return -mag if s else mag


def test_e2m3_patterns_of_the_integers_by_hand_and_by_value():
    # By hand: 1 = 2^0 * 1.000 -> e = 1, m = 0 -> 0b0_01_000 = 8;  3 = 2^1 * 1.100b -> e = 2, m = 4 -> 0b0_10_100 = 20;
    # -7 = -(2^2 * 1.110b) -> s = 1, e = 3, m = 6 -> 0b1_11_110 = 62.  Three codes fill bits 0..17 of the row:
    # 8 | 62 << 6 | 20 << 12 = 0x014F88 -> bytes 88 4F 01.
    packed = oracle.pack_e2m3(np.array([[1, -7, 3]], np.int8))
    assert packed.shape == (1, 1, 96) and oracle.e2m3_blocks(3) == 1
    assert packed[0, 0, :3].tolist() == [0x88, 0x4F, 0x01] and not packed[0, 0, 3:].any()
    # Every integer of the range: the stored pattern's value under the format's definition is the integer,
    # zero has a clear sign bit, and the patterns are the 15 distinct ones with integer values up to 7.
    for v in range(-7, 8):
        pattern = int(oracle.pack_e2m3(np.array([[v]], np.int8))[0, 0, 0]) & 63
        assert _e2m3_value(pattern) == v, (v, pattern)
        if v == 0:
            assert pattern == 0
    for bad in (-8, 8, 100):
        with pytest.raises(ValueError):
            oracle.pack_e2m3(np.array([[bad]], np.int8))


def test_e2m3_block_layout_by_hand():
    # 256 codes = two 96-byte blocks.  Code k sits in block k // 128, group g = (k % 128) // 32, at bits
    # [6 j, 6 j + 6) of the group's 24-byte string (j = k % 32); string bytes 0..15 at block offset 16 g,
    # bytes 16..23 at block offset 64 + 8 g.  Storage is block-major: packed[block][row][96].
    codes = np.zeros((3, 256), np.int8)
    codes[0, 32] = 1      # group 1, j = 0: bits 0..5 of string byte 0 -> block offset 16, value 8
    codes[0, 21] = 7      # group 0, j = 21: bits 126..131: pattern 30 = 0b011110; its bits 0,1 -> byte 15 bits 6,7 (0x80),
    #                       its bits 2..5 (0b0111) -> byte 16 = block offset 64, value 0x07
    codes[0, 255] = -1    # block 1, group 3, j = 31: bits 186..191 = byte 23 bits 2..7: pattern 40 = 0b101000 -> 0xA0
    #                       at block offset 64 + 24 + 7 = 95 of block 1
    codes[2, 128] = 2     # row 2, block 1, group 0, j = 0: pattern 16 at offset 0 of row 2 in plane 1
    packed = oracle.pack_e2m3(codes)
    assert packed.shape == (2, 3, 96)
    want = np.zeros((2, 3, 96), np.uint8)
    want[0, 0, 16], want[0, 0, 15], want[0, 0, 64], want[1, 0, 95], want[1, 2, 0] = 0x08, 0x80, 0x07, 0xA0, 0x10
    assert np.array_equal(packed, want)
    # as flat bytes: plane b starts at 96 * rows * b
    flat = packed.reshape(-1)
    assert flat[96 * 3 * 1 + 96 * 2 + 0] == 0x10 and flat[96 * 3 * 1 + 95] == 0xA0
    assert np.array_equal(oracle.unpack_e2m3(packed, 256), codes)


@pytest.mark.parametrize("K", [1, 31, 32, 33, 127, 128, 129, 384, 500])
def test_e2m3_round_trip_and_zero_padding(K):
    rng = np.random.default_rng(K)
    codes = rng.integers(-7, 8, size=(5, K)).astype(np.int8)
    packed = oracle.pack_e2m3(codes)
    assert packed.shape == ((K + 127) // 128, 5, 96)
    assert np.array_equal(oracle.unpack_e2m3(packed, K), codes)
    # Independent decode of the bit string: gather each group's 24 bytes, read 6-bit fields, map by value.
    by_value = {p: int(_e2m3_value(p)) for p in range(64) if _e2m3_value(p).denominator == 1}
    Kp = (K + 127) // 128 * 128
    full = np.zeros((5, Kp), np.int64)
    for r in range(5):
        for blk in range(Kp // 128):
            b = packed[blk, r]
            for g in range(4):
                string = int.from_bytes(bytes(b[16 * g:16 * g + 16]) + bytes(b[64 + 8 * g:72 + 8 * g]), "little")
                for j in range(32):
                    full[r, blk * 128 + 32 * g + j] = by_value[(string >> (6 * j)) & 63]
    assert np.array_equal(full[:, :K], codes) and not full[:, K:].any()


def test_bits_8_reduces_to_the_pinned_8_bit_functions_and_4_bit_range():
    rng = np.random.default_rng(21)
    B, L, K, N = 2, 9, 32, 12
    x = _f16(rng.standard_normal((B * L, K)) * 2)
    w = _f16(rng.standard_normal((N, K)) * 0.05)
    m = (0.5 + rng.random(K)).astype(np.float32)
    s_tok = (0.01 + 0.02 * rng.random(L)).astype(np.float32)
    wq8, sw8, im8 = oracle.fold_smoothing(w, m)
    wq, sw, im = oracle.fold_smoothing_bits(w, m, 8)
    assert np.array_equal(wq, wq8) and np.array_equal(sw, sw8) and np.array_equal(im, im8)
    assert np.array_equal(oracle.quantize_pts_bits(x, im, s_tok, B, L, 8), oracle.quantize_pts(x, im, s_tok, B, L))
    wq4, sw4, _ = oracle.fold_smoothing_bits(w, m, 4)
    assert np.all(np.abs(wq4).max(axis=1) == 7) and np.abs(wq4).max() == 7       # full +-7 range, never -8
    wf = w.astype(np.float32) * m[None, :]
    assert np.array_equal(sw4, (np.abs(wf).max(axis=1) / np.float32(7.0)).astype(np.float32))
    assert np.all(np.abs(wf - wq4 * sw4[:, None]) <= 0.5 * sw4[:, None] * (1 + 1e-6))   # half-step reconstruction
    xq4 = oracle.quantize_pts_bits(x, im, s_tok * np.float32(16), B, L, 4)
    assert xq4.min() >= -7 and xq4.max() <= 7


def test_w4a4_on_grid_end_to_end_is_exact():
    # Power-of-two steps and integer grids: fold(4 bit) -> quantize(4 bit) -> pack -> unpack -> integer
    # GEMM -> dequantize must reproduce X W^T + b exactly (checked in rational arithmetic).
    rng = np.random.default_rng(22)
    B, L, K, N = 2, 5, 16, 6
    m = (2.0 ** rng.integers(-2, 3, K)).astype(np.float32)
    s_tok = (2.0 ** rng.integers(-4, 0, L)).astype(np.float32)
    s_w_true = (2.0 ** rng.integers(-6, -2, N)).astype(np.float32)
    qx = rng.integers(-7, 8, (B * L, K))
    qw = rng.integers(-7, 8, (N, K))
    qw[np.arange(N), rng.integers(0, K, N)] = 7                           # pins each row's step
    x = _f16(qx * np.tile(s_tok, B)[:, None] * m[None, :])
    w = _f16(qw * s_w_true[:, None] / m[None, :])
    bias = _f16(rng.integers(-8, 9, N) * 0.125)
    wq, s_w, inv_m = oracle.fold_smoothing_bits(w, m, 4)
    xq = oracle.quantize_pts_bits(x, inv_m, s_tok, B, L, 4)
    assert np.array_equal(wq, qw) and np.array_equal(xq, qx) and np.array_equal(s_w, s_w_true)
    xq_rt = oracle.unpack_int4(oracle.pack_int4(xq))
    wq_rt = oracle.unpack_int4(oracle.pack_int4(wq))
    y, y64 = oracle.dequant(oracle.int8_gemm(xq_rt, wq_rt), s_tok, s_w, bias, B, L)
    for r in range(B * L):
        for o in range(N):
            exact = sum(Fraction(float(x[r, k])) * Fraction(float(w[o, k])) for k in range(K)) + Fraction(float(bias[o]))
            assert Fraction(float(y64[r, o])) == exact


# --------------------------------------------------------------------------------------
# per-token zero offset (Sec. 5.1 names it; quantizer form of Sec. 2.3)
# --------------------------------------------------------------------------------------
def test_offset_quantizer_on_grid_and_clip_range():
    # x = s_t (j - z_t) for every int8 code j must come back as code j: pins the sign of the offset
    # and the [-128, 127] range.  Values beyond the range saturate at both ends.
    L, K = 3, 256
    s_tok = np.array([0.5, 0.25, 2.0], np.float32)
    z_tok = np.array([-128, 5, 100], np.int32)
    j = np.arange(-128, 128)
    x = _f16(np.stack([s_tok[t] * (j - int(z_tok[t])) for t in range(L)]))
    xq = oracle.quantize_pts_offset(x, None, s_tok, z_tok, 1, L)
    assert np.array_equal(xq, np.tile(j.astype(np.int8), (L, 1)))
    far = _f16([[1e4, -1e4, np.inf, -np.inf, np.nan]] * L)
    q = oracle.quantize_pts_offset(far, None, s_tok, z_tok, 1, L)
    assert np.array_equal(q[:, :4], np.tile(np.array([127, -128, 127, -128], np.int8), (L, 1)))
    assert np.array_equal(q[:, 4], z_tok.astype(np.int8))                  # NaN -> rounded value 0 -> code z


def test_offset_zero_reduces_to_pts_inside_the_symmetric_range():
    rng = np.random.default_rng(31)
    B, L, K = 3, 7, 48
    x = _f16(rng.standard_normal((B * L, K)))
    s_tok = (0.1 + 0.05 * rng.random(L)).astype(np.float32)                # |codes| stay far below 127
    inv_m = (0.5 + rng.random(K)).astype(np.float32)
    a = oracle.quantize_pts_offset(x, inv_m, s_tok, np.zeros(L, np.int32), B, L)
    assert np.abs(a.astype(int)).max() < 127
    assert np.array_equal(a, oracle.quantize_pts(x, inv_m, s_tok, B, L))


def test_offset_dequantization_equals_the_product_of_reconstructed_operands():
    # sum_k s_t (q - z_t) * s_w w = s_t s_w (acc - z_t rowsum): evaluate the left side in exact
    # rational arithmetic from the codes.  Catches a wrong sign or a column/row mix-up in the
    # correction term and an offset indexed by r div L.
    rng = np.random.default_rng(32)
    B, L, K, N = 2, 4, 24, 5
    xq = rng.integers(-128, 128, (B * L, K)).astype(np.int8)
    wq = rng.integers(-127, 128, (N, K)).astype(np.int8)
    s_tok = (2.0 ** rng.integers(-6, -2, L)).astype(np.float32)
    s_w = (2.0 ** rng.integers(-8, -4, N)).astype(np.float32)
    z_tok = rng.integers(-128, 128, L).astype(np.int32)
    bias = _f16(rng.integers(-4, 5, N) * 0.25)
    rowsum = oracle.weight_rowsum(wq)
    assert np.array_equal(rowsum, wq.astype(np.int64).sum(axis=1))
    y, y64 = oracle.dequant_offset(oracle.int8_gemm(xq, wq), s_tok, z_tok, rowsum, s_w, bias, B, L)
    for r in range(B * L):
        t = r % L
        for o in range(N):
            exact = sum(Fraction(float(s_tok[t])) * (int(xq[r, k]) - int(z_tok[t])) * Fraction(float(s_w[o])) * int(wq[o, k])
                        for k in range(K)) + Fraction(float(bias[o]))
            assert Fraction(float(y64[r, o])) == exact
    assert np.array_equal(y, y64.astype(np.float16))                       # power-of-two steps: y64 is exact


def test_offset_shift_identity():
    # Adding c steps to every element of a token and c to its offset leaves the reconstruction
    # s (q - z) of the unshifted values unchanged: the code moves by exactly c.
    L, K, c = 2, 64, 17
    s_tok = np.array([0.125, 0.5], np.float32)
    rng = np.random.default_rng(33)
    base = rng.integers(-60, 60, (L, K))
    x0 = _f16(base * s_tok[:, None])
    x1 = _f16((base + c) * s_tok[:, None])
    q0 = oracle.quantize_pts_offset(x0, None, s_tok, np.array([3, -9], np.int32), 1, L)
    q1 = oracle.quantize_pts_offset(x1, None, s_tok, np.array([3 - c, -9 - c], np.int32), 1, L)
    assert np.array_equal(q0, q1)
