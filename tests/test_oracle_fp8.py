"""The FP8 oracle (oracle/fp8.py) against what the format, the mathematics and brute force fix: the E4M3 table of the
format's definition (tests/golden/e4m3_facts.txt), rounding on hand-worked ties, scale choice at its boundaries,
error bounds of a quantise / dequantise round trip, exactness on inputs the format represents, and the LCMA form
against the plain quantised product where the two must agree exactly."""
import math

import numpy as np
import pytest

import lcma_inputs as inp
import oracle
from oracle import fp8 as F
from oracle import schemes as S


def test_e4m3_table_matches_the_format(golden):
    g = golden("e4m3_facts.txt")
    for key, vals in g.items():
        if key == "finite_magnitudes":
            finite = F.e4m3_decode(np.arange(128, dtype=np.uint8))
            assert np.isfinite(finite).sum() == int(vals[0]) and np.isnan(finite[127])
            continue
        code, value = int(vals[0], 16), float(vals[1])
        got = float(F.e4m3_decode(np.array([code], np.uint8))[0])
        assert (math.isnan(got) and math.isnan(value)) or got == value, key
        if not math.isnan(value):
            assert int(F.e4m3_encode(np.array([value]))[0]) == code, key
    # strictly increasing over the positive codes, symmetric in the sign bit, subnormal spacing 2^-9, 8 values per binade
    pos = F.e4m3_decode(np.arange(127, dtype=np.uint8))
    assert np.all(np.diff(pos) > 0)
    assert np.array_equal(F.e4m3_decode(np.arange(127, dtype=np.uint8) | np.uint8(0x80)), -pos)
    assert np.all(np.diff(pos[:9]) == 2.0 ** -9)
    for e in range(-6, 9):
        assert ((pos >= 2.0 ** e) & (pos < 2.0 ** (e + 1))).sum() == (8 if e < 8 else 7)  # the last binade stops at 448


def test_e4m3_rounding_is_nearest_ties_to_even():
    enc = lambda v: float(F.e4m3_decode(F.e4m3_encode(np.array([v], np.float64)))[0])
    # between 16 (mantissa 000) and 18 (001): the tie 17 goes to 16; between 18 and 20 (010): the tie 19 goes to 20
    assert enc(17.0) == 16.0 and enc(19.0) == 20.0 and enc(17.0001) == 18.0 and enc(16.9999) == 16.0
    assert enc(-17.0) == -16.0 and enc(-19.0) == -20.0
    # ties at a binade boundary: 15 (1.875 * 8) and 16: 15.5 -> 16 (even mantissa 000)
    assert enc(15.5) == 16.0 and enc(15.49) == 15.0
    # subnormals: spacing 2^-9; 1.5 * 2^-9 ties to 2 * 2^-9 (even), 0.5 * 2^-9 ties to 0, 2.5 * 2^-9 ties to 2 * 2^-9
    u = 2.0 ** -9
    assert enc(1.5 * u) == 2 * u and enc(0.5 * u) == 0.0 and enc(2.5 * u) == 2 * u and enc(0.51 * u) == u
    # saturation and the top of the range: 448 stays, 464 (the midpoint to the absent 480) and beyond give 448
    assert enc(448.0) == 448.0 and enc(447.0) == 448.0 and enc(432.0) == 448.0 and enc(431.9) == 416.0
    assert enc(1e9) == 448.0 and enc(-1e9) == -448.0
    # every representable value encodes to itself; every midpoint goes to the even neighbour
    pos = F.e4m3_decode(np.arange(127, dtype=np.uint8))
    assert np.array_equal(F.e4m3_encode(pos), np.arange(127, dtype=np.uint8))
    mids = (pos[:-1] + pos[1:]) / 2
    got = F.e4m3_encode(mids)
    assert np.all(got % 2 == 0) and np.all((got == np.arange(126)) | (got == np.arange(1, 127)))
    # brute force against the definition on a dense sweep: no representable value is closer than the chosen one
    xs = np.concatenate([np.linspace(0, 450, 20011), np.geomspace(1e-4, 448, 5003)])
    chosen = F.e4m3_decode(F.e4m3_encode(xs))
    best = np.abs(pos[None, :] - xs[:, None]).min(axis=1)
    assert np.all(np.abs(chosen - np.minimum(xs, 448.0)) <= best + 0.0)


def test_scale_exponent_boundaries():
    se = lambda v: int(F.scale_exponent(np.array([v], np.float64))[0])
    assert se(448.0) == 0 and se(448.0 * (1 + 2.0 ** -20)) == 1 and se(224.0) == -1 and se(224.0000001) == 0
    assert se(3.0) == -7 and se(3.5) == -7 and se(3.5000001) == -6 and se(6.0) == -6      # 3 * 128 = 384, 6 * 64 = 384
    assert se(1.0) == -8 and se(0.02) == -14 and se(0.0) == 0
    assert se(1e-45) == -127 and se(3e38) == 120
    # definition by brute force: the smallest e with amax <= 448 * 2^e
    rng = np.random.default_rng(3)
    for v in np.exp(rng.uniform(-40, 40, 500)):
        e = se(v)
        assert v <= 448.0 * 2.0 ** e and v > 448.0 * 2.0 ** (e - 1)


def test_quantize_round_trip_bounds_and_exact_cases():
    rng = np.random.default_rng(11)
    X = inp.widen(inp.store(rng.standard_normal((37, 384)) * np.exp(rng.uniform(-6, 6, (37, 1))), "bf16"), "bf16")
    q, s = F.quantize_1x128(X)
    assert q.shape == (37, 384) and s.shape == (37, 3) and q.dtype == np.uint8 and s.dtype == np.uint8
    back = F.dequantize_1x128(q, s)
    scale = np.repeat(2.0 ** (s.astype(np.float64) - 127), 128, axis=1)
    y = np.abs(X) / scale
    # the largest element of a block lands in (224, 448]: full use of the range, nothing saturates
    top = y.reshape(37, 3, 128).max(axis=2)
    assert np.all((top > 224.0) & (top <= 448.0))
    # error: half a unit in the last place, relative 2^-4 for normal results, absolute 2^-10 (scaled) below 2^-6
    err = np.abs(back - X) / scale
    assert np.all(err <= np.where(y >= 2.0 ** -6, y * 2.0 ** -4, 2.0 ** -10) + 0.0)
    # integers up to 6 are represented exactly in a block whose largest magnitude is at most 7 (scale 2^-6: k * 64)
    Xi = inp.integers(5, 1, (9, 256), -6, 6).astype(np.float64)
    qi, si = F.quantize_1x128(Xi)
    assert np.array_equal(F.dequantize_1x128(qi, si), Xi)
    # a block of zeros keeps scale byte 127 and zero codes; scaling a block by 2^5 moves only the scale byte
    Z = np.zeros((2, 128))
    qz, sz = F.quantize_1x128(Z)
    assert not qz.any() and np.all(sz == 127)
    q2, s2 = F.quantize_1x128(X * 32.0)
    assert np.array_equal(q2, q) and np.array_equal(s2.astype(int), s.astype(int) + 5)
    with pytest.raises(ValueError):
        F.quantize_1x128(np.zeros((4, 100)))


def test_quantized_gemm_is_the_product_of_the_dequantised_operands():
    # integer operands that the format holds exactly: the quantised product equals the integer product
    M, N, K = 24, 40, 256
    Ai, Wi = inp.integers(21, 1, (M, K)), inp.integers(21, 2, (N, K))
    qa, sa = F.quantize_1x128(Ai.astype(np.float64))
    qw, sw = F.quantize_1x128(Wi.astype(np.float64))
    assert np.array_equal(F.gemm_fp8(qa, sa, qw, sw), (Ai @ Wi.T).astype(np.float64))
    # a single non-zero element on each side isolates one term: code value times code value times both scales
    A = np.zeros((2, 256)); W = np.zeros((3, 256))
    A[1, 130] = 0.3; W[2, 130] = -5.0
    qa, sa = F.quantize_1x128(A); qw, sw = F.quantize_1x128(W)
    C = F.gemm_fp8(qa, sa, qw, sw)
    a_hat = float(F.e4m3_decode(qa[1:2, 130])[0]) * 2.0 ** (int(sa[1, 1]) - 127)
    assert a_hat == 320 * 2.0 ** -10                 # 0.3 / 2^-10 = 307.2, nearest code value 320
    assert C[1, 2] == a_hat * -5.0 and np.count_nonzero(C) == 1
    # float operands: error of the quantised product against the unquantised one stays near 2^-4 / sqrt(3) per operand
    rng = np.random.default_rng(5)
    A = inp.widen(inp.store(rng.standard_normal((32, 512)), "bf16"), "bf16")
    W = inp.widen(inp.store(rng.standard_normal((48, 512)) * 0.02, "bf16"), "bf16")
    qa, sa = F.quantize_1x128(A); qw, sw = F.quantize_1x128(W)
    err = oracle.rel_frobenius(F.gemm_fp8(qa, sa, qw, sw), oracle.gemm(A, np.ascontiguousarray(W.T)))
    assert 5e-3 < err < 6e-2


@pytest.mark.parametrize("name", ["strassen", "laderman", "strassen2"])
def test_lcma_fp8_exact_on_integers_and_reduces_to_the_plain_form(name):
    s = S.by_name(name)
    M, N, K = 8 * s.m, 6 * s.n, 128 * s.k
    Ai, Wi = inp.integers(31, 1, (M, K)), inp.integers(31, 2, (N, K))
    if name == "laderman":      # 7-term sums of entries in [-1, 1] stay within what one block scale represents exactly
        Ai, Wi = inp.integers(31, 1, (M, K), -1, 1), inp.integers(31, 2, (N, K), -1, 1)
    if name == "strassen2":
        Ai, Wi = inp.integers(31, 1, (M, K), -1, 1), inp.integers(31, 2, (N, K), -1, 1)
    C = F.lcma_fp8(s, Ai.astype(np.float64), Wi.astype(np.float64))
    assert np.array_equal(C, (Ai @ Wi.T).astype(np.float64))
    # the quantised combinations are the combinations, where the format holds them exactly
    qa, sa = F.combine_a_quantized(s, Ai.astype(np.float64))
    Bt = oracle.combine_b(s, np.ascontiguousarray(Wi.T))
    qw, sw = F.combine_w_quantized(s, Wi.astype(np.float64))
    for r in range(s.R):
        assert np.array_equal(F.dequantize_1x128(qw[r], sw[r]), Bt[r].T.astype(np.float64))
    # the classical scheme has one block on each side of every product: its LCMA form is the plain quantised product
    c = S.classical(2, 2, 2)
    rng = np.random.default_rng(9)
    A = inp.widen(inp.store(rng.standard_normal((16, 256)), "bf16"), "bf16")
    W = inp.widen(inp.store(rng.standard_normal((12, 256)), "bf16"), "bf16")
    qa, sa = F.quantize_1x128(A); qw, sw = F.quantize_1x128(W)
    assert np.allclose(F.lcma_fp8(c, A, W), F.gemm_fp8(qa, sa, qw, sw), rtol=1e-13, atol=1e-13)
    # storing the products in fp16 changes the result by at most the rounding of the at most R terms of a block of C
    full, half = F.lcma_fp8(s, Ai.astype(np.float64), Wi.astype(np.float64)), F.lcma_fp8(s, Ai.astype(np.float64), Wi.astype(np.float64), np.float16)
    assert np.array_equal(full, half)      # integers below 2048 are fp16 values
