"""CPU oracle of the FP8 path.  TEST INFRASTRUCTURE ONLY (see the package header).

The paper's FP8 workflow (Sec. 4.1, experimental setup): operands arrive in bf16, are quantised to FP8 E4M3 with
one scale per 1 x 128 block along K, and multiplied block-scaled; in the LCMA form the quantisation is fused into the
Combine A stage (Sec. 4.3, end-to-end results), i.e. the left operands At_r of Eq. 3 are formed from bf16 blocks and
stored as E4M3 codes with their scales.  What the paper leaves open is fixed here the way this build reads it:

  * E4M3 is the OCP 8-bit format with 4 exponent bits (bias 7), 3 mantissa bits, subnormals, no infinities, largest
    finite value 448 (code 0x7E) and one NaN (0x7F).  Rounding is to nearest, ties to the even mantissa.
  * A scale is a power of two 2^e, stored as the byte e + 127 (the E8M0 scale type of the OCP microscaling formats,
    which MI355X's matrix instructions apply in hardware): e is the smallest integer with amax <= 448 * 2^e, where
    amax is the largest magnitude of the 128 values; an all-zero block takes e = 0.  e is clamped to [-127, 127].
    Dividing by a power of two is exact, so the only rounding of the quantisation is the one to E4M3, and the codes of
    two implementations can be compared bit for bit.
  * Both operands are scaled 1 x 128 along K: A per row, B per column (a row of the N x K weight matrix).
  * The sums of Eq. 3 / Eq. 4 are formed in fp32, ascending block order, before they are quantised.
  * A product is  sum over the K/128 blocks kb of  2^(ea[i,kb] + eb[j,kb]) * sum_{k in kb} qa[i,k] qb[j,k]  (Eq. 5 on
    the dequantised operands); the oracle evaluates it in fp64.

Nothing here is shared with the GPU library.
"""
from __future__ import annotations

import numpy as np

from . import gemm
from .schemes import Scheme

BLOCK = 128          # elements per scale block along K
E4M3_MAX = 448.0     # largest finite magnitude


def _table() -> np.ndarray:
    """Value of every non-negative code 0x00..0x7E (0x7F is NaN), from the format's definition."""
    out = np.empty(127, np.float64)
    for code in range(127):
        e, m = code >> 3, code & 7
        out[code] = m * 2.0 ** -9 if e == 0 else (8 + m) * 2.0 ** (e - 10)   # subnormal: 0.m * 2^-6; normal: 1.m * 2^(e-7)
    return out


_POS = _table()


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """fp64 value of each E4M3 code (NaN for 0x7F / 0xFF)."""
    codes = np.asarray(codes, np.uint8)
    mag = codes & np.uint8(0x7F)
    val = np.where(mag == 0x7F, np.nan, _POS[np.minimum(mag, 126)])
    return np.where(codes & np.uint8(0x80), -val, val)


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of each value: the representable magnitude closest to |x|, of two equally close ones the one
    with the even code (= even mantissa), magnitudes beyond 448 saturate to 448; the sign bit is kept (also on zero)."""
    x = np.asarray(x, np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.clip(np.searchsorted(_POS, a, side="left"), 0, 126)       # first code whose value is >= a
    lo = np.maximum(hi - 1, 0)
    d_hi, d_lo = _POS[hi] - a, a - _POS[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    return code | np.where(np.signbit(x), np.uint8(0x80), np.uint8(0))


def scale_exponent(amax: np.ndarray) -> np.ndarray:
    """Smallest integer e with amax <= 448 * 2^e, per element (0 where amax is 0), clamped to [-127, 127]."""
    amax = np.asarray(amax, np.float64)
    safe = np.where(amax > 0, amax, 1.0)
    e = np.ceil(np.log2(safe / E4M3_MAX)).astype(np.int64)
    # log2 is inexact near the boundary: settle it with exact comparisons
    e = np.where(safe > E4M3_MAX * np.exp2(e.astype(np.float64)), e + 1, e)
    e = np.where(safe <= E4M3_MAX * np.exp2((e - 1).astype(np.float64)), e - 1, e)
    e = np.where(amax > 0, e, 0)
    return np.clip(e, -127, 127)


def quantize_1x128(X: np.ndarray):
    """1 x 128 block quantisation of the rows of X (values exactly representable in fp32; K a multiple of 128):
    returns (codes uint8 [rows, K], scale bytes uint8 [rows, K/128]) with X ~ decode(code) * 2^(byte - 127)."""
    X = np.asarray(X, np.float64)
    rows, K = X.shape
    if K % BLOCK:
        raise ValueError(f"K = {K} is not a multiple of {BLOCK}")
    blocks = X.reshape(rows, K // BLOCK, BLOCK)
    e = scale_exponent(np.abs(blocks).max(axis=2))
    y = blocks * np.exp2(-e.astype(np.float64))[:, :, None]               # exact: a power of two
    return e4m3_encode(y).reshape(rows, K), (e + 127).astype(np.uint8)


def dequantize_1x128(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """fp64 values decode(code) * 2^(scale byte - 127)."""
    rows, K = codes.shape
    e = scales.astype(np.int64) - 127
    return (e4m3_decode(codes).reshape(rows, K // BLOCK, BLOCK) * np.exp2(e.astype(np.float64))[:, :, None]).reshape(rows, K)


def gemm_fp8(qa: np.ndarray, sa: np.ndarray, qw: np.ndarray, sw: np.ndarray) -> np.ndarray:
    """C = dequantised A times dequantised W transposed (A: M x K codes, W: N x K codes, both scaled 1 x 128 along K),
    by the fp64 triple loop of Eq. 1."""
    return gemm(dequantize_1x128(qa, sa), np.ascontiguousarray(dequantize_1x128(qw, sw).T))


def _combine_fp32(coef: np.ndarray, blocks, rows: int, cols: int) -> np.ndarray:
    """Signed sum of blocks in fp32, ascending block order (the order `blocks` yields them in)."""
    acc = None
    for c, blk in zip(coef, blocks):
        c = int(c)
        if not c:
            continue
        term = np.float32(c) * blk
        acc = term if acc is None else (acc + term).astype(np.float32)
    return np.zeros((rows, cols), np.float32) if acc is None else acc


def combine_a_quantized(s: Scheme, A: np.ndarray):
    """Combine A with the quantisation fused in (Eq. 3; Sec. 4.3): At_r = sum_{i,l} U[r,i,l] A_{i,l} in fp32 (ascending
    (i, l)), quantised 1 x 128 along K/k.  A: M x K values representable in bf16; K/k a multiple of 128.
    Returns (codes [R, M/m, K/k], scale bytes [R, M/m, K/k/128])."""
    A32 = np.asarray(A, np.float64).astype(np.float32)
    M, K = A32.shape
    if M % s.m or K % (s.k * BLOCK):
        raise ValueError("shape not divisible by the scheme grid and the scale block")
    bm, bk = M // s.m, K // s.k
    blocks = [A32[i * bm:(i + 1) * bm, l * bk:(l + 1) * bk] for i in range(s.m) for l in range(s.k)]
    q = [quantize_1x128(_combine_fp32(s.U[r].reshape(-1), blocks, bm, bk)) for r in range(s.R)]
    return np.stack([c for c, _ in q]), np.stack([e for _, e in q])


def combine_w_quantized(s: Scheme, Wt: np.ndarray):
    """Combine B for weights stored N x K (Wt[n][k] = B[k][n]) with the quantisation fused in (Eq. 4): the transposed
    right operand Bt_r^T = sum_{l,j} V[r,l,j] (block (j, l) of Wt) in fp32 (ascending (l, j)), quantised 1 x 128 along
    K/k.  Returns (codes [R, N/n, K/k], scale bytes [R, N/n, K/k/128])."""
    W32 = np.asarray(Wt, np.float64).astype(np.float32)
    N, K = W32.shape
    if N % s.n or K % (s.k * BLOCK):
        raise ValueError("shape not divisible by the scheme grid and the scale block")
    bn, bk = N // s.n, K // s.k
    blocks = [W32[j * bn:(j + 1) * bn, l * bk:(l + 1) * bk] for l in range(s.k) for j in range(s.n)]
    q = [quantize_1x128(_combine_fp32(s.V[r].reshape(-1), blocks, bn, bk)) for r in range(s.R)]
    return np.stack([c for c, _ in q]), np.stack([e for _, e in q])


def lcma_fp8(s: Scheme, A: np.ndarray, Wt: np.ndarray, h_dtype=None) -> np.ndarray:
    """C = A x Wt^T by the four stages of Algorithm 1 on FP8 operands: quantised Combine A, quantised Combine B, the R
    block products on the dequantised operands (Eq. 5, fp64), and C_{i,j} = sum_r W[r,i,j] H_r (Eq. 6).  h_dtype
    (np.float16 / np.float32 / None) is the type the products are stored in between stages 3 and 4 (None: unrounded).
    Returns fp64, before the final rounding of C."""
    qa, sa = combine_a_quantized(s, A)
    qw, sw = combine_w_quantized(s, Wt)
    bm, bn = qa.shape[1], qw.shape[1]
    C = np.zeros((s.m * bm, s.n * bn), np.float64)
    with np.errstate(over="ignore"):
        for r in range(s.R):
            H = gemm_fp8(qa[r], sa[r], qw[r], sw[r])
            if h_dtype is not None:
                H = H.astype(h_dtype).astype(np.float64)
            for i in range(s.m):
                for j in range(s.n):
                    w = int(s.W[r, i, j])
                    if w:
                        C[i * bm:(i + 1) * bm, j * bn:(j + 1) * bn] += w * H
    return C
