"""CPU oracle for the LCMA GEMM path.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with the GPU library and never imports it.

The arithmetic lives in lcma_oracle.c (plain C, fp64 / int64, compiled with gcc);
this module builds it, loads it through ctypes and wraps the calls for numpy
arrays.  Every wrapper names the passage of the paper it evaluates.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from . import schemes  # noqa: F401  (re-exported)
from .schemes import Scheme

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lcma_oracle.c")
_LIB = os.path.join(_HERE, "liblcma_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile lcma_oracle.c with gcc (OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, p, i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        for fn in (lib.oracle_gemm_f64, lib.oracle_gemm_i64):
            fn.argtypes = [i64, i64, i64, p, i64, p, i64, p, i64]
            fn.restype = None
        for fn in (lib.oracle_lcma_f64, lib.oracle_lcma_i64):
            fn.argtypes = [i32, i32, i32, i32, p, p, p, i64, i64, i64, p, i64, p, i64, p, i64]
            fn.restype = ctypes.c_int
        lib.oracle_brent_residual.argtypes = [i32, i32, i32, i32, p, p, p, ctypes.POINTER(i64)]
        lib.oracle_brent_residual.restype = i64
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _ptr(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _rowmajor(a: np.ndarray, dtype) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype != dtype or a.ndim != 2 or a.strides[1] != a.itemsize or a.strides[0] % a.itemsize:
        a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ld(a: np.ndarray) -> int:
    return a.strides[0] // a.itemsize if a.shape[0] > 1 else max(a.shape[1], 1)


def gemm(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C = A x B by the triple loop (paper Eq. 1).  int64 inputs stay exact
    integers; anything else is evaluated in fp64 on the values as given."""
    integer = A.dtype == np.int64 and B.dtype == np.int64
    dt = np.int64 if integer else np.float64
    A, B = _rowmajor(A, dt), _rowmajor(B, dt)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    C = np.empty((M, N), dt)
    fn = _load().oracle_gemm_i64 if integer else _load().oracle_gemm_f64
    fn(M, N, K, _ptr(A), _ld(A), _ptr(B), _ld(B), _ptr(C), N)
    return C


def gemm_rows(A: np.ndarray, B: np.ndarray, rows) -> np.ndarray:
    """Selected rows of C = A x B (same triple loop, on a row subset of A)."""
    rows = np.asarray(rows, dtype=np.int64)
    return gemm(np.ascontiguousarray(np.asarray(A)[rows]).astype(np.float64), np.asarray(B).astype(np.float64))


def lcma(s: Scheme, A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C by the four-stage LCMA workflow (paper Eq. 3-6 / Algorithm 1)."""
    integer = A.dtype == np.int64 and B.dtype == np.int64
    dt = np.int64 if integer else np.float64
    A, B = _rowmajor(A, dt), _rowmajor(B, dt)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    U = np.ascontiguousarray(s.U, np.int32)
    V = np.ascontiguousarray(s.V, np.int32)
    W = np.ascontiguousarray(s.W, np.int32)
    C = np.empty((M, N), dt)
    fn = _load().oracle_lcma_i64 if integer else _load().oracle_lcma_f64
    rc = fn(s.m, s.k, s.n, s.R, _ptr(U), _ptr(V), _ptr(W), M, N, K,
            _ptr(A), _ld(A), _ptr(B), _ld(B), _ptr(C), N)
    if rc == 1:
        raise ValueError(f"shape ({M},{N},{K}) is not divisible by the scheme grid ({s.m},{s.n},{s.k})")
    if rc:
        raise MemoryError("oracle_lcma: out of memory")
    return C


def combine_b(s: Scheme, B: np.ndarray) -> np.ndarray:
    """Combine B (paper Eq. 4; Algorithm 2 stage 2): Bt[r] = sum_{l,j} V[r,l,j] * B_{l,j}, r = 0..R-1.

    Returns an array of shape (R, K/k, N/n) in fp64 (int64 for integer input): the exact right
    operands of the R products.  The paper's end-to-end evaluation runs this stage once, offline,
    for static weights."""
    integer = B.dtype == np.int64
    B = np.asarray(B, np.int64 if integer else np.float64)
    K, N = B.shape
    if K % s.k or N % s.n:
        raise ValueError(f"shape ({K},{N}) is not divisible by the scheme grid ({s.k},{s.n})")
    bk, bn = K // s.k, N // s.n
    out = np.zeros((s.R, bk, bn), B.dtype)
    for r in range(s.R):
        for l in range(s.k):
            for j in range(s.n):
                v = int(s.V[r, l, j])
                if v:
                    out[r] += v * B[l * bk:(l + 1) * bk, j * bn:(j + 1) * bn]
    return out


def combine_b_stored(s: Scheme, B: np.ndarray, dtype: str) -> np.ndarray:
    """Combine B as a 16-bit / fp32 library has to store it: the terms of Eq. 4 are added in fp32, in
    ascending (l, j) order, and the sum is rounded once (nearest-even) to the type the products are
    multiplied in: fp16 for bf16 and fp16 storage, fp32 for fp32 storage.  B holds values already
    representable in the storage type.  Returns (R, K/k, N/n) in fp64 (the stored values, widened).
    This fixes the precision in which the rounding decision is taken, so that an implementation can be
    compared bit for bit."""
    B = np.asarray(B, np.float64)
    K, N = B.shape
    if K % s.k or N % s.n:
        raise ValueError(f"shape ({K},{N}) is not divisible by the scheme grid ({s.k},{s.n})")
    bk, bn = K // s.k, N // s.n
    B32 = B.astype(np.float32)
    out = np.empty((s.R, bk, bn), np.float64)
    with np.errstate(over="ignore"):
        for r in range(s.R):
            acc = None
            for l in range(s.k):
                for j in range(s.n):
                    v = int(s.V[r, l, j])
                    if not v:
                        continue
                    term = np.float32(v) * B32[l * bk:(l + 1) * bk, j * bn:(j + 1) * bn]
                    acc = term if acc is None else (acc + term).astype(np.float32)
            if acc is None:
                acc = np.zeros((bk, bn), np.float32)
            out[r] = acc.astype(np.float16).astype(np.float64) if dtype in ("bf16", "f16") else acc.astype(np.float64)
    return out


def combine_a_stored(s: Scheme, A: np.ndarray, dtype: str) -> np.ndarray:
    """Combine A (paper Eq. 3; Algorithm 1 stage 1) as a library that materialises At_r has to store it:
    terms added in fp32 in ascending (i, l) order, the sum rounded once (nearest-even) to fp16 (bf16 and
    fp16 storage) or kept in fp32.  A holds values representable in the storage type.  Returns
    (R, M/m, K/k) in fp64 (the stored values, widened)."""
    A = np.asarray(A, np.float64)
    M, K = A.shape
    if M % s.m or K % s.k:
        raise ValueError(f"shape ({M},{K}) is not divisible by the scheme grid ({s.m},{s.k})")
    bm, bk = M // s.m, K // s.k
    A32 = A.astype(np.float32)
    out = np.empty((s.R, bm, bk), np.float64)
    with np.errstate(over="ignore"):
        for r in range(s.R):
            acc = None
            for i in range(s.m):
                for l in range(s.k):
                    u = int(s.U[r, i, l])
                    if not u:
                        continue
                    term = np.float32(u) * A32[i * bm:(i + 1) * bm, l * bk:(l + 1) * bk]
                    acc = term if acc is None else (acc + term).astype(np.float32)
            if acc is None:
                acc = np.zeros((bm, bk), np.float32)
            out[r] = acc.astype(np.float16).astype(np.float64) if dtype in ("bf16", "f16") else acc.astype(np.float64)
    return out


def lcma_unfused(s: Scheme, A: np.ndarray, B: np.ndarray, dtype: str, level: int, h_dtype: str | None = None,
                 residual_products: tuple = ()) -> np.ndarray:
    """C by the dataflows that keep intermediate results in memory, with the roundings that storing
    them implies (values in fp64, before the final rounding of C to the storage type):
      level 1  Algorithm 1: At_r and Bt_r stored (combine_a_stored, combine_b_stored), H_r = At_r Bt_r
               (Eq. 5; exact product, rounded once when it is stored: Algorithm 1 does not say in which type, so the
               caller names it with h_dtype "f16" or "f32"; None: fp16 for 16-bit storage, fp32 for fp32 storage),
               C_{i,j} = sum_r W[r,i,j] H_r (Eq. 6);
      level 2  Algorithm 2 as printed: At_r and Bt_r stored, H_r kept unrounded on chip.
    residual_products (level 1, 16-bit storage): products r whose left combination is kept as TWO stored values, the
    rounded sum and the rounded remainder of that rounding, each multiplied with Bt_r and both products (each rounded as
    H_r is) entering Eq. 6 with W[r]: the error compensation for combinations of many blocks.
    A and B hold values representable in the storage type; shapes divisible by the grid."""
    if level not in (1, 2):
        raise ValueError("level is 1 (Algorithm 1) or 2 (Algorithm 2)")
    At = combine_a_stored(s, A, dtype)       # [r, x, y]
    Bt = combine_b_stored(s, B, dtype)       # [r, y, z]
    bm, bn = At.shape[1], Bt.shape[2]
    C = np.zeros((s.m * bm, s.n * bn), np.float64)
    ht = h_dtype or ("f16" if dtype in ("bf16", "f16") else "f32")
    if ht not in ("f16", "f32"):
        raise ValueError("h_dtype is f16 or f32")
    stored_h = lambda H: (H.astype(np.float16) if ht == "f16" else H.astype(np.float32)).astype(np.float64)
    At32 = combine_a_stored(s, A, "f32") if residual_products else None   # the fp32 sums of Eq. 3 before they are rounded
    if residual_products and (level != 1 or dtype not in ("bf16", "f16")):
        raise ValueError("residual products belong to level 1 with 16-bit storage")
    with np.errstate(over="ignore"):
        for r in range(s.R):
            H = gemm(np.ascontiguousarray(At[r]), np.ascontiguousarray(Bt[r]))
            if level == 1:
                H = stored_h(H)
                if r in residual_products:
                    # the unrounded fp32 sum of Eq. 3 minus its stored value, stored in fp16 itself
                    rest = (At32[r] - At[r]).astype(np.float16).astype(np.float64)
                    H = H + stored_h(gemm(np.ascontiguousarray(rest), np.ascontiguousarray(Bt[r])))
            for i in range(s.m):
                for j in range(s.n):
                    w = int(s.W[r, i, j])
                    if w:
                        C[i * bm:(i + 1) * bm, j * bn:(j + 1) * bn] += w * H
    return C


def brent(s: Scheme):
    """(number of violated Brent equations, flat index of the first or -1)."""
    U = np.ascontiguousarray(s.U, np.int32)
    V = np.ascontiguousarray(s.V, np.int32)
    W = np.ascontiguousarray(s.W, np.int32)
    first = ctypes.c_int64(-1)
    bad = _load().oracle_brent_residual(s.m, s.k, s.n, s.R, _ptr(U), _ptr(V), _ptr(W),
                                        ctypes.byref(first))
    return int(bad), int(first.value)


def rel_frobenius(C: np.ndarray, Cref: np.ndarray) -> float:
    """||C - Cref||_F / ||Cref||_F in fp64 (the parity metric)."""
    C = np.asarray(C, np.float64)
    Cref = np.asarray(Cref, np.float64)
    den = float(np.sqrt(np.sum(Cref * Cref)))
    num = float(np.sqrt(np.sum((C - Cref) ** 2)))
    return num / den if den > 0 else num
