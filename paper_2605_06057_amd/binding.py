"""Thin ctypes binding of liblcma.so: argument marshalling only, same names as include/lcma.h.

Every step of the GEMM runs in the library's HIP kernels.  There is no CPU or PyTorch
fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblcma.so")

LCMA_OK = 0
STATUS_NAMES = ["OK", "ERR_ARG", "ERR_IO", "ERR_PARSE", "ERR_BRENT", "ERR_SHAPE", "ERR_DTYPE",
                "ERR_NOKERNEL", "ERR_HIP"]
(LCMA_ERR_ARG, LCMA_ERR_IO, LCMA_ERR_PARSE, LCMA_ERR_BRENT, LCMA_ERR_SHAPE, LCMA_ERR_DTYPE,
 LCMA_ERR_NOKERNEL, LCMA_ERR_HIP) = range(1, 9)
LCMA_F32, LCMA_BF16, LCMA_F16 = 0, 1, 2
LCMA_PLAIN, LCMA_STRASSEN, LCMA_STRASSEN2, LCMA_LADERMAN = 0, 1, 2, 3
DTYPE_IDS = {"f32": LCMA_F32, "bf16": LCMA_BF16, "f16": LCMA_F16}
SCHEME_NAMES = {LCMA_PLAIN: "plain", LCMA_STRASSEN: "strassen", LCMA_STRASSEN2: "strassen2",
                LCMA_LADERMAN: "laderman"}

EXPORTS = [
    "lcma_scheme_load", "lcma_scheme_verify", "lcma_scheme_free", "lcma_scheme_info", "lcma_scheme_coeffs",
    "lcma_gemm", "lcma_variant_count", "lcma_variant_name", "lcma_variant_info", "lcma_gemm_variant",
    "lcma_select", "lcma_hw_mi355x", "lcma_model_stages", "lcma_model_intensity", "lcma_predict_seconds",
    "lcma_sched_waves", "lcma_sched_range", "lcma_status_str", "lcma_last_error",
    "lcma_scheme_name", "lcma_scheme_id_max", "lcma_variant_prepared", "lcma_prepared_b_bytes", "lcma_prepare_b", "lcma_prepare_bt", "lcma_gemm_prepared",
    "lcma_gemm_nt", "lcma_variant_b_layout", "lcma_unfused_workspace_bytes", "lcma_gemm_unfused",
    "lcma_predict_unfused_seconds", "lcma_select_dataflow", "lcma_gemm_ex", "lcma_set_tuning",
    "lcma_static_scratch_bytes", "lcma_gemm_unfused_static", "lcma_split_group_scratch_bytes", "lcma_gemm_nt_ws", "lcma_gemm_ws", "lcma_fp16_range_flags", "lcma_mfma_probe",
    "lcma_fp8_code_pitch", "lcma_fp8_scale_pitch", "lcma_fp8_quantize", "lcma_fp8_gemm_nt", "lcma_fp8_prepared_w_bytes",
    "lcma_fp8_prepare_w", "lcma_fp8_workspace_bytes", "lcma_fp8_gemm_lcma",
]


class LcmaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"LCMA_{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {message}")
        self.status = status


class lcma_hw(ctypes.Structure):
    _fields_ = [("flops_mul", ctypes.c_double), ("flops_add", ctypes.c_double), ("beta", ctypes.c_double)]


class lcma_choice(ctypes.Structure):
    _fields_ = [("scheme_id", ctypes.c_int), ("dataflow", ctypes.c_int), ("seconds", ctypes.c_double)]


class lcma_stage_costs(ctypes.Structure):
    _fields_ = [("flops", ctypes.c_double * 4), ("elems", ctypes.c_double * 4), ("seconds", ctypes.c_double * 4)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library (raises if it has not been built: run `python -m paper_2605_06057_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_06057_amd.build`")
        # PyTorch ships its own HIP runtime; it must be the one already in the process when
        # this library's dependency on libamdhip64 is resolved, or two runtimes would coexist.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, vp, cp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_char_p
        pi32, pi64, pd = ctypes.POINTER(i32), ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)
        L.lcma_scheme_load.argtypes = [cp, ctypes.POINTER(vp)]
        L.lcma_scheme_verify.argtypes = [vp, pi64]
        L.lcma_scheme_free.argtypes = [vp]
        L.lcma_scheme_free.restype = None
        L.lcma_scheme_info.argtypes = [vp] + [pi32] * 7
        L.lcma_scheme_coeffs.argtypes = [vp, vp, vp, vp]
        L.lcma_gemm.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp, vp]
        L.lcma_gemm_nt.argtypes = L.lcma_gemm.argtypes
        L.lcma_gemm_ex.argtypes = [ctypes.c_float, ctypes.c_float, i32] + L.lcma_gemm.argtypes
        L.lcma_variant_b_layout.argtypes = [i32]
        L.lcma_unfused_workspace_bytes.argtypes = [i64, i64, i64, i32, vp]
        L.lcma_unfused_workspace_bytes.restype = i64
        L.lcma_predict_unfused_seconds.argtypes = [i32, i64, i64, i64, i32, i32]
        L.lcma_predict_unfused_seconds.restype = ctypes.c_double
        L.lcma_select_dataflow.argtypes = [i64, i64, i64, i32, i32, ctypes.POINTER(lcma_choice)]
        L.lcma_gemm_unfused.argtypes = [i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp, vp, i64, i32, vp]
        L.lcma_variant_count.argtypes = []
        L.lcma_variant_name.argtypes = [i32]
        L.lcma_variant_name.restype = cp
        L.lcma_variant_info.argtypes = [i32] + [pi32] * 8
        L.lcma_gemm_variant.argtypes = [cp, i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
        L.lcma_scheme_name.argtypes = [i32]
        L.lcma_scheme_name.restype = cp
        L.lcma_scheme_id_max.argtypes = []
        L.lcma_variant_prepared.argtypes = [i32]
        L.lcma_prepared_b_bytes.argtypes = [vp, i64, i64, i32]
        L.lcma_prepared_b_bytes.restype = i64
        L.lcma_prepare_b.argtypes = [i64, i64, vp, i64, i32, vp, vp, vp]
        L.lcma_prepare_bt.argtypes = [i64, i64, vp, i64, i32, vp, vp, vp]
        L.lcma_gemm_prepared.argtypes = [i64, i64, i64, vp, i64, vp, vp, i64, i32, vp, vp]
        L.lcma_select.argtypes = [i64, i64, i64, i32]
        L.lcma_hw_mi355x.argtypes = [i32, ctypes.POINTER(lcma_hw)]
        L.lcma_model_stages.argtypes = [vp, i64, i64, i64, ctypes.POINTER(lcma_hw), ctypes.POINTER(lcma_stage_costs)]
        L.lcma_model_intensity.argtypes = [vp, i64, i64, i64, pd, pd, pd]
        L.lcma_predict_seconds.argtypes = [i32, i64, i64, i64, i32]
        L.lcma_predict_seconds.restype = ctypes.c_double
        L.lcma_sched_waves.argtypes = [i64, i32, i32, pi64, pi64]
        L.lcma_sched_range.argtypes = [i64, i32, i32, i32, pi64, pi64]
        L.lcma_status_str.argtypes = [i32]
        L.lcma_status_str.restype = cp
        L.lcma_last_error.argtypes = []
        L.lcma_last_error.restype = cp
        L.lcma_set_tuning.argtypes = [cp, cp]
        L.lcma_gemm_nt_ws.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp, i64, vp]
        L.lcma_gemm_ws.argtypes = [i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp, vp, i64, ctypes.POINTER(ctypes.c_int), vp]
        L.lcma_fp16_range_flags.argtypes = [i64, i64, vp, i64, vp, vp]
        L.lcma_mfma_probe.argtypes = [vp, vp, i64, ctypes.POINTER(ctypes.c_double), vp]
        L.lcma_split_group_scratch_bytes.argtypes = []
        L.lcma_split_group_scratch_bytes.restype = i64
        L.lcma_static_scratch_bytes.argtypes = []
        L.lcma_static_scratch_bytes.restype = i64
        L.lcma_gemm_unfused_static.argtypes = [i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, i32, vp, i32, vp]
        L.lcma_fp8_code_pitch.argtypes = [i64]
        L.lcma_fp8_code_pitch.restype = i64
        L.lcma_fp8_scale_pitch.argtypes = [i64]
        L.lcma_fp8_scale_pitch.restype = i64
        L.lcma_fp8_quantize.argtypes = [i64, i64, vp, i64, vp, vp, vp]
        L.lcma_fp8_gemm_nt.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, i64, vp]
        L.lcma_fp8_prepared_w_bytes.argtypes = [vp, i64, i64]
        L.lcma_fp8_prepared_w_bytes.restype = i64
        L.lcma_fp8_prepare_w.argtypes = [i64, i64, vp, i64, vp, vp, vp]
        L.lcma_fp8_workspace_bytes.argtypes = [vp, i64, i64, i64]
        L.lcma_fp8_workspace_bytes.restype = i64
        L.lcma_fp8_gemm_lcma.argtypes = [i64, i64, i64, vp, i64, vp, vp, i64, vp, vp, i64, vp]
        _lib = L
        # schemes that kernels were generated for beyond the paper's three
        for sid in range(4, int(L.lcma_scheme_id_max()) + 1):
            name = L.lcma_scheme_name(sid)
            if name:
                SCHEME_NAMES[sid] = name.decode()
    return _lib


def _check(status: int):
    if status != LCMA_OK:
        raise LcmaError(status, lib().lcma_last_error().decode())


class Scheme:
    """Owns an lcma_scheme handle."""

    def __init__(self, spec: str):
        self.handle = ctypes.c_void_p()
        _check(lib().lcma_scheme_load(spec.encode(), ctypes.byref(self.handle)))

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.lcma_scheme_free(self.handle)
            self.handle = None


def lcma_scheme_load(spec: str) -> Scheme:
    return Scheme(spec)


def lcma_scheme_verify(s: Scheme) -> int:
    """Returns -1 when the Brent identity holds, raises LcmaError(ERR_BRENT) otherwise
    (the error carries .first_bad)."""
    first = ctypes.c_int64(-1)
    st = lib().lcma_scheme_verify(s.handle, ctypes.byref(first))
    if st != LCMA_OK:
        err = LcmaError(st, lib().lcma_last_error().decode())
        err.first_bad = int(first.value)
        raise err
    return int(first.value)


def lcma_scheme_info(s: Scheme) -> dict:
    v = [ctypes.c_int() for _ in range(7)]
    _check(lib().lcma_scheme_info(s.handle, *[ctypes.byref(x) for x in v]))
    return dict(zip(["m", "k", "n", "R", "nnzU", "nnzV", "nnzW"], [int(x.value) for x in v]))


def lcma_scheme_coeffs(s: Scheme):
    import numpy as np
    d = lcma_scheme_info(s)
    U = np.zeros((d["R"], d["m"], d["k"]), np.int8)
    V = np.zeros((d["R"], d["k"], d["n"]), np.int8)
    W = np.zeros((d["R"], d["m"], d["n"]), np.int8)
    _check(lib().lcma_scheme_coeffs(s.handle, U.ctypes.data, V.ctypes.data, W.ctypes.data))
    return U, V, W


def _dtype_of(t) -> int:
    import torch
    return {torch.float32: LCMA_F32, torch.bfloat16: LCMA_BF16, torch.float16: LCMA_F16}[t.dtype]


def _marshal(A, B, C, b_nk: bool = False):
    """(M, N, K, ptrs and leading dimensions, stream) of three row-major device tensors; with b_nk the
    second one is the N x K weight matrix."""
    import torch
    assert A.is_cuda and B.is_cuda and C.is_cuda, "matrices must live on the GPU"
    assert A.dim() == B.dim() == C.dim() == 2 and A.stride(1) == B.stride(1) == C.stride(1) == 1
    assert A.dtype == B.dtype == C.dtype
    M, K = A.shape
    K2, N = B.shape[::-1] if b_nk else B.shape
    assert K == K2 and tuple(C.shape) == (M, N)
    stream = torch.cuda.current_stream(A.device).cuda_stream
    return M, N, K, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0), C.data_ptr(), C.stride(0), stream


def lcma_gemm(A, B, C, scheme: Scheme | None = None):
    """C = A x B on the current stream (torch tensors carry pointers and strides only)."""
    M, N, K, pa, lda, pb, ldb, pc, ldc, stream = _marshal(A, B, C)
    _check(lib().lcma_gemm(M, N, K, pa, lda, pb, ldb, pc, ldc, _dtype_of(A),
                           scheme.handle if scheme is not None else None, stream))
    return C


def lcma_gemm_ex(alpha: float, beta: float, A, B, C, scheme: Scheme | None = None, b_nk: bool = False):
    """C = alpha * (A x B) + beta * C on the current stream; b_nk: the second operand is the N x K weight matrix."""
    M, N, K, pa, lda, pb, ldb, pc, ldc, stream = _marshal(A, B, C, b_nk)
    _check(lib().lcma_gemm_ex(alpha, beta, 2 if b_nk else 0, M, N, K, pa, lda, pb, ldb, pc, ldc, _dtype_of(A),
                              scheme.handle if scheme is not None else None, stream))
    return C


def lcma_gemm_nt(A, W, C, scheme: Scheme | None = None):
    """C = A x W^T for the N x K weight tensor W, on the current stream."""
    M, N, K, pa, lda, pw, ldw, pc, ldc, stream = _marshal(A, W, C, True)
    _check(lib().lcma_gemm_nt(M, N, K, pa, lda, pw, ldw, pc, ldc, _dtype_of(A),
                              scheme.handle if scheme is not None else None, stream))
    return C


def lcma_predict_unfused_seconds(scheme_id: int, M: int, N: int, K: int, dtype: int, combine_b_offline: bool = False) -> float:
    return float(lib().lcma_predict_unfused_seconds(scheme_id, M, N, K, dtype, int(combine_b_offline)))


def lcma_select_dataflow(M: int, N: int, K: int, dtype: int, combine_b_offline: bool = False) -> dict:
    """{'scheme_id', 'dataflow' (0 fused / plain, 1 Algorithm 1), 'seconds'} with the smallest predicted time."""
    c = lcma_choice()
    _check(lib().lcma_select_dataflow(M, N, K, dtype, int(combine_b_offline), ctypes.byref(c)))
    return {"scheme_id": int(c.scheme_id), "dataflow": int(c.dataflow), "seconds": float(c.seconds)}


def lcma_unfused_workspace_bytes(scheme: Scheme, M: int, N: int, K: int, dtype: int) -> int:
    return int(lib().lcma_unfused_workspace_bytes(M, N, K, dtype, scheme.handle))


def lcma_gemm_unfused(level: int, A, B, C, scheme: Scheme, workspace, reuse_bt: bool = False):
    """C = A x B by Algorithm 1 (level 1) or Algorithm 2 as printed (level 2); `workspace` is a device
    tensor of at least lcma_unfused_workspace_bytes bytes."""
    M, N, K, pa, lda, pb, ldb, pc, ldc, stream = _marshal(A, B, C)
    assert workspace.is_cuda and workspace.is_contiguous()
    _check(lib().lcma_gemm_unfused(level, M, N, K, pa, lda, pb, ldb, pc, ldc, _dtype_of(A), scheme.handle,
                                   workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                   int(reuse_bt), stream))
    return C


def lcma_gemm_ws(A, B, C, scheme, workspace=None, b_nk: bool = False) -> int:
    """lcma_gemm (b_nk: lcma_gemm_nt, B is the N x K weight matrix) with a workspace (uint8 device tensor or None);
    returns the dataflow that ran: 0 fused, 1 Algorithm 1."""
    M, N, K, pa, lda, pb, ldb, pc, ldc, stream = _marshal(A, B, C, b_nk)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    flow = ctypes.c_int(0)
    _check(lib().lcma_gemm_ws(2 if b_nk else 0, M, N, K, pa, lda, pb, ldb, pc, ldc, _dtype_of(A), scheme.handle if scheme is not None else None,
                              ws_ptr, ws_n, ctypes.byref(flow), stream))
    return int(flow.value)


def lcma_gemm_nt_ws(A, W, C, workspace=None):
    """Plain C = A x W^T (W: N x K) on the plane GEMM; `workspace` (uint8 device tensor) allows the Split-Group schedule."""
    M, N, K, pa, lda, pw, ldw, pc, ldc, stream = _marshal(A, W, C, True)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_n = workspace.numel() if workspace is not None else 0
    _check(lib().lcma_gemm_nt_ws(M, N, K, pa, lda, pw, ldw, pc, ldc, _dtype_of(A), ws_ptr, ws_n, stream))
    return C


def lcma_fp16_range_flags(X) -> int:
    """Bit 0: some |x| > 32752 in the bf16 device tensor X; bit 1: some 0 < |x| < 2^-14 (synchronises to read the word)."""
    import torch
    assert X.is_cuda and X.dtype == torch.bfloat16 and X.dim() == 2 and X.stride(1) == 1
    flags = torch.empty((1,), dtype=torch.int32, device=X.device)
    stream = torch.cuda.current_stream(X.device).cuda_stream
    _check(lib().lcma_fp16_range_flags(X.shape[0], X.shape[1], X.data_ptr(), X.stride(0), flags.data_ptr(), stream))
    return int(flags.item())


def lcma_mfma_probe(operands, sink, iters: int) -> float:
    """Launches the matrix-pipe probe on the fp16 values in `operands` (device, >= 64 KiB); returns the flops of the launch."""
    import torch
    assert operands.is_cuda and operands.is_contiguous() and operands.numel() * operands.element_size() >= 65536
    assert sink.is_cuda and sink.is_contiguous() and sink.numel() * sink.element_size() >= 2 * 1024 * 1024
    flops = ctypes.c_double(0.0)
    stream = torch.cuda.current_stream(operands.device).cuda_stream
    _check(lib().lcma_mfma_probe(operands.data_ptr(), sink.data_ptr(), iters, ctypes.byref(flops), stream))
    return flops.value


def lcma_split_group_scratch_bytes() -> int:
    return int(lib().lcma_split_group_scratch_bytes())


def lcma_static_scratch_bytes() -> int:
    return int(lib().lcma_static_scratch_bytes())


def lcma_gemm_unfused_static(level: int, A, B, C, scheme: Scheme, reuse_bt: bool = False):
    """lcma_gemm_unfused on the library's static device buffer: allocates nothing, takes no workspace."""
    M, N, K, pa, lda, pb, ldb, pc, ldc, stream = _marshal(A, B, C)
    _check(lib().lcma_gemm_unfused_static(level, M, N, K, pa, lda, pb, ldb, pc, ldc, _dtype_of(A), scheme.handle,
                                          int(reuse_bt), stream))
    return C


def lcma_gemm_variant(variant: str, A, B, C, b_nk: bool = False):
    """Runs the named kernel; b_nk: B is the N x K matrix (for variants whose b_layout is 2)."""
    M, N, K, pa, lda, pb, ldb, pc, ldc, stream = _marshal(A, B, C, b_nk)
    _check(lib().lcma_gemm_variant(variant.encode(), M, N, K, pa, lda, pb, ldb, pc, ldc, stream))
    return C


def lcma_variants() -> list[dict]:
    out = []
    for i in range(lib().lcma_variant_count()):
        v = [ctypes.c_int() for _ in range(8)]
        _check(lib().lcma_variant_info(i, *[ctypes.byref(x) for x in v]))
        d = dict(zip(["scheme_id", "dtype", "TM", "TN", "TK", "mult_M", "mult_N", "mult_K"],
                     [int(x.value) for x in v]))
        d["name"] = lib().lcma_variant_name(i).decode()
        d["prepared"] = int(lib().lcma_variant_prepared(i))
        d["b_layout"] = int(lib().lcma_variant_b_layout(i))  # 0: K x N, 1: prepared planes, 2: N x K
        out.append(d)
    return out


def lcma_prepared_b_bytes(scheme: Scheme, N: int, K: int, dtype: int) -> int:
    return int(lib().lcma_prepared_b_bytes(scheme.handle, N, K, dtype))


def lcma_prepare_b(B, scheme: Scheme, Bt=None, transposed: bool = False):
    """Offline Combine B of the K x N device tensor B (or, with transposed=True, of the N x K weight
    tensor W = B^T); returns the prepared operand, a device tensor of shape (R, N/n, K/k), padded to
    whole tiles, in the compute type (allocated here unless Bt is given)."""
    import torch
    assert B.is_cuda and B.dim() == 2 and B.stride(1) == 1
    (N, K) = B.shape if transposed else B.shape[::-1]
    dt = _dtype_of(B)
    nbytes = lcma_prepared_b_bytes(scheme, N, K, dt)
    if nbytes < 0:
        raise LcmaError(LCMA_ERR_SHAPE, f"lcma_prepare_b: N = {N} and K = {K} must be whole 16-byte vectors of elements")
    info = lcma_scheme_info(scheme)
    ct = torch.float32 if B.dtype == torch.float32 else torch.float16
    if Bt is None:  # planes of N/n rows and K/k columns, both padded to whole tiles of the Combine-B kernel
        kt = 64 // B.element_size()
        cols = -(-K // (info["k"] * kt)) * kt
        rows = nbytes // (info["R"] * cols * B.element_size())
        Bt = torch.empty((info["R"], rows, cols), device=B.device, dtype=ct)
    assert Bt.is_cuda and Bt.is_contiguous() and Bt.dtype == ct and Bt.numel() * Bt.element_size() == nbytes
    stream = torch.cuda.current_stream(B.device).cuda_stream
    fn = lib().lcma_prepare_bt if transposed else lib().lcma_prepare_b
    _check(fn(N, K, B.data_ptr(), B.stride(0), dt, scheme.handle, Bt.data_ptr(), stream))
    return Bt


def lcma_prepare_bt(W, scheme: Scheme, Bt=None):
    """lcma_prepare_b for weights stored N x K (a linear layer's weight)."""
    return lcma_prepare_b(W, scheme, Bt, transposed=True)


def _marshal_prepared(A, Bt, C):
    import torch
    assert A.is_cuda and Bt.is_cuda and C.is_cuda, "matrices must live on the GPU"
    assert A.dim() == C.dim() == 2 and A.stride(1) == C.stride(1) == 1 and Bt.is_contiguous()
    assert A.dtype == C.dtype
    M, K = A.shape
    M2, N = C.shape
    assert M == M2
    stream = torch.cuda.current_stream(A.device).cuda_stream
    return M, N, K, A.data_ptr(), A.stride(0), Bt.data_ptr(), C.data_ptr(), C.stride(0), stream


def lcma_gemm_prepared(A, Bt, C, scheme: Scheme):
    """C = A x B with the prepared operand Bt = lcma_prepare_b(B, scheme), on the current stream."""
    M, N, K, pa, lda, pbt, pc, ldc, stream = _marshal_prepared(A, Bt, C)
    _check(lib().lcma_gemm_prepared(M, N, K, pa, lda, pbt, pc, ldc, _dtype_of(A), scheme.handle, stream))
    return C


def lcma_gemm_variant_prepared(variant: str, A, Bt, C):
    """lcma_gemm_variant for a variant that takes the prepared operand."""
    M, N, K, pa, lda, pbt, pc, ldc, stream = _marshal_prepared(A, Bt, C)
    _check(lib().lcma_gemm_variant(variant.encode(), M, N, K, pa, lda, pbt, N, pc, ldc, stream))
    return C


def lcma_select(M: int, N: int, K: int, dtype: int) -> int:
    return int(lib().lcma_select(M, N, K, dtype))


def lcma_predict_seconds(scheme_id: int, M: int, N: int, K: int, dtype: int) -> float:
    return float(lib().lcma_predict_seconds(scheme_id, M, N, K, dtype))


def lcma_hw_mi355x(dtype: int) -> lcma_hw:
    hw = lcma_hw()
    _check(lib().lcma_hw_mi355x(dtype, ctypes.byref(hw)))
    return hw


def lcma_model_stages(s: Scheme | None, M: int, N: int, K: int, hw: lcma_hw) -> lcma_stage_costs:
    out = lcma_stage_costs()
    _check(lib().lcma_model_stages(s.handle if s else None, M, N, K, ctypes.byref(hw), ctypes.byref(out)))
    return out


def lcma_model_intensity(s: Scheme | None, M: int, N: int, K: int):
    e = [ctypes.c_double() for _ in range(3)]
    _check(lib().lcma_model_intensity(s.handle if s else None, M, N, K, *[ctypes.byref(x) for x in e]))
    return tuple(float(x.value) for x in e)


# ---------------------------------------------------------------- FP8 (E4M3 codes, 1 x 128 power-of-two scales)
def lcma_fp8_quantize(X, Q=None, S=None):
    """Codes (rows x code pitch, uint8) and scale bytes (rows x scale pitch, uint8) of the bf16 device tensor X."""
    import torch
    assert X.is_cuda and X.dim() == 2 and X.stride(1) == 1 and X.dtype == torch.bfloat16
    rows, K = X.shape
    kp, ls = int(lib().lcma_fp8_code_pitch(K)), int(lib().lcma_fp8_scale_pitch(K))
    if Q is None:
        Q = torch.empty((rows, kp), dtype=torch.uint8, device=X.device)
    if S is None:
        S = torch.empty((rows, ls), dtype=torch.uint8, device=X.device)
    assert Q.is_contiguous() and S.is_contiguous() and tuple(Q.shape) == (rows, kp) and tuple(S.shape) == (rows, ls)
    stream = torch.cuda.current_stream(X.device).cuda_stream
    _check(lib().lcma_fp8_quantize(rows, K, X.data_ptr(), X.stride(0), Q.data_ptr(), S.data_ptr(), stream))
    return Q, S


def lcma_fp8_gemm_nt(Aq, Sa, Wq, Sw, C, K: int):
    """C (bf16, M x N) = dequantised A (codes Aq, scales Sa) times dequantised W (N x K) transposed."""
    import torch
    M, N = C.shape
    assert Aq.is_contiguous() and Wq.is_contiguous() and Sa.is_contiguous() and Sw.is_contiguous()
    assert Aq.shape[0] == M and Wq.shape[0] == N and C.dtype == torch.bfloat16 and C.stride(1) == 1
    stream = torch.cuda.current_stream(C.device).cuda_stream
    _check(lib().lcma_fp8_gemm_nt(M, N, K, Aq.data_ptr(), Sa.data_ptr(), Wq.data_ptr(), Sw.data_ptr(), C.data_ptr(),
                                  C.stride(0), stream))
    return C


def lcma_fp8_prepare_w(W, scheme: Scheme, Wp=None):
    """Offline Combine B of the N x K bf16 weight tensor with the quantisation fused in; returns the prepared operand
    (uint8, lcma_fp8_prepared_w_bytes bytes)."""
    import torch
    assert W.is_cuda and W.dim() == 2 and W.stride(1) == 1 and W.dtype == torch.bfloat16
    N, K = W.shape
    nbytes = int(lib().lcma_fp8_prepared_w_bytes(scheme.handle, N, K))
    if Wp is None:
        Wp = torch.empty((nbytes,), dtype=torch.uint8, device=W.device)
    assert Wp.is_contiguous() and Wp.numel() == nbytes
    stream = torch.cuda.current_stream(W.device).cuda_stream
    _check(lib().lcma_fp8_prepare_w(N, K, W.data_ptr(), W.stride(0), scheme.handle, Wp.data_ptr(), stream))
    return Wp


def lcma_fp8_workspace_bytes(scheme: Scheme, M: int, N: int, K: int) -> int:
    return int(lib().lcma_fp8_workspace_bytes(scheme.handle, M, N, K))


def lcma_fp8_gemm_lcma(A, Wp, C, scheme: Scheme, workspace):
    """C (bf16) = A (bf16, M x K) x W^T with the prepared weights Wp = lcma_fp8_prepare_w(W, scheme)."""
    import torch
    assert A.is_cuda and A.dtype == torch.bfloat16 and C.dtype == torch.bfloat16 and A.stride(1) == C.stride(1) == 1
    M, K = A.shape
    M2, N = C.shape
    assert M == M2 and workspace.is_contiguous() and Wp.is_contiguous()
    stream = torch.cuda.current_stream(A.device).cuda_stream
    _check(lib().lcma_fp8_gemm_lcma(M, N, K, A.data_ptr(), A.stride(0), Wp.data_ptr(), C.data_ptr(), C.stride(0),
                                    scheme.handle, workspace.data_ptr(), workspace.numel(), stream))
    return C


def lcma_set_tuning(key: str, value: str = ""):
    """Measurement aid: "variant", "unfused_variant", "panel" or "batch_order"; an empty value restores the default."""
    _check(lib().lcma_set_tuning(key.encode(), value.encode()))


def lcma_sched_waves(groups: int, R: int, units: int):
    a, b = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().lcma_sched_waves(groups, R, units, ctypes.byref(a), ctypes.byref(b)))
    return int(a.value), int(b.value)


def lcma_sched_range(groups: int, R: int, units: int, unit: int):
    a, b = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().lcma_sched_range(groups, R, units, unit, ctypes.byref(a), ctypes.byref(b)))
    return int(a.value), int(b.value)
