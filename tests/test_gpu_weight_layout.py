"""lcma_gemm_nt (B given as the N x K weight matrix W, C = A W^T) through the C ABI: exact on integer
inputs against the oracle, and bit for bit what lcma_gemm returns for B = W^T on floating-point inputs
(same tiles, same arithmetic, only the way the B tiles reach LDS differs).  Every kernel of this layout is
also covered, by name, by the per-variant parity tests."""
import numpy as np
import pytest

import lcma_inputs as inp
import oracle
from oracle import schemes as S

pytestmark = pytest.mark.gpu

CASES = [  # scheme, dtype, (M, N, K): whole tiles, and ragged in every direction
    (None, "bf16", (512, 512, 256)), (None, "f32", (300, 264, 200)),
    ("strassen", "bf16", (512, 384, 512)), ("strassen", "f16", (260, 200, 328)), ("strassen", "f32", (250, 132, 260)),
    ("strassen2", "bf16", (512, 512, 256)), ("strassen2", "f32", (130, 260, 132)),
    ("laderman", "f16", (384, 384, 192)), ("laderman", "bf16", (100, 392, 200)), ("laderman", "f32", (390, 100, 100)),
]


@pytest.fixture(scope="module")
def B():
    from paper_2605_06057_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("name,dt,shape", CASES, ids=lambda c: str(c))
def test_weight_layout_matches_oracle_and_lcma_gemm(B, name, dt, shape):
    import torch
    import gpu_util as G
    M, N, K = shape
    print(f"lcma_gemm_nt {name} {dt} {M}x{N}x{K}", flush=True)
    h = B.lcma_scheme_load("builtin:" + name) if name else None
    vec = 4 if dt == "f32" else 8
    # integers: exact
    Ai, Bi = inp.integers(77, 1, (M, K)), inp.integers(77, 2, (K, N))
    want = inp.store(oracle.gemm(Ai, Bi).astype(np.float64), dt)
    a = G.to_device(inp.store(Ai, dt), dt)
    b = G.to_device(inp.store(Bi, dt), dt)
    wide = torch.full((N + 1, K + vec), float("nan"), dtype=b.dtype, device="cuda")  # NaN wherever W must not be read
    w = wide[:N, :K]
    w.copy_(b.t())
    big_c = G.empty_like_c(M + 2, N + 2 * vec, dt, fill=7.0)
    c = big_c[1:M + 1, vec:vec + N]
    B.lcma_gemm_nt(a, w, c, h)
    got = G.to_host_stored(c, dt)
    assert np.array_equal(got.view(np.uint8), want.view(np.uint8))
    guard = big_c.clone()
    guard[1:M + 1, vec:vec + N] = 7.0
    assert torch.all(guard == 7.0).item(), "wrote outside C"
    # normal floats: the same bits as the K x N entry point
    Af, Bf = inp.normal(78, 1, (M, K)), inp.normal(78, 2, (K, N))
    a, b = G.to_device(inp.store(Af, dt), dt), G.to_device(inp.store(Bf, dt), dt)
    w.copy_(b.t())
    c1, c2 = G.empty_like_c(M, N, dt, fill=float("nan")), G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm(a, b, c1, h)
    B.lcma_gemm_nt(a, w, c2, h)
    assert torch.equal(c1.view(torch.uint8), c2.view(torch.uint8))


def test_weight_layout_error_paths(B):
    import torch
    a = torch.zeros((64, 64), dtype=torch.float16, device="cuda")
    c = torch.zeros((64, 128), dtype=torch.float16, device="cuda")
    w = torch.zeros((128, 64), dtype=torch.float16, device="cuda")
    B.lcma_gemm_nt(a, w, c)                                  # fine
    L = B.lib()
    st = torch.cuda.current_stream().cuda_stream
    # leading dimension of W smaller than K
    assert L.lcma_gemm_nt(64, 128, 64, a.data_ptr(), 64, w.data_ptr(), 56, c.data_ptr(), 128, B.LCMA_F16, None, st) == B.LCMA_ERR_ARG
    # a scheme without kernels for this layout
    h = B.lcma_scheme_load("builtin:strassen_wide")
    assert L.lcma_gemm_nt(64, 128, 64, a.data_ptr(), 64, w.data_ptr(), 64, c.data_ptr(), 128, B.LCMA_F16, h.handle, st) == B.LCMA_ERR_NOKERNEL
    assert "N x K" in B.lib().lcma_last_error().decode()
