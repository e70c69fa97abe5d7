"""lcma_gemm_ex, C = alpha * (A B) + beta * C, through the C ABI against the oracle (the fp64 product, scaled and
added in fp64, rounded once): exact on integer inputs with integer factors, within the storage type's rounding on
floats; alpha = 1, beta = 0 must give lcma_gemm's bits and must not read C."""
import numpy as np
import pytest

import lcma_inputs as inp
import oracle

pytestmark = pytest.mark.gpu

CASES = [  # scheme, dtype, (M, N, K), B given N x K?
    (None, "bf16", (300, 264, 200), False), (None, "f32", (256, 256, 64), True),
    ("strassen", "bf16", (512, 384, 512), False), ("strassen", "f16", (260, 200, 328), True),
    ("strassen", "f32", (250, 132, 260), False), ("winograd", "f32", (256, 256, 256), True),
    ("strassen2", "bf16", (256, 512, 256), False), ("laderman", "f16", (384, 200, 192), False),
    ("laderman", "f32", (390, 100, 100), True),
]
EPS = {"f32": 2.0 ** -24, "bf16": 2.0 ** -9, "f16": 2.0 ** -11}


@pytest.fixture(scope="module")
def B():
    from paper_2605_06057_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("name,dt,shape,nk", CASES, ids=lambda c: str(c))
def test_scaled_gemm(B, name, dt, shape, nk):
    import torch
    import gpu_util as G
    M, N, K = shape
    print(f"lcma_gemm_ex {name} {dt} {M}x{N}x{K} nk={nk}", flush=True)
    h = B.lcma_scheme_load("builtin:" + name) if name else None
    second = (lambda b: b.t().contiguous()) if nk else (lambda b: b)
    # integers: exact
    Ai, Bi, Ci = inp.integers(31, 1, (M, K)), inp.integers(31, 2, (K, N)), inp.integers(31, 3, (M, N))
    a, b = G.to_device(inp.store(Ai, dt), dt), G.to_device(inp.store(Bi, dt), dt)
    c = G.to_device(inp.store(Ci, dt), dt)
    B.lcma_gemm_ex(2.0, -1.0, a, second(b), c, h, b_nk=nk)
    want = inp.store((2 * oracle.gemm(Ai, Bi) - Ci).astype(np.float64), dt)
    assert np.array_equal(G.to_host_stored(c, dt).view(np.uint8), want.view(np.uint8))
    # floats: one rounding of the fp64 value, plus the fp32 accumulation
    As, Bs, Cs = (inp.store(inp.normal(32, i, s), dt) for i, s in ((1, (M, K)), (2, (K, N)), (3, (M, N))))
    Aw, Bw, Cw = inp.widen(As, dt), inp.widen(Bs, dt), inp.widen(Cs, dt)
    a, b, c = G.to_device(As, dt), G.to_device(Bs, dt), G.to_device(Cs, dt)
    B.lcma_gemm_ex(0.5, 1.5, a, second(b), c, h, b_nk=nk)
    ref = 0.5 * oracle.gemm(Aw, Bw) + 1.5 * Cw
    plain = G.empty_like_c(M, N, dt, fill=0.0)
    B.lcma_gemm(a, b, plain, h)                       # the unscaled product, for the size of the scheme's own error
    err_product = oracle.rel_frobenius(G.to_host_f64(plain, dt), oracle.gemm(Aw, Bw))
    err = oracle.rel_frobenius(G.to_host_f64(c, dt), ref)
    print(f"relF scaled {err:.3e}, unscaled product {err_product:.3e}", flush=True)
    assert err <= 2.0 * EPS[dt] + err_product
    # alpha = 1, beta = 0: lcma_gemm's bits, and C is not read (it holds NaN)
    c1 = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_ex(1.0, 0.0, a, second(b), c1, h, b_nk=nk)
    assert torch.equal(c1.view(torch.uint8), plain.view(torch.uint8))
    # beta != 0 reads C: NaN in, NaN out (and only there)
    c2 = G.to_device(Cs, dt)
    c2[3, 5] = float("nan")
    B.lcma_gemm_ex(1.0, 1.0, a, second(b), c2, h, b_nk=nk)
    bad = torch.isnan(c2)
    assert bad[3, 5].item() and int(bad.sum().item()) == 1


def test_scaled_gemm_refusals(B):
    import torch
    a = torch.zeros((64, 64), dtype=torch.float16, device="cuda")
    c = torch.full((64, 64), 3.0, dtype=torch.float16, device="cuda")
    L = B.lib()
    st = torch.cuda.current_stream().cuda_stream
    args = (64, 64, 64, a.data_ptr(), 64, a.data_ptr(), 64, c.data_ptr(), 64, B.LCMA_F16, None, st)
    assert L.lcma_gemm_ex(1.0, 0.0, 1, *args) == B.LCMA_ERR_ARG            # the prepared layout has its own entry point
    assert L.lcma_gemm_ex(float("nan"), 0.0, 0, *args) == B.LCMA_ERR_ARG
    assert L.lcma_gemm_ex(1.0, float("nan"), 0, *args) == B.LCMA_ERR_ARG
    torch.cuda.synchronize()
    assert torch.all(c == 3.0).item()
    assert L.lcma_gemm_ex(0.0, 2.0, 0, *args) == B.LCMA_OK                 # alpha = 0: C is scaled
    torch.cuda.synchronize()
    assert torch.all(c == 6.0).item()
