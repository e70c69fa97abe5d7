"""lcma_gemm_unfused (Algorithm 1 and Algorithm 2 as printed, intermediate results in device memory)
through the C ABI against the oracle: exact on integer inputs; on floating-point inputs within the
storage type's rounding of the oracle's evaluation of the same dataflow (oracle.lcma_unfused, which
rounds At_r, Bt_r and, at level 1, H_r where the dataflow stores them) and within the project's error
bounds of the fp64 product."""
import numpy as np
import pytest

import lcma_inputs as inp
import oracle
from oracle import schemes as S

pytestmark = pytest.mark.gpu

CASES = [  # scheme, dtype, (M, N, K): whole planes, and ragged in every direction
    ("strassen", "bf16", (512, 512, 256)), ("strassen", "f16", (260, 200, 328)), ("strassen", "f32", (250, 132, 260)),
    ("strassen2", "bf16", (1024, 512, 512)), ("strassen2", "f32", (130, 260, 132)),
    ("laderman", "f16", (384, 768, 192)), ("laderman", "bf16", (100, 392, 200)), ("laderman", "f32", (390, 100, 100)),
]
TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 2e-2}
EPS = {"f32": 2.0 ** -24, "bf16": 2.0 ** -9, "f16": 2.0 ** -11}


@pytest.fixture(scope="module")
def B():
    from paper_2605_06057_amd import binding
    binding.lib()
    return binding


def padded(x, rows, cols):
    out = np.zeros((rows, cols), x.dtype)
    out[:x.shape[0], :x.shape[1]] = x
    return out


@pytest.mark.parametrize("level", [1, 2])
@pytest.mark.parametrize("name,dt,shape", CASES, ids=lambda c: str(c))
def test_unfused_against_oracle(B, name, dt, shape, level):
    import torch
    import gpu_util as G
    M, N, K = shape
    print(f"lcma_gemm_unfused level {level} {name} {dt} {M}x{N}x{K}", flush=True)
    s = S.by_name(name)
    h = B.lcma_scheme_load("builtin:" + name)
    vec = 4 if dt == "f32" else 8
    nbytes = B.lcma_unfused_workspace_bytes(h, M, N, K, B.DTYPE_IDS[dt])
    assert nbytes > 0
    ws = torch.full((nbytes,), 0x7f, dtype=torch.uint8, device="cuda")   # stale bytes: every plane must be written in full
    # integers: exact
    Ai, Bi = inp.integers(91, 1, (M, K)), inp.integers(91, 2, (K, N))
    want = inp.store(oracle.gemm(Ai, Bi).astype(np.float64), dt)
    a, b = G.to_device(inp.store(Ai, dt), dt), G.to_device(inp.store(Bi, dt), dt)
    big_c = G.empty_like_c(M + 2, N + 2 * vec, dt, fill=7.0)
    c = big_c[1:M + 1, vec:vec + N]
    B.lcma_gemm_unfused(level, a, b, c, h, ws)
    got = G.to_host_stored(c, dt)
    assert np.array_equal(got.view(np.uint8), want.view(np.uint8))
    guard = big_c.clone()
    guard[1:M + 1, vec:vec + N] = 7.0
    assert torch.all(guard == 7.0).item(), "wrote outside C"
    # floats
    As, Bs = inp.store(inp.normal(92, 1, (M, K)), dt), inp.store(inp.normal(92, 2, (K, N)), dt)
    Aw, Bw = inp.widen(As, dt), inp.widen(Bs, dt)
    a, b = G.to_device(As, dt), G.to_device(Bs, dt)
    c = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_unfused(level, a, b, c, h, ws)
    got = G.to_host_f64(c, dt)
    ref = oracle.gemm(Aw, Bw)
    err = oracle.rel_frobenius(got, ref)
    # the same dataflow in the oracle, on the inputs padded to whole blocks
    up = lambda x, g: -(-x // g) * g
    Mp, Np, Kp = up(M, s.m), up(N, s.n), up(K, s.k)
    # (the products H_r of level 1 are kept in fp32 for fp16 storage, in fp16 for bf16 storage)
    # and <3,3,3;23> with fp16 storage multiplies the rounding residuals of the left combinations of products 4 and 7 as well
    comp = (3, 6) if (name, dt, level) == ("laderman", "f16", 1) else ()
    model = oracle.lcma_unfused(s, padded(Aw, Mp, Kp), padded(Bw, Kp, Np), dt, level, h_dtype="f32" if dt == "f16" else None,
                                residual_products=comp)[:M, :N]
    err_model = oracle.rel_frobenius(got, model)
    print(f"relF vs fp64 product {err:.3e}, vs the oracle's level-{level} evaluation {err_model:.3e}", flush=True)
    assert err <= TOL[dt]
    # what remains between the two is the final rounding of C, the fp32 accumulation of the MFMA (a random
    # walk of K/k roundings) and, at level 1, the few H_r elements whose rounding falls the other way
    assert err_model <= 2.0 * EPS[dt] + 2.0 ** -24 * np.sqrt(K)
    # static weights: the second call reuses the Bt planes and returns the same bits
    c2 = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_unfused(level, a, b, c2, h, ws, reuse_bt=True)
    assert torch.equal(c.view(torch.uint8), c2.view(torch.uint8))


def test_unfused_error_paths_launch_nothing(B):
    import torch
    h = B.lcma_scheme_load("builtin:strassen")
    a = torch.zeros((256, 256), dtype=torch.float16, device="cuda")
    c = torch.full((256, 256), 3.0, dtype=torch.float16, device="cuda")
    need = B.lcma_unfused_workspace_bytes(h, 256, 256, 256, B.LCMA_F16)
    assert need == 7 * 128 * 128 * (2 + 2 + 4)   # At and Bt in fp16, the products in fp32
    small = torch.zeros((need - 256,), dtype=torch.uint8, device="cuda")
    ws = torch.zeros((need,), dtype=torch.uint8, device="cuda")
    for args in ((1, a, a, c, h, small), (3, a, a, c, h, ws), (0, a, a, c, h, ws)):
        with pytest.raises(B.LcmaError) as e:
            B.lcma_gemm_unfused(*args)
        assert e.value.status == B.LCMA_ERR_ARG
    with pytest.raises(B.LcmaError) as e:
        B.lcma_gemm_unfused(1, a, a, c, B.lcma_scheme_load("builtin:strassen_wide"), ws)
    assert e.value.status == B.LCMA_ERR_NOKERNEL
    with pytest.raises(B.LcmaError) as e:       # a stage kernel cannot be run by name
        stage = [v["name"] for v in B.lcma_variants() if v["b_layout"] == 3][0]
        B.lcma_gemm_variant(stage, a, a, c)
    assert e.value.status == B.LCMA_ERR_ARG
    torch.cuda.synchronize()
    assert torch.all(c == 3.0).item()
    assert B.lcma_unfused_workspace_bytes(h, 0, 256, 256, B.LCMA_F16) == -1


def test_batch_order_changes_nothing_but_time(B):
    """The batched GEMM of level 1 in group-major instead of product-major order (lcma_set_tuning("batch_order", "1"),
    kept to measure the paper's Cache-Aware ordering): the same bits.  (bf16 storage: both kernels keep the products in
    fp16; for fp16 storage the default kernel keeps them in fp32 and the results differ in the last bits.)"""
    import torch
    h = B.lcma_scheme_load("builtin:laderman")
    M, N, K = 520, 392, 200
    a = torch.randn(M, K, device="cuda").bfloat16()
    b = torch.randn(K, N, device="cuda").bfloat16()
    ws = torch.empty((B.lcma_unfused_workspace_bytes(h, M, N, K, B.LCMA_BF16),), dtype=torch.uint8, device="cuda")
    c0 = torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
    c1 = torch.empty_like(c0)
    B.lcma_gemm_unfused(1, a, b, c0, h, ws)
    B.lcma_set_tuning("batch_order", "1")
    try:
        B.lcma_gemm_unfused(1, a, b, c1, h, ws)
    finally:
        B.lcma_set_tuning("batch_order", "")
    torch.cuda.synchronize()
    assert torch.equal(c0.view(torch.uint8), c1.view(torch.uint8))
