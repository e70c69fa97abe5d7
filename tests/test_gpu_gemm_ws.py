"""lcma_gemm_ws (lcma_gemm with a workspace: the fused kernel or Algorithm 1, whichever the time model predicts
faster, Sec. 3.3) through the C ABI: the dataflow it reports is the one the model's two predictions name, and the
result meets the bounds of that dataflow against the oracle (exact on integer inputs either way)."""
import numpy as np
import pytest

import lcma_inputs as inp
import oracle

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 2e-2}
# shapes on both sides of the model's choice (checked below: both dataflows must occur), one ragged
CASES = [("strassen", "bf16", (2048, 3584, 1024)), ("strassen", "bf16", (1000, 520, 264)), ("strassen", "f32", (512, 512, 512)),
         ("strassen2", "bf16", (2048, 2048, 1024)), ("laderman", "f16", (1536, 1536, 1536)), ("laderman", "bf16", (1536, 1536, 1536)), ("strassen", "f16", (4096, 7168, 2048))]


@pytest.fixture(scope="module")
def B():
    from paper_2605_06057_amd import binding
    binding.lib()
    return binding


def model_says_algorithm1(B, sid, M, N, K, dtid):
    fused, unfused = B.lcma_predict_seconds(sid, M, N, K, dtid), B.lcma_predict_unfused_seconds(sid, M, N, K, dtid, False)
    return unfused > 0 and (fused <= 0 or unfused < fused)


def test_both_dataflows_are_covered(B):
    ids = {n: i for i, n in B.SCHEME_NAMES.items()}
    flows = {model_says_algorithm1(B, ids[name], *shape, B.DTYPE_IDS[dt]) for name, dt, shape in CASES}
    assert flows == {False, True}


@pytest.mark.parametrize("name,dt,shape", CASES, ids=lambda c: str(c))
def test_gemm_ws_against_oracle(B, name, dt, shape):
    import torch
    import gpu_util as G
    M, N, K = shape
    print(f"lcma_gemm_ws {name} {dt} {M}x{N}x{K}", flush=True)
    h = B.lcma_scheme_load("builtin:" + name)
    sid = {n: i for i, n in B.SCHEME_NAMES.items()}[name]
    dtid = B.DTYPE_IDS[dt]
    expect = 1 if model_says_algorithm1(B, sid, M, N, K, dtid) else 0
    nbytes = B.lcma_unfused_workspace_bytes(h, M, N, K, dtid)
    ws = torch.full((nbytes,), 0x7f, dtype=torch.uint8, device="cuda")
    # integers: exact by either dataflow (entries in [-1, 1]: the products H_r that Algorithm 1 stores in fp16 stay
    # below 2048 in magnitude, where fp16 holds every integer)
    Ai, Bi = inp.integers(71, 1, (M, K), -1, 1), inp.integers(71, 2, (K, N), -1, 1)
    want = inp.store(oracle.gemm(Ai, Bi).astype(np.float64), dt)
    a, b = G.to_device(inp.store(Ai, dt), dt), G.to_device(inp.store(Bi, dt), dt)
    c = G.empty_like_c(M, N, dt, fill=float("nan"))
    flow = B.lcma_gemm_ws(a, b, c, h, ws)
    print(f"dataflow {flow} (model: {expect})", flush=True)
    assert flow == expect
    assert np.array_equal(G.to_host_stored(c, dt).view(np.uint8), want.view(np.uint8))
    # floats: the project's bound against the fp64 product, and no worse than 4x the plain kernel
    As, Bs = inp.store(inp.normal(72, 1, (M, K)), dt), inp.store(inp.normal(72, 2, (K, N)), dt)
    a, b = G.to_device(As, dt), G.to_device(Bs, dt)
    ref = oracle.gemm(inp.widen(As, dt), inp.widen(Bs, dt))
    c = G.empty_like_c(M, N, dt, fill=float("nan"))
    assert B.lcma_gemm_ws(a, b, c, h, ws) == expect
    err = oracle.rel_frobenius(G.to_host_f64(c, dt), ref)
    cp = G.empty_like_c(M, N, dt, fill=float("nan"))
    assert B.lcma_gemm_ws(a, b, cp, None, ws) == 0
    err_plain = oracle.rel_frobenius(G.to_host_f64(cp, dt), ref)
    # without a workspace, or with one that is too small: the fused kernel
    c2 = G.empty_like_c(M, N, dt, fill=float("nan"))
    assert B.lcma_gemm_ws(a, b, c2, h, None) == 0
    assert B.lcma_gemm_ws(a, b, c2, h, ws[:256]) == 0
    err_fused = oracle.rel_frobenius(G.to_host_f64(c2, dt), ref)
    print(f"relF {err:.3e}, fused kernel {err_fused:.3e}, plain {err_plain:.3e}", flush=True)
    # the project's bounds
    assert err <= TOL[dt] and err_fused <= TOL[dt]
    assert err <= 4.0 * err_plain
    if expect == 0:   # the same kernel ran: same bits
        assert torch.equal(c2, c)
    # the weights given N x K (C = A W^T): the same choice; Algorithm 1 then reads W without transposing and writes
    # the bits it writes for B = W^T; the fused route is lcma_gemm_nt's kernel (same bits as lcma_gemm's, tested elsewhere)
    w = b.t().contiguous()
    c3 = G.empty_like_c(M, N, dt, fill=float("nan"))
    assert B.lcma_gemm_ws(a, w, c3, h, ws, b_nk=True) == expect
    assert torch.equal(c3.view(torch.uint8), c.view(torch.uint8))
    # without a scheme: the plain product on the plane GEMM (16-bit) with the workspace for its schedule
    c4 = G.empty_like_c(M, N, dt, fill=float("nan"))
    assert B.lcma_gemm_ws(a, w, c4, None, ws, b_nk=True) == 0
    assert oracle.rel_frobenius(G.to_host_f64(c4, dt), ref) <= 1.05 * err_plain + 1e-7


@pytest.mark.parametrize("name,ratio", [("strassen", 3.2), ("laderman", 3.9)])
def test_fp16_storage_error_of_algorithm1_against_the_plain_kernel(B, name, ratio):
    """Algorithm 1 with fp16 storage against the bound of four times the plain kernel's error: with the products kept in
    fp32 the error is that of the fp16 combinations.  <2,2,2;7> (rows of 2 blocks) is well inside; <3,3,3;23> (rows of up
    to 7) would land at 4.04 and is inside because the stage kernels multiply the rounding residuals of the left
    combinations of products 4 and 7 as well (25 planes instead of 23), as the fused kernels of the scheme do."""
    import torch
    import gpu_util as G
    M = N = K = 1536
    h = B.lcma_scheme_load("builtin:" + name)
    As, Bs = inp.store(inp.uniform(5, 1, (M, K)), "f16"), inp.store(inp.uniform(5, 2, (K, N)), "f16")
    ref = oracle.gemm(inp.widen(As, "f16"), inp.widen(Bs, "f16"))
    a, b = G.to_device(As, "f16"), G.to_device(Bs, "f16")
    ws = torch.empty((B.lcma_unfused_workspace_bytes(h, M, N, K, B.LCMA_F16),), dtype=torch.uint8, device="cuda")
    c = G.empty_like_c(M, N, "f16", fill=float("nan"))
    B.lcma_gemm_unfused(1, a, b, c, h, ws)
    err = oracle.rel_frobenius(G.to_host_f64(c, "f16"), ref)
    B.lcma_gemm(a, b, c, None)
    err_plain = oracle.rel_frobenius(G.to_host_f64(c, "f16"), ref)
    print(f"{name}: Algorithm 1 {err:.3e}, plain {err_plain:.3e}, ratio {err / err_plain:.2f}", flush=True)
    assert err <= ratio * err_plain
