"""Split-Group Parallelism in a kernel (Sec. 3.2): the plane GEMM hands the steps of all tile-products to persistent
work-groups in contiguous ranges of ceil(total / work-groups) steps, a tile-product that straddles work-groups is put
together from fp32 pieces by a second kernel in ascending work-group order.  Checked here through the plain GEMM for
N x K weights (lcma_gemm_nt_ws) and through Algorithm 1 (lcma_gemm_unfused level 1): that schedule, the launch with a
work-group per tile-product and the persistent work-groups that take whole tile-products in turn, each against the
oracle's exact product on integer inputs (identical bits), and against each other on float inputs."""
import numpy as np
import pytest

import lcma_inputs as inp
import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_06057_amd import binding
    binding.lib()
    return binding


# few tiles and long K (the split-K case: every tile is cut into many pieces), a single tile, more tiles than
# work-groups (pieces only where a range ends inside a tile; the persistent work-groups take several whole
# tile-products each, 306 and 323 of them: a number no multiple of 8, the last XCD's share shorter), ragged M and N
PLAIN_SHAPES = [(256, 256, 4096), (100, 72, 1024), (2048, 4096, 2048), (4352, 4608, 320), (4800, 4200, 192), (520, 392, 1216)]


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("shape", PLAIN_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_plain_gemm_both_schedules(B, dt, shape):
    import torch
    import gpu_util as G
    M, N, K = shape
    Ai, Wi = inp.integers(71, 1, (M, K)), inp.integers(71, 2, (N, K))
    want = inp.store((Ai @ Wi.T).astype(np.float64), dt)
    a, w = G.to_device(inp.store(Ai, dt), dt), G.to_device(inp.store(Wi, dt), dt)
    rng = np.random.default_rng(M + K)
    Af, Wf = inp.store(rng.standard_normal((M, K)), dt), inp.store(rng.standard_normal((N, K)) * 0.05, dt)
    af, wf = G.to_device(Af, dt), G.to_device(Wf, dt)
    ws = torch.empty((B.lcma_split_group_scratch_bytes(),), dtype=torch.uint8, device="cuda")
    ref = oracle.gemm(inp.widen(Af, dt), np.ascontiguousarray(inp.widen(Wf, dt).T))
    got = {}
    try:
        for sched in ("static", "split", "persist"):
            B.lcma_set_tuning("schedule", sched)
            big = G.empty_like_c(M + 3, N + 8, dt, fill=float("nan"))
            print(f"plane gemm {dt} {M}x{N}x{K} schedule {sched}", flush=True)
            B.lcma_gemm_nt_ws(a, w, big[:M, :N], ws)
            torch.cuda.synchronize()
            assert np.array_equal(G.to_host_stored(big[:M, :N], dt).view(np.uint8), want.view(np.uint8)), sched
            assert torch.isnan(big[M:]).all().item() and torch.isnan(big[:, N:]).all().item(), "wrote outside C"
            c = G.empty_like_c(M, N, dt, fill=float("nan"))
            B.lcma_gemm_nt_ws(af, wf, c, ws)
            torch.cuda.synchronize()
            got[sched] = G.to_host_f64(c, dt)
            assert oracle.rel_frobenius(got[sched], ref) <= 2e-2
    finally:
        B.lcma_set_tuning("schedule", "")
    # the same bits as lcma_gemm_nt on integers, and the two schedules within two roundings of C of each other
    c0 = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_nt(a, w, c0, None)
    assert np.array_equal(G.to_host_stored(c0, dt).view(np.uint8), want.view(np.uint8))
    eps = 2.0 ** -8 if dt == "bf16" else 2.0 ** -11
    assert oracle.rel_frobenius(got["split"], got["static"]) <= eps
    # no workspace: never split, still right
    B.lcma_set_tuning("schedule", "")
    c1 = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_nt_ws(a, w, c1, None)
    assert np.array_equal(G.to_host_stored(c1, dt).view(np.uint8), want.view(np.uint8))


@pytest.mark.parametrize("name,shape", [("strassen", (520, 776, 328)), ("strassen", (4104, 4608, 128)), ("laderman", (768, 768, 1536)),
                                        ("strassen2", (2048, 1024, 4096))])
def test_algorithm1_both_schedules(B, name, shape):
    import torch
    import gpu_util as G
    dt = "bf16"
    M, N, K = shape
    h = B.lcma_scheme_load("builtin:" + name)
    # entries in [-1, 1]: the products H_r, which Algorithm 1 stores in fp16, stay integers below 2048
    Ai, Bi = inp.integers(73, 1, (M, K), -1, 1), inp.integers(73, 2, (K, N), -1, 1)
    want = inp.store(oracle.gemm(Ai, Bi).astype(np.float64), dt)
    a, b = G.to_device(inp.store(Ai, dt), dt), G.to_device(inp.store(Bi, dt), dt)
    nb = B.lcma_unfused_workspace_bytes(h, M, N, K, B.LCMA_BF16) + B.lcma_split_group_scratch_bytes()
    ws = torch.empty((nb,), dtype=torch.uint8, device="cuda")
    try:
        for sched in ("static", "split", "persist"):
            B.lcma_set_tuning("schedule", sched)
            c = G.empty_like_c(M, N, dt, fill=float("nan"))
            print(f"algorithm 1 {name} {M}x{N}x{K} schedule {sched}", flush=True)
            B.lcma_gemm_unfused(1, a, b, c, h, ws)
            torch.cuda.synchronize()
            assert np.array_equal(G.to_host_stored(c, dt).view(np.uint8), want.view(np.uint8)), sched
    finally:
        B.lcma_set_tuning("schedule", "")


def test_split_needs_its_scratch(B):
    import torch
    a = torch.ones((256, 256), dtype=torch.bfloat16, device="cuda")
    c = torch.full((256, 256), 3.0, dtype=torch.bfloat16, device="cuda")
    small = torch.empty((1 << 20,), dtype=torch.uint8, device="cuda")
    B.lcma_set_tuning("schedule", "split")
    try:
        with pytest.raises(B.LcmaError) as e:
            B.lcma_gemm_nt_ws(a, a, c, small)
        assert e.value.status == B.LCMA_ERR_ARG and "scratch" in str(e.value)
    finally:
        B.lcma_set_tuning("schedule", "")
    torch.cuda.synchronize()
    assert torch.all(c == 3.0).item()
