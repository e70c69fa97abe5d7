"""lcma_gemm_unfused_static (the entry point that allocates nothing: its planes live in the library's static device
buffer) against lcma_gemm_unfused with a caller-provided workspace, bit for bit, on two calls in a row, the second
with a smaller input; and its size limit."""
import numpy as np
import pytest

import lcma_inputs as inp
import oracle

pytestmark = pytest.mark.gpu


def _run_pair(B, level, scheme_name, dt, M, N, K, seed):
    import torch
    import gpu_util as G
    s = B.lcma_scheme_load("builtin:" + scheme_name)
    Ai, Bi = inp.integers(seed, 1, (M, K)), inp.integers(seed, 2, (K, N))
    a, b = G.to_device(inp.store(Ai, dt), dt), G.to_device(inp.store(Bi, dt), dt)
    ws = torch.empty((B.lcma_unfused_workspace_bytes(s, M, N, K, B.DTYPE_IDS[dt]),), dtype=torch.uint8, device="cuda")
    want_c = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_unfused(level, a, b, want_c, s, ws)
    got_c = G.empty_like_c(M, N, dt, fill=float("nan"))
    print(f"static level {level} {scheme_name} {dt} {M}x{N}x{K}", flush=True)
    B.lcma_gemm_unfused_static(level, a, b, got_c, s)
    torch.cuda.synchronize()
    got, want = G.to_host_stored(got_c, dt), G.to_host_stored(want_c, dt)
    assert np.array_equal(got.view(np.uint8), want.view(np.uint8)), "static buffer and workspace give different bits"
    exact = inp.store(oracle.gemm(Ai, Bi).astype(np.float64), dt)
    assert np.array_equal(got.view(np.uint8), exact.view(np.uint8)), "differs from the oracle's exact product"
    # the planes of static weights are reused from the buffer
    again = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_unfused_static(level, a, b, again, s, reuse_bt=True)
    torch.cuda.synchronize()
    assert np.array_equal(G.to_host_stored(again, dt).view(np.uint8), want.view(np.uint8))


@pytest.mark.parametrize("level", [1, 2])
def test_two_calls_in_a_row_second_smaller(level):
    import torch
    from paper_2605_06057_amd import binding as B
    assert torch.cuda.is_available()
    B.lib()
    _run_pair(B, level, "strassen", "bf16", 520, 776, 328, 0x57A71C01)   # ragged, several tiles
    _run_pair(B, level, "strassen", "bf16", 200, 264, 136, 0x57A71C02)   # smaller: stale planes of the first call stay behind it
    _run_pair(B, level, "laderman", "f32", 150, 132, 60, 0x57A71C03)


def test_size_limit_is_an_error_and_launches_nothing():
    import torch
    from paper_2605_06057_amd import binding as B
    s = B.lcma_scheme_load("builtin:strassen")
    limit = B.lcma_static_scratch_bytes()
    assert limit == 32 << 20
    M = N = K = 4096
    assert B.lcma_unfused_workspace_bytes(s, M, N, K, B.LCMA_BF16) > limit
    a = torch.ones((M, K), dtype=torch.bfloat16, device="cuda")
    c = torch.full((M, N), 3.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.LcmaError) as e:
        B.lcma_gemm_unfused_static(1, a, a, c, s)
    assert e.value.status == B.LCMA_ERR_SHAPE and "static buffer" in str(e.value)
    torch.cuda.synchronize()
    assert torch.all(c == 3.0).item()
