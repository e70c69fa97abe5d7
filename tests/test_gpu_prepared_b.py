"""GPU parity of the offline Combine-B path: lcma_prepare_b against the oracle's Combine B as stored
(bit for bit: both add in fp32 in the same order and round once), and lcma_gemm_prepared against the
oracle's product (integers bit-exact, floats within the bounds of the fused path)."""
import numpy as np
import pytest

import lcma_inputs as inp
import oracle
from oracle import schemes as S

pytestmark = pytest.mark.gpu

REL_BOUND = {"f32": 1e-5, "bf16": 2e-2, "f16": 2e-2}


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_06057_amd import binding
    binding.lib()
    return binding


def prepared_to_host(bt) -> np.ndarray:
    """(R, N/n, K/k) device tensor -> (R, K/k, N/n) fp64, the oracle's orientation."""
    return bt.cpu().numpy().astype(np.float64).transpose(0, 2, 1)


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("kind", ["uniform", "weights", "int"])
def test_prepare_b_equals_oracle_bit_for_bit(B, dt, kind):
    import torch
    import gpu_util as G
    s = S.strassen()
    N, K = 3 * 128, 5 * 64  # 3 x 5 tiles of the Combine-B kernel per block (5 x 10 for fp32)
    print(f"prepare_b {dt} {kind} N={N} K={K}", flush=True)
    _, Bs = inp.matrices("uniform", kind, 64, N, K, dt, seed=11)
    want = oracle.combine_b_stored(s, inp.widen(Bs, dt), dt)
    # B as a strided view (ldb > N)
    pad = 16 // (4 if dt == "f32" else 2)
    big = torch.zeros((K, N + 3 * pad), dtype=G.empty_like_c(1, 1, dt).dtype, device="cuda")
    big[:, pad:pad + N] = G.to_device(Bs, dt)
    h = B.lcma_scheme_load("builtin:strassen")
    bt = B.lcma_prepare_b(big[:, pad:pad + N], h)
    assert tuple(bt.shape) == (7, N // 2, K // 2)
    assert bt.dtype == (torch.float32 if dt == "f32" else torch.float16)
    assert B.lcma_prepared_b_bytes(h, N, K, B.DTYPE_IDS[dt]) == bt.numel() * bt.element_size()
    got = prepared_to_host(bt)
    assert np.array_equal(got, want)
    if kind == "int":  # and then the stored values are the exact sums
        assert np.array_equal(got, oracle.combine_b(s, inp.widen(Bs, dt)))


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
def test_gemm_prepared_integer_bit_exact_and_float_bounds(B, dt):
    import gpu_util as G
    h = B.lcma_scheme_load("builtin:strassen")
    M, N, K = 768, 512, 384
    print(f"gemm_prepared {dt} {M}x{N}x{K}", flush=True)
    Ai, Bi = inp.integers(101, 1, (M, K)), inp.integers(101, 2, (K, N))
    want = inp.store(oracle.gemm(Ai, Bi).astype(np.float64), dt)
    a, b = G.to_device(inp.store(Ai, dt), dt), G.to_device(inp.store(Bi, dt), dt)
    bt = B.lcma_prepare_b(b, h)
    c = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_prepared(a, bt, c, h)
    assert np.array_equal(G.to_host_stored(c, dt).view(np.uint8), want.view(np.uint8))

    kinds = ("uniform", "uniform") if dt != "bf16" else ("normal", "weights")
    As, Bs = inp.matrices(kinds[0], kinds[1], M, N, K, dt, seed=13)
    ref = oracle.gemm(inp.widen(As, dt), inp.widen(Bs, dt))
    a, b = G.to_device(As, dt), G.to_device(Bs, dt)
    bt = B.lcma_prepare_b(b, h)
    c = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_prepared(a, bt, c, h)
    err = oracle.rel_frobenius(G.to_host_f64(c, dt), ref)
    cp = G.empty_like_c(M, N, dt)
    B.lcma_gemm(a, b, cp, None)
    err_plain = oracle.rel_frobenius(G.to_host_f64(cp, dt), ref)
    cf = G.empty_like_c(M, N, dt)
    B.lcma_gemm(a, b, cf, h)
    err_fused = oracle.rel_frobenius(G.to_host_f64(cf, dt), ref)
    print(f"relF prepared {err:.3e} fused {err_fused:.3e} plain {err_plain:.3e}", flush=True)
    assert err <= REL_BOUND[dt] and err <= 4.0 * err_plain
    # the prepared operand is rounded once from an fp32 sum: never worse than the fused kernel's packed adds
    assert err <= 1.05 * err_fused


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
def test_prepare_b_ragged_n(B, dt):
    """N that is not a whole number of tiles: the planes hold the padded rows, filled with zeros."""
    import gpu_util as G
    s = S.strassen()
    h = B.lcma_scheme_load("builtin:strassen")
    vec = 4 if dt == "f32" else 8
    N, K = 128 + 5 * vec, 128 + 3 * vec
    _, Bs = inp.matrices("uniform", "uniform", 64, N, K, dt, seed=17)
    bt = B.lcma_prepare_b(G.to_device(Bs, dt), h)
    kt = 16 if dt == "f32" else 32                       # K/k is padded to whole tiles of the Combine-B kernel
    Kp = -(-K // (2 * kt)) * 2 * kt
    assert tuple(bt.shape) == (7, 128, Kp // 2)          # N/n padded from 64 + 2.5 vec to 128
    got = prepared_to_host(bt)
    padded = np.zeros((Kp, 256))
    # blocks are cut from the padded matrix: block row l starts at l * Kp/2, block column j at j * 128
    padded[:K, :N] = inp.widen(Bs, dt)
    want = oracle.combine_b_stored(s, padded, dt)
    assert np.array_equal(got, want)
    # and the product against it, ragged in all three directions
    M = 200 + 3
    Ai, Bi = inp.integers(9, 5, (M, K)), inp.integers(9, 6, (K, N))
    a, b = G.to_device(inp.store(Ai, dt), dt), G.to_device(inp.store(Bi, dt), dt)
    c = G.empty_like_c(M, N, dt, fill=float("nan"))
    B.lcma_gemm_prepared(a, B.lcma_prepare_b(b, h), c, h)
    want = inp.store(oracle.gemm(Ai, Bi).astype(np.float64), dt)
    assert np.array_equal(G.to_host_stored(c, dt).view(np.uint8), want.view(np.uint8))


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
def test_prepare_bt_takes_the_weight_layout(B, dt):
    """Weights stored N x K (W = B^T, strided view): same planes as lcma_prepare_b, bit for bit, and
    equal to the oracle's stored Combine B, for a full and a ragged shape."""
    import torch
    import gpu_util as G
    s = S.strassen()
    h = B.lcma_scheme_load("builtin:strassen")
    vec = 4 if dt == "f32" else 8
    for N, K in ((256, 192), (128 + 5 * vec, 128 + 3 * vec)):
        print(f"prepare_bt {dt} N={N} K={K}", flush=True)
        _, Bs = inp.matrices("uniform", "weights", 64, N, K, dt, seed=23)
        b = G.to_device(Bs, dt)
        big = torch.zeros((N, K + 2 * vec), dtype=b.dtype, device="cuda")
        big[:, vec:vec + K] = b.t()
        bt_w = B.lcma_prepare_bt(big[:, vec:vec + K], h)
        bt_b = B.lcma_prepare_b(b, h)
        assert bt_w.shape == bt_b.shape
        assert torch.equal(bt_w.view(torch.uint8), bt_b.view(torch.uint8))
        kt = 16 if dt == "f32" else 32
        Kp, Np = -(-K // (2 * kt)) * 2 * kt, -(-N // 128) * 128
        padded = np.zeros((Kp, Np))
        padded[:K, :N] = inp.widen(Bs, dt)
        assert np.array_equal(prepared_to_host(bt_w), oracle.combine_b_stored(s, padded, dt))


def test_prepared_error_paths_launch_nothing(B):
    import torch
    h = B.lcma_scheme_load("builtin:strassen")
    b = torch.ones((256, 256), dtype=torch.float16, device="cuda")
    with pytest.raises(B.LcmaError) as e:
        B.lcma_prepare_b(b[:100, :252], h)                  # N = 252: rows are not whole 16-byte vectors
    assert e.value.status == B.LCMA_ERR_SHAPE
    with pytest.raises(B.LcmaError) as e:
        B.lcma_prepare_b(b[:, 1:129], h)                    # misaligned pointer
    assert e.value.status == B.LCMA_ERR_ARG
    h2 = B.lcma_scheme_load("builtin:laderman")
    assert B.lcma_prepared_b_bytes(h2, 384, 384, B.LCMA_F16) == 23 * 128 * 128 * 2
    assert B.lcma_prepared_b_bytes(h2, 256, 384, B.LCMA_F16) == 23 * 128 * 128 * 2   # N padded to 3 * 128
    assert B.lcma_prepared_b_bytes(h2, 250, 384, B.LCMA_F16) == -1   # rows of B must stay 16-byte granular
    h3 = B.lcma_scheme_load("builtin:strassen2")
    bt3 = torch.zeros((49, 64, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(B.LcmaError) as e:                   # two-level Strassen has no fp16 kernels
        B.lcma_prepare_b(torch.ones((256, 256), dtype=torch.float16, device="cuda"), h3, bt3)
    assert e.value.status == B.LCMA_ERR_NOKERNEL
    bt = B.lcma_prepare_b(b, h)
    c = torch.full((200, 256), 3.0, dtype=torch.float16, device="cuda")
    with pytest.raises(B.LcmaError) as e:
        B.lcma_gemm_prepared(b[:200, :100], bt, c, h)       # K = 100: rows of A are not whole 16-byte vectors
    assert e.value.status == B.LCMA_ERR_SHAPE
    torch.cuda.synchronize()
    assert torch.all(c == 3.0) and torch.all(bt3 == 0)
    B.lcma_gemm_prepared(b[:0], bt, torch.empty((0, 256), dtype=torch.float16, device="cuda"), h)  # M = 0


@pytest.mark.parametrize("name,dt", [("laderman", "bf16"), ("laderman", "f16"), ("laderman", "f32"), ("strassen2", "bf16"),
                                     ("strassen2", "f32")])
def test_prepare_b_of_the_high_rank_schemes_bit_for_bit(B, name, dt):
    """Combine B of <3,3,3;23> and <4,4,4;49> in both layouts of B against the oracle's stored Combine B, bit for bit; K/k is
    one and a half times what a work-group of the K x N kernel covers, so its last work-group writes half a line."""
    import torch
    import gpu_util as G
    s = S.by_name(name)
    h = B.lcma_scheme_load("builtin:" + name)
    kt = 16 if dt == "f32" else 32
    N, K = s.n * 128, s.k * 3 * kt
    print(f"prepare_b {name} {dt} N={N} K={K}", flush=True)
    _, Bs = inp.matrices("uniform", "weights", 64, N, K, dt, seed=31)
    want = oracle.combine_b_stored(s, inp.widen(Bs, dt), dt)
    b = G.to_device(Bs, dt)
    bt_b = B.lcma_prepare_b(b, h)
    bt_w = B.lcma_prepare_bt(b.t().contiguous(), h)
    assert tuple(bt_b.shape) == (s.R, N // s.n, K // s.k)
    assert np.array_equal(prepared_to_host(bt_b), want)
    assert torch.equal(bt_w.view(torch.uint8), bt_b.view(torch.uint8))
