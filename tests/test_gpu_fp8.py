"""GPU parity of the FP8 path (E4M3 codes, 1 x 128 power-of-two block scales) against oracle/fp8.py, through the C ABI.

Codes and scale bytes are compared bit for bit (the scale decision is integer logic on the block maximum and the one
rounding is the conversion to E4M3, so both sides take every decision on the same fp32 values).  Products are compared
(i) exactly on integer-valued inputs that the format holds exactly, (ii) against the oracle's fp64 product of the SAME
codes within FP8_ACC_TOL, the allowance for fp32 accumulation in the matrix unit (derivation in the test), and (iii)
against the unquantised product, where the LCMA form may be at most 4 times as far off as the plain form."""
import numpy as np
import pytest

import lcma_inputs as inp
import oracle
from oracle import fp8 as F
from oracle import schemes as S

pytestmark = pytest.mark.gpu

# The matrix unit adds the exact products of a 64-element slice into an fp32 accumulator.  A probe on MI355X put the
# deviation of one such slice sum at no more than 2^-12.5 of the sum of the magnitudes of its terms in the worst of 1024
# outputs; for operands with zero mean the magnitudes of K terms sum to about sqrt(K) times the size of the result and
# the slice deviations add in quadrature, which gives a relative Frobenius deviation below 2^-12.5 * 8 / sqrt(K / 64),
# 4e-4 from K = 1024 on (the measured deviation is far smaller: 3e-5 at most in these tests, next to the 1.7e-3 of the
# final rounding of C to bf16, which is accounted for separately).
FP8_ACC_TOL = 4e-4


def up(x, g):
    return (x + g - 1) // g * g


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2605_06057_amd import binding
    binding.lib()
    return binding


def bf16_dev(values):
    import gpu_util as G
    return G.to_device(inp.store(values, "bf16"), "bf16")


def bf16_values(values):
    return inp.widen(inp.store(values, "bf16"), "bf16")


def padded(X, rows, cols):
    out = np.zeros((rows, cols), np.float64)
    out[:X.shape[0], :X.shape[1]] = X
    return out


@pytest.mark.parametrize("rows,K", [(16, 128), (37, 392), (300, 1024), (5, 8)])
def test_quantize_codes_and_scales_bit_exact(B, rows, K):
    rng = np.random.default_rng(rows * 1000 + K)
    X = bf16_values(rng.standard_normal((rows, K)) * np.exp(rng.uniform(-8, 8, (rows, 1))))
    X[0, : min(K, 128)] = 0.0                       # an all-zero block
    X[-1, 0] = 448.0 if K >= 128 else X[-1, 0]      # a block maximum exactly at the top of the range
    print(f"fp8 quantize {rows}x{K}", flush=True)
    Q, Sc = B.lcma_fp8_quantize(bf16_dev(X))
    kp = up(K, 128)
    want_q, want_s = F.quantize_1x128(padded(X, rows, kp))
    got_q, got_s = Q.cpu().numpy(), Sc.cpu().numpy()
    assert got_q.shape == (rows, kp) and got_s.shape[1] == up(kp // 128, 4)
    assert np.array_equal(got_s[:, : kp // 128], want_s)
    assert np.array_equal(got_q, want_q)


def test_plain_fp8_gemm_exact_on_integers(B):
    import torch
    M, N, K = 300, 264, 392                          # ragged in all three directions, several tiles
    Ai, Wi = inp.integers(41, 1, (M, K)), inp.integers(41, 2, (N, K))
    qa, sa = B.lcma_fp8_quantize(bf16_dev(Ai.astype(np.float64)))
    qw, sw = B.lcma_fp8_quantize(bf16_dev(Wi.astype(np.float64)))
    big = torch.full((M + 2, N + 8), float("nan"), dtype=torch.bfloat16, device="cuda")
    print(f"fp8 plain gemm {M}x{N}x{K}", flush=True)
    B.lcma_fp8_gemm_nt(qa, sa, qw, sw, big[:M, :N], K)
    torch.cuda.synchronize()
    import gpu_util as G
    want = inp.store((Ai @ Wi.T).astype(np.float64), "bf16")
    assert np.array_equal(G.to_host_stored(big[:M, :N], "bf16"), want)
    assert torch.isnan(big[M:]).all().item() and torch.isnan(big[:, N:]).all().item(), "wrote outside C"


@pytest.mark.parametrize("shape", [(256, 256, 512), (520, 392, 1160), (1024, 2048, 1024)])
def test_plain_fp8_gemm_against_the_oracle_on_the_same_codes(B, shape):
    import torch
    import gpu_util as G
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    A = bf16_values(rng.standard_normal((M, K)))
    W = bf16_values(rng.standard_normal((N, K)) * 0.02)
    qa, sa = B.lcma_fp8_quantize(bf16_dev(A))
    qw, sw = B.lcma_fp8_quantize(bf16_dev(W))
    c = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    print(f"fp8 plain gemm {M}x{N}x{K}", flush=True)
    B.lcma_fp8_gemm_nt(qa, sa, qw, sw, c, K)
    torch.cuda.synchronize()
    kp = up(K, 128)
    ref_q = F.gemm_fp8(qa.cpu().numpy(), sa.cpu().numpy()[:, : kp // 128], qw.cpu().numpy(), sw.cpu().numpy()[:, : kp // 128])
    got = G.to_host_f64(c, "bf16")
    assert not np.isnan(got).any()
    dev = oracle.rel_frobenius(got, ref_q)
    rounded = oracle.rel_frobenius(inp.widen(inp.store(ref_q, "bf16"), "bf16"), ref_q)   # what the bf16 rounding of C alone costs
    err = oracle.rel_frobenius(got, oracle.gemm(A, np.ascontiguousarray(W.T)))
    print(f"  vs oracle on the same codes {dev:.3e} (bf16 rounding alone {rounded:.3e}); vs unquantised {err:.3e}", flush=True)
    assert dev <= rounded + FP8_ACC_TOL
    assert err <= 6e-2


@pytest.mark.parametrize("name", ["strassen", "laderman", "strassen2"])
def test_prepared_weights_bit_exact(B, name):
    s, h = S.by_name(name), B.lcma_scheme_load("builtin:" + name)
    N, K = 3 * s.n * 40, s.k * 200                   # ragged: blocks padded to 128 rows and 256 columns
    rng = np.random.default_rng(7)
    W = bf16_values(rng.standard_normal((N, K)) * 0.02)
    print(f"fp8 prepare_w {name} {N}x{K}", flush=True)
    Wp = B.lcma_fp8_prepare_w(bf16_dev(W), h).cpu().numpy()
    bn, bk = up(-(-N // s.n), 128), up(-(-K // s.k), 128)
    ls = up(bk // 128, 4)
    want_q, want_s = F.combine_w_quantized(s, padded(W, s.n * bn, s.k * bk))
    nq = up(s.R * bn * bk, 256)
    got_q = Wp[: s.R * bn * bk].reshape(s.R, bn, bk)
    got_s = Wp[nq: nq + s.R * bn * ls].reshape(s.R, bn, ls)[:, :, : bk // 128]
    assert np.array_equal(got_s, want_s)
    assert np.array_equal(got_q, want_q)


@pytest.mark.parametrize("name,lo,hi", [("strassen", -3, 3), ("strassen2", -3, 3), ("laderman", -2, 2)])
def test_lcma_fp8_exact_on_integers(B, name, lo, hi):
    """Entries small enough that every combination (at most 14 in magnitude) is an E4M3 value at its block scale: the
    whole path is exact and C equals the integer product."""
    import torch
    import gpu_util as G
    s, h = S.by_name(name), B.lcma_scheme_load("builtin:" + name)
    M, N, K = s.m * 150, s.n * 136, s.k * 264
    Ai, Wi = inp.integers(51, 1, (M, K), lo, hi), inp.integers(51, 2, (N, K), lo, hi)
    Wp = B.lcma_fp8_prepare_w(bf16_dev(Wi.astype(np.float64)), h)
    ws = torch.empty((B.lcma_fp8_workspace_bytes(h, M, N, K),), dtype=torch.uint8, device="cuda")
    big = torch.full((M + 2, N + 8), float("nan"), dtype=torch.bfloat16, device="cuda")
    print(f"fp8 lcma {name} {M}x{N}x{K}", flush=True)
    B.lcma_fp8_gemm_lcma(bf16_dev(Ai.astype(np.float64)), Wp, big[:M, :N], h, ws)
    torch.cuda.synchronize()
    want = inp.store((Ai @ Wi.T).astype(np.float64), "bf16")
    assert np.array_equal(G.to_host_stored(big[:M, :N], "bf16"), want)
    assert torch.isnan(big[M:]).all().item() and torch.isnan(big[:, N:]).all().item(), "wrote outside C"


@pytest.mark.parametrize("name,shape", [("strassen", (512, 768, 1024)), ("strassen", (1100, 520, 776)),
                                        ("laderman", (384, 768, 1152)), ("strassen2", (1024, 1024, 2048))])
def test_lcma_fp8_against_the_oracle(B, name, shape):
    import torch
    import gpu_util as G
    s, h = S.by_name(name), B.lcma_scheme_load("builtin:" + name)
    M, N, K = shape
    rng = np.random.default_rng(M + 3 * N + 5 * K)
    A = bf16_values(rng.standard_normal((M, K)))
    W = bf16_values(rng.standard_normal((N, K)) * 0.02)
    a, w = bf16_dev(A), bf16_dev(W)
    Wp = B.lcma_fp8_prepare_w(w, h)
    ws = torch.empty((B.lcma_fp8_workspace_bytes(h, M, N, K),), dtype=torch.uint8, device="cuda")
    c = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    print(f"fp8 lcma {name} {M}x{N}x{K}", flush=True)
    B.lcma_fp8_gemm_lcma(a, Wp, c, h, ws)
    qa, sa = B.lcma_fp8_quantize(a)
    qw, sw = B.lcma_fp8_quantize(w)
    cp = torch.empty_like(c)
    B.lcma_fp8_gemm_nt(qa, sa, qw, sw, cp, K)
    torch.cuda.synchronize()
    bm, bn, bk = up(-(-M // s.m), 128), up(-(-N // s.n), 128), up(-(-K // s.k), 128)
    ref_q = F.lcma_fp8(s, padded(A, s.m * bm, s.k * bk), padded(W, s.n * bn, s.k * bk), np.float16)[:M, :N]
    got, got_plain = G.to_host_f64(c, "bf16"), G.to_host_f64(cp, "bf16")
    assert not np.isnan(got).any()
    dev = oracle.rel_frobenius(got, ref_q)
    rounded = oracle.rel_frobenius(inp.widen(inp.store(ref_q, "bf16"), "bf16"), ref_q)
    exact = oracle.gemm(A, np.ascontiguousarray(W.T))
    err, err_plain = oracle.rel_frobenius(got, exact), oracle.rel_frobenius(got_plain, exact)
    print(f"  vs oracle (same dataflow) {dev:.3e} (bf16 rounding alone {rounded:.3e}); vs unquantised: lcma {err:.3e} "
          f"plain fp8 {err_plain:.3e} ratio {err / err_plain:.2f}", flush=True)
    # the W-combination adds up to nnz(W column) products, each with its own accumulation allowance
    assert dev <= rounded + FP8_ACC_TOL * np.sqrt(float(np.abs(s.W).sum(axis=0).max()))
    assert err <= 4.0 * err_plain


def test_fp8_argument_checks(B):
    import torch
    h = B.lcma_scheme_load("builtin:strassen")
    wide = B.lcma_scheme_load("builtin:strassen_wide")
    L = B.lib()
    P = 0x100000
    assert L.lcma_fp8_quantize(16, 100, P, 100, P, P, None) == B.LCMA_ERR_ARG          # ldx * 2 not a multiple of 16
    assert L.lcma_fp8_quantize(16, 100, P, 104, P, P, None) == B.LCMA_ERR_SHAPE        # K not a multiple of 8
    assert L.lcma_fp8_quantize(16, 128, None, 128, P, P, None) == B.LCMA_ERR_ARG
    assert L.lcma_fp8_gemm_nt(128, 128, 128, P, P, P, P, None, 128, None) == B.LCMA_ERR_ARG
    assert L.lcma_fp8_prepare_w(256, 256, P, 256, wide.handle, P, None) == B.LCMA_ERR_NOKERNEL
    assert L.lcma_fp8_gemm_lcma(256, 256, 256, P, 256, P, P, 256, h.handle, P, 16, None) == B.LCMA_ERR_ARG
    assert b"needed" in L.lcma_last_error()
    assert L.lcma_fp8_workspace_bytes(h.handle, 0, 256, 256) == -1 and L.lcma_fp8_code_pitch(130) == 256
    assert L.lcma_fp8_scale_pitch(130) == 4 and L.lcma_fp8_scale_pitch(128 * 5) == 8
    # K = 0: zeros
    c = torch.full((8, 16), float("nan"), dtype=torch.bfloat16, device="cuda")
    e = torch.empty((0,), dtype=torch.uint8, device="cuda")
    assert L.lcma_fp8_gemm_nt(8, 16, 0, None, None, None, None, c.data_ptr(), 16, None) == B.LCMA_OK
    torch.cuda.synchronize()
    assert torch.all(c == 0).item()


@pytest.mark.parametrize("name,shape", [("strassen", (300, 272, 528)), ("strassen", (1024, 1536, 4096)), ("laderman", (768, 768, 1536))])
def test_split_group_schedule_gives_the_same_product(B, name, shape):
    """The batched GEMM handed out as contiguous ranges of steps to persistent work-groups (Sec. 3.2, Split-Group: a
    tile-product straddles work-groups, pieces are added in a fixed order by a second kernel) against one tile-product per
    work-group: identical bits on integer inputs (every partial sum is exact), equal within the accumulation allowance
    on float inputs."""
    import torch
    import gpu_util as G
    s, h = S.by_name(name), B.lcma_scheme_load("builtin:" + name)
    M, N, K = shape
    lo, hi = (-2, 2) if name == "laderman" else (-3, 3)
    Ai, Wi = inp.integers(61, 1, (M, K), lo, hi), inp.integers(61, 2, (N, K), lo, hi)
    rng = np.random.default_rng(M)
    Af, Wf = bf16_values(rng.standard_normal((M, K))), bf16_values(rng.standard_normal((N, K)) * 0.02)
    ws = torch.empty((B.lcma_fp8_workspace_bytes(h, M, N, K),), dtype=torch.uint8, device="cuda")
    out = {}
    try:
        for sched in ("static", "split"):
            B.lcma_set_tuning("schedule", sched)
            for tag, (A, W) in (("int", (Ai.astype(np.float64), Wi.astype(np.float64))), ("float", (Af, Wf))):
                Wp = B.lcma_fp8_prepare_w(bf16_dev(W), h)
                c = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
                print(f"fp8 lcma {name} {M}x{N}x{K} schedule {sched} {tag}", flush=True)
                B.lcma_fp8_gemm_lcma(bf16_dev(A), Wp, c, h, ws)
                torch.cuda.synchronize()
                out[(sched, tag)] = G.to_host_stored(c, "bf16")
    finally:
        B.lcma_set_tuning("schedule", "")
    want = inp.store((Ai @ Wi.T).astype(np.float64), "bf16")
    assert np.array_equal(out[("static", "int")], want)
    assert np.array_equal(out[("split", "int")], want)
    a, b = inp.widen(out[("static", "float")], "bf16"), inp.widen(out[("split", "float")], "bf16")
    assert not np.isnan(b).any()
    assert oracle.rel_frobenius(b, a) <= 2.4e-3 + FP8_ACC_TOL      # two independent roundings to bf16 of nearly equal sums
