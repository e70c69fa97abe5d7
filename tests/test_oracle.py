"""Pins for the CPU oracle: none of these compares the oracle with itself.

GEMM triple loop  -> closed forms, exact integers, a library matmul.
Brent checker     -> the classical algorithm must pass, planted errors must fail,
                     an independent tensor-contraction form of the same identity.
Schemes           -> the facts the paper prints (tests/golden/paper_facts.txt).
LCMA evaluator    -> brute force on tiny integer matrices, bit-exact; special cases
                     that isolate one Brent equation; recursive two-level Strassen.
"""
import itertools

import numpy as np
import pytest

import lcma_inputs as inp
import oracle
from oracle import schemes as S

PAPER = ["strassen", "laderman", "strassen2"]      # the schemes the paper names
ALL = PAPER + ["strassen_wide", "winograd"]          # plus the two further schemes the package ships


# ---------------------------------------------------------------- GEMM triple loop
def test_gemm_all_ones_closed_form():
    for M, N, K in [(1, 1, 1), (3, 5, 7), (16, 9, 33)]:
        C = oracle.gemm(np.ones((M, K)), np.ones((K, N)))
        assert C.shape == (M, N) and np.all(C == K)


def test_gemm_dot_product_closed_forms():
    K = 100
    p = np.arange(1, K + 1, dtype=np.float64)
    assert oracle.gemm(p[None, :], np.ones((K, 1)))[0, 0] == K * (K + 1) / 2
    assert oracle.gemm(p[None, :], p[:, None])[0, 0] == K * (K + 1) * (2 * K + 1) / 6


def test_gemm_identity_and_rank_one():
    rng = np.random.default_rng(1)
    A = rng.standard_normal((6, 6))
    assert np.array_equal(oracle.gemm(A, np.eye(6)), A)
    assert np.array_equal(oracle.gemm(np.eye(6), A), A)
    u, v = rng.standard_normal((5, 1)), rng.standard_normal((1, 4))
    assert np.array_equal(oracle.gemm(u, v), u * v)  # one product per entry, no sum


def test_gemm_not_commutative_and_not_transposed():
    # A = e_0 e_1^T, B = e_1 e_2^T : AB = e_0 e_2^T, BA = 0.  Catches swapped / transposed operands.
    A = np.zeros((3, 3)); A[0, 1] = 2.0
    B = np.zeros((3, 3)); B[1, 2] = 3.0
    want = np.zeros((3, 3)); want[0, 2] = 6.0
    assert np.array_equal(oracle.gemm(A, B), want)
    assert np.array_equal(oracle.gemm(B, A), np.zeros((3, 3)))


def test_gemm_matches_library_matmul():
    rng = np.random.default_rng(2)
    for M, N, K in [(17, 13, 29), (64, 48, 80), (1, 7, 200)]:
        A, B = rng.standard_normal((M, K)), rng.standard_normal((K, N))
        C = oracle.gemm(A, B)
        ref = A @ B
        assert np.max(np.abs(C - ref)) <= 1e-13 * K * np.max(np.abs(ref)) + 1e-300


def test_gemm_integer_exact_and_fp64_agree():
    A = inp.integers(3, 1, (23, 31))
    B = inp.integers(3, 2, (31, 19))
    Ci = oracle.gemm(A, B)
    assert Ci.dtype == np.int64
    assert np.array_equal(Ci, A @ B)
    assert np.array_equal(oracle.gemm(A.astype(np.float64), B.astype(np.float64)), Ci.astype(np.float64))


def test_gemm_strided_views():
    rng = np.random.default_rng(4)
    big_a, big_b = rng.standard_normal((20, 30)), rng.standard_normal((30, 40))
    A, B = big_a[3:11, 5:17], big_b[2:14, 7:29]
    assert np.allclose(oracle.gemm(A, B), A @ B, rtol=0, atol=1e-12)


def test_gemm_rows_subset():
    rng = np.random.default_rng(5)
    A, B = rng.standard_normal((12, 9)), rng.standard_normal((9, 7))
    rows = [0, 5, 11]
    assert np.array_equal(oracle.gemm_rows(A, B, rows), oracle.gemm(A, B)[rows])


# ---------------------------------------------------------------- Brent checker
def brent_by_contraction(s):
    """Same identity through a library tensor contraction instead of loops."""
    T = np.einsum("ria,rbj,rcd->iabjcd", s.U.astype(np.int64), s.V.astype(np.int64), s.W.astype(np.int64))
    want = np.einsum("ab,ic,jd->iabjcd", np.eye(s.k, dtype=np.int64), np.eye(s.m, dtype=np.int64),
                     np.eye(s.n, dtype=np.int64))
    return T, want


@pytest.mark.parametrize("mkn", [(1, 1, 1), (2, 2, 2), (2, 3, 4), (3, 1, 2)])
def test_brent_accepts_classical(mkn):
    s = S.classical(*mkn)
    assert oracle.brent(s) == (0, -1)


@pytest.mark.parametrize("name", ALL)
def test_brent_accepts_named_schemes(name):
    s = S.by_name(name)
    assert oracle.brent(s) == (0, -1)
    T, want = brent_by_contraction(s)
    assert np.array_equal(T, want)


def test_brent_rejects_planted_errors_and_reports_index():
    base = S.strassen()
    for which, pos in [("U", (0, 0, 0)), ("V", (2, 1, 1)), ("W", (6, 0, 0)), ("W", (1, 1, 1))]:
        T = {"U": base.U.copy(), "V": base.V.copy(), "W": base.W.copy()}
        T[which][pos] = 1 - T[which][pos] if T[which][pos] in (0, 1) else 0
        s = S.Scheme(2, 2, 2, 7, T["U"], T["V"], T["W"])
        bad, first = oracle.brent(s)
        Tc, want = brent_by_contraction(s)
        diff = (Tc != want).reshape(-1)
        assert bad == int(diff.sum()) and bad > 0
        assert first == int(np.argmax(diff))


def test_brent_rejects_sign_flip_and_transposed_w():
    s = S.strassen()
    assert oracle.brent(S.Scheme(2, 2, 2, 7, s.U, -s.V, s.W))[0] > 0
    assert oracle.brent(S.Scheme(2, 2, 2, 7, s.U, s.V, s.W.transpose(0, 2, 1).copy()))[0] > 0
    assert oracle.brent(S.Scheme(2, 2, 2, 7, s.V, s.U, s.W))[0] > 0  # operands swapped
    assert oracle.brent(S.Scheme(2, 2, 2, 6, s.U[:6], s.V[:6], s.W[:6]))[0] > 0  # dropped product


# ---------------------------------------------------------------- schemes vs the paper's printed facts
def test_schemes_match_paper_facts(golden):
    g = golden("paper_facts.txt")
    for name in PAPER:
        s = S.by_name(name)
        assert [s.m, s.k, s.n] == [int(x) for x in g[f"{name}_grid"]]
        assert s.R == int(g[f"{name}_rank"][0])
    st = S.strassen()
    assert st.nnz()[0] == int(g["strassen_nnzU"][0])
    assert st.nnz()[0] - st.R == int(g["strassen_addsA"][0])
    c11 = [r + 1 for r in range(st.R) if st.W[r, 0, 0] != 0]
    assert c11 == [int(x) for x in g["strassen_c11_products"]]


def test_scheme_sparsity_counts():
    assert S.strassen().nnz() == (12, 12, 12)
    assert S.laderman().nnz() == (51, 51, 51)
    assert S.strassen2().nnz() == (144, 144, 144)
    for name in ALL:
        s = S.by_name(name)
        assert set(np.unique(s.U)) | set(np.unique(s.V)) | set(np.unique(s.W)) <= {-1, 0, 1}


def test_text_round_trip():
    s = S.laderman()
    rows = [l for l in S.to_text(s).splitlines()]
    assert rows[0] == "3 3 3 23" and len(rows) == 1 + 3 * 23
    U = np.array([[int(x) for x in r.split()] for r in rows[1:24]]).reshape(23, 3, 3)
    assert np.array_equal(U, s.U)


# ---------------------------------------------------------------- LCMA evaluator
def brute(A, B):
    M, K = A.shape
    N = B.shape[1]
    C = np.zeros((M, N), dtype=np.int64)
    for i in range(M):
        for j in range(N):
            acc = 0
            for p in range(K):
                acc += int(A[i, p]) * int(B[p, j])
            C[i, j] = acc
    return C


@pytest.mark.parametrize("name", ALL)
def test_lcma_equals_brute_force_on_integers(name):
    s = S.by_name(name)
    for mult in [(1, 1, 1), (2, 1, 3), (3, 2, 1)]:
        M, N, K = s.m * mult[0], s.n * mult[1], s.k * mult[2]
        A = inp.integers(11, 1, (M, K))
        B = inp.integers(11, 2, (K, N))
        assert np.array_equal(oracle.lcma(s, A, B), brute(A, B))


@pytest.mark.parametrize("name", ["strassen", "laderman"])
def test_lcma_single_entry_inputs(name):
    """A = E_{ia}, B = E_{bj}: the result is [a == b] E_{ij}; one Brent equation family per case."""
    s = S.by_name(name)
    for i, a, b, j in itertools.product(range(s.m), range(s.k), range(s.k), range(s.n)):
        A = np.zeros((s.m, s.k), np.int64); A[i, a] = 1
        B = np.zeros((s.k, s.n), np.int64); B[b, j] = 1
        want = np.zeros((s.m, s.n), np.int64)
        if a == b:
            want[i, j] = 1
        assert np.array_equal(oracle.lcma(s, A, B), want)


@pytest.mark.parametrize("name", ALL)
def test_lcma_identity_and_rectangular(name):
    s = S.by_name(name)
    M, N, K = 2 * s.m, 3 * s.n, 2 * s.k
    A = inp.integers(5, 1, (M, K))
    assert np.array_equal(oracle.lcma(s, A, np.eye(K, dtype=np.int64)), A)
    B = inp.integers(5, 2, (K, N))
    assert np.array_equal(oracle.lcma(s, np.eye(K, dtype=np.int64), B), B)


def test_lcma_classical_scheme_is_block_gemm():
    s = S.classical(2, 3, 2)
    A = inp.integers(6, 1, (4, 9))
    B = inp.integers(6, 2, (9, 6))
    assert np.array_equal(oracle.lcma(s, A, B), A @ B)


def test_lcma_fp64_close_to_gemm():
    rng = np.random.default_rng(7)
    for name in ALL:
        s = S.by_name(name)
        M, N, K = 8 * s.m, 4 * s.n, 8 * s.k
        A, B = rng.standard_normal((M, K)), rng.standard_normal((K, N))
        assert oracle.rel_frobenius(oracle.lcma(s, A, B), oracle.gemm(A, B)) < 1e-13


def test_flat_two_level_equals_recursive_strassen():
    """Applying Strassen to each of Strassen's 7 block products == the flat <4,4,4;49> scheme."""
    s1, s2 = S.strassen(), S.strassen2()
    M = N = K = 8
    A = inp.integers(9, 1, (M, K))
    B = inp.integers(9, 2, (K, N))

    def blocks(X, r, c):
        h, w = X.shape[0] // r, X.shape[1] // c
        return [[X[i * h:(i + 1) * h, j * w:(j + 1) * w] for j in range(c)] for i in range(r)]

    Ab, Bb = blocks(A, 2, 2), blocks(B, 2, 2)
    H = []
    for r in range(7):
        At = sum(int(s1.U[r, i, l]) * Ab[i][l] for i in range(2) for l in range(2))
        Bt = sum(int(s1.V[r, l, j]) * Bb[l][j] for l in range(2) for j in range(2))
        H.append(oracle.lcma(s1, np.ascontiguousarray(At), np.ascontiguousarray(Bt)))
    C = np.zeros((M, N), np.int64)
    for i in range(2):
        for j in range(2):
            C[i * 4:(i + 1) * 4, j * 4:(j + 1) * 4] = sum(int(s1.W[r, i, j]) * H[r] for r in range(7))
    flat = oracle.lcma(s2, A, B)
    assert np.array_equal(flat, C)
    assert np.array_equal(flat, brute(A, B))


def test_lcma_rejects_non_divisible_shape():
    with pytest.raises(ValueError):
        oracle.lcma(S.strassen(), np.ones((3, 4)), np.ones((4, 4)))


def test_lcma_with_wrong_scheme_disagrees():
    """A planted coefficient error must show in the evaluator, not only in the checker."""
    s = S.strassen()
    W = s.W.copy(); W[4, 0, 0] = 1  # C11 = H1+H4+H5+H7 instead of -H5
    bad = S.Scheme(2, 2, 2, 7, s.U, s.V, W)
    A = inp.integers(13, 1, (4, 4)); B = inp.integers(13, 2, (4, 4))
    assert not np.array_equal(oracle.lcma(bad, A, B), brute(A, B))


# ---------------------------------------------------------------- input generators
def test_inputs_are_deterministic_and_distributed():
    a1 = inp.normal(42, 1, (200, 300))
    a2 = inp.normal(42, 1, (200, 300))
    assert np.array_equal(a1, a2)
    assert abs(a1.mean()) < 0.02 and abs(a1.std() - 1.0) < 0.02
    u = inp.uniform(42, 1, (200, 300))
    assert u.min() > -1 and u.max() < 1 and abs(u.mean()) < 0.02 and abs(u.var() - 1 / 3) < 0.01
    assert not np.array_equal(inp.normal(42, 2, (4, 4)), inp.normal(42, 1, (4, 4)))
    k = inp.integers(1, 1, (1000,))
    assert k.min() == -3 and k.max() == 3


def test_storage_rounding():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 0.0, 3.0])
    b = inp.store(x, "bf16")
    back = inp.widen(b, "bf16")
    # ties go to even: 1+2^-8 -> 1, 1+3*2^-8 -> 1+2^-6
    assert list(back) == [1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -2.5, 0.0, 3.0]
    assert np.array_equal(inp.widen(inp.store(x, "f16"), "f16"), x.astype(np.float16).astype(np.float64))
    ints = inp.integers(2, 1, (50,)).astype(np.float64)
    for dt in inp.DTYPES:
        assert np.array_equal(inp.widen(inp.store(ints, dt), dt), ints)


# ----------------------------------------------------------------------------- Combine B (Eq. 4)
def test_combine_b_strassen_textbook_operands():
    """Right operands of Strassen's seven products as every textbook prints them."""
    B = inp.integers(9, 3, (6, 8))
    b11, b12, b21, b22 = B[:3, :4], B[:3, 4:], B[3:, :4], B[3:, 4:]
    want = [b11 + b22, b11, b12 - b22, b21 - b11, b22, b11 + b12, b21 + b22]
    got = oracle.combine_b(S.strassen(), B)
    assert got.shape == (7, 3, 4)
    for r in range(7):
        assert np.array_equal(got[r], want[r]), r


@pytest.mark.parametrize("name", ALL)
def test_combine_b_rebuilds_the_product(name):
    """Eq. 3-6 with Combine B taken from the oracle and the other stages written as einsums here:
    the result must be A @ B.  A wrong sign, index or transposition in combine_b breaks it."""
    s = S.by_name(name)
    M, N, K = 2 * s.m, 3 * s.n, 2 * s.k
    A = inp.integers(7, 4, (M, K))
    B = inp.integers(7, 5, (K, N))
    Ab = A.reshape(s.m, M // s.m, s.k, K // s.k)           # [i, x, l, y]
    At = np.einsum("ril,ixly->rxy", s.U.astype(np.int64), Ab)
    Bt = oracle.combine_b(s, B)                             # [r, y, z]
    H = np.einsum("rxy,ryz->rxz", At, Bt)
    Cb = np.einsum("rij,rxz->ixjz", s.W.astype(np.int64), H)
    assert np.array_equal(Cb.reshape(M, N), A @ B)


def test_combine_b_single_entry():
    """B = E_{bj} (one block set to ones): Bt[r] = V[r,b,j] * ones."""
    s = S.laderman()
    for b, j in itertools.product(range(s.k), range(s.n)):
        B = np.zeros((2 * s.k, 3 * s.n), np.int64)
        B[2 * b:2 * b + 2, 3 * j:3 * j + 3] = 1
        got = oracle.combine_b(s, B)
        for r in range(s.R):
            assert np.array_equal(got[r], int(s.V[r, b, j]) * np.ones((2, 3), np.int64))


def test_combine_b_stored_rounds_once_to_nearest_even():
    s = S.strassen()
    small = inp.integers(9, 6, (4, 4)).astype(np.float64)
    for dt in ("bf16", "f16", "f32"):  # representable sums are stored exactly
        assert np.array_equal(oracle.combine_b_stored(s, small, dt), oracle.combine_b(s, small))
    # fp16 keeps 11 significant bits: 2048 + 1 -> 2048, 2048 + 3 -> 2052 (tie to even), 2048 + 5 -> 2052
    B = np.zeros((2, 2))
    for add, want in ((1.0, 2048.0), (3.0, 2052.0), (5.0, 2052.0)):
        B[0, 0], B[1, 1] = 2048.0, add
        assert oracle.combine_b_stored(s, B, "f16")[0, 0, 0] == want      # product 1: b11 + b22
        assert oracle.combine_b_stored(s, B, "bf16")[0, 0, 0] == want
        assert oracle.combine_b_stored(s, B, "f32")[0, 0, 0] == 2048.0 + add
    B[0, 0], B[1, 1] = 2.0 ** 24, 1.0                                      # fp32 keeps 24 bits
    assert oracle.combine_b_stored(s, B, "f32")[0, 0, 0] == 2.0 ** 24
    B[0, 0], B[1, 1] = 60000.0, 60000.0                                    # beyond fp16's range
    assert np.isinf(oracle.combine_b_stored(s, B, "f16")[0, 0, 0])


# ----------------------------------------------------------------------------- unfused dataflows (Algorithm 1; Algorithm 2 as printed)
def test_combine_a_strassen_textbook_operands_and_rounding():
    """Left operands of Strassen's seven products as every textbook prints them; sums that fp16 cannot
    hold are rounded once to nearest-even."""
    s = S.strassen()
    A = inp.integers(9, 7, (6, 4)).astype(np.float64)
    a11, a12, a21, a22 = A[:3, :2], A[:3, 2:], A[3:, :2], A[3:, 2:]
    want = [a11 + a22, a21 + a22, a11, a22, a11 + a12, a21 - a11, a12 - a22]
    for dt in ("bf16", "f16", "f32"):
        got = oracle.combine_a_stored(s, A, dt)
        assert got.shape == (7, 3, 2)
        for r in range(7):
            assert np.array_equal(got[r], want[r]), (dt, r)
    A = np.zeros((2, 2))
    for add, want16 in ((1.0, 2048.0), (3.0, 2052.0), (5.0, 2052.0)):
        A[0, 0], A[1, 1] = 2048.0, add
        assert oracle.combine_a_stored(s, A, "f16")[0, 0, 0] == want16   # product 1: a11 + a22
        assert oracle.combine_a_stored(s, A, "bf16")[0, 0, 0] == want16
        assert oracle.combine_a_stored(s, A, "f32")[0, 0, 0] == 2048.0 + add


@pytest.mark.parametrize("name", ALL)
def test_combine_a_rebuilds_the_product(name):
    """Eq. 3-6 with Combine A taken from the oracle and the other stages written as einsums here."""
    s = S.by_name(name)
    M, N, K = 2 * s.m, 3 * s.n, 2 * s.k
    A = inp.integers(17, 4, (M, K))
    B = inp.integers(17, 5, (K, N))
    At = oracle.combine_a_stored(s, A.astype(np.float64), "f32")           # [r, x, y], exact on small integers
    Bb = B.reshape(s.k, K // s.k, s.n, N // s.n)                            # [l, y, j, z]
    Bt = np.einsum("rlj,lyjz->ryz", s.V.astype(np.int64), Bb)
    H = np.einsum("rxy,ryz->rxz", At, Bt.astype(np.float64))
    Cb = np.einsum("rij,rxz->ixjz", s.W.astype(np.float64), H)
    assert np.array_equal(Cb.reshape(M, N), (A @ B).astype(np.float64))


@pytest.mark.parametrize("name", ALL)
@pytest.mark.parametrize("level", [1, 2])
def test_unfused_is_exact_on_small_integers(name, level):
    s = S.by_name(name)
    M, N, K = 3 * s.m, 2 * s.n, 4 * s.k
    A, B = inp.integers(21, 1, (M, K)), inp.integers(21, 2, (K, N))
    for dt in ("bf16", "f16", "f32"):
        got = oracle.lcma_unfused(s, A.astype(np.float64), B.astype(np.float64), dt, level)
        assert np.array_equal(got, (A @ B).astype(np.float64)), (dt, level)


def test_unfused_rounding_points():
    """One-element blocks, Strassen, values worked out by hand: the stored left operand of product 1,
    fp16(2048 + 1) = 2048, changes C11 and C22 at both levels; a product that fp16 cannot hold changes
    C11 at level 1 only."""
    s = S.strassen()
    A = np.array([[2048.0, 0.0], [0.0, 1.0]])
    B = np.eye(2)
    # stored operands: At1 = fp16(a11 + a22) = 2048 (not 2049), Bt1 = b11 + b22 = 2
    # M1 = 4096, M2 = (a21 + a22) b11 = 1, M3 = a11 (b12 - b22) = -2048, M4 = a22 (b21 - b11) = -1,
    # M5 = (a11 + a12) b22 = 2048, M6 = (a21 - a11)(b11 + b12) = -2048, M7 = (a12 - a22)(b21 + b22) = -1
    # C11 = M1 + M4 - M5 + M7 = 4096 - 1 - 2048 - 1 = 2046 (exact: 2048): the rounding of At1 shows
    # C22 = M1 - M2 + M3 + M6 = 4096 - 1 - 2048 - 2048 = -1 (exact: 1)
    for level in (1, 2):
        got = oracle.lcma_unfused(s, A, B, "f16", level)
        assert np.array_equal(got, np.array([[2046.0, 0.0], [0.0, -1.0]])), level
        assert np.array_equal(oracle.lcma_unfused(s, A, B, "f32", level), A)
    # level 1 also rounds the stored products: a11 = b11 = 45.25 (exact in fp16), everything else 0:
    # M1 = M3' ... only products with a11 and b11: M1 = a11 b11, M3 = a11 (0 - 0) = 0, M5 = a11 * 0 = 0,
    # M6 = -a11 b11.  a11 b11 = 2047.5625 -> fp16 2048 (spacing 1 in [1024, 2048], tie-free).
    A = np.array([[45.25, 0.0], [0.0, 0.0]])
    B = np.array([[45.25, 0.0], [0.0, 0.0]])
    exact = 45.25 * 45.25
    assert exact == 2047.5625
    got1 = oracle.lcma_unfused(s, A, B, "f16", 1)
    got2 = oracle.lcma_unfused(s, A, B, "f16", 2)
    assert got1[0, 0] == 2048.0 and got2[0, 0] == exact       # C11 = M1 + M4 - M5 + M7 = M1
    assert got1[1, 1] == 0.0 and got2[1, 1] == 0.0            # C22 = M1 - M2 + M3 + M6 = M1 - M1


# ---------------------------------------------------------------- the parity metric itself
def test_rel_frobenius_hand_values():
    """||C - Cref||_F / ||Cref||_F on cases worked by hand: each fails for a dropped square root, a swapped
    numerator and denominator, a max-norm or a 1-norm in place of the Frobenius norm, or a missing square."""
    import math
    # zero reference: the metric is the absolute norm; sqrt(3^2 + 4^2) = 5 (9 + 16 = 25 without the root, 7 as a 1-norm)
    assert oracle.rel_frobenius(np.array([[3.0, 0.0], [0.0, 4.0]]), np.zeros((2, 2))) == 5.0
    # difference (1, 1, 0, 0), reference (1, 2, 2, 4): sqrt(2) / 5, irrational only through the square root
    ref = np.array([[1.0, 2.0], [2.0, 4.0]])
    got = ref + np.array([[1.0, 1.0], [0.0, 0.0]])
    assert oracle.rel_frobenius(got, ref) == pytest.approx(math.sqrt(2.0) / 5.0, rel=1e-15)
    assert oracle.rel_frobenius(got, ref) != pytest.approx(2.0 / 25.0, rel=1e-3)       # no roots
    assert oracle.rel_frobenius(got, ref) != pytest.approx(1.0 / 4.0, rel=1e-3)        # max norms
    assert oracle.rel_frobenius(got, ref) != pytest.approx(2.0 / 9.0, rel=1e-3)        # 1-norms
    # not symmetric: the reference is the second argument (swapped: sqrt(2) / sqrt(4 + 9 + 4 + 16))
    assert oracle.rel_frobenius(ref, got) == pytest.approx(math.sqrt(2.0 / 33.0), rel=1e-15)
    # identical matrices: exactly zero; scaling both leaves the ratio unchanged; a uniform relative error eps gives eps
    assert oracle.rel_frobenius(ref, ref) == 0.0
    assert oracle.rel_frobenius(1024.0 * got, 1024.0 * ref) == pytest.approx(math.sqrt(2.0) / 5.0, rel=1e-15)
    assert oracle.rel_frobenius(ref * (1.0 + 2.0 ** -10), ref) == pytest.approx(2.0 ** -10, rel=1e-12)
    # one wrong element among many: |d| / ||ref||_F, the whole matrix counts (a mean instead of a sum would divide by 10^4)
    big = np.ones((100, 100))
    bad = big.copy()
    bad[17, 3] = 3.0
    assert oracle.rel_frobenius(bad, big) == pytest.approx(2.0 / 100.0, rel=1e-15)
    # narrower storage types are widened, not compared in their own precision
    assert oracle.rel_frobenius(np.array([[1.0]], np.float32), np.array([[1.0 + 2.0 ** -30]])) == pytest.approx(2.0 ** -30, rel=1e-6)
