"""Host-side logic of liblcma.so, no GPU needed: exported symbols, scheme store and Brent
verifier (against the oracle's independent tables), Table 2 / Eq. 8-10 closed forms, the
Split-Group worked example, selector sanity."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from oracle import schemes as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2605_06057_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_06057_amd import build
        build.build()
    binding.lib()
    return binding


def test_every_declared_symbol_is_exported(B):
    header = open(os.path.join(ROOT, "include", "lcma.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(lcma_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib(), name), name


@pytest.mark.parametrize("name", ["strassen", "strassen2", "laderman", "strassen_wide"])
def test_builtin_schemes_equal_the_oracles(B, name):
    s = B.lcma_scheme_load("builtin:" + name)
    assert B.lcma_scheme_verify(s) == -1
    U, V, W = B.lcma_scheme_coeffs(s)
    ref = S.by_name(name)
    assert np.array_equal(U, ref.U) and np.array_equal(V, ref.V) and np.array_equal(W, ref.W)
    info = B.lcma_scheme_info(s)
    assert (info["m"], info["k"], info["n"], info["R"]) == (ref.m, ref.k, ref.n, ref.R)
    assert (info["nnzU"], info["nnzV"], info["nnzW"]) == ref.nnz()


def test_paper_facts_from_the_library(B, golden):
    g = golden("paper_facts.txt")
    info = B.lcma_scheme_info(B.lcma_scheme_load("builtin:strassen"))
    assert info["R"] == int(g["strassen_rank"][0]) and info["nnzU"] == int(g["strassen_nnzU"][0])
    assert info["nnzU"] - info["R"] == int(g["strassen_addsA"][0])
    _, _, W = B.lcma_scheme_coeffs(B.lcma_scheme_load("builtin:strassen"))
    assert [r + 1 for r in range(7) if W[r, 0, 0]] == [int(x) for x in g["strassen_c11_products"]]
    assert B.lcma_scheme_info(B.lcma_scheme_load("builtin:laderman"))["R"] == int(g["laderman_rank"][0])
    assert B.lcma_scheme_info(B.lcma_scheme_load("builtin:strassen2"))["R"] == int(g["strassen2_rank"][0])


def test_file_schemes_and_verifier_verdicts(B, tmp_path):
    good = tmp_path / "classical.txt"
    good.write_text("# classical 2x3x2\n" + S.to_text(S.classical(2, 3, 2)))
    s = B.lcma_scheme_load(str(good))
    assert B.lcma_scheme_verify(s) == -1
    assert B.lcma_scheme_info(s)["R"] == 12
    base = S.laderman()
    for which, pos in [("U", (3, 1, 0)), ("V", (10, 2, 2)), ("W", (5, 0, 0))]:
        T = {"U": base.U.copy(), "V": base.V.copy(), "W": base.W.copy()}
        T[which][pos] = 0 if T[which][pos] else 1
        bad = S.Scheme(3, 3, 3, 23, T["U"], T["V"], T["W"])
        path = tmp_path / f"bad_{which}.txt"
        path.write_text(S.to_text(bad))
        with pytest.raises(B.LcmaError) as e:
            B.lcma_scheme_verify(B.lcma_scheme_load(str(path)))
        assert e.value.status == B.LCMA_ERR_BRENT
        assert e.value.first_bad == oracle.brent(bad)[1]  # same first violated equation as the oracle finds
    # a file with a built-in's coefficients is recognised as that built-in (kernels exist for it)
    same = tmp_path / "strassen_copy.txt"
    same.write_text(S.to_text(S.strassen()))
    assert B.lcma_scheme_verify(B.lcma_scheme_load(str(same))) == -1


def test_loader_error_paths(B, tmp_path):
    for text, status in [("2 2 2\n", B.LCMA_ERR_PARSE), ("2 2 2 7\n1 0 0 1\n", B.LCMA_ERR_PARSE),
                         ("2 2 2 1\n1 0 0 x\n", B.LCMA_ERR_PARSE), ("1 1 1 1\n300\n1\n1\n", B.LCMA_ERR_PARSE),
                         ("0 1 1 1\n1\n1\n1\n", B.LCMA_ERR_PARSE)]:
        p = tmp_path / "t.txt"
        p.write_text(text)
        with pytest.raises(B.LcmaError) as e:
            B.lcma_scheme_load(str(p))
        assert e.value.status == status, text
    with pytest.raises(B.LcmaError) as e:
        B.lcma_scheme_load(str(tmp_path / "missing.txt"))
    assert e.value.status == B.LCMA_ERR_IO
    with pytest.raises(B.LcmaError) as e:
        B.lcma_scheme_load("builtin:nonesuch")
    assert e.value.status == B.LCMA_ERR_IO
    assert B.lib().lcma_status_str(B.LCMA_ERR_BRENT).decode().startswith("scheme violates")


def test_split_group_worked_example(B, golden):
    g = {k: v[0] for k, v in golden("split_group_example.txt").items()}
    tile, R, units = int(g["tile"]), int(g["R"]), int(g["units"])
    groups = (int(g["M"]) // 2 // tile) * (int(g["N"]) // 2 // tile)
    assert groups == int(g["groups"]) and groups * R == int(g["h_tiles"])
    tile_level, group_level = B.lcma_sched_waves(groups, R, units)
    assert tile_level == int(g["waves_tile_level"]) and group_level == int(g["waves_group_level"])
    assert round(100.0 * (group_level - tile_level) / tile_level, 1) == float(g["waste_percent"])
    # Split-Group ranges: contiguous, cover every tile-product once, capacity ceil(total/units)
    cap = -(-groups * R // units)
    prev_end = 0
    for u in range(units):
        b, e = B.lcma_sched_range(groups, R, units, u)
        assert b == prev_end and 0 <= e - b <= cap
        prev_end = e
    assert prev_end == groups * R
    straddle = [sum(1 for u in range(units) if (lambda be: be[0] < (gi + 1) * R and be[1] > gi * R)(B.lcma_sched_range(groups, R, units, u)))
                for gi in range(groups)]
    assert max(straddle) <= 2  # a group is split across at most two units


def test_table2_and_intensity_closed_forms(B):
    M, N, K = 4096, 2048, 1024
    s = B.lcma_scheme_load("builtin:strassen")
    hw = B.lcma_hw()
    hw.flops_mul, hw.flops_add, hw.beta = 148e12, 20e12, 2e12  # H20 bf16 figures of the roofline section: 4 TB/s = 2e12 elements/s
    c = B.lcma_model_stages(s, M, N, K, hw)
    # Table 2 with ||U||0 = ||V||0 = ||W||0 = 12, R = 7, m = k = n = 2
    assert c.flops[0] == 5 * (M / 2) * (K / 2) and c.elems[0] == M * K * (1 + 7 / 4)
    assert c.flops[1] == 5 * (N / 2) * (K / 2) and c.elems[1] == N * K * (1 + 7 / 4)
    assert c.flops[2] == 2 * 7 * M * N * K / 8 and c.elems[2] == 7 * (M * K / 4 + N * K / 4 + M * N / 4)
    assert c.flops[3] == (12 - 4) * (M / 2) * (N / 2) and c.elems[3] == M * N * (1 + 7 / 4)
    for i in range(4):
        rate = hw.flops_mul if i == 2 else hw.flops_add
        assert c.seconds[i] == max(c.flops[i] / rate, c.elems[i] / hw.beta)
    p = B.lcma_model_stages(None, M, N, K, hw)
    assert p.flops[2] == 2 * M * N * K and p.elems[2] == M * K + N * K + M * N
    eq8, eq9, eq10 = B.lcma_model_intensity(s, M, N, K)
    assert eq8 == pytest.approx(2 * M * N * K / (M * K + N * K + M * N))
    assert eq9 == pytest.approx(2 * M * N * K * (1 - 7 / 8) / (M * K * 2.75 + N * K * 2.75 + M * N * 2.75))
    assert eq10 == pytest.approx(2 * M * N * K * (1 - 7 / 8) / (M * K * 2.75 + N * K * 2.75 + M * N))
    assert eq10 > eq9  # fusing Combine H removes the R/mn term
    # Eq. 9 is the simplification of "sum of stage times < plain time" when combines are memory-bound:
    lhs = c.elems[0] / hw.beta + c.elems[1] / hw.beta + c.flops[2] / hw.flops_mul + c.elems[3] / hw.beta
    assert (lhs < p.flops[2] / hw.flops_mul) == (eq9 > hw.flops_mul / hw.beta)


def test_selector_sanity(B):
    for dt in (B.LCMA_F32, B.LCMA_BF16, B.LCMA_F16):
        assert B.lcma_select(64, 64, 64, dt) == B.LCMA_PLAIN        # memory/launch bound: Eq. 8 short-circuit
        assert B.lcma_select(8, 4096, 4096, dt) == B.LCMA_PLAIN
        pick = B.lcma_select(8192, 14336, 4096, dt)
        assert pick in (B.LCMA_PLAIN, B.LCMA_STRASSEN, B.LCMA_STRASSEN2, B.LCMA_LADERMAN)
        t_pick = B.lcma_predict_seconds(pick, 8192, 14336, 4096, dt)
        for other in range(4):
            t = B.lcma_predict_seconds(other, 8192, 14336, 4096, dt)
            assert t < 0 or t_pick <= t  # the pick is the argmin of the model
    assert B.lcma_select(0, 1, 1, B.LCMA_F32) < 0 and B.lcma_select(1, 1, 1, 9) < 0
    hw = B.lcma_hw_mi355x(B.LCMA_BF16)
    assert hw.flops_mul == pytest.approx(2516.6e12) and hw.beta == pytest.approx(4e12)
    assert B.lcma_hw_mi355x(B.LCMA_F32).flops_mul == pytest.approx(157.3e12)


def test_further_scheme_files_get_ids_and_kernels(B):
    """A scheme file present at build time (here the rectangular <2,2,4;14>) is known by name, gets an
    id after the paper's three, and has kernels for every dtype; a copy of its text is recognised."""
    L = B.lib()
    assert L.lcma_scheme_name(0) == b"plain" and L.lcma_scheme_name(1) == b"strassen"
    assert L.lcma_scheme_name(3) == b"laderman" and L.lcma_scheme_name(99) is None
    ids = {L.lcma_scheme_name(i).decode(): i for i in range(L.lcma_scheme_id_max() + 1)}
    assert ids["strassen_wide"] >= 4
    vs = [v for v in B.lcma_variants() if v["scheme_id"] == ids["strassen_wide"]]
    assert {v["dtype"] for v in vs} == {B.LCMA_F32, B.LCMA_BF16, B.LCMA_F16}
    assert all(v["mult_N"] == 4 * v["TN"] and v["mult_M"] == 2 * v["TM"] for v in vs)
    assert B.SCHEME_NAMES[ids["strassen_wide"]] == "strassen_wide"
    s = B.lcma_scheme_load("builtin:strassen_wide")
    info = B.lcma_scheme_info(s)
    assert (info["m"], info["k"], info["n"], info["R"]) == (2, 2, 4, 14)


def test_variant_registry(B):
    vs = B.lcma_variants()
    names = [v["name"] for v in vs]
    assert len(set(names)) == len(names) > 0
    for v in vs:
        assert v["mult_M"] % v["TM"] == 0 and v["mult_N"] % v["TN"] == 0 and v["mult_K"] % v["TK"] == 0
    # every BASELINE configuration has a kernel: (scheme id, dtype id, M, N, K)
    for sid, dt, M, N, K in [(1, 0, 256, 256, 256), (1, 1, 4096, 4096, 4096), (1, 1, 8192, 14336, 4096),
                             (2, 1, 8192, 14336, 4096), (3, 2, 6144, 6144, 6144), (0, 1, 2048, 4096, 14336)]:
        assert any(v["scheme_id"] == sid and v["dtype"] == dt and M % v["mult_M"] == 0 and N % v["mult_N"] == 0
                   and K % v["mult_K"] == 0 for v in vs), (sid, dt, M, N, K)


def test_prepared_b_host_side(B):
    """Sizes and argument checks of the offline Combine-B entry points (nothing here launches)."""
    s = B.lcma_scheme_load("builtin:strassen")
    assert B.lcma_prepared_b_bytes(s, 4096, 4096, B.LCMA_BF16) == 7 * 2048 * 2048 * 2
    assert B.lcma_prepared_b_bytes(s, 4096, 4096, B.LCMA_F32) == 7 * 2048 * 2048 * 4
    assert B.lcma_prepared_b_bytes(s, 4095, 4096, B.LCMA_BF16) == -1
    assert B.lcma_prepared_b_bytes(s, 4096, 0, B.LCMA_BF16) == -1
    assert B.lcma_prepared_b_bytes(s, 4096, 4096, 17) == -1
    L = B.lib()
    # null pointers, a missing scheme and an unknown dtype are refused before anything is launched
    assert L.lcma_prepare_b(256, 256, None, 256, B.LCMA_F16, s.handle, None, None) == B.LCMA_ERR_ARG
    assert L.lcma_prepare_b(256, 256, None, 256, B.LCMA_F16, None, None, None) == B.LCMA_ERR_ARG
    assert L.lcma_prepare_b(256, 256, None, 256, 17, s.handle, None, None) == B.LCMA_ERR_DTYPE
    assert L.lcma_prepare_bt(256, 256, None, 256, B.LCMA_F16, s.handle, None, None) == B.LCMA_ERR_ARG
    assert L.lcma_prepare_bt(256, 512, 0x1000, 256, B.LCMA_F16, s.handle, 0x2000, None) == B.LCMA_ERR_ARG  # ldw < K
    # the rows of the planes are the y dimension of the Combine kernels' grids (at most 65535 work-groups of 16 rows of W,
    # or of 64 columns of B): taller matrices are refused, however short their rows
    P = 0x100000
    assert L.lcma_prepare_bt(2 * 16 * 65536 + 128, 64, P, 64, B.LCMA_F16, s.handle, P, None) == B.LCMA_ERR_SHAPE
    assert b"N is too large" in L.lcma_last_error()
    assert L.lcma_prepare_b(2 * 64 * 65536 + 128, 64, P, 2 * 64 * 65536 + 128, B.LCMA_F16, s.handle, P, None) == B.LCMA_ERR_SHAPE
    assert b"N is too large" in L.lcma_last_error()
    assert L.lcma_gemm_prepared(256, 256, 256, None, 256, None, None, 256, B.LCMA_F16, None, None) == B.LCMA_ERR_ARG
    assert L.lcma_gemm_prepared(256, 256, 256, None, 256, None, None, 256, B.LCMA_F16, s.handle, None) == B.LCMA_ERR_ARG
    assert b"null" in L.lcma_last_error()
    vs = B.lcma_variants()
    assert any(v["prepared"] for v in vs) and any(not v["prepared"] for v in vs)
    assert B.lib().lcma_variant_prepared(len(vs)) == -1


def test_gemm_argument_checks_before_any_launch(B):
    """Every refusal below is decided on the host from sizes, strides and pointer values alone:
    the fake (never dereferenced) pointers prove that nothing is launched or read."""
    L = B.lib()
    s = B.lcma_scheme_load("builtin:strassen")
    P = 0x100000  # 16-byte aligned, not a real allocation
    ok_shape = (256, 256, 256)

    def gemm(M, N, K, a=P, lda=None, b=P, ldb=None, c=P, ldc=None, dt=B.LCMA_F16, sch=s.handle):
        return L.lcma_gemm(M, N, K, a, K if lda is None else lda, b, N if ldb is None else ldb,
                           c, N if ldc is None else ldc, dt, sch, None)

    assert gemm(*ok_shape, a=None) == B.LCMA_ERR_ARG                    # null matrix
    assert gemm(*ok_shape, lda=255) == B.LCMA_ERR_ARG                   # leading dimension below the row
    assert gemm(*ok_shape, a=P + 2) == B.LCMA_ERR_ARG                   # pointer not 16-byte aligned
    assert gemm(*ok_shape, ldc=260) == B.LCMA_ERR_ARG                   # ldc * 2 bytes not a multiple of 16
    assert gemm(-1, 256, 256) == B.LCMA_ERR_ARG
    assert gemm(256, 256, 0, c=None) == B.LCMA_ERR_ARG                  # K = 0 writes zeros: C is needed
    assert gemm(256, 256, 0, ldc=255) == B.LCMA_ERR_ARG
    assert gemm(256, 256, 252, lda=256) == B.LCMA_ERR_SHAPE             # K = 252: rows of A not 16-byte granular
    assert gemm(256, 250, 256) == B.LCMA_ERR_SHAPE                      # N = 250: rows not 16-byte granular
    assert gemm(*ok_shape, dt=9) == B.LCMA_ERR_DTYPE
    assert gemm(0, 256, 256, a=None, b=None, c=None) == B.LCMA_OK       # M = 0: nothing to do
    # a matrix whose rows span 2 GiB or more: 256 rows with a leading dimension of 2^23 fp16 elements
    assert gemm(*ok_shape, lda=1 << 23) == B.LCMA_ERR_SHAPE
    assert b"2 GiB" in L.lcma_last_error()
    assert gemm(*ok_shape, ldc=1 << 23) == B.LCMA_ERR_SHAPE
    # the largest accepted extent is just below 2 GiB
    lda_max = ((1 << 31) // 2 - 256) // 255 // 8 * 8
    assert (255 * lda_max + 256) * 2 < (1 << 31)
    assert gemm(*ok_shape, c=P + 256 * 256 * 2 - 16) == B.LCMA_ERR_ARG    # C overlaps the end of A (and of B)
    assert b"overlaps" in L.lcma_last_error()
    # (accepted arguments would launch: not tried here without a GPU)
    # two-level Strassen has no fp16 kernel
    s2 = B.lcma_scheme_load("builtin:strassen2")
    assert gemm(*ok_shape, sch=s2.handle) == B.LCMA_ERR_NOKERNEL
    # lcma_gemm_variant: unknown name, null name
    assert L.lcma_gemm_variant(b"no_such_kernel", 256, 256, 256, P, 256, P, 256, P, 256, None) == B.LCMA_ERR_NOKERNEL
    assert L.lcma_gemm_variant(None, 256, 256, 256, P, 256, P, 256, P, 256, None) == B.LCMA_ERR_ARG


def test_weight_layout_and_unfused_host_side(B):
    """lcma_gemm_nt and lcma_gemm_unfused: sizes and refusals decided on the host (fake pointers, nothing launched)."""
    L = B.lib()
    s = B.lcma_scheme_load("builtin:strassen")
    P = 0x100000
    # N x K layout: the leading dimension of W is checked against K, not N
    assert L.lcma_gemm_nt(256, 512, 128, P, 128, P, 120, P, 512, B.LCMA_F16, s.handle, None) == B.LCMA_ERR_ARG
    assert L.lcma_gemm_nt(256, 512, 128, None, 128, P, 128, P, 512, B.LCMA_F16, s.handle, None) == B.LCMA_ERR_ARG
    assert L.lcma_gemm_nt(256, 512, 128, P, 128, P, 128, P, 512, 17, s.handle, None) == B.LCMA_ERR_DTYPE
    wide = B.lcma_scheme_load("builtin:strassen_wide")
    assert L.lcma_gemm_nt(256, 512, 128, P, 128, P, 128, P, 512, B.LCMA_F16, wide.handle, None) == B.LCMA_ERR_NOKERNEL
    layouts = [v["b_layout"] for v in B.lcma_variants()]
    assert set(layouts) == {0, 1, 2, 3} and L.lcma_variant_b_layout(len(layouts)) == -1
    # every selectable kernel of the paper's schemes that takes B has a twin for the N x K layout
    names = {v["name"] for v in B.lcma_variants()}
    for v in B.lcma_variants():
        if v["b_layout"] == 2 and not v["name"].endswith("dt"):   # the direct-load kernels exist for this layout only
            base = v["name"].replace("to2", "o2") if v["name"].endswith("to2") else v["name"][:-1]
            assert base in names, v["name"]
    # workspace of the unfused dataflows: At, Bt and H planes, blocks padded to 128 rows and 64 (fp32: 16) columns
    assert B.lcma_unfused_workspace_bytes(s, 4096, 4096, 4096, B.LCMA_BF16) == 3 * 7 * 2048 * 2048 * 2
    assert B.lcma_unfused_workspace_bytes(s, 100, 200, 72, B.LCMA_F32) == 7 * (128 * 48 + 128 * 48 + 128 * 128) * 4
    lad = B.lcma_scheme_load("builtin:laderman")
    # fp16 storage: planes of At and Bt in fp16, the products in fp32; 25 planes (two compensated products)
    assert B.lcma_unfused_workspace_bytes(lad, 384, 384, 192, B.LCMA_F16) == 25 * (128 * 64 * 2 * 2 + 128 * 128 * 4)
    assert B.lcma_unfused_workspace_bytes(lad, 384, 384, 192, B.LCMA_BF16) == 23 * (128 * 64 * 2 + 128 * 128) * 2
    assert B.lcma_unfused_workspace_bytes(s, 4096, 4096, 4096, 17) == -1

    def unfused(level=1, M=256, N=256, K=256, a=P, ws=P, nbytes=1 << 30, dt=B.LCMA_F16, sch=s.handle, lda=None):
        return L.lcma_gemm_unfused(level, M, N, K, a, K if lda is None else lda, P, N, P, N, dt, sch, ws, nbytes, 0, None)

    assert unfused(level=0) == B.LCMA_ERR_ARG and unfused(level=3) == B.LCMA_ERR_ARG
    assert unfused(sch=None) == B.LCMA_ERR_ARG
    assert unfused(sch=wide.handle) == B.LCMA_ERR_NOKERNEL
    assert unfused(dt=17) == B.LCMA_ERR_DTYPE
    assert unfused(a=None) == B.LCMA_ERR_ARG and unfused(ws=None) == B.LCMA_ERR_ARG
    assert unfused(ws=P + 16) == B.LCMA_ERR_ARG                 # the workspace must be 256-byte aligned
    assert unfused(nbytes=3 * 7 * 128 * 128 * 2 - 1) == B.LCMA_ERR_ARG
    assert b"needed" in L.lcma_last_error()
    assert unfused(K=252, lda=256) == B.LCMA_ERR_SHAPE
    # more than 65535 x 16 rows per block of A: the rows are the y dimension of Combine A's grid
    assert unfused(M=2 * 16 * 65536 + 256, N=256, K=64, nbytes=1 << 40, dt=B.LCMA_BF16) == B.LCMA_ERR_SHAPE
    assert b"M is too large" in L.lcma_last_error()
    assert L.lcma_gemm_unfused(1, 256, 256, 0, P, 0, P, 256, None, 256, B.LCMA_F16, s.handle, P, 1 << 30, 0, None) == B.LCMA_ERR_ARG  # K = 0 writes zeros: C is needed
    assert unfused(M=0) == B.LCMA_OK                            # nothing to write

    # lcma_gemm_ws: layout argument, refusals of the call it routes to, nothing to do
    import ctypes
    flow = ctypes.c_int(7)

    def ws_call(layout=0, M=256, N=256, K=256, a=P, ldb=256, sch=s.handle, ws=P, nbytes=1 << 30, dt=B.LCMA_F16):
        return L.lcma_gemm_ws(layout, M, N, K, a, K, P, ldb, P, N, dt, sch, ws, nbytes, ctypes.byref(flow), None)
    assert ws_call(layout=1) == B.LCMA_ERR_ARG and b"b_layout" in L.lcma_last_error() and flow.value == 0
    assert ws_call(layout=3) == B.LCMA_ERR_ARG
    assert ws_call(a=None) == B.LCMA_ERR_ARG and ws_call(layout=2, a=None) == B.LCMA_ERR_ARG
    assert ws_call(dt=17) == B.LCMA_ERR_DTYPE
    assert ws_call(layout=2, N=512, K=128, ldb=120) == B.LCMA_ERR_ARG      # W is N x K: its pitch is checked against K
    assert ws_call(M=0) == B.LCMA_OK and ws_call(layout=2, M=0, sch=None, ws=None, nbytes=0) == B.LCMA_OK
    # <3,3,3;23> with fp16 storage works on 25 planes (two compensated products), with bf16 storage on 23
    assert B.lcma_unfused_workspace_bytes(lad, 768, 768, 768, B.LCMA_F16) == 25 * 256 * 256 * (2 + 2 + 4)
    assert B.lcma_unfused_workspace_bytes(lad, 768, 768, 768, B.LCMA_BF16) == 23 * 256 * 256 * (2 + 2 + 2)


def test_selector_over_both_dataflows(B):
    """lcma_select_dataflow and the Algorithm 1 cost model: pure host arithmetic."""
    bf16, f32 = B.LCMA_BF16, B.LCMA_F32
    # large LLM shapes, 16-bit: the plain GEMM; fp32: the fused Strassen kernel
    assert B.lcma_select_dataflow(8192, 14336, 4096, bf16, True) == {"scheme_id": 0, "dataflow": 0,
                                                                    "seconds": B.lcma_predict_seconds(0, 8192, 14336, 4096, bf16)}
    c = B.lcma_select_dataflow(4096, 4096, 4096, f32)
    assert (c["scheme_id"], c["dataflow"]) == (B.LCMA_STRASSEN, 0)
    # few rows, long K, static weights: the plain kernel has half a round of tiles, Algorithm 1 seven times as many jobs
    c = B.lcma_select_dataflow(2048, 4096, 14336, bf16, True)
    assert (c["scheme_id"], c["dataflow"]) == (B.LCMA_STRASSEN, 1)
    assert c["seconds"] == B.lcma_predict_unfused_seconds(B.LCMA_STRASSEN, 2048, 4096, 14336, bf16, True)
    # Combine B per call costs what its bytes cost
    on = B.lcma_predict_unfused_seconds(1, 8192, 14336, 4096, bf16, False)
    off = B.lcma_predict_unfused_seconds(1, 8192, 14336, 4096, bf16, True)
    assert abs((on - off) - ((4096 * 14336 + 7 * 7168 * 2048) * 2 / 4.5e12 + 2e-6)) < 1e-9
    # the stage sum: Combine A + batched GEMM + Combine H, three launches
    g = 13 * (32 + 3.5) * 1.62e-6   # 3136 tiles of 256 x 256 on 256 CUs: 13 rounds of 32 steps of 128 bytes, 3.5 more per tile
    want = (8192 * 4096 + 7 * 4096 * 2048) * 2 / 5.6e12 + g + (7 * 4096 * 7168 + 8192 * 14336) * 2 / 5.2e12 + 3 * 2e-6
    assert abs(off - want) < 1e-9 * want + 1e-12
    # no stage kernels: plain, further schemes, unknown ids
    ids = {n: i for i, n in B.SCHEME_NAMES.items()}
    for sid in (0, ids["strassen_wide"], 99):
        assert B.lcma_predict_unfused_seconds(sid, 4096, 4096, 4096, bf16) < 0
    assert B.lcma_predict_unfused_seconds(1, 0, 4096, 4096, bf16) < 0
    L = B.lib()
    assert L.lcma_select_dataflow(4096, 4096, 4096, 17, 0, None) == B.LCMA_ERR_ARG
    import ctypes
    out = B.lcma_choice()
    assert L.lcma_select_dataflow(4096, 4096, 4096, 17, 0, ctypes.byref(out)) == B.LCMA_ERR_DTYPE
    assert L.lcma_select_dataflow(0, 4096, 4096, bf16, 0, ctypes.byref(out)) == B.LCMA_ERR_ARG


def test_mfma_probe_argument_checks(B):
    """The matrix-pipe probe refuses bad arguments before it launches anything, and reports the flops of a launch."""
    import ctypes
    L = B.lib()
    P = 0x100000
    flops = ctypes.c_double(-1.0)
    assert L.lcma_mfma_probe(None, P, 10, ctypes.byref(flops), None) == B.LCMA_ERR_ARG
    assert L.lcma_mfma_probe(P, None, 10, ctypes.byref(flops), None) == B.LCMA_ERR_ARG
    assert L.lcma_mfma_probe(P + 8, P, 10, ctypes.byref(flops), None) == B.LCMA_ERR_ARG
    assert L.lcma_mfma_probe(P, P, 0, ctypes.byref(flops), None) == B.LCMA_ERR_ARG
    assert L.lcma_mfma_probe(P, P, 10 ** 7 + 1, ctypes.byref(flops), None) == B.LCMA_ERR_ARG
    assert flops.value == -1.0


def test_wide_buffer_stores_have_a_literal_zero_scalar_offset():
    """A buffer store of more than 8 bytes whose scalar-offset operand is a register was seen to have its data
    registers overwritten by the next vector instruction (the compiler keeps the distance only without a scalar
    offset); every such store in the kernels therefore passes a literal 0 there.  This keeps it that way."""
    import glob
    import re
    csrc = os.path.join(ROOT, "paper_2605_06057_amd", "csrc")
    calls = 0
    for path in glob.glob(os.path.join(csrc, "*.hpp")) + glob.glob(os.path.join(csrc, "*.hip")):
        text = open(path).read()
        for m in re.finditer(r"raw_buffer_store_b128\((.*?)\);", text, re.S):
            args = [a.strip() for a in m.group(1).rsplit(",", 2)]
            # (..., scalar offset, cache policy): the policy may be the non-temporal one of H_r and C
            assert args[-2] == "0" and args[-1] in ("0", "kStreamed"), f"{os.path.basename(path)}: {m.group(0)}"
            calls += 1
    assert calls >= 5
