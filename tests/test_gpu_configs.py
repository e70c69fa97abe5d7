"""The BASELINE configurations at full size, through lcma_gemm's default kernel choice (the launch
configuration bench.py times), checked on sampled rows of C that the oracle computes one by one:
a few rows inside every block row of the scheme grid, all N columns, so every C block, every tile
column and every y step takes part."""
import numpy as np
import pytest

import lcma_inputs as inp
import oracle

pytestmark = pytest.mark.gpu

CONFIGS = [
    # id, scheme, dtype, M, N, K, A kind, B kind, seed, relF bound
    ("c1_strassen_f32_256", "strassen", "f32", 256, 256, 256, "uniform", "uniform", 0x5EED0001, 1e-5),
    ("c2_strassen_bf16_4096", "strassen", "bf16", 4096, 4096, 4096, "normal", "normal", 0x5EED0002, 2e-2),
    ("c3_strassen_bf16_ffn", "strassen", "bf16", 8192, 14336, 4096, "normal", "weights", 0x5EED0003, 2e-2),
    ("c3_strassen2_bf16_ffn", "strassen2", "bf16", 8192, 14336, 4096, "normal", "weights", 0x5EED0003, 2e-2),
    ("c4_laderman_f16_6144", "laderman", "f16", 6144, 6144, 6144, "uniform", "uniform", 0x5EED0004, 2e-2),
    ("c5_plain_bf16_2048x4096x14336", None, "bf16", 2048, 4096, 14336, "normal", "weights", 0x5EED0005, 2e-2),
    # close to the largest C the 32-bit offsets allow (0.98 GB, padded 0.99 GB), ragged in all three directions
    ("big_ragged_strassen_bf16", "strassen", "bf16", 30001, 16376, 2056, "normal", "weights", 0x5EED0006, 2e-2),
    ("big_ragged_strassen_f32", "strassen", "f32", 15001, 16380, 1028, "uniform", "uniform", 0x5EED0007, 1e-5),
]


@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c[0])
def test_full_size_config_on_sampled_rows(cfg):
    import torch
    import gpu_util as G
    from paper_2605_06057_amd import binding as B
    name, scheme, dt, M, N, K, ka, kb, seed, bound = cfg
    print(f"config {name}: generating inputs", flush=True)
    As, Bs = inp.matrices(ka, kb, M, N, K, dt, seed)
    a, b = G.to_device(As, dt), G.to_device(Bs, dt)
    c = G.empty_like_c(M, N, dt, fill=float("nan"))
    cp = G.empty_like_c(M, N, dt, fill=float("nan"))
    s = B.lcma_scheme_load("builtin:" + scheme) if scheme else None
    grid_m = B.lcma_scheme_info(s)["m"] if s else 1
    print(f"config {name}: launching", flush=True)
    B.lcma_gemm(a, b, c, s)
    B.lcma_gemm(a, b, cp, None)
    torch.cuda.synchronize()
    bm = M // grid_m
    rows = np.unique(np.concatenate([(np.array([0, 1, 63, 64, 127, 128, bm // 2 + 5, bm - 1]) % bm) + i * bm
                                     for i in range(grid_m)]))
    ref = oracle.gemm_rows(inp.widen(As, dt), inp.widen(Bs, dt), rows)
    idx = torch.from_numpy(rows).cuda()
    got = G.to_host_f64(c[idx], dt)
    got_plain = G.to_host_f64(cp[idx], dt)
    assert not np.isnan(G.to_host_f64(c[:: max(1, M // 64)], dt)).any(), "part of C was never written"
    err, err_plain = oracle.rel_frobenius(got, ref), oracle.rel_frobenius(got_plain, ref)
    print(f"config {name}: relF {err:.3e} plain {err_plain:.3e} ratio {err / err_plain:.2f}", flush=True)
    assert err <= bound and err_plain <= bound
    assert err <= 4.0 * err_plain
    c2 = G.empty_like_c(M, N, dt, fill=0.0)
    B.lcma_gemm(a, b, c2, s)
    assert torch.equal(c2.view(torch.uint8), c.view(torch.uint8)), "two runs differ"


def test_selector_sweep_runs_its_pick():
    """Shape sweep of the Decision Module (bf16): whatever lcma_select picks must run and be right."""
    import torch
    import gpu_util as G
    from paper_2605_06057_amd import binding as B
    dt = "bf16"
    for M in (2048, 8192):
        for N, K in ((4096, 4096), (4096, 14336)):
            pick = B.lcma_select(M, N, K, B.LCMA_BF16)
            assert pick in (0, 1, 2, 3)
            As, Bs = inp.matrices("normal", "weights", M, N, K, dt, 0x5EED0100 + M + N)
            a, b = G.to_device(As, dt), G.to_device(Bs, dt)
            c = G.empty_like_c(M, N, dt, fill=float("nan"))
            s = B.lcma_scheme_load("builtin:" + B.SCHEME_NAMES[pick]) if pick else None
            B.lcma_gemm(a, b, c, s)
            rows = np.array([0, M // 3, M - 1])
            ref = oracle.gemm_rows(inp.widen(As, dt), inp.widen(Bs, dt), rows)
            err = oracle.rel_frobenius(G.to_host_f64(c[torch.from_numpy(rows).cuda()], dt), ref)
            print(f"sweep {M}x{N}x{K}: pick {B.SCHEME_NAMES[pick]} relF {err:.3e}", flush=True)
            assert err <= 2e-2


def test_selector_pick_is_close_to_the_measured_best():
    """Decision Module (Sec. 3.3) against the clock: on a few shapes, time every scheme lcma_select chooses
    among (plain and the paper's three) and require its pick to be within 15 % of the fastest (best of three timings each) (all timings
    from this one run)."""
    import torch
    from paper_2605_06057_amd import binding as B

    def seconds(fn, iters=16, warm=8, repeats=3):
        """Best of `repeats` timings of `iters` calls: a box whose clocks move between legs cannot turn the comparison."""
        for _ in range(warm):
            fn()
        best = None
        for _ in range(repeats):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) / iters * 1e-3
            best = t if best is None else min(best, t)
        return best

    schemes = {i: (B.lcma_scheme_load("builtin:" + n) if i else None) for i, n in B.SCHEME_NAMES.items() if i <= 3}
    cases = [("bf16", 4096, 4096, 4096), ("bf16", 2048, 14336, 4096), ("bf16", 1000, 4096, 4096),
             ("f16", 3072, 3072, 3072), ("f32", 4096, 4096, 4096), ("f32", 1024, 1024, 1024), ("f32", 3000, 4096, 2040)]
    heat = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
    for _ in range(300):  # settle the clocks
        torch.mm(heat, heat)
    for dt, M, N, K in cases:
        td = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dt]
        a = torch.randn(M, K, device="cuda").to(td)
        b = (torch.randn(K, N, device="cuda") * 0.05).to(td)
        c = torch.empty(M, N, device="cuda", dtype=td)
        times = {}
        for i, s in schemes.items():
            try:
                times[i] = seconds(lambda: B.lcma_gemm(a, b, c, s))
            except B.LcmaError:
                pass  # no kernel of this scheme for the dtype or shape
        pick = B.lcma_select(M, N, K, B.DTYPE_IDS[dt])
        best = min(times, key=times.get)
        tf = {B.SCHEME_NAMES[i]: round(2.0 * M * N * K / t / 1e12, 1) for i, t in times.items()}
        print(f"{dt} {M}x{N}x{K}: pick {B.SCHEME_NAMES[pick]}, measured TFLOP/s {tf}", flush=True)
        assert pick in times
        assert times[pick] <= 1.15 * times[best], (dt, M, N, K, B.SCHEME_NAMES[pick], B.SCHEME_NAMES[best])


def test_dataflow_choice_is_close_to_the_measured_best():
    """lcma_select_dataflow against the clock: plain, the fused kernels and Algorithm 1 (Combine B offline) of the
    paper's schemes, all timed in this run; the choice must be within 15 % of the fastest (best of three timings each)."""
    import torch
    from paper_2605_06057_amd import binding as B

    def seconds(fn, iters=16, warm=8, repeats=3):
        """Best of `repeats` timings of `iters` calls: a box whose clocks move between legs cannot turn the comparison."""
        for _ in range(warm):
            fn()
        best = None
        for _ in range(repeats):
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) / iters * 1e-3
            best = t if best is None else min(best, t)
        return best

    names = {0: "plain", 1: "strassen", 2: "strassen2", 3: "laderman"}
    handles = {i: (B.lcma_scheme_load("builtin:" + n) if i else None) for i, n in names.items()}
    heat = torch.randn(4096, 4096, device="cuda", dtype=torch.bfloat16)
    for _ in range(300):  # settle the clocks
        torch.mm(heat, heat)
    for dt, M, N, K in (("bf16", 2048, 4096, 14336), ("bf16", 8192, 4096, 4096), ("f16", 3072, 3072, 3072), ("f32", 2048, 2048, 2048)):
        td = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[dt]
        a = torch.randn(M, K, device="cuda").to(td)
        b = (torch.randn(K, N, device="cuda") * 0.05).to(td)
        c = torch.empty(M, N, device="cuda", dtype=td)
        times = {}
        for i, h in handles.items():
            try:
                times[(i, 0)] = seconds(lambda: B.lcma_gemm(a, b, c, h))
            except B.LcmaError:
                pass
            if i and B.lcma_predict_unfused_seconds(i, M, N, K, B.DTYPE_IDS[dt], True) > 0:
                ws = torch.empty((B.lcma_unfused_workspace_bytes(h, M, N, K, B.DTYPE_IDS[dt]),), dtype=torch.uint8, device="cuda")
                B.lcma_gemm_unfused(1, a, b, c, h, ws)
                times[(i, 1)] = seconds(lambda: B.lcma_gemm_unfused(1, a, b, c, h, ws, reuse_bt=True))
                del ws
        ch = B.lcma_select_dataflow(M, N, K, B.DTYPE_IDS[dt], True)
        pick = (ch["scheme_id"], ch["dataflow"])
        best = min(times, key=times.get)
        tf = {f"{names[i]}/{'alg1' if d else 'fused'}": round(2.0 * M * N * K / t / 1e12, 1) for (i, d), t in times.items()}
        print(f"{dt} {M}x{N}x{K}: choice {names[pick[0]]}/{'alg1' if pick[1] else 'fused'}, measured TFLOP/s {tf}", flush=True)
        assert pick in times
        assert times[pick] <= 1.15 * times[best], (dt, M, N, K, pick, best)
