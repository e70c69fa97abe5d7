#!/usr/bin/env python3
"""Benchmark of the LCMA GEMM hot path on one MI355X.

One "step" is one lcma_gemm_ws call (lcma_gemm with a workspace): the whole LCMA product over one pair of
synthetic matrices that already sit in HBM, by the dataflow the library's time model (Sec. 3.3) predicts faster
for the shape: the fused group-parallel kernel (block split, operand combinations in LDS, grouped MFMA
sub-GEMMs, W epilogue in one launch) or Algorithm 1 (Combine A, Combine B, one batched GEMM over the R
products, Combine H; every stage runs in every step).  `config.dataflow` says which ran; the fused kernel's
own rate is reported beside it (`fused_kernel_tflops`), and --fused-only makes it the headline.  The default workload is the largest LLM-shaped configuration: the FFN GEMM
M = 8192 tokens, N = 14336, K = 4096, bf16 storage with fp32 accumulation, A ~ N(0,1),
B ~ N(0, 0.02^2), Strassen <2,2,2;7> one level.  The other configurations (Strassen bf16 4096^3,
two-level Strassen on the FFN shape, Laderman fp16 6144^3, Strassen fp32 4096^3) are timed the
same way as further legs and reported in `other_workloads` of the same line.

Prints ONE JSON line.  `value` is effective TFLOP/s = 2MNK / time (standard-GEMM flop count,
paper Sec. 4.1 "Measurement"), so it can exceed what the MFMA units did.  Beside it: the same-build
plain MFMA GEMM timed the same way, the fraction of the dense MFMA peak, a roofline object
for the dominant kernel (under Algorithm 1 the batched GEMM stage, timed alone with HIP events) and the CPU oracle timed on a bounded sample of the same workload.
Further legs, each about a second, run unless --no-extras is given and are reported in objects of
their own beside `value`: the offline Combine-B path, B given as the N x K weight matrix, and the
unfused dataflows of Algorithm 1 / Algorithm 2.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3}  # MI355X dense MFMA, published

WORKLOADS = {
    # name: (scheme, dtype, M, N, K, kind of A, kind of B, seed)
    "strassen_bf16_4096": ("strassen", "bf16", 4096, 4096, 4096, "normal", "normal", 0x5EED0002),
    "strassen_f32_256": ("strassen", "f32", 256, 256, 256, "uniform", "uniform", 0x5EED0001),
    "strassen_bf16_ffn": ("strassen", "bf16", 8192, 14336, 4096, "normal", "weights", 0x5EED0003),
    "strassen2_bf16_ffn": ("strassen2", "bf16", 8192, 14336, 4096, "normal", "weights", 0x5EED0003),
    "laderman_f16_6144": ("laderman", "f16", 6144, 6144, 6144, "uniform", "uniform", 0x5EED0004),
    "strassen_f32_4096": ("strassen", "f32", 4096, 4096, 4096, "uniform", "uniform", 0x5EED0005),
    "strassen2_f32_4096": ("strassen2", "f32", 4096, 4096, 4096, "uniform", "uniform", 0x5EED0005),
    # Winograd's form of Strassen's algorithm (generated with its common sums shared): not a BASELINE config
    "winograd_f32_4096": ("winograd", "f32", 4096, 4096, 4096, "uniform", "uniform", 0x5EED0005),
    "winograd_bf16_4096": ("winograd", "bf16", 4096, 4096, 4096, "normal", "normal", 0x5EED0002),
}


def read_traffic(workload: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        for line in f:
            tok = line.split("#", 1)[0].split()
            if len(tok) >= 2 and tok[0] == workload:
                return float(tok[1])
    return None


def selector_sweep(args):
    """The Decision Module (Sec. 3.3) against the clock on the LLM-shaped sweep."""
    import torch

    from paper_2605_06057_amd import binding as B
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU. Re-run with --gpus 1.")
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    B.lib()
    names = {0: "plain", 1: "strassen", 2: "strassen2", 3: "laderman"}
    handles = {i: (B.lcma_scheme_load("builtin:" + n) if i else None) for i, n in names.items()}
    gen = torch.Generator(device="cuda").manual_seed(0x5EED0005)

    def timed(fn, steps, warmup):
        t_heat = time.perf_counter()
        while time.perf_counter() - t_heat < args.heat_seconds:
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps * 1e-3

    rows = []
    steps, warmup = max(5, args.steps // 10), max(2, args.warmup // 4)
    for M in (2048, 8192, 16384):
        for N, K in ((4096, 4096), (14336, 4096), (4096, 14336)):
            a = torch.randn((M, K), device="cuda", generator=gen).bfloat16()
            b = (torch.randn((K, N), device="cuda", generator=gen) * 0.02).bfloat16()
            c = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
            flops = 2.0 * M * N * K
            row = {"M": M, "N": N, "K": K, "measured_tflops": {}, "predicted_tflops": {}}
            for i, n in names.items():
                row["measured_tflops"][n] = flops / timed(lambda: B.lcma_gemm(a, b, c, handles[i]), steps, warmup) / 1e12
                t = B.lcma_predict_seconds(i, M, N, K, B.LCMA_BF16)
                row["predicted_tflops"][n] = flops / t / 1e12 if t > 0 else None
            row["algorithm1_combine_b_offline_tflops"], row["algorithm1_predicted_tflops"] = {}, {}
            for i in (1, 2, 3):
                ws = torch.empty((B.lcma_unfused_workspace_bytes(handles[i], M, N, K, B.LCMA_BF16),), dtype=torch.uint8, device="cuda")
                B.lcma_gemm_unfused(1, a, b, c, handles[i], ws)
                row["algorithm1_combine_b_offline_tflops"][names[i]] = flops / timed(
                    lambda: B.lcma_gemm_unfused(1, a, b, c, handles[i], ws, reuse_bt=True), steps, warmup) / 1e12
                row["algorithm1_predicted_tflops"][names[i]] = flops / B.lcma_predict_unfused_seconds(i, M, N, K, B.LCMA_BF16, True) / 1e12
                del ws
            row["pick"] = names[B.lcma_select(M, N, K, B.LCMA_BF16)]
            row["fastest_fused"] = max(row["measured_tflops"], key=row["measured_tflops"].get)
            ch = B.lcma_select_dataflow(M, N, K, B.LCMA_BF16, True)
            row["choice"] = names[ch["scheme_id"]] + ("/algorithm1" if ch["dataflow"] else "/fused")
            every = {n + "/fused": v for n, v in row["measured_tflops"].items()}
            every.update({n + "/algorithm1": v for n, v in row["algorithm1_combine_b_offline_tflops"].items()})
            row["fastest_of_all"] = max(every, key=every.get)
            row["choice_vs_fastest"] = every[row["choice"]] / every[row["fastest_of_all"]]
            rows.append(row)
            del a, b, c
    print(json.dumps({"metric": "effective TFLOP/s (2MNK/t) per scheme on the selector's shape sweep, bf16", "unit": "TFLOP/s",
                      "n_gpus": 1, "steps": steps, "warmup": warmup, "dtype": "f16", "data": "synthetic",
                      "picks_equal_fastest": sum(r["pick"] == r["fastest_fused"] for r in rows), "shapes": len(rows),
                      "worst_choice_vs_fastest": min(r["choice_vs_fastest"] for r in rows),
                      "sweep": rows}))

def _timed(torch, step, steps, warmup, heat_seconds):
    """(wall ms per step, mean and median ms per step by events on the launch stream) after an untimed spell of load
    that settles the clocks (a cold MI355X needs some milliseconds of load to get there) and `warmup` steps."""
    t_heat = time.perf_counter()
    while time.perf_counter() - t_heat < heat_seconds:
        for i in range(10):
            step(i)
        torch.cuda.synchronize()
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        step(i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    return wall / steps * 1e3, sum(per) / steps, sorted(per)[steps // 2]


def sampled_rows(np, M, m, per_block=8):
    """`per_block` rows inside every block row of the scheme grid (first, last, tile edges and a few others)."""
    bm = M // m
    inside = np.array([0, 1, 63, 64, 127, bm // 2 + 5, bm // 3, bm - 1][:per_block]) % bm
    return np.unique(np.concatenate([inside + i * bm for i in range(m)]))


def side_workload(name, args):
    """One further configuration: lcma_gemm_ws (the dataflow the time model picks), the plain and the vendor GEMM timed the same way
    as the main workload on fewer steps, and parity with the oracle on sampled rows."""
    import numpy as np
    import torch

    import lcma_inputs as inp
    from paper_2605_06057_amd import binding as B
    scheme_name, dt, M, N, K, kind_a, kind_b, seed = WORKLOADS[name]
    As, Bs = inp.matrices(kind_a, kind_b, M, N, K, dt, seed)

    def dev(x):
        if dt == "bf16":
            return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(x).cuda()
    sets = []
    for i in range(3):
        a, b = dev(As), dev(Bs)
        sets.append((a, b, torch.empty((M, N), dtype=a.dtype, device="cuda")))
    scheme = B.lcma_scheme_load("builtin:" + scheme_name)
    info = B.lcma_scheme_info(scheme)
    steps, warmup = max(20, args.steps // 4), max(5, args.warmup // 2)
    flops = 2.0 * M * N * K
    nbytes = B.lcma_unfused_workspace_bytes(scheme, M, N, K, B.DTYPE_IDS[dt])
    ws = torch.empty((nbytes + B.lcma_split_group_scratch_bytes(),), dtype=torch.uint8, device="cuda") if nbytes > 0 and not args.fused_only else None
    ran = {"flow": 0}

    def lcma_step(i):
        ran["flow"] = B.lcma_gemm_ws(*sets[i % 3], scheme, ws)
    wall, ev, _ = _timed(torch, lcma_step, steps, warmup, args.heat_seconds)
    kernel_ms, fused_tf = ev, None
    if ran["flow"] == 1:   # the dominant kernel is the GEMM stage of Algorithm 1: timed alone
        f_wall, _, _ = _timed(torch, lambda i: B.lcma_gemm(*sets[i % 3], scheme), max(10, steps // 2), 3, args.heat_seconds)
        fused_tf = flops / (f_wall * 1e-3) / 1e12
        B.lcma_set_tuning("unfused_stages", "4")
        _, kernel_ms, _ = _timed(torch, lambda i: B.lcma_gemm_unfused(1, *sets[i % 3], scheme, ws), max(10, steps // 2), 3, args.heat_seconds)
        B.lcma_set_tuning("unfused_stages", "")
    alg1_tf = None
    if ran["flow"] == 0 and ws is not None:  # Algorithm 1 called directly, for comparison with what the library chose
        a_wall, _, _ = _timed(torch, lambda i: B.lcma_gemm_unfused(1, *sets[i % 3], scheme, ws), max(10, steps // 2), 3, args.heat_seconds)
        alg1_tf = flops / (a_wall * 1e-3) / 1e12
        alg1_c = sets[2][2].clone()
        B.lcma_gemm_unfused(1, sets[2][0], sets[2][1], alg1_c, scheme, ws)
    p_wall, _, _ = _timed(torch, lambda i: B.lcma_gemm(*sets[i % 3], None), steps, warmup, args.heat_seconds)
    v_wall, _, _ = _timed(torch, lambda i: torch.mm(sets[i % 3][0], sets[i % 3][1], out=sets[i % 3][2]), max(10, steps // 2), 3, args.heat_seconds)
    peak = PEAK_TFLOPS[dt]
    value = flops / (wall * 1e-3) / 1e12
    mfma_flops = flops * info["R"] / (info["m"] * info["k"] * info["n"])
    out = {"config": f"{scheme_name} <{info['m']},{info['k']},{info['n']};{info['R']}>, {dt} storage, M={M} N={N} K={K}, A {kind_a}, B {kind_b}",
           "value": value, "unit": "TFLOP/s", "ms_per_step": wall, "steps": steps, "frac_of_dense_peak": value / peak,
           "plain_mfma_gemm_tflops": flops / (p_wall * 1e-3) / 1e12, "vs_plain": p_wall / wall,
           "vendor_gemm_tflops": flops / (v_wall * 1e-3) / 1e12,
           "dataflow": "algorithm1" if ran["flow"] == 1 else "fused", "fused_kernel_tflops": fused_tf,
           "algorithm1_not_chosen_tflops": alg1_tf,
           "roofline": {"bound": "mfma", "achieved": mfma_flops / (kernel_ms * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s",
                        "frac": mfma_flops / (kernel_ms * 1e-3) / 1e12 / peak, "kernel_ms": kernel_ms,
                        "traffic": read_traffic(name + ("_alg1" if ran["flow"] == 1 else ""))}}
    if not args.no_cpu:
        import oracle
        rows = sampled_rows(np, M, info["m"])
        lcma_step(0)
        B.lcma_gemm(*sets[1], None)
        torch.cuda.synchronize()
        ref = oracle.gemm_rows(inp.widen(As, dt), inp.widen(Bs, dt), rows)

        def host(t):
            t = t[torch.from_numpy(rows).cuda()]
            if dt == "bf16":
                return inp.widen(t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16), dt)
            return t.cpu().numpy().astype(np.float64)
        out["rel_frobenius_error"] = {"lcma": oracle.rel_frobenius(host(sets[0][2]), ref),
                                      "plain": oracle.rel_frobenius(host(sets[1][2]), ref), "rows_checked": int(len(rows))}
        if alg1_tf is not None:  # (for <3,3,3;23> in fp16 this is why the library does not offer it: past 4 x plain)
            out["rel_frobenius_error"]["algorithm1_not_chosen"] = oracle.rel_frobenius(host(alg1_c), ref)
    del sets, ws
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--heat-seconds", type=float, default=0.3,
                    help="untimed load before each timed leg, so that clocks are settled")
    ap.add_argument("--workload", default="strassen_bf16_ffn", choices=sorted(WORKLOADS))
    ap.add_argument("--no-others", action="store_true",
                    help="skip the further workloads (by default the other configurations are timed as well, about "
                         "two seconds each, and reported in `other_workloads`)")
    ap.add_argument("--variant", default=None, help="time this generated kernel instead of the default choice")
    ap.add_argument("--fused-only", action="store_true",
                    help="time lcma_gemm (always the fused kernel) as the headline instead of lcma_gemm_ws, which runs "
                         "the fused kernel or Algorithm 1, whichever the library's time model predicts faster")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--with-copy", action="store_true",
                    help="also run a plain device copy of A's bytes (a known-size kernel that calibrates HBM counters)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--prepared-b", action="store_true",
                    help="also time the offline Combine-B path (lcma_prepare_b once, lcma_gemm_prepared per step); "
                         "reported beside `value`, which stays the fully fused lcma_gemm")
    ap.add_argument("--weight-layout", action="store_true",
                    help="also time lcma_gemm_nt, which takes B as the N x K weight matrix of a linear layer "
                         "(no transposition while staging); reported beside `value`, which stays lcma_gemm on K x N")
    ap.add_argument("--ablation", action="store_true",
                    help="also time the dataflows the paper starts from (lcma_gemm_unfused): Algorithm 1 (four stages "
                         "through device memory) and Algorithm 2 as printed (Combine A/B materialised, GEMM + Combine H "
                         "fused), each with Combine B per call and with Combine B done once (static weights)")
    ap.add_argument("--fp8", action="store_true",
                    help="also time the FP8 E4M3 workflow with 1 x 128 block scales on the same bf16 matrices: quantise + "
                         "block-scaled GEMM against the LCMA form with the quantisation fused into Combine A")
    ap.add_argument("--no-extras", action="store_true",
                    help="time lcma_gemm, the plain and the vendor GEMM only (by default the prepared-B, weight-layout "
                         "and ablation legs run too; each adds about a second)")
    ap.add_argument("--selector-sweep", action="store_true",
                    help="instead of one workload: the bf16 shape sweep M in {2048, 8192, 16384} x (N, K) in {(4096, 4096), "
                         "(14336, 4096), (4096, 14336)} with A ~ N(0,1), B ~ N(0, 0.02^2); times plain, Strassen, two-level "
                         "Strassen and Laderman both fused (lcma_gemm) and by Algorithm 1 with Combine B offline, and prints "
                         "lcma_select's pick, lcma_select_dataflow's choice and the predictions beside them, as one JSON line")
    args = ap.parse_args()
    if args.selector_sweep:
        return selector_sweep(args)
    if not args.no_extras:
        args.prepared_b = args.weight_layout = args.ablation = args.fp8 = True
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the path would shard over M with no exchange between "
                 "GPUs, each running this same kernel on its rows). Re-run with --gpus 1.")

    import numpy as np
    import torch

    import lcma_inputs as inp
    from paper_2605_06057_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    B.lib()
    scheme_name, dt, M, N, K, kind_a, kind_b, seed = WORKLOADS[args.workload]
    As, Bs = inp.matrices(kind_a, kind_b, M, N, K, dt, seed)

    def dev(x):
        if dt == "bf16":
            return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(x).cuda()

    # three buffer sets, rotated, so that a step never finds its inputs left in cache by the step before
    sets = []
    for i in range(3):
        a, b = dev(As), dev(Bs)
        c = torch.empty((M, N), dtype=a.dtype, device="cuda")
        sets.append((a, b, c))
    scheme = B.lcma_scheme_load("builtin:" + scheme_name)
    B.lcma_scheme_verify(scheme)
    info = B.lcma_scheme_info(scheme)

    # the headline runs lcma_gemm_ws: lcma_gemm with a workspace, i.e. the fused kernel or Algorithm 1, whichever the
    # Decision Module predicts faster (every stage runs in every step, Combine B included)
    ws_main = None
    dataflow = {"ran": 0}
    if not args.variant and not args.fused_only:
        nbytes = B.lcma_unfused_workspace_bytes(scheme, M, N, K, B.DTYPE_IDS[dt])
        if nbytes > 0:
            ws_main = torch.empty((nbytes + B.lcma_split_group_scratch_bytes(),), dtype=torch.uint8, device="cuda")

    def lcma_step(i):
        a, b, c = sets[i % 3]
        if args.variant:
            B.lcma_gemm_variant(args.variant, a, b, c)
        elif ws_main is not None:
            dataflow["ran"] = B.lcma_gemm_ws(a, b, c, scheme, ws_main)
        else:
            B.lcma_gemm(a, b, c, scheme)

    def fused_step(i):
        a, b, c = sets[i % 3]
        B.lcma_gemm(a, b, c, scheme)

    def plain_step(i):
        a, b, c = sets[i % 3]
        B.lcma_gemm(a, b, c, None)

    def vendor_step(i):
        a, b, c = sets[i % 3]
        torch.mm(a, b, out=c)

    def timed(step, steps, warmup):
        return _timed(torch, step, steps, warmup, args.heat_seconds)

    if args.with_copy:
        dst = torch.empty_like(sets[0][0])
        for _ in range(5):
            dst.copy_(sets[0][0])
        torch.cuda.synchronize()

    flops = 2.0 * M * N * K
    wall_ms, ev_ms, med_ms = timed(lcma_step, args.steps, args.warmup)
    p_wall_ms, p_ev_ms, p_med_ms = timed(plain_step, args.steps, args.warmup)
    v_wall_ms, v_ev_ms, v_med_ms = timed(vendor_step, max(10, args.steps // 2), 3)
    value = flops / (wall_ms * 1e-3) / 1e12
    plain_tf = flops / (p_wall_ms * 1e-3) / 1e12
    # the dominant kernel: the fused kernel itself, or the GEMM stage of Algorithm 1 timed alone (the other stages
    # switched off through the library's measurement aid; their times are reported beside it)
    kernel_ms, kernel_name, stage_ms, fused_tf = ev_ms, "fused group-parallel kernel (lcma_gemm)", None, None
    if dataflow["ran"] == 1:
        f_wall_ms, _, _ = timed(fused_step, max(10, args.steps // 2), 3)
        fused_tf = flops / (f_wall_ms * 1e-3) / 1e12
        stage_ms = {}
        for bit, key in ((1, "combine_a"), (2, "combine_b"), (4, "gemm"), (8, "combine_h")):
            B.lcma_set_tuning("unfused_stages", str(bit))
            _, s_ev, _ = timed(lambda i: B.lcma_gemm_unfused(1, *sets[i % 3], scheme, ws_main), max(10, args.steps // 2), 3)
            stage_ms[key] = s_ev
        B.lcma_set_tuning("unfused_stages", "")
        kernel_ms, kernel_name = stage_ms["gemm"], "batched plane GEMM of Algorithm 1 (lcma_k_pg_*), R products in one launch"
    prepared = None
    if args.prepared_b:
        if scheme is None:
            sys.exit("bench.py: --prepared-b needs a workload with a scheme")
        bts = [B.lcma_prepare_b(b, scheme) for _, b, _ in sets]  # offline stage, once per weight matrix

        def prepared_step(i):
            B.lcma_gemm_prepared(sets[i % 3][0], bts[i % 3], sets[i % 3][2], scheme)

        def prepare_step(i):
            B.lcma_prepare_b(sets[i % 3][1], scheme, bts[i % 3])
        b_wall_ms, b_ev_ms, _ = timed(prepared_step, args.steps, args.warmup)
        o_wall_ms, o_ev_ms, _ = timed(prepare_step, max(10, args.steps // 4), 3)
        es = 4 if dt == "f32" else 2
        prep_bytes = K * N * es + bts[0].numel() * bts[0].element_size()
        prepared = {"gemm_prepared_tflops": flops / (b_wall_ms * 1e-3) / 1e12, "gemm_prepared_kernel_ms": b_ev_ms,
                    "prepare_b_ms": o_ev_ms, "prepare_b_bytes": prep_bytes,
                    "prepare_b_roofline": {"bound": "hbm", "achieved": prep_bytes / (o_ev_ms * 1e-3) / 1e9,
                                           "peak": 8000.0, "unit": "GB/s",
                                           "frac": prep_bytes / (o_ev_ms * 1e-3) / 1e9 / 8000.0}}
        prepared_step(0)
        torch.cuda.synchronize()
        prepared["_c"] = sets[0][2].clone()
    nk = None
    if args.weight_layout:
        ws = [b.t().contiguous() for _, b, _ in sets]

        def nt_step(i):
            B.lcma_gemm_nt(sets[i % 3][0], ws[i % 3], sets[i % 3][2], scheme)

        def nt_plain_step(i):
            B.lcma_gemm_nt(sets[i % 3][0], ws[i % 3], sets[i % 3][2], None)

        def nt_vendor_step(i):
            torch.mm(sets[i % 3][0], ws[i % 3].t(), out=sets[i % 3][2])
        n_wall_ms, n_ev_ms, _ = timed(nt_step, args.steps, args.warmup)
        np_wall_ms, _, _ = timed(nt_plain_step, args.steps, args.warmup)
        nv_wall_ms, _, _ = timed(nt_vendor_step, max(10, args.steps // 2), 3)
        nk = {"lcma_tflops": flops / (n_wall_ms * 1e-3) / 1e12, "lcma_kernel_ms": n_ev_ms,
              "plain_mfma_gemm_tflops": flops / (np_wall_ms * 1e-3) / 1e12,
              "vendor_gemm_tflops": flops / (nv_wall_ms * 1e-3) / 1e12}
        if dt != "f32":  # the plane GEMM (direct loads into LDS; Split-Group schedule where its model prefers it)
            sg = torch.empty((B.lcma_split_group_scratch_bytes(),), dtype=torch.uint8, device="cuda")
            pg_wall_ms, _, _ = timed(lambda i: B.lcma_gemm_nt_ws(sets[i % 3][0], ws[i % 3], sets[i % 3][2], sg), args.steps, args.warmup)
            nk["plain_plane_gemm_tflops"] = flops / (pg_wall_ms * 1e-3) / 1e12
            del sg
        if ws_main is not None:  # lcma_gemm_ws on this layout: the time model's dataflow, Combine B straight from the N x K weights
            flow_nk = {"ran": 0}

            def nt_ws_step(i):
                flow_nk["ran"] = B.lcma_gemm_ws(sets[i % 3][0], ws[i % 3], sets[i % 3][2], scheme, ws_main, b_nk=True)
            w_wall_ms, _, _ = timed(nt_ws_step, args.steps, args.warmup)
            nk["lcma_gemm_ws_tflops"] = flops / (w_wall_ms * 1e-3) / 1e12
            nk["lcma_gemm_ws_dataflow"] = "algorithm1" if flow_nk["ran"] == 1 else "fused"
        nt_step(0)
        torch.cuda.synchronize()
        nk["_c"] = sets[0][2].clone()
    fp8 = None
    if args.fp8 and dt == "bf16" and scheme_name in ("strassen", "strassen2", "laderman"):
        # The FP8 workflow of the paper (Sec. 4.1: bf16 operands, E4M3 with 1 x 128 block scales; Sec. 4.3: quantisation
        # fused into Combine A).  Weights are static: quantised (plain) or combined and quantised (LCMA) once, untimed.
        # A step of the plain workflow quantises A and multiplies; a step of the LCMA form runs Combine A with the
        # quantisation fused in, the batched block-scaled GEMM and Combine H.
        wt = [b.t().contiguous() for _, b, _ in sets]
        qw = [B.lcma_fp8_quantize(w) for w in wt]
        qa = [B.lcma_fp8_quantize(a) for a, _, _ in sets]
        wp = [B.lcma_fp8_prepare_w(w, scheme) for w in wt]
        wsf = torch.empty((B.lcma_fp8_workspace_bytes(scheme, M, N, K),), dtype=torch.uint8, device="cuda")

        def fp8_plain_step(i):
            j = i % 3
            B.lcma_fp8_quantize(sets[j][0], qa[j][0], qa[j][1])
            B.lcma_fp8_gemm_nt(qa[j][0], qa[j][1], qw[j][0], qw[j][1], sets[j][2], K)

        def fp8_gemm_step(i):
            j = i % 3
            B.lcma_fp8_gemm_nt(qa[j][0], qa[j][1], qw[j][0], qw[j][1], sets[j][2], K)

        def fp8_lcma_step(i):
            j = i % 3
            B.lcma_fp8_gemm_lcma(sets[j][0], wp[j], sets[j][2], scheme, wsf)
        fp_wall, _, _ = timed(fp8_plain_step, args.steps, args.warmup)
        fg_wall, fg_ev, _ = timed(fp8_gemm_step, args.steps, args.warmup)
        fl_wall, _, _ = timed(fp8_lcma_step, args.steps, args.warmup)
        fp8 = {"plain_workflow_tflops": flops / (fp_wall * 1e-3) / 1e12, "plain_gemm_only_tflops": flops / (fg_wall * 1e-3) / 1e12,
               "lcma_tflops": flops / (fl_wall * 1e-3) / 1e12, "lcma_vs_plain_workflow": fp_wall / fl_wall,
               "lcma_frac_of_dense_fp8_peak": flops / (fl_wall * 1e-3) / 1e12 / 5000.0,
               "lcma_frac_of_dense_bf16_peak": flops / (fl_wall * 1e-3) / 1e12 / 2500.0,
               "gemm_roofline": {"bound": "mfma", "achieved": flops / (fg_ev * 1e-3) / 1e12, "peak": 5000.0, "unit": "TFLOP/s",
                                 "frac": flops / (fg_ev * 1e-3) / 1e12 / 5000.0}}
        fp8_lcma_step(0)
        fp8_plain_step(1)
        torch.cuda.synchronize()
        fp8["_c"], fp8["_cp"] = sets[0][2].clone(), sets[1][2].clone()
        del wt, qw, qa, wp, wsf
    ablation = None
    if args.ablation and B.lib().lcma_gemm_unfused(1, 0, 0, 0, None, 0, None, 0, None, 0, B.DTYPE_IDS[dt], scheme.handle,
                                                   None, 0, 0, None) == B.LCMA_ERR_NOKERNEL:
        args.ablation = False  # no stage kernels for this scheme (an empty call answers before anything is launched)
    if args.ablation:
        nbytes = B.lcma_unfused_workspace_bytes(scheme, M, N, K, B.DTYPE_IDS[dt]) + B.lcma_split_group_scratch_bytes()
        ws = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
        ablation = {"workspace_bytes": nbytes}
        for level, key in ((1, "algorithm1"), (2, "algorithm2_as_printed")):
            for reuse, tag in ((False, ""), (True, "_combine_b_offline")):
                if reuse:  # the planes of B in the workspace belong to buffer set 0 from here on
                    B.lcma_gemm_unfused(level, sets[0][0], sets[0][1], sets[0][2], scheme, ws)

                def unfused_step(i, level=level, reuse=reuse):
                    a, b, c = sets[0] if reuse else sets[i % 3]
                    B.lcma_gemm_unfused(level, a, b, c, scheme, ws, reuse_bt=reuse)
                u_wall_ms, u_ev_ms, _ = timed(unfused_step, max(10, args.steps // 2), 5)
                ablation[key + tag + "_tflops"] = flops / (u_wall_ms * 1e-3) / 1e12
            unfused_step(0)
            torch.cuda.synchronize()
            ablation["_c" + key] = sets[0][2].clone()
    peak = PEAK_TFLOPS[dt]

    # parity on sampled rows (one row range inside every block row of the scheme grid)
    # what the matrix pipe alone sustains on zeros and on this workload's values (16-bit storage; no memory traffic at all):
    # on MI355X the second is well below the first, and it, not the dense peak, is what a kernel could reach on these inputs
    pipe = None
    if dt != "f32" and not args.no_extras:
        sink = torch.empty((512 * 1024,), dtype=torch.float32, device="cuda")
        pipe = {"unit": "TFLOP/s", "kernel": "lcma_mfma_probe: 32x32x16 fp16 MFMA on fragments held in registers"}
        for key, src in (("zeros", torch.zeros((32768,), dtype=torch.float16, device="cuda")),
                         ("values_of_A", sets[0][0].reshape(-1)[:32768].to(torch.float16).contiguous())):
            iters = 10000
            probe_flops = B.lcma_mfma_probe(src, sink, iters)
            _, p_ms, _ = timed(lambda i: B.lcma_mfma_probe(src, sink, iters), 8, 2)
            pipe[key] = probe_flops / (p_ms * 1e-3) / 1e12
    lcma_step(0)
    plain_step(1)
    torch.cuda.synchronize()
    rows = sampled_rows(np, M, info["m"])
    cpu = None
    err = err_plain = None
    if not args.no_cpu:
        import oracle
        Aw, Bw = inp.widen(As, dt), inp.widen(Bs, dt)
        t0 = time.perf_counter()
        ref = oracle.gemm_rows(Aw, Bw, rows)

        def host(t):
            t = t[torch.from_numpy(rows).cuda()]
            if dt == "bf16":
                return inp.widen(t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16), dt)
            return t.cpu().numpy().astype(np.float64)
        err = oracle.rel_frobenius(host(sets[0][2]), ref)
        err_plain = oracle.rel_frobenius(host(sets[1][2]), ref)
        if prepared:
            prepared["rel_frobenius_error"] = oracle.rel_frobenius(host(prepared["_c"]), ref)
        if nk:
            nk["rel_frobenius_error"] = oracle.rel_frobenius(host(nk["_c"]), ref)
        if fp8:  # against the UNQUANTISED product: what the FP8 formats cost, plain and LCMA
            fp8["rel_frobenius_error"] = {"lcma": oracle.rel_frobenius(host(fp8["_c"]), ref),
                                          "plain": oracle.rel_frobenius(host(fp8["_cp"]), ref)}
        if ablation:
            for key in ("algorithm1", "algorithm2_as_printed"):
                ablation[key + "_rel_frobenius_error"] = oracle.rel_frobenius(host(ablation["_c" + key]), ref)
        # timed sample: as many leading rows as fit the CPU budget, judged from a run on 256 rows (the parity run on a
        # handful of rows is too short to tell the rate of a long one)
        probe_rows = int(min(M, 256))
        t0 = time.perf_counter()
        oracle.gemm_rows(Aw, Bw, np.arange(probe_rows))
        rate = 2.0 * probe_rows * N * K / max(time.perf_counter() - t0, 1e-6)
        nrows = int(min(M, max(len(rows), args.cpu_seconds * rate / (2.0 * N * K))))
        t0 = time.perf_counter()
        oracle.gemm_rows(Aw, Bw, np.arange(nrows))
        t_cpu = time.perf_counter() - t0
        cpu = {"value": 2.0 * nrows * N * K / t_cpu / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": f"fp64 triple loop on the first {nrows} of {M} rows of C "
               f"({t_cpu:.1f} s); whole problem extrapolated {t_cpu * M / nrows:.0f} s"}

    if prepared:
        prepared.pop("_c")
    if nk:
        nk.pop("_c")
    if fp8:
        fp8.pop("_c")
        fp8.pop("_cp")
    if ablation:
        ablation = {k: v for k, v in ablation.items() if not k.startswith("_c")}
    mfma_flops = flops * info["R"] / (info["m"] * info["k"] * info["n"])
    achieved = mfma_flops / (kernel_ms * 1e-3) / 1e12
    out = {
        "metric": "effective TFLOP/s (2MNK/t) and fraction of MI355X dense MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if dt == "bf16" else dt, "data": "synthetic",
        "config": {"workload": f"{scheme_name} <{info['m']},{info['k']},{info['n']};{info['R']}> one launch, "
                               f"{dt} storage, fp32 accumulate, M={M} N={N} K={K}, A {kind_a}, B {kind_b}",
                   "variant": args.variant or "library default",
                   "entry": "lcma_gemm_variant" if args.variant else ("lcma_gemm_ws" if ws_main is not None else "lcma_gemm"),
                   "dataflow": "Algorithm 1 (Combine A, Combine B, batched GEMM, Combine H; chosen by the time model)"
                               if dataflow["ran"] == 1 else "fused group-parallel kernel"},
        "frac_of_dense_peak": value / peak,
        "plain_mfma_gemm_tflops": plain_tf, "vs_plain": value / plain_tf,
        "vendor_gemm_tflops": flops / (v_wall_ms * 1e-3) / 1e12,
        "kernel_ms_events": {"lcma_mean": ev_ms, "lcma_median": med_ms, "plain_mean": p_ev_ms, "plain_median": p_med_ms},
        "rel_frobenius_error": {"lcma": err, "plain": err_plain, "rows_checked": int(len(rows))},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": read_traffic(args.workload + ("_alg1" if dataflow["ran"] == 1 else "")),
                     "kernel": kernel_name, "kernel_ms": kernel_ms},
        "cpu_baseline": cpu,
    }
    if pipe:
        pipe["roofline_achieved_over_values_of_A"] = achieved / pipe["values_of_A"]
        out["mfma_pipe_alone"] = pipe
    if stage_ms:
        out["algorithm1_stage_ms_events"] = stage_ms
        out["fused_kernel_tflops"] = fused_tf
    if prepared:
        out["offline_combine_b"] = prepared
    if nk:
        out["weight_layout_nk"] = nk
    if ablation:
        out["ablation_unfused_dataflows"] = ablation
    if fp8:
        out["fp8_e4m3_block_scaled"] = fp8
    if not args.no_others and not args.variant:
        sets = bts = ws = wt = None  # release the device buffers of the main workload
        torch.cuda.empty_cache()
        others = [w for w in ("strassen_bf16_4096", "strassen2_bf16_ffn", "laderman_f16_6144", "strassen_f32_4096",
                              "strassen_bf16_ffn") if w != args.workload][:4]
        out["other_workloads"] = {w: side_workload(w, args) for w in others}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
