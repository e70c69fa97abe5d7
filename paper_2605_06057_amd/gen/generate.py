"""Kernel generator: one gfx950 HIP translation unit per (scheme, dtype, tile, chunking).

This is the build-time counterpart of the paper's Automated Code Generation (Sec. 3.1):
the coefficient tensors U, V, W of a scheme are turned into straight-line code, so zero
coefficients cost nothing and no coefficient is read at run time.  The scheme-agnostic
part (tile staging, MFMA loop, stores) is csrc/lcma_device.hpp; what is emitted here is

  * per chunk of products: which raw blocks A_{i,l}, B_{l,j} to stage, and the signed sums
    of Eq. 3 / Eq. 4 on 16-byte register vectors;
  * after each chunk: the signed accumulation of Eq. 6 into fp32 tiles of C, each tile
    stored as soon as its last product has arrived (the "register reuse" reordering);
  * on-chip resource planning: accumulator registers and LDS bytes of every variant are
    computed and checked against the gfx950 budget before anything is written.

Also emitted: builtin_schemes.inc (the scheme texts the library embeds) and registry.cc.
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
PKG = os.path.dirname(HERE)
SCHEME_DIR = os.path.join(PKG, "schemes")

SCHEME_IDS = {"plain": 0, "strassen": 1, "strassen2": 2, "laderman": 3}  # further scheme files: 4, 5, ... by name
DTYPE_IDS = {"f32": 0, "bf16": 1, "f16": 2}
ACC_REG_BUDGET = 400      # of 512 unified VGPR/AGPR per lane at one wave per SIMD
LDS_BUDGET = 160 * 1024


# ----------------------------------------------------------------------------- schemes
@dataclass
class Scheme:
    name: str
    m: int
    k: int
    n: int
    R: int
    U: np.ndarray
    V: np.ndarray
    W: np.ndarray

    def text(self) -> str:
        rows = [f"{self.m} {self.k} {self.n} {self.R}"]
        for T in (self.U, self.V, self.W):
            rows += [" ".join(str(int(v)) for v in T[r].reshape(-1)) for r in range(self.R)]
        return "\n".join(rows) + "\n"


def parse_scheme(name: str, text: str) -> Scheme:
    nums = []
    for line in text.splitlines():
        nums += [int(t) for t in line.split("#", 1)[0].replace(",", " ").split()]
    m, k, n, R = nums[:4]
    body = np.array(nums[4:], dtype=np.int64)
    assert body.size == R * (m * k + k * n + m * n), f"{name}: wrong number of coefficients"
    a, b = R * m * k, R * m * k + R * k * n
    return Scheme(name, m, k, n, R, body[:a].reshape(R, m, k), body[a:b].reshape(R, k, n),
                  body[b:].reshape(R, m, n))


def compose(outer: Scheme, inner: Scheme, name: str) -> Scheme:
    """Scheme of applying `inner` to each block product of `outer` (flat Kronecker form)."""
    def kron(X, Y):
        R1, p1, q1 = X.shape
        R2, p2, q2 = Y.shape
        Z = np.zeros((R1 * R2, p1 * p2, q1 * q2), np.int64)
        for r1 in range(R1):
            for r2 in range(R2):
                Z[r1 * R2 + r2] = np.kron(X[r1], Y[r2])
        return Z
    return Scheme(name, outer.m * inner.m, outer.k * inner.k, outer.n * inner.n, outer.R * inner.R,
                  kron(outer.U, inner.U), kron(outer.V, inner.V), kron(outer.W, inner.W))


def multiplies_matrices(s: Scheme) -> bool:
    """Brent identity, exact (checked again by the library when a scheme is loaded)."""
    for i in range(s.m):
        for a in range(s.k):
            for b in range(s.k):
                for j in range(s.n):
                    got = np.tensordot(s.U[:, i, a] * s.V[:, b, j], s.W, axes=(0, 0))
                    want = np.zeros((s.m, s.n), np.int64)
                    if a == b:
                        want[i, j] = 1
                    if not np.array_equal(got, want):
                        return False
    return True


def load_schemes() -> dict[str, Scheme]:
    """The schemes kernels are generated for: Strassen and Laderman from their files, two-level
    Strassen composed from Strassen, and every further scheme file: any other *.txt in schemes/ and the
    paths listed (colon-separated) in the environment variable LCMA_EXTRA_SCHEMES.  A further scheme is
    known to the library by its file name without the extension ("builtin:<name>") and gets ids from 4
    up in name order."""
    out = {}
    for name in ("strassen", "laderman"):
        with open(os.path.join(SCHEME_DIR, name + ".txt")) as f:
            out[name] = parse_scheme(name, f.read())
    out["strassen2"] = compose(out["strassen"], out["strassen"], "strassen2")
    one = np.ones((1, 1, 1), np.int64)
    out["plain"] = Scheme("plain", 1, 1, 1, 1, one, one, one)
    extra = [os.path.join(SCHEME_DIR, f) for f in os.listdir(SCHEME_DIR) if f.endswith(".txt")]
    extra += [p for p in os.environ.get("LCMA_EXTRA_SCHEMES", "").split(":") if p]
    for path in sorted(extra, key=os.path.basename):
        name = os.path.splitext(os.path.basename(path))[0]
        if name in out:
            continue
        assert name.isidentifier(), f"{path}: the file name must be usable as an identifier"
        with open(path) as f:
            out[name] = parse_scheme(name, f.read())
    for s in out.values():
        assert multiplies_matrices(s), f"scheme {s.name} violates the Brent equations"
    nxt = max(SCHEME_IDS.values()) + 1
    for name in sorted(out):
        if name not in SCHEME_IDS:
            SCHEME_IDS[name] = nxt
            nxt += 1
    return out


def further_schemes(schemes: dict[str, Scheme]) -> list[str]:
    return sorted(n for n in schemes if SCHEME_IDS[n] > 3)


# ----------------------------------------------------------------------------- variants
@dataclass
class Variant:
    scheme: str
    dtype: str
    TM: int
    TN: int
    TK: int
    wgm: int = 2
    wgn: int = 2
    chunk: int = 1            # products per chunk (consecutive in the chunk order)
    stages: int = 2
    rank: int = 0             # >= 90: ablation variant, only reachable by name
    eff: float = 0.1          # measured fraction of the dtype's MFMA peak its MFMA work sustains (large shapes)
    pipe: int = 0             # 0: staging in one phase, 2: staging spread over the MFMA phase (with fc)
    occ: int = 1              # work-groups per CU the kernel is compiled for
    fc: int = 0               # 1: LDS holds raw blocks, waves combine MFMA fragments (needs chunk >= R)
    comp: tuple = ()          # products (0-based) whose left operand also gets its rounding residual multiplied
    pb: int = 0               # 1: B side comes from the offline Combine-B kernel (needs fc, pipe 2)
    dl: int = 0               # 1 (with pb): tiles are loaded from memory straight into LDS
    tb: int = 0               # 1: B is given as the N x K weight matrix (k-contiguous rows)
    pa: int = 0               # 1 (with pb, staged loop): the left operands come ready-made from planes too
    batch: int = 0            # 1 (plain, tb): the grid covers R products on planes (Algorithm 1's batched GEMM)
    name: str = field(default="")

    def finish(self):
        if not self.name:
            self.name = (f"{self.scheme}_{self.dtype}_t{self.TM}x{self.TN}x{self.TK}_c{self.chunk}"
                         + (f"x{len(self.comp)}" if self.comp else "") + (f"w{self.wgm}x{self.wgn}" if (self.wgm, self.wgn) != (2, 2) else "") + ("f" if self.fc else "") + ("i" if self.pipe == 2 else "") + ("s3" if self.stages == 3 else "") + ("a" if self.pa else "") + ("b" if self.pb else "") + ("d" if self.dl else "") + ("t" if self.tb else "") + ("g" if self.batch else "") + (f"o{self.occ}" if self.occ > 1 else ""))
        return self


def with_residuals(s: Scheme, comp: tuple) -> tuple[Scheme, set]:
    """Error compensation for 16-bit operands.  For each product r in `comp` a further product is
    appended whose left operand is the rounding residual of the r-th combination (its fp32 value minus
    its fp16 value, itself rounded to fp16) and whose right operand and W row are those of r; the sum
    of the two products is the product with an (almost) unrounded left operand.  Returns the longer
    scheme and the indices of the residual products."""
    if not comp:
        return s, set()
    rows = list(range(s.R)) + list(comp)
    ext = Scheme(s.name, s.m, s.k, s.n, len(rows), s.U[rows], s.V[rows], s.W[rows])
    return ext, set(range(s.R, len(rows)))


def chunks_of(s: Scheme, v: Variant) -> list[list[int]]:
    order = list(range(s.R))
    if v.chunk >= s.R:
        return [order]
    return [order[i:i + v.chunk] for i in range(0, s.R, v.chunk)]


def plan(s: Scheme, v: Variant):
    """On-chip resource planning: (accumulator registers per lane, LDS bytes, peak live C tiles)."""
    es = 4 if v.dtype == "f32" else 2
    tile_regs = (v.TM // v.wgm // 32) * (v.TN // v.wgn // 32) * 16
    chunks = chunks_of(s, v)
    nslot = max(len(c) for c in chunks)
    if len(chunks) == 1:
        live_c = 0
    else:
        first, last = {}, {}
        for ci, ch in enumerate(chunks):
            for r in ch:
                for i in range(s.m):
                    for j in range(s.n):
                        if s.W[r, i, j]:
                            first.setdefault((i, j), ci)
                            last[(i, j)] = ci
        live_c = max(sum(1 for key in first if first[key] <= ci <= last[key]) for ci in range(len(chunks)))
    regs = (live_c + nslot) * tile_regs
    if v.fc:
        assert len(chunks) == 1, "fragment combine keeps every product's accumulator live"
        nsa = len({(i, l) for r in chunks[0] for i in range(s.m) for l in range(s.k) if s.U[r, i, l]})
        nsb = len({(l, j) for r in chunks[0] for l in range(s.k) for j in range(s.n) if s.V[r, l, j]})
        if v.pb:
            nsb = len(chunks[0])  # one LDS slot per product's right operand
    else:
        nsa = nsb = nslot
    lds = v.stages * (nsa * v.TM * v.TK + nsb * v.TK * v.TN) * es
    return regs, lds, live_c, nslot, nsa, nsb


# ----------------------------------------------------------------------------- code emission
CPP_TYPES = {"f32": ("F32", "F32"), "f16": ("F16", "F16"), "bf16": ("BF16", "F16")}


def signed_sum(terms: list[tuple[int, str]], wide: bool = False, fn: bool = False) -> str:
    """[(coef, expr)] -> C++ expression; +-1 become additions, anything else a multiply.
    wide: form the sum in fp32 and round once (used for fp16 sums of three or more terms)."""
    if wide and len(terms) >= 3:
        return "Wide<V>::down(" + signed_sum([(c, f"Wide<V>::up({e})") for c, e in terms]) + ")"
    terms = sorted(terms, key=lambda t: t[0] < 0)  # a positive term first when there is one
    out = ""
    for idx, (c, e) in enumerate(terms):
        mag = e if abs(c) == 1 else f"{e} * {abs(c)}"
        if idx == 0:
            out = mag if c > 0 else f"-{mag}"
        elif fn:
            out = f"{'vadd' if c > 0 else 'vsub'}({out}, {mag})"
        else:
            out += (" + " if c > 0 else " - ") + mag
    return out


def share_sums(rows: list[dict[int, int]], n_in: int):
    """Common sums of a set of signed sums with +-1 coefficients (the "register reuse" of Sec. 3.1): while
    some pair of variables occurs with the same relative sign in two or more rows, it becomes a shared
    temporary t = x +- y that replaces the pair everywhere.  Variables 0..n_in-1 are the inputs, the
    temporaries follow.  Returns (temps [(x, y, sign)], rewritten rows).  Winograd's form of Strassen's
    algorithm comes out at its 4 + 4 additions this way; schemes without common pairs are left as they are."""
    rows = [dict(r) for r in rows]
    temps = []
    while True:
        count = {}
        for r in rows:
            vs = sorted(r)
            for a in range(len(vs)):
                for b in range(a + 1, len(vs)):
                    key = (vs[a], vs[b], r[vs[a]] * r[vs[b]])
                    count[key] = count.get(key, 0) + 1
        best = max(count.items(), key=lambda kv: (kv[1], -kv[0][0], -kv[0][1]), default=None)
        if best is None or best[1] < 2:
            return temps, rows
        (x, y, rel), _ = best
        users = [r for r in rows if x in r and y in r and r[x] * r[y] == rel]
        lone = sum(r[x] for r in users if len(r) == 2)  # rows that are this pair alone would need a negation
        if rel < 0 and (lone < 0 or (lone == 0 and sum(r[x] for r in users) < 0)):
            x, y = y, x  # a difference is taken the way round that saves negations
        t = n_in + len(temps)
        temps.append((x, y, rel))
        for r in users:
            cx = r.pop(x)
            r.pop(y)
            r[t] = cx


def emit_comb(w, fn_name: str, n_name: str, rows: list[list[tuple[int, int]]], n_in: int, wide: bool):
    """out[s] = signed sum of in[...] for every row [(coef, input index)], with common sums shared when every
    coefficient is +-1 and the sums are not formed in a wider type."""
    w(f"    template <class V> static LCMA_DEV void {fn_name}(const V (&in)[{n_name}], V (&out)[NP]) {{")
    shareable = not wide and all(abs(c) == 1 for row in rows for c, _ in row)
    temps, new_rows = share_sums([{i: c for c, i in row} for row in rows], n_in) if shareable else ([], None)
    name = lambda i: f"in[{i}]" if i < n_in else f"t{i - n_in}"
    for ti, (x, y, rel) in enumerate(temps):
        w(f"        const V t{ti} = {'vadd' if rel > 0 else 'vsub'}({name(x)}, {name(y)});")
    for si, row in enumerate(rows):
        terms = [(c, name(i)) for i, c in sorted(new_rows[si].items())] if temps else [(c, f"in[{i}]") for c, i in row]
        w(f"        out[{si}] = {signed_sum(terms, wide, True)};")
    w("    }")


def emit_kernel(s: Scheme, v: Variant) -> str:
    s, residual = with_residuals(s, v.comp)
    in_t, ct_t = CPP_TYPES[v.dtype]
    if s.name == "plain":
        ct_t = in_t  # nothing is added: multiply in the storage type
    regs, lds, live_c, nslot, nsa, nsb = plan(s, v)
    chunks = chunks_of(s, v)
    single = len(chunks) == 1
    # bf16 inputs carry 8 significant bits, so their sums are (nearly) exact in packed fp16 adds;
    # fp16 inputs need the fp32 detour to be rounded only once.
    wide = v.dtype == "f16"
    L = []
    w = L.append
    w(f"// GENERATED by gen/generate.py - do not edit.  Scheme {s.name} <{s.m},{s.k},{s.n};{s.R}>, dtype {v.dtype},")
    w(f"// tile {v.TM}x{v.TN}x{v.TK}, {len(chunks)} chunk(s) of up to {nslot} products; planned accumulator registers")
    w(f"// per lane {regs}, LDS {lds} bytes, peak live C tiles {live_c}.")
    w('#include "lcma_device.hpp"')
    w("namespace {")
    w("using namespace lcma;")
    w(f"using T = Tile<{in_t}, {ct_t}, {v.TM}, {v.TN}, {v.TK}, {v.wgm}, {v.wgn}, {nsa}, {nsb}, {v.pipe}, {v.fc}, {v.stages}, {v.pb}, {v.dl}, {v.tb}, {v.pa}, {v.batch}>;")
    for ci, ch in enumerate(chunks):
        a_blocks = sorted({(i, l) for r in ch for i in range(s.m) for l in range(s.k) if s.U[r, i, l]})
        b_blocks = sorted({(l, j) for r in ch for l in range(s.k) for j in range(s.n) if s.V[r, l, j]})
        w(f"struct Chunk{ci} {{  // products {', '.join(str(r + 1) for r in ch)}")
        if v.pb:
            b_blocks = []
        if v.pa:
            a_blocks = []
        w(f"    static constexpr int NA = {len(a_blocks)}, NB = {len(b_blocks)}, NP = {len(ch)};")
        for fn, vals in (("a_i", [b[0] for b in a_blocks]), ("a_l", [b[1] for b in a_blocks]),
                         ("b_l", [b[0] for b in b_blocks]), ("b_j", [b[1] for b in b_blocks])):
            if not vals:
                continue
            w(f"    static LCMA_DEV constexpr int {fn}(int t) {{ constexpr int v[] = {{{', '.join(map(str, vals))}}}; return v[t]; }}")
        if v.pa:
            assert not v.comp, "residual products are formed by the fused kernels only"
            w(f"    static LCMA_DEV constexpr int a_plane(int s) {{ constexpr int v[] = {{{', '.join(map(str, ch))}}}; return v[s]; }}")
        elif not any(r in residual for r in ch):
            emit_comb(w, "comb_a", "NA", [[(int(s.U[r, i, l]), a_blocks.index((i, l))) for (i, l) in a_blocks if s.U[r, i, l]]
                                          for r in ch], len(a_blocks), wide)
        else:
            w("    template <class V> static LCMA_DEV void comb_a(const V (&in)[NA], V (&out)[NP]) {")
            for si, r in enumerate(ch):
                terms = [(int(s.U[r, i, l]), f"in[{a_blocks.index((i, l))}]") for (i, l) in a_blocks if s.U[r, i, l]]
                if r in residual:
                    assert wide and len(terms) >= 2, "residual products need fp16 sums formed in fp32"
                    wsum = signed_sum([(c, f"Wide<V>::up({e})") for c, e in terms])
                    w(f"        out[{si}] = Wide<V>::residual({wsum});")
                else:
                    w(f"        out[{si}] = {signed_sum(terms, wide, True)};")
            w("    }")
        if v.pb:
            n_orig = s.R - len(v.comp)  # a residual product multiplies the same right operand as its source
            planes = [r if r < n_orig else v.comp[r - n_orig] for r in ch]
            w(f"    static LCMA_DEV constexpr int b_plane(int s) {{ constexpr int v[] = {{{', '.join(map(str, planes))}}}; return v[s]; }}")
        if not v.pb:
            emit_comb(w, "comb_b", "NB", [[(int(s.V[r, l, j]), b_blocks.index((l, j))) for (l, j) in b_blocks if s.V[r, l, j]]
                                          for r in ch], len(b_blocks), wide)
        w("};")
    w("")
    w("} // namespace")
    w("")
    w("// the kernel carries the variant's name so that profiles tell the variants apart")
    w(f'extern "C" __global__ __launch_bounds__({64 * v.wgm * v.wgn}, {v.occ}) void lcma_k_{v.name}(const lcma::Params p) {{')
    w("    __shared__ __attribute__((aligned(16))) char smem[T::LDS_BYTES];")
    w("    const Ctx<T> cx(p, (LCMA_LDS char *)smem);")
    if single:
        ch = chunks[0]
        w(f"    T::Acc h[{len(ch)}];")
        w(f"    for (auto &t : h) zero_acc(t);")
        w("    run_chunk<T, Chunk0>(cx, h);")
        for i in range(s.m):
            for j in range(s.n):
                terms = [(int(s.W[r, i, j]), f"h[{si}].v[mi][ni]") for si, r in enumerate(ch) if s.W[r, i, j]]
                w(f"    cx.store_c({i}, {j}, [&](int mi, int ni) {{ return {signed_sum(terms)}; }});")
    else:
        first, last = {}, {}
        for ci, ch in enumerate(chunks):
            for r in ch:
                for i in range(s.m):
                    for j in range(s.n):
                        if s.W[r, i, j]:
                            first.setdefault((i, j), (ci, r))
                            last[(i, j)] = (ci, r)
        w(f"    T::Acc c[{s.m * s.n}];")
        for ci, ch in enumerate(chunks):
            w("    {")
            w(f"        T::Acc h[{len(ch)}];")
            w("        for (auto &t : h) zero_acc(t);")
            w(f"        run_chunk<T, Chunk{ci}>(cx, h);")
            for si, r in enumerate(ch):
                for i in range(s.m):
                    for j in range(s.n):
                        coef = int(s.W[r, i, j])
                        if not coef:
                            continue
                        op = "set" if first[(i, j)] == (ci, r) else "add"
                        w(f"        acc_{op}(c[{i * s.n + j}], h[{si}], {float(coef)}f);")
                        if last[(i, j)] == (ci, r):
                            w(f"        cx.store_c({i}, {j}, [&](int mi, int ni) {{ return c[{i * s.n + j}].v[mi][ni]; }});")
            w("    }")
    w("}")
    w("")
    w(f'extern "C" int lcma_launch_{v.name}(const lcma::Params *p, int grid, void *stream) {{')
    w(f"    lcma_k_{v.name}<<<dim3(grid), dim3({64 * v.wgm * v.wgn}), 0, (hipStream_t)stream>>>(*p);")
    w("    return (int)hipGetLastError();")
    w("}")
    return "\n".join(L) + "\n"


def emit_registry(schemes: dict[str, Scheme], variants: list[Variant]) -> str:
    L = ["// GENERATED by gen/generate.py - do not edit.", '#include "host_common.h"', ""]
    for v in variants:
        L.append(f'extern "C" int lcma_launch_{v.name}(const lcma::Params *p, int grid, void *stream);')
    L += ["", "namespace lcma {", "const Variant kVariants[] = {"]
    for v in variants:
        s = schemes[v.scheme]
        hash_expr = "0" if s.name == "plain" else f"0x{scheme_hash(s):016x}ull"
        L.append(f'    {{"{v.name}", {SCHEME_IDS[v.scheme]}, {DTYPE_IDS[v.dtype]}, {s.m}, {s.k}, {s.n}, {s.R}, '
                 f"{hash_expr}, {v.TM}, {v.TN}, {v.TK}, {min(v.chunk, s.R)}, {v.rank}, {v.eff}, {v.occ}, {s.R + len(v.comp)}, {v.pb}, {v.tb}, {v.pa}, {v.batch}, lcma_launch_{v.name}}},")
    L += ["};", f"const int kVariantCount = {len(variants)};"]
    preps = prep_kernels(variants)
    L.append("const PrepKernel kPrepKernels[] = {")
    for sch, dt in preps:
        L.append(f"    {{{SCHEME_IDS[sch]}, {DTYPE_IDS[dt]}, lcma_launch_prep_b_{sch}_{dt}, lcma_launch_prep_bt_{sch}_{dt}}},")
    if not preps:
        L.append("    {0, 0, nullptr, nullptr},")
    L += ["};", f"const int kPrepKernelCount = {len(preps)};"]
    stages = stage_kernels(variants)
    L.append("const StageKernel kStageKernels[] = {")
    for sch, dt in stages:
        ra, rb, rh = STAGE_RATES.get((sch, dt != "f32"), (4.0e12, 3.0e12, 5.0e12))
        h32 = f"lcma_launch_comb_h32_{sch}_{dt}" if dt != "f32" else "nullptr"
        ext = (sch, dt) in STAGE_COMP
        cb, cbt = (f"lcma_launch_comb_b_{sch}_{dt}", f"lcma_launch_comb_bt_{sch}_{dt}") if ext else ("nullptr", "nullptr")
        L.append(f"    {{{SCHEME_IDS[sch]}, {DTYPE_IDS[dt]}, {stage_planes(schemes[sch], dt)}, lcma_launch_comb_a_{sch}_{dt}, {cb}, {cbt}, "
                 f"lcma_launch_comb_h_{sch}_{dt}, {h32}, {ra}, {rb}, {rh}}},")
    if not stages:
        L.append("    {0, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr, 0.0, 0.0, 0.0},")
    L += ["};", f"const int kStageKernelCount = {len(stages)};"]
    fp8 = sorted({sch for sch, dt in stages if dt == "bf16"} & {sch for sch, dt in preps if dt == "bf16"})
    L.append("const Fp8Kernel kFp8Kernels[] = {")
    for sch in fp8:
        L.append(f"    {{{SCHEME_IDS[sch]}, lcma_launch_fp8_comb_a_{sch}, lcma_launch_fp8_prep_w_{sch}}},")
    if not fp8:
        L.append("    {0, nullptr, nullptr},")
    L += ["};", f"const int kFp8KernelCount = {len(fp8)};", "} // namespace lcma", ""]
    for sch in fp8:
        L.insert(3, f'extern "C" int lcma_launch_fp8_comb_a_{sch}(const lcma::Fp8QuantParams *p, int gx, int gy, void *stream);')
        L.insert(3, f'extern "C" int lcma_launch_fp8_prep_w_{sch}(const lcma::Fp8QuantParams *p, int gx, int gy, void *stream);')
    for sch, dt in stages:
        L.insert(3, f'extern "C" int lcma_launch_comb_a_{sch}_{dt}(const lcma::PrepParams *p, int gx, int gy, void *stream);')
        L.insert(3, f'extern "C" int lcma_launch_comb_h_{sch}_{dt}(const lcma::CombHParams *p, int gx, int gy, void *stream);')
        if dt != "f32":
            L.insert(3, f'extern "C" int lcma_launch_comb_h32_{sch}_{dt}(const lcma::CombHParams *p, int gx, int gy, void *stream);')
        if (sch, dt) in STAGE_COMP:
            L.insert(3, f'extern "C" int lcma_launch_comb_b_{sch}_{dt}(const lcma::PrepParams *p, int gx, int gy, void *stream);')
            L.insert(3, f'extern "C" int lcma_launch_comb_bt_{sch}_{dt}(const lcma::PrepParams *p, int gx, int gy, void *stream);')
    for sch, dt in preps:
        L.insert(3, f'extern "C" int lcma_launch_prep_b_{sch}_{dt}(const lcma::PrepParams *p, int gx, int gy, void *stream);')
        L.insert(3, f'extern "C" int lcma_launch_prep_bt_{sch}_{dt}(const lcma::PrepParams *p, int gx, int gy, void *stream);')
    return "\n".join(L)


def prep_kernels(variants: list[Variant]) -> list[tuple[str, str]]:
    """(scheme, dtype) pairs that need an offline Combine-B kernel: those with a prepared-B GEMM kernel."""
    return sorted({(v.scheme, v.dtype) for v in variants if v.pb})


# Measured rates of the stand-alone Combine-A / Combine-B / Combine-H kernels (algorithmic bytes per second at LLM
# sizes on MI355X, rocprofv3), per scheme and element size; used by the cost model of the unfused dataflow.
STAGE_RATES = {  # (scheme, 16-bit?) -> (Combine A, Combine B, Combine H)
    ("strassen", True): (5.6e12, 4.5e12, 5.2e12), ("strassen", False): (5.0e12, 4.5e12, 5.8e12),
    ("laderman", True): (6.0e12, 4.5e12, 4.6e12), ("laderman", False): (5.0e12, 3.0e12, 5.0e12),
    ("strassen2", True): (6.3e12, 4.2e12, 5.1e12), ("strassen2", False): (3.5e12, 3.0e12, 5.6e12),
}


def stage_kernels(variants: list[Variant]) -> list[tuple[str, str]]:
    """(scheme, dtype) pairs that get the stand-alone Combine-A and Combine-H kernels of the unfused
    dataflows: those with a GEMM kernel that takes both operands from planes."""
    return sorted({(v.scheme, v.dtype) for v in variants if v.pa})


def float_sum(terms: list[tuple[int, str]]) -> str:
    """Left-to-right fp32 sum of signed terms, parenthesised so that the order is the written one."""
    expr = ""
    for c, e in terms:
        mag = e if abs(c) == 1 else f"{float(abs(c))}f * {e}"
        if not expr:
            expr = mag if c > 0 else f"-{mag}"
        else:
            expr = f"({expr} {'+' if c > 0 else '-'} {mag})"
    return expr or "0.f"


# Algorithm 1 with fp16 storage: products whose left combination also gets its rounding residual multiplied (as a further
# plane pair: the residual of At_r beside a second copy of Bt_r, with the W row of r), the compensation the fused kernels
# of the scheme use (see with_residuals): without it <3,3,3;23> lands at 4.04 x the plain kernel's error.
STAGE_COMP = {("laderman", "f16"): (3, 6)}


def stage_planes(s: Scheme, dtype: str) -> int:
    return s.R + len(STAGE_COMP.get((s.name, dtype), ()))


def emit_stage(s0: Scheme, dtype: str) -> str:
    """Stand-alone Combine A (Eq. 3; sums in fp32, ascending (i, l), one rounding to the compute type) and
    Combine H (Eq. 6; sums in fp32, ascending r, one rounding to the storage type) for one scheme and
    storage type: stages 1 and 4 of Algorithm 1.  With compensated products (STAGE_COMP) every stage works on
    the longer list of planes, and the Combine B kernels for it are emitted here as well."""
    in_t, ct_t = CPP_TYPES[dtype]
    s, residual = with_residuals(s0, STAGE_COMP.get((s0.name, dtype), ()))
    a_blocks = sorted({(i, l) for r in range(s.R) for i in range(s.m) for l in range(s.k) if s.U[r, i, l]})
    L = []
    w = L.append
    w(f"// GENERATED by gen/generate.py - do not edit.  Stand-alone Combine A and Combine H of scheme {s.name} <{s.m},{s.k},{s.n};{s.R}>, dtype {dtype}.")
    w('#include "lcma_combine_h.hpp"')
    if dtype == "bf16":
        w('#include "lcma_fp8.hpp"')
    w("namespace {")
    w("using namespace lcma;")
    w("struct CombA {  // block A_{i,l} takes the place of block (j, l) of an N x K weight matrix")
    w(f"    static constexpr int NB = {len(a_blocks)}, NP = {s.R};")
    w("    // planes that hold what rounding the sum to the compute type loses (the sum is that of the plane's source product)")
    w(f"    static LCMA_DEV constexpr bool residual(int r) {{ return r >= {s0.R}; }}")
    for fn, vals in (("b_j", [b[0] for b in a_blocks]), ("b_l", [b[1] for b in a_blocks])):
        w(f"    static LCMA_DEV constexpr int {fn}(int t) {{ constexpr int v[] = {{{', '.join(map(str, vals))}}}; return v[t]; }}")
    w("    static LCMA_DEV float comb(const float (&in)[NB], int r) {")
    w("#pragma clang fp contract(off)")
    w("        switch (r) {")
    for r in range(s.R):
        terms = [(int(s.U[r, i, l]), f"in[{a_blocks.index((i, l))}]") for (i, l) in a_blocks if s.U[r, i, l]]
        w(f"        case {r}: return {float_sum(terms)};")
    w("        default: return 0.f;")
    w("        }")
    w("    }")
    w("};")
    w("struct CombH {")
    w(f"    static constexpr int NP = {s.R}, NC = {s.m * s.n};")
    w(f"    static LCMA_DEV constexpr int c_i(int o) {{ return o / {s.n}; }}")
    w(f"    static LCMA_DEV constexpr int c_j(int o) {{ return o % {s.n}; }}")
    w("    static LCMA_DEV float comb(const float (&in)[NP], int o) {")
    w("#pragma clang fp contract(off)")
    w("        switch (o) {")
    for i in range(s.m):
        for j in range(s.n):
            terms = [(int(s.W[r, i, j]), f"in[{r}]") for r in range(s.R) if s.W[r, i, j]]
            w(f"        case {i * s.n + j}: return {float_sum(terms)};")
    w("        default: return 0.f;")
    w("        }")
    w("    }")
    w("};")
    if residual:
        L += comb_b_struct(s, "CombB")
    w("} // namespace")
    w("")
    if residual:
        for kind, fn in (("b", "prepare_b_tile"), ("bt", "prepare_bt_tile")):
            w(f'extern "C" __global__ __launch_bounds__(256) void lcma_k_comb_{kind}_{s.name}_{dtype}(const lcma::PrepParams p) {{')
            w(f"    {fn}<{in_t}, {ct_t}, CombB>(p);")
            w("}")
            w("")
            w(f'extern "C" int lcma_launch_comb_{kind}_{s.name}_{dtype}(const lcma::PrepParams *p, int gx, int gy, void *stream) {{')
            seg = " / kPrepBSegments + (gy % kPrepBSegments != 0)" if kind == "b" else ""
            w(f"    lcma_k_comb_{kind}_{s.name}_{dtype}<<<dim3(gy{seg}, gx), dim3(256), 0, (hipStream_t)stream>>>(*p);")
            w("    return (int)hipGetLastError();")
            w("}")
            w("")
    w(f'extern "C" __global__ __launch_bounds__(256) void lcma_k_comb_a_{s.name}_{dtype}(const lcma::PrepParams p) {{')
    w(f"    prepare_bt_tile<{in_t}, {ct_t}, CombA>(p);")
    w("}")
    w("")
    w(f'extern "C" int lcma_launch_comb_a_{s.name}_{dtype}(const lcma::PrepParams *p, int gx, int gy, void *stream) {{')
    w(f"    lcma_k_comb_a_{s.name}_{dtype}<<<dim3(gy, gx), dim3(256), 0, (hipStream_t)stream>>>(*p);")
    w("    return (int)hipGetLastError();")
    w("}")
    w("")
    if dtype == "bf16":
        w("// Combine A with the FP8 quantisation fused in (Eq. 3; E4M3 codes and 1 x 128 power-of-two scales)")
        w(f'extern "C" __global__ __launch_bounds__(256) void lcma_k_fp8_comb_a_{s.name}(const lcma::Fp8QuantParams p) {{')
        w("    fp8_combine_quantize_tile<CombA>(p);")
        w("}")
        w("")
        w(f'extern "C" int lcma_launch_fp8_comb_a_{s.name}(const lcma::Fp8QuantParams *p, int gx, int gy, void *stream) {{')
        w(f"    lcma_k_fp8_comb_a_{s.name}<<<dim3(gy, gx), dim3(256), 0, (hipStream_t)stream>>>(*p);")
        w("    return (int)hipGetLastError();")
        w("}")
        w("")
    w(f'extern "C" __global__ __launch_bounds__(256) void lcma_k_comb_h_{s.name}_{dtype}(const lcma::CombHParams p) {{')
    w(f"    combine_h_tile<{in_t}, {ct_t}, CombH>(p);")
    w("}")
    w("")
    w(f'extern "C" int lcma_launch_comb_h_{s.name}_{dtype}(const lcma::CombHParams *p, int gx, int gy, void *stream) {{')
    w(f"    lcma_k_comb_h_{s.name}_{dtype}<<<dim3(gy, gx), dim3(256), 0, (hipStream_t)stream>>>(*p);")
    w("    return (int)hipGetLastError();")
    w("}")
    if dtype != "f32":  # the same sums from planes that hold the products in fp32
        w("")
        w(f'extern "C" __global__ __launch_bounds__(256) void lcma_k_comb_h32_{s.name}_{dtype}(const lcma::CombHParams p) {{')
        w(f"    combine_h_tile<{in_t}, F32, CombH>(p);")
        w("}")
        w("")
        w(f'extern "C" int lcma_launch_comb_h32_{s.name}_{dtype}(const lcma::CombHParams *p, int gx, int gy, void *stream) {{')
        w(f"    lcma_k_comb_h32_{s.name}_{dtype}<<<dim3(gy, gx), dim3(256), 0, (hipStream_t)stream>>>(*p);")
        w("    return (int)hipGetLastError();")
        w("}")
    return "\n".join(L) + "\n"


def comb_b_struct(s: Scheme, name: str) -> list[str]:
    """The generated description of Combine B (Eq. 4) for the kernels of csrc/lcma_prepare_b.hpp: raw blocks, planes,
    the signed fp32 sum of plane r in ascending (l, j) order."""
    b_blocks = sorted({(l, j) for r in range(s.R) for l in range(s.k) for j in range(s.n) if s.V[r, l, j]})
    L = []
    w = L.append
    w(f"struct {name} {{")
    w(f"    static constexpr int NB = {len(b_blocks)}, NP = {s.R};")
    for fn, vals in (("b_l", [b[0] for b in b_blocks]), ("b_j", [b[1] for b in b_blocks])):
        w(f"    static LCMA_DEV constexpr int {fn}(int t) {{ constexpr int v[] = {{{', '.join(map(str, vals))}}}; return v[t]; }}")
    w("    static LCMA_DEV constexpr bool residual(int) { return false; }")
    w("    // Bt_r at one element position; r is a literal at every call site, so the switch folds")
    w("    static LCMA_DEV float comb(const float (&in)[NB], int r) {")
    w("#pragma clang fp contract(off)")
    w("        switch (r) {")
    for r in range(s.R):
        # ascending (l, j), left to right: the order the stored result is defined in
        terms = [(int(s.V[r, l, j]), f"in[{b_blocks.index((l, j))}]") for (l, j) in b_blocks if s.V[r, l, j]]
        w(f"        case {r}: return {float_sum(terms)};")
    w("        default: return 0.f;")
    w("        }")
    w("    }")
    w("};")
    return L


def emit_prep_b(s: Scheme, dtype: str) -> str:
    """Offline Combine B (Eq. 4) for one scheme and storage type; sums in fp32, ascending (l, j)."""
    in_t, ct_t = CPP_TYPES[dtype]
    L = []
    w = L.append
    w(f"// GENERATED by gen/generate.py - do not edit.  Offline Combine B of scheme {s.name} <{s.m},{s.k},{s.n};{s.R}>, dtype {dtype}.")
    w('#include "lcma_prepare_b.hpp"')
    if dtype == "bf16":
        w('#include "lcma_fp8.hpp"')
    w("namespace {")
    w("using namespace lcma;")
    L += comb_b_struct(s, "Comb")
    w("} // namespace")
    w("")
    w(f'extern "C" __global__ __launch_bounds__(256) void lcma_k_prep_b_{s.name}_{dtype}(const lcma::PrepParams p) {{')
    w(f"    prepare_b_tile<{in_t}, {ct_t}, Comb>(p);")
    w("}")
    w("")
    w(f'extern "C" int lcma_launch_prep_b_{s.name}_{dtype}(const lcma::PrepParams *p, int gx, int gy, void *stream) {{')
    w("    // gy counts 64-byte segments of a row of a plane; a work-group writes kPrepBSegments of them")
    w(f"    lcma_k_prep_b_{s.name}_{dtype}<<<dim3(gy / kPrepBSegments + (gy % kPrepBSegments != 0), gx), dim3(256), 0, (hipStream_t)stream>>>(*p);")
    w("    return (int)hipGetLastError();")
    w("}")
    w("")
    w("// the same for a weight matrix stored N x K")
    w(f'extern "C" __global__ __launch_bounds__(256) void lcma_k_prep_bt_{s.name}_{dtype}(const lcma::PrepParams p) {{')
    w(f"    prepare_bt_tile<{in_t}, {ct_t}, Comb>(p);")
    w("}")
    w("")
    w(f'extern "C" int lcma_launch_prep_bt_{s.name}_{dtype}(const lcma::PrepParams *p, int gx, int gy, void *stream) {{')
    w(f"    lcma_k_prep_bt_{s.name}_{dtype}<<<dim3(gy, gx), dim3(256), 0, (hipStream_t)stream>>>(*p);")
    w("    return (int)hipGetLastError();")
    w("}")
    if dtype == "bf16":
        w("")
        w("// Combine B for N x K weights with the FP8 quantisation fused in (Eq. 4; E4M3 codes and 1 x 128 power-of-two scales)")
        w(f'extern "C" __global__ __launch_bounds__(256) void lcma_k_fp8_prep_w_{s.name}(const lcma::Fp8QuantParams p) {{')
        w("    fp8_combine_quantize_tile<Comb>(p);")
        w("}")
        w("")
        w(f'extern "C" int lcma_launch_fp8_prep_w_{s.name}(const lcma::Fp8QuantParams *p, int gx, int gy, void *stream) {{')
        w(f"    lcma_k_fp8_prep_w_{s.name}<<<dim3(gy, gx), dim3(256), 0, (hipStream_t)stream>>>(*p);")
        w("    return (int)hipGetLastError();")
        w("}")
    return "\n".join(L) + "\n"


def scheme_hash(s: Scheme) -> int:
    """FNV-1a over (m,k,n,R) as int32 and the int8 coefficients, matching the library's."""
    h = 0xCBF29CE484222325
    data = np.array([s.m, s.k, s.n, s.R], np.int32).tobytes()
    for T in (s.U, s.V, s.W):
        data += T.astype(np.int8).tobytes()
    for byte in data:
        h = ((h ^ byte) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def emit_builtin_inc(schemes: dict[str, Scheme]) -> str:
    names = ["strassen", "strassen2", "laderman"] + further_schemes(schemes)
    L = ["// GENERATED by gen/generate.py from schemes/*.txt - do not edit."]
    L.append("static const char *const kBuiltinNames[] = {" + ", ".join(f'"{n}"' for n in names) + "};")
    L.append("static const int kBuiltinIds[] = {" + ", ".join(str(SCHEME_IDS[n]) for n in names) + "};")
    L.append("static const char *const kBuiltinTexts[] = {")
    for n in names:
        body = "".join(f'    "{line}\\n"\n' for line in schemes[n].text().splitlines())
        L.append(body.rstrip("\n") + ",")
    L.append("};")
    L.append(f"static const int kBuiltinCount = {len(names)};")
    return "\n".join(L) + "\n"


def manifest(schemes: dict[str, Scheme] | None = None) -> list[Variant]:
    """The kernels that are built.  `eff` is the fraction of the dtype's dense MFMA peak that the
    variant's own MFMA work sustained on MI355X at large shapes (4096^3 and up, this library's
    bench); the library launches, among the variants of a scheme whose tile divides the shape, the one
    with the smallest predicted time (eff and wave quantisation).  Eight-wave work-groups (two waves
    per SIMD) beat four-wave ones throughout."""
    V = []
    for dt in ("bf16", "f16"):
        e = (lambda bf, f: bf if dt == "bf16" else f)  # bf16 pays for its conversion to fp16
        V += [
            Variant("plain", dt, 256, 256, 64, wgm=2, wgn=4, eff=e(0.447, 0.426)),
            Variant("plain", dt, 256, 128, 32, occ=2, eff=e(0.375, 0.363)),
            Variant("plain", dt, 128, 128, 64, occ=2, eff=e(0.332, 0.317)),
            Variant("plain", dt, 64, 64, 32, eff=e(0.172, 0.163)),
            # fragment-combine kernels: raw blocks in LDS, every wave forms the 7 operand pairs;
            # "i": staging spread over the MFMA phase
            Variant("strassen", dt, 128, 64, 32, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, eff=e(0.268, 0.291)),
            Variant("strassen", dt, 64, 128, 32, chunk=7, fc=1, wgm=2, wgn=4, pipe=2, eff=e(0.265, 0.287)),
            Variant("strassen", dt, 64, 64, 32, chunk=7, fc=1, occ=2, pipe=2, eff=e(0.241, 0.263)),
            # B from the offline Combine-B kernel (static weights): only the A side is combined on fragments
            Variant("strassen", dt, 128, 64, 32, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, pb=1, eff=e(0.264, 0.252)),
            Variant("strassen", dt, 64, 64, 32, chunk=7, fc=1, pipe=2, pb=1, eff=e(0.202, 0.194)),
            Variant("strassen", dt, 128, 64, 32, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, pb=1, dl=1, eff=e(0.233, 0.243), rank=90),
            # ablation variants: staging in one phase; a third LDS stage; combinations formed while staging
            Variant("strassen", dt, 128, 64, 32, chunk=7, fc=1, wgm=4, wgn=2, eff=e(0.261, 0.280), rank=90),
            Variant("strassen", dt, 128, 64, 32, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, stages=3, eff=e(0.268, 0.286), rank=90),
            Variant("strassen", dt, 64, 64, 32, chunk=7, eff=e(0.099, 0.114), rank=90),
            # Algorithm 2's r loop: one product at a time, combinations formed while staging
            Variant("strassen", dt, 128, 128, 32, chunk=1, eff=e(0.149, 0.179)),
            Variant("laderman", dt, 128, 64, 32, chunk=1, eff=e(0.060, 0.068), rank=90 if dt == "f16" else 0),
            Variant("laderman", dt, 64, 64, 32, chunk=1, eff=e(0.039, 0.043), rank=90 if dt == "f16" else 0),
        ]
    # Laderman with fp16 storage: rounding its 3- and 7-term combinations to fp16 costs 4.05x the error
    # of the plain kernel; multiplying the residual of the left operand of products 4 and 7 (both
    # three-term on each side) as well brings it under the 4x bound for 2 extra products out of 23.
    # The uncompensated kernels above stay as ablation variants (rank 90).
    V += [Variant("laderman", "bf16", 128, 64, 32, chunk=1, pb=1, eff=0.088),
          Variant("laderman", "f16", 128, 64, 32, chunk=1, pb=1, comp=(3, 6), eff=0.09)]
    V += [Variant("strassen2", "bf16", 64, 64, 32, chunk=7, pb=1, eff=0.104),
          Variant("strassen2", "f32", 64, 64, 16, chunk=7, pb=1, eff=0.579),
          Variant("laderman", "f32", 64, 64, 16, chunk=1, pb=1, eff=0.473)]
    V += [Variant("laderman", "f16", 128, 64, 32, chunk=1, comp=(3, 6), eff=0.064),
          Variant("laderman", "f16", 64, 64, 32, chunk=1, comp=(3, 6), eff=0.041)]
    # two-level Strassen: with fp16 storage its four-term sums exceed the 4x error bound, so it is
    # generated for bf16 (sums nearly exact in fp16) and fp32 only
    V += [
        Variant("strassen2", "bf16", 64, 64, 32, chunk=7, eff=0.065),
        Variant("strassen2", "bf16", 64, 64, 32, chunk=1, eff=0.030),
    ]
    V += [
        Variant("plain", "f32", 256, 128, 16, wgm=2, wgn=4, eff=0.917),
        Variant("plain", "f32", 128, 128, 16, occ=2, eff=0.916),
        Variant("plain", "f32", 64, 64, 16, eff=0.856),
        Variant("strassen", "f32", 64, 64, 16, chunk=7, fc=1, occ=2, pipe=2, eff=0.87),
        Variant("strassen", "f32", 128, 64, 16, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, eff=0.802),
        Variant("strassen", "f32", 128, 64, 16, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, pb=1, eff=0.875),
        Variant("strassen", "f32", 64, 64, 16, chunk=7, fc=1, pipe=2, pb=1, eff=0.74),
        Variant("strassen", "f32", 128, 64, 16, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, pb=1, dl=1, eff=0.852, rank=90),
        Variant("strassen", "f32", 64, 64, 16, chunk=7, fc=1, occ=2, eff=0.795, rank=90),
        Variant("strassen", "f32", 64, 64, 16, chunk=7, eff=0.656, rank=90),
        Variant("strassen", "f32", 128, 64, 16, chunk=1, eff=0.613),
        Variant("laderman", "f32", 64, 64, 16, chunk=1, eff=0.399),
        Variant("strassen2", "f32", 64, 64, 16, chunk=7, eff=0.534),
    ]
    # Further scheme files get Algorithm 2's r loop (one product at a time, the m*n C tiles in registers)
    # on a 64 x 64 tile, which fits any grid up to m*n = 24.
    schemes = load_schemes() if schemes is None else schemes
    for name in further_schemes(schemes):
        sch = schemes[name]
        assert (sch.m * sch.n + 1) * 16 <= ACC_REG_BUDGET, f"{name}: {sch.m}x{sch.n} C tiles do not fit the registers"
        V += [Variant(name, "bf16", 64, 64, 32, chunk=1, eff=0.04), Variant(name, "f16", 64, 64, 32, chunk=1, eff=0.04),
              Variant(name, "f32", 64, 64, 16, chunk=1, eff=0.4)]
    # Both raw operands straight into LDS by direct loads, three stages ("s3dt"): needs B given N x K and a storage
    # type that is multiplied as it is.  fp16: +3% over the register-staged twin, chosen by lcma_gemm_nt; fp32: +1%
    # over its twin but below the 64 x 64 kernel, kept by name.  (bf16 would have to be converted on the fragments:
    # measured 626 against 764 TFLOP/s, not generated.)
    # the plain fp16 kernel the same way: +3% over the register-staged N x K kernel (batched over planes, for the
    # GEMM stage of lcma_gemm_unfused, it measured +3% at 4096^3 and -1 to -3% at the larger shapes: not generated)
    V += [Variant("plain", "f16", 256, 256, 32, wgm=2, wgn=4, fc=1, pipe=2, stages=3, dl=1, tb=1, eff=0.45)]
    V += [Variant("strassen", "f16", 128, 64, 32, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, stages=3, dl=1, tb=1, eff=0.318),
          Variant("strassen", "f32", 128, 64, 16, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, stages=3, dl=1, tb=1, eff=0.847, rank=90)]
    # Winograd's form of Strassen's algorithm (a further scheme file): the fragment-combine kernels with the
    # common sums shared, 4 + 4 additions per fragment set instead of 5 + 5.  fp16 storage forms its 3- and
    # 4-term sums in fp32 (no sharing) and keeps the default r-loop kernel only.
    if "winograd" in schemes:
        for tb in (0, 1):
            V += [Variant("winograd", "bf16", 128, 64, 32, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, tb=tb, eff=0.282 if tb else 0.271),
                  Variant("winograd", "bf16", 64, 64, 32, chunk=7, fc=1, occ=2, pipe=2, tb=tb, eff=0.250 if tb else 0.243),
                  Variant("winograd", "f32", 64, 64, 16, chunk=7, fc=1, occ=2, pipe=2, tb=tb, eff=0.90),
                  Variant("winograd", "f32", 128, 64, 16, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, tb=tb, eff=0.88)]
        V += [Variant("winograd", "bf16", 128, 64, 32, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, pb=1, eff=0.27),
              Variant("winograd", "f32", 128, 64, 16, chunk=7, fc=1, wgm=4, wgn=2, pipe=2, pb=1, eff=0.88)]
    # The unfused dataflows the paper starts from, built to be measured against the fused kernels
    # (lcma_gemm_unfused; rank 95: never chosen by lcma_gemm, not callable by name).  Algorithm 1: a
    # batched plain GEMM over the R planes written by the stand-alone Combine-A / Combine-B kernels ("g");
    # Algorithm 2 as printed: a GEMM + Combine-H kernel that takes both operands from planes ("ab").
    for dt in ("f16", "f32"):
        tk = 64 if dt == "f16" else 16
        V += [Variant("plain", dt, 256, 256 if dt == "f16" else 128, tk, wgm=2, wgn=4, tb=1, batch=1, rank=95,
                      eff=0.477 if dt == "f16" else 0.88),
              Variant("plain", dt, 128, 128, tk, occ=2, tb=1, batch=1, rank=95, eff=0.35 if dt == "f16" else 0.86)]
    for dt in ("bf16", "f16", "f32"):
        tk = 16 if dt == "f32" else 32
        # (eff: what the GEMM stage of lcma_gemm_unfused level 2 sustains with each at 4096^3 and at the FFN shape: the choice
        # between the two goes by it)
        V += [Variant("strassen", dt, 64, 64, tk, chunk=7, pa=1, pb=1, rank=95, eff=0.16 if dt != "f32" else 0.70),
              Variant("strassen", dt, 128, 128 if dt != "f32" else 64, tk, chunk=1, pa=1, pb=1, rank=95,
                      eff=0.30 if dt != "f32" else 0.85),
              Variant("laderman", dt, 128 if dt != "f32" else 64, 64, tk, chunk=1, pa=1, pb=1, rank=95)]
        if dt != "f16":
            V += [Variant("strassen2", dt, 64, 64, tk, chunk=7, pa=1, pb=1, rank=95)]
    # Every kernel that lcma_gemm can pick for the paper's schemes also exists for B given as the N x K
    # weight matrix ("t"): its B tiles are staged like A's, with 16-byte loads and no transposition.
    from dataclasses import replace
    V += [replace(v, tb=1, name="") for v in V if not v.pb and not v.tb and v.rank < 90 and SCHEME_IDS[v.scheme] <= 3]
    return [v.finish() for v in V]


def generate(out_dir: str) -> list[str]:
    """Writes the generated sources into out_dir; returns the .hip files to compile."""
    os.makedirs(out_dir, exist_ok=True)
    schemes = load_schemes()
    variants = manifest(schemes)
    hips = []

    def put(name, text):
        path = os.path.join(out_dir, name)
        old = None
        if os.path.exists(path):
            with open(path) as f:
                old = f.read()
        if old != text:
            with open(path, "w") as f:
                f.write(text)
        return path

    for v in variants:
        s = schemes[v.scheme]
        regs, lds = plan(with_residuals(s, v.comp)[0], v)[:2]
        assert regs <= ACC_REG_BUDGET, f"{v.name}: {regs} accumulator registers exceed the budget"
        assert lds <= LDS_BUDGET, f"{v.name}: {lds} bytes of LDS exceed the budget"
        hips.append(put(f"k_{v.name}.hip", emit_kernel(s, v)))
    for sch, dt in prep_kernels(variants):
        hips.append(put(f"k_prep_b_{sch}_{dt}.hip", emit_prep_b(schemes[sch], dt)))
    for sch, dt in stage_kernels(variants):
        hips.append(put(f"k_stage_{sch}_{dt}.hip", emit_stage(schemes[sch], dt)))
    put("registry.cc", emit_registry(schemes, variants))
    put("builtin_schemes.inc", emit_builtin_inc(schemes))
    keep = {os.path.basename(h) for h in hips} | {"registry.cc", "builtin_schemes.inc"}
    for f in os.listdir(out_dir):
        if f not in keep and (f.endswith(".hip") or f.endswith(".o")) and f[:-len(os.path.splitext(f)[1])] + ".hip" not in keep:
            os.remove(os.path.join(out_dir, f))
    return hips


if __name__ == "__main__":
    import sys
    for path in generate(sys.argv[1] if len(sys.argv) > 1 else os.path.join(PKG, "csrc", "generated")):
        print(path)
