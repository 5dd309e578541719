"""Generates gaunt_table.h: coupling tables for the tensor product with features up to degree 2 or 3.

The coupling of path p = (l1, l2, l3) is the real Gaunt integral
    G[m1, m2, m3] = (1/4pi) Int Y_{l1 m1} Y_{l2 m2} Y_{l3 m3} dOmega
scaled by a positive factor so that sum G^2 = 2 l3 + 1.  Here it is evaluated in closed form:
every real harmonic (component normalisation, order m = -l..l) is a polynomial in (x, y, z),
the triple product is expanded into monomials, and each monomial is integrated exactly with
    <x^a y^b z^c> = (a-1)!! (b-1)!! (c-1)!! / (a+b+c+1)!!   (all exponents even, else 0).
Coefficients carry square roots, so arithmetic is done in floats of 50 digits (decimal) and
printed to float precision with entries below 1e-12 dropped.

Run:  python gen_gaunt.py   (rewrites gaunt_table.h next to this file)
"""
from __future__ import annotations

import os
from decimal import Decimal, getcontext
from itertools import product

getcontext().prec = 50
D = Decimal


def dfact(n: int) -> int:  # double factorial with (-1)!! = 1
    r = 1
    while n > 1:
        r *= n
        n -= 2
    return r


def mono_mean(a: int, b: int, c: int) -> Decimal:
    if a % 2 or b % 2 or c % 2:
        return D(0)
    return D(dfact(a - 1) * dfact(b - 1) * dfact(c - 1)) / D(dfact(a + b + c + 1))


s3, s5, s15 = D(3).sqrt(), D(5).sqrt(), D(15).sqrt()
c35, c105, c21, c7 = (D(35) / 8).sqrt(), D(105).sqrt(), (D(21) / 8).sqrt(), D(7).sqrt() / 2
# polynomials: dict {(a,b,c): coeff}, homogeneous (1 = x^2 + y^2 + z^2 put in where the textbook form is not)
Y = [
    {(0, 0, 0): D(1)},
    {(0, 1, 0): s3}, {(0, 0, 1): s3}, {(1, 0, 0): s3},
    {(1, 1, 0): s15}, {(0, 1, 1): s15},
    # (sqrt5/2)(3 z^2 - 1)  ->  (sqrt5/2)(2 z^2 - x^2 - y^2)
    {(0, 0, 2): s5, (2, 0, 0): -s5 / 2, (0, 2, 0): -s5 / 2},
    {(1, 0, 1): s15}, {(2, 0, 0): s15 / 2, (0, 2, 0): -s15 / 2},
    # degree 3, m = -3..3: sqrt(35/8) y (3x^2 - y^2); sqrt105 xyz; sqrt(21/8) y (5z^2 - 1); (sqrt7/2) z (5z^2 - 3);
    # sqrt(21/8) x (5z^2 - 1); (sqrt105/2) z (x^2 - y^2); sqrt(35/8) x (x^2 - 3y^2)
    {(2, 1, 0): 3 * c35, (0, 3, 0): -c35},
    {(1, 1, 1): c105},
    {(0, 1, 2): 4 * c21, (2, 1, 0): -c21, (0, 3, 0): -c21},
    {(0, 0, 3): 2 * c7, (2, 0, 1): -3 * c7, (0, 2, 1): -3 * c7},
    {(1, 0, 2): 4 * c21, (3, 0, 0): -c21, (1, 2, 0): -c21},
    {(2, 0, 1): c105 / 2, (0, 2, 1): -c105 / 2},
    {(3, 0, 0): c35, (1, 2, 0): -3 * c35},
]
OFF = [0, 1, 4, 9]


def paths_of(lmax):
    return [(l1, l2, l3) for l1 in range(lmax + 1) for l2 in range(lmax + 1) for l3 in range(lmax + 1)
            if abs(l1 - l2) <= l3 <= l1 + l2 and (l1 + l2 + l3) % 2 == 0]


def pmul(p, q):
    r = {}
    for (a, c1), (b, c2) in product(p.items(), q.items()):
        k = (a[0] + b[0], a[1] + b[1], a[2] + b[2])
        r[k] = r.get(k, D(0)) + c1 * c2
    return r


def integral(p):
    return sum(c * mono_mean(*k) for k, c in p.items())


def tables(lmax):
    out = []
    for (l1, l2, l3) in paths_of(lmax):
        ent = {}
        for m1 in range(2 * l1 + 1):
            for m2 in range(2 * l2 + 1):
                pq = pmul(Y[OFF[l1] + m1], Y[OFF[l2] + m2])
                for m3 in range(2 * l3 + 1):
                    g = integral(pmul(pq, Y[OFF[l3] + m3]))
                    if abs(g) > D("1e-30"):
                        ent[(OFF[l1] + m1, OFF[l2] + m2, OFF[l3] + m3)] = g
        norm = sum(g * g for g in ent.values())
        scale = (D(2 * l3 + 1) / norm).sqrt()
        out.append({k: g * scale for k, g in ent.items()})
    return out


def f(c: Decimal) -> str:
    t = f"{float(c):.9g}"
    if "." not in t and "e" not in t:
        t += ".0"
    return t + "f"


def emit_tab(lmax, L):
    PATHS = paths_of(lmax)
    T = tables(lmax)
    nm = (lmax + 1) ** 2
    nnz = sum(len(t) for t in T)
    npp = (len(PATHS) + 3) // 4 * 4
    cy_ld = (nnz + 1 + 3) // 4 * 4
    L.append(f"// ---- l <= {lmax}: {len(PATHS)} paths, {nnz} non-zero coupling entries, {nm} components")
    L.append(f"template <>\nstruct Tab<{lmax}> {{")
    L.append(f"  static constexpr int LMAX = {lmax};")
    L.append(f"  static constexpr int NM = {nm};        // components of a feature vector")
    L.append(f"  static constexpr int NPATH = {len(PATHS)};")
    L.append(f"  static constexpr int NPP = {npp};      // path values per channel as stored (padded to a multiple of four)")
    L.append(f"  static constexpr int NNZ = {nnz};")
    L.append(f"  static constexpr int CY_LD = {cy_ld};  // floats per edge in a table of per-edge products: NNZ entries, one more value, padding to 16 bytes")
    L.append(f"  static constexpr int TAB_LOADS = {(cy_ld + 63) // 64};  // 64-float pieces a wave fetches to hold one table")
    L.append("  // l1, l2, l3 of each path")
    L.append("  static constexpr int PATH_L[NPATH][3] = {" + ", ".join("{%d,%d,%d}" % p for p in PATHS) + "};")
    ents, slots = [], []
    for p, t in enumerate(T):
        by = {}
        for (a, b, c), g in t.items():
            by.setdefault(c, []).append((a, b, g))
        for c, terms in sorted(by.items()):
            slots.append((p, c))
            for a, b, g in terms:
                ents.append((p, a, b, c, g, len(slots) - 1))
    assert len(ents) == nnz
    yslots = sorted({(e[0], e[2]) for e in ents})
    arr = lambda name, typ, vals: L.append(f"  static constexpr {typ} {name}[{len(vals)}] = {{" + ", ".join(vals) + "};")
    L.append("  // entry tables: T^p[m1, m2, m3] = ENT_COEF[n] for n = 0..NNZ-1; slot s = (path, m3), yslot = (path, m2);")
    L.append("  // ENT_*FIRST[n]: entry n is the first of its slot / its path / its yslot in this order")
    L.append(f"  static constexpr int NSLOT = {len(slots)};")
    L.append(f"  static constexpr int NYSLOT = {len(yslots)};")
    arr("ENT_M1", "int", [str(e[1]) for e in ents])
    arr("ENT_M2", "int", [str(e[2]) for e in ents])
    arr("ENT_SLOT", "int", [str(e[5]) for e in ents])
    arr("ENT_COEF", "float", [f(e[4]) for e in ents])
    ys_of = [yslots.index((e[0], e[2])) for e in ents]
    arr("ENT_YSLOT", "int", [str(y) for y in ys_of])
    arr("ENT_SFIRST", "bool", ["true" if n == 0 or ents[n - 1][5] != e[5] else "false" for n, e in enumerate(ents)])
    arr("ENT_PFIRST", "bool", ["true" if n == 0 or ents[n - 1][0] != e[0] else "false" for n, e in enumerate(ents)])
    arr("ENT_YFIRST", "bool", ["true" if ys_of.index(y) == n else "false" for n, y in enumerate(ys_of)])
    arr("ENT_SLAST", "bool", ["true" if n == nnz - 1 or ents[n + 1][5] != e[5] else "false" for n, e in enumerate(ents)])
    # the entries once more, ordered by (path, m2): runs of one yslot are contiguous, and so are the paths
    yord = sorted(range(nnz), key=lambda n: (ents[n][0], ents[n][2], n))
    L.append("  // YORD: the entries ordered by (path, m2); YORD_*: position k of that order starts / ends a run of one yslot or one path")
    arr("YORD", "int", [str(n) for n in yord])
    arr("YORD_YFIRST", "bool", ["true" if k == 0 or ys_of[yord[k - 1]] != ys_of[n] else "false" for k, n in enumerate(yord)])
    arr("YORD_YLAST", "bool", ["true" if k == nnz - 1 or ys_of[yord[k + 1]] != ys_of[n] else "false" for k, n in enumerate(yord)])
    arr("YORD_PFIRST", "bool", ["true" if k == 0 or ents[yord[k - 1]][0] != ents[n][0] else "false" for k, n in enumerate(yord)])
    arr("YORD_PLAST", "bool", ["true" if k == nnz - 1 or ents[yord[k + 1]][0] != ents[n][0] else "false" for k, n in enumerate(yord)])
    arr("SLOT_P", "int", [str(sl[0]) for sl in slots])
    arr("SLOT_M3", "int", [str(sl[1]) for sl in slots])
    arr("YSLOT_P", "int", [str(ys[0]) for ys in yslots])
    arr("YSLOT_M2", "int", [str(ys[1]) for ys in yslots])
    L.append("  // parity (-1)^l2 of each path: the couplings of the inverted direction are PATH_SIGN[p] times these")
    arr("PATH_SIGN", "float", ["-1.0f" if pp[1] % 2 else "1.0f" for pp in PATHS])
    L.append("  // the paths (l, l, 0), the only ones that reach the l = 0 output: their indices, and each path's position among them (-1: none)")
    last = [PATHS.index((l, l, 0)) for l in range(lmax + 1)]
    arr("LAST_PATHS", "int", [str(x) for x in last])
    arr("LAST_K", "int", [str(last.index(k)) if k in last else "-1" for k in range(len(PATHS))])
    L.append("  // parity (-1)^l of each component")
    arr("M_SIGN", "float", ["-1.0f" if l % 2 else "1.0f" for l in range(lmax + 1) for _ in range(2 * l + 1)])
    L.append("  // first component of each degree, and one past the last")
    arr("L_OFF", "int", [str(l * l) for l in range(lmax + 2)])
    L.append("};")
    L.append(f"// ENT_M2 and ENT_COEF of Tab<{lmax}> in device memory, for indexing at run time")
    L.append(f"static __device__ const int ENT_M2_DEV_{lmax}[{nnz}] = {{" + ", ".join(str(e[2]) for e in ents) + "};")
    L.append(f"static __device__ const float ENT_COEF_DEV_{lmax}[{nnz}] = {{" + ", ".join(f(e[4]) for e in ents) + "};")
    return PATHS, T


def emit():
    L = []
    L.append("// GENERATED by gen_gaunt.py -- do not edit.  Real Gaunt couplings of the even-parity paths (l1, l2, l3) with every")
    L.append("// degree <= LMAX (2 or 3), ordered by (l1, l2, l3), each scaled to sum of squares 2 l3 + 1.  Components are indexed")
    L.append("// 0..8 = (l=0; l=1: y,z,x; l=2: xy,yz,z2,xz,x2-y2) and 9..15 = the seven degree-3 harmonics m = -3..3.")
    L.append("// With the per-edge products cy[n] = ENT_COEF[n] * Y[ENT_M2[n]] precomputed (they do not depend on the channel),")
    L.append("// each coupling term costs one multiply-add.")
    L.append("#pragma once")
    L.append("#include <hip/hip_runtime.h>")
    L.append("namespace gaunt {")
    L.append("template <int LMAX>\nstruct Tab;")
    emit_tab(2, L)
    emit_tab(3, L)
    L.append("template <int LMAX> __device__ __forceinline__ int ent_m2_dev(int n);")
    L.append("template <> __device__ __forceinline__ int ent_m2_dev<2>(int n) { return ENT_M2_DEV_2[n]; }")
    L.append("template <> __device__ __forceinline__ int ent_m2_dev<3>(int n) { return ENT_M2_DEV_3[n]; }")
    L.append("template <int LMAX> __device__ __forceinline__ float ent_coef_dev(int n);")
    L.append("template <> __device__ __forceinline__ float ent_coef_dev<2>(int n) { return ENT_COEF_DEV_2[n]; }")
    L.append("template <> __device__ __forceinline__ float ent_coef_dev<3>(int n) { return ENT_COEF_DEV_3[n]; }")
    L.append("}  // namespace gaunt")
    return "\n".join(L) + "\n"


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.path.join(here, "gaunt_table.h"), "w") as fh:
        fh.write(emit())
    print("wrote gaunt_table.h")
