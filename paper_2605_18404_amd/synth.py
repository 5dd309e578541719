"""Seeded synthetic inputs for the four-phase MLIP training step.

This module only *draws numbers*: structures, species, parameter values, reference
labels and stage boundary tensors.  It contains none of the model's arithmetic (no
basis functions, no message passing, no derivatives), so both the CPU oracle's tests
and the HIP path's tests can take their inputs from it without sharing method code.

Random numbers come from a counter-based generator: value = splitmix64-finaliser of
(key(seed, stream) + (counter+1)*golden).  A uniform is the top 53 bits / 2^53, a normal
is Box-Muller on two consecutive uniforms.  Streams: 1 positions, 2 species, 3 params,
4 E_ref, 5 F_ref, 6 h_in, 7 g_out, 8 hdot_in, 9 v, 10 lam_out.

The five workloads stand in for the paper's mixed ODAC23 / OMat24 / OMol25 micro-batches
(Sec. 5.1 "Experimental Setup"), which are not available: periodic cubic cells of fixed
number density with a hard minimum distance, i.e. the shape (atoms, neighbours per atom,
channels, layers) rather than the chemistry.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

STREAM_POS, STREAM_SPECIES, STREAM_PARAMS, STREAM_EREF, STREAM_FREF = 1, 2, 3, 4, 5
STREAM_H_IN, STREAM_G_OUT, STREAM_HDOT_IN, STREAM_V, STREAM_LAM_OUT = 6, 7, 8, 9, 10
STREAM_ALPHA = 12  # (11 is taken by the graph-size recipe)
STREAM_CELL = 13

BASE_SEED = 18404000

KIND_INVARIANT, KIND_EQUIVARIANT, KIND_STAGE = 0, 1, 2
N_PATHS_LMAX2 = 11  # (l1,l2,l3) with l<=2, triangle rule, l1+l2+l3 even


def n_paths(l_max: int) -> int:
    """Number of coupling paths (l1, l2, l3), every degree <= l_max, triangle rule, l1 + l2 + l3 even (11 for 2, 23 for 3)."""
    return sum(1 for l1 in range(l_max + 1) for l2 in range(l_max + 1) for l3 in range(l_max + 1)
               if abs(l1 - l2) <= l3 <= l1 + l2 and (l1 + l2 + l3) % 2 == 0)


def _finalise(z: np.ndarray) -> np.ndarray:
    z = z ^ (z >> np.uint64(30))
    z = z * _M1
    z = z ^ (z >> np.uint64(27))
    z = z * _M2
    z = z ^ (z >> np.uint64(31))
    return z


def raw_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """`count` 64-bit words for counters start .. start+count-1 of (seed, stream)."""
    with np.errstate(over="ignore"):
        key = _finalise(np.array([seed], dtype=np.uint64) ^ (np.uint64(stream) * _GOLDEN))
        ctr = np.arange(start + 1, start + 1 + count, dtype=np.uint64)
        return _finalise(key + ctr * _GOLDEN)


def uniform(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 uniforms in [0, 1)."""
    return (raw_u64(seed, stream, start, count) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 standard normals; value i uses uniforms 2i and 2i+1 (Box-Muller, cosine branch)."""
    u = uniform(seed, stream, 2 * start, 2 * count).reshape(count, 2)
    u1 = u[:, 0] + 0.5 / 9007199254740992.0  # keep log() finite
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u[:, 1])


@dataclass(frozen=True)
class Workload:
    """Shape of one synthetic workload and of the model that runs on it."""
    name: str
    index: int
    kind: int                 # KIND_*
    n_structs: int
    atoms_per_struct: int
    box: float                # cubic cell edge, Angstrom
    n_species: int
    species_dist: str         # "uniform" | "zipf1.2"
    cutoff: float
    n_rbf: int
    channels: int
    n_layers: int
    edge_hidden: int
    edge_depth: int           # 2: K->H->C ; 3: K->H->H->C
    l_max: int
    gemm_bf16: bool
    force_weight: float = 10.0
    min_dist: float = 1.0
    cell_kind: str = "cubic"  # "cubic" | "triclinic" (sheared lattice, per structure) | "free" (molecule in vacuum: zero cell)
    gate: int = 0             # 1 (equivariant model): gated nonlinearity in the node update instead of the linear residual
    filter_fp32: int = 0      # bf16 workloads: 1 keeps the radial-filter jets in fp32 (rounding touches GEMM operands only)
    n_experts: int = 0        # > 0: the node-level matrices of every layer (update MLP / per-l mixing) are banks of this many experts

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def n_atoms(self) -> int:
        return self.n_structs * self.atoms_per_struct


def _box(n: int, density: float) -> float:
    return float((n / density) ** (1.0 / 3.0))


WORKLOADS: List[Workload] = [
    Workload("cfg0_tiny_invariant", 0, KIND_INVARIANT, 1, 64, 12.0, 2, "uniform", 5.0, 16, 32, 2, 32, 2, 0, False),
    Workload("cfg1_invariant_batch", 1, KIND_INVARIANT, 32, 192, _box(192, 0.08), 8, "zipf1.2", 6.0, 32, 128, 4, 128, 2, 0, False),
    Workload("cfg2_equivariant_batch", 2, KIND_EQUIVARIANT, 16, 256, _box(256, 0.08), 8, "zipf1.2", 6.0, 32, 64, 4, 64, 2, 2, True),
    Workload("cfg3_invariant_stage", 3, KIND_STAGE, 64, 128, _box(128, 0.08), 1, "uniform", 6.0, 32, 512, 4, 512, 3, 0, True),
    Workload("cfg4_equivariant_large", 4, KIND_EQUIVARIANT, 1, 20000, _box(20000, 0.1), 4, "uniform", 6.0, 32, 128, 6, 128, 2, 2, True),
]


def shrink(w: Workload, **kw) -> Workload:
    """A smaller variant of a workload (same recipe, other sizes) for oracle-speed parity cases."""
    return replace(w, **kw)


# ----------------------------------------------------------------------------- structures

def _periodic_dists(cands_new: np.ndarray, placed: np.ndarray, box: float, n_img: int) -> np.ndarray:
    """All distances (float64) from one point to placed points over images -n_img..n_img per axis."""
    d0 = placed - cands_new[None, :]
    if n_img == 0:
        d0 = d0 - box * np.round(d0 / box)
        return np.sqrt((d0 * d0).sum(-1))
    rng = np.arange(-n_img, n_img + 1, dtype=np.float64) * box
    sh = np.stack(np.meshgrid(rng, rng, rng, indexing="ij"), -1).reshape(-1, 3)
    d = d0[:, None, :] + sh[None, :, :]
    return np.sqrt((d * d).sum(-1)).reshape(-1)


def make_structure(seed: int, struct_index: int, n: int, box: float, cutoff: float,
                   min_dist: float = 1.0, shell: float = 1e-4) -> np.ndarray:
    """Random sequential insertion of n points in a periodic cube.

    A candidate (three uniforms scaled by the box, rounded to float32) is rejected if it
    comes closer than `min_dist` to a placed point, or if any pair distance (all images)
    falls within `shell` of the cutoff -- so that float32 and float64 neighbour tests
    agree on every pair.  Returns float32 [n,3], sorted by a coarse spatial grid.
    """
    min_image_ok = box >= 2.0 * (cutoff + shell)
    pts = np.zeros((n, 3), dtype=np.float64)
    placed = 0
    cand = 0
    base = struct_index * (1 << 32)
    chunk = 256
    while placed < n:
        u = uniform(seed, STREAM_POS, base + 3 * cand, 3 * chunk).reshape(chunk, 3)
        xyz = (u * box).astype(np.float32)
        xyz = np.where(xyz >= np.float32(box), np.float32(0.0), xyz).astype(np.float64)
        for k in range(chunk):
            cand += 1
            p = xyz[k]
            if placed:
                if min_image_ok:
                    dist = _periodic_dists(p, pts[:placed], box, 0)
                else:
                    dist = _periodic_dists(p, pts[:placed], box, 1)
                if dist.min() < min_dist or np.any(np.abs(dist - cutoff) < shell):
                    continue
            pts[placed] = p
            placed += 1
            if placed == n:
                break
    # coarse spatial order (part of the input): cells of edge >= 3 Angstrom, z-major
    nb = max(1, int(box / 3.0))
    b = np.minimum((pts / box * nb).astype(np.int64), nb - 1)
    key = (b[:, 2] * nb + b[:, 1]) * nb + b[:, 0]
    order = np.argsort(key, kind="stable")
    return pts[order].astype(np.float32)


def make_lattice(w: "Workload", struct_index: int) -> np.ndarray:
    """Cell matrix (rows = lattice vectors, float32) of one structure.  "triclinic": the cube of
    edge `box` sheared by seeded amounts of up to 0.3 box (volume unchanged, all perpendicular
    heights stay above 0.9 box); "free": zeros, which marks a molecule in vacuum."""
    if w.cell_kind == "cubic":
        return (np.eye(3) * w.box).astype(np.float32)
    if w.cell_kind == "free":
        return np.zeros((3, 3), np.float32)
    if w.cell_kind != "triclinic":
        raise ValueError(w.cell_kind)
    t = 2.0 * uniform(w.seed, STREAM_CELL, 3 * struct_index, 3) - 1.0
    lat = np.eye(3) * w.box
    lat[1, 0] = 0.3 * w.box * t[0]
    lat[2, 0] = 0.2 * w.box * t[1]
    lat[2, 1] = 0.25 * w.box * t[2]
    return lat.astype(np.float32)


def make_structure_general(seed: int, struct_index: int, n: int, lat: np.ndarray, box: float, cutoff: float,
                           min_dist: float = 1.0, shell: float = 1e-4) -> np.ndarray:
    """Random sequential insertion for a general lattice (rows of `lat`) or, with lat = 0, for a
    molecule in vacuum inside a cube of edge `box` whose corner sits at a seeded offset (so that
    coordinates of either sign occur).  Same rejection rules as make_structure; periodic
    candidates keep fractional coordinates 0.1 % clear of the cell faces, so that "inside the
    cell" has the same answer in float32 and float64.  Returns float32 [n,3] in a coarse
    spatial order."""
    lat64 = np.asarray(lat, dtype=np.float32).astype(np.float64)
    periodic = bool(lat64.any())
    if periodic:
        rng = np.array([-1.0, 0.0, 1.0])
        img = np.stack(np.meshgrid(rng, rng, rng, indexing="ij"), -1).reshape(27, 3) @ lat64
        origin = np.zeros(3)
    else:
        img = np.zeros((1, 3))
        origin = (40.0 * uniform(seed, STREAM_CELL, (1 << 20) + 3 * struct_index, 3) - 20.0).astype(np.float32).astype(np.float64)
    pts = np.zeros((n, 3), dtype=np.float64)
    frac = np.zeros((n, 3), dtype=np.float64)
    placed = 0
    cand = 0
    base = struct_index * (1 << 32)
    chunk = 256
    while placed < n:
        u = uniform(seed, STREAM_POS, base + 3 * cand, 3 * chunk).reshape(chunk, 3)
        if periodic:
            u = 1e-3 + u * (1.0 - 2e-3)
            xyz = (u @ lat64).astype(np.float32).astype(np.float64)
        else:
            xyz = (origin + u * box).astype(np.float32).astype(np.float64)
        for k in range(chunk):
            cand += 1
            p = xyz[k]
            if placed:
                d = (pts[:placed, None, :] + img[None, :, :]) - p[None, None, :]
                dist = np.sqrt((d * d).sum(-1)).reshape(-1)
                if dist.min() < min_dist or np.any(np.abs(dist - cutoff) < shell):
                    continue
            pts[placed] = p
            frac[placed] = u[k]
            placed += 1
            if placed == n:
                break
    nb = max(1, int(box / 3.0))
    b = np.minimum((frac * nb).astype(np.int64), nb - 1)
    key = (b[:, 2] * nb + b[:, 1]) * nb + b[:, 0]
    order = np.argsort(key, kind="stable")
    return pts[order].astype(np.float32)


def draw_species(seed: int, n: int, n_species: int, dist: str) -> np.ndarray:
    u = uniform(seed, STREAM_SPECIES, 0, n)
    if dist == "uniform":
        p = np.full(n_species, 1.0 / n_species)
    elif dist == "zipf1.2":
        p = np.arange(1, n_species + 1, dtype=np.float64) ** -1.2
        p /= p.sum()
    else:
        raise ValueError(dist)
    cdf = np.cumsum(p)
    cdf[-1] = 1.0
    return np.searchsorted(cdf, u, side="right").astype(np.int32)


# ----------------------------------------------------------------------------- parameters

def param_shapes(w: Workload) -> List[Tuple[str, Tuple[int, ...], int, int]]:
    """Flat parameter layout: list of (name, shape, fan_in, fan_out); row-major [out, in]."""
    C, H, K, S = w.channels, w.edge_hidden, w.n_rbf, w.n_species
    out: List[Tuple[str, Tuple[int, ...], int, int]] = []
    if w.kind != KIND_STAGE:
        out.append(("emb", (S, C), S, C))
    for l in range(w.n_layers):
        if w.kind == KIND_EQUIVARIANT:
            out.append((f"l{l}.W1", (H, K), K, H))
            npth = n_paths(w.l_max)
            out.append((f"l{l}.W2", (npth * C, H), H, npth * C))
            for lam in range(w.l_max + 1):
                out.append((f"l{l}.Wl{lam}", (w.n_experts, C, C) if w.n_experts > 0 else (C, C), C, C))
        else:
            out.append((f"l{l}.W1", (H, K), K, H))
            if w.edge_depth == 3:
                out.append((f"l{l}.W2", (H, H), H, H))
                out.append((f"l{l}.W3", (C, H), H, C))
            else:
                out.append((f"l{l}.W2", (C, H), H, C))
            vshape = (w.n_experts, C, C) if w.n_experts > 0 else (C, C)
            out.append((f"l{l}.V1", vshape, C, C))
            out.append((f"l{l}.V2", vshape, C, C))
    if w.kind != KIND_STAGE:
        out.append(("U", (C, C), C, C))
        out.append(("w_o", (C,), C, 1))
    return out


def param_count(w: Workload) -> int:
    return int(sum(int(np.prod(s)) for _, s, _, _ in param_shapes(w)))


def param_slices(w: Workload) -> Dict[str, Tuple[int, Tuple[int, ...]]]:
    """name -> (offset into the flat vector, shape)."""
    off, res = 0, {}
    for name, shape, _, _ in param_shapes(w):
        res[name] = (off, shape)
        off += int(np.prod(shape))
    return res


def draw_params(w: Workload) -> np.ndarray:
    """Xavier-uniform per tensor, bound sqrt(6/(fan_in+fan_out)), float32 flat vector."""
    parts, ctr = [], 0
    for _, shape, fin, fout in param_shapes(w):
        n = int(np.prod(shape))
        a = np.sqrt(6.0 / (fin + fout))
        parts.append(((2.0 * uniform(w.seed, STREAM_PARAMS, ctr, n) - 1.0) * a).astype(np.float32))
        ctr += n
    return np.concatenate(parts)


# ----------------------------------------------------------------------------- whole workload

@dataclass
class Inputs:
    workload: Workload
    pos: np.ndarray          # [N,3] f32
    species: np.ndarray      # [N] i32
    struct_ptr: np.ndarray   # [B+1] i32
    cell: np.ndarray         # [B,3,3] f32 (rows = lattice vectors)
    params: np.ndarray       # [n_params] f32
    E_ref: np.ndarray        # [B] f32
    F_ref: np.ndarray        # [N,3] f32
    stage: Dict[str, np.ndarray] = field(default_factory=dict)  # h_in, g_out, hdot_in, v, lam_out
    alpha: Optional[np.ndarray] = None  # [B, n_experts] f32 mixing coefficients (rows sum to 1), n_experts > 0


def make_inputs(w: Workload) -> Inputs:
    B, n, N = w.n_structs, w.atoms_per_struct, w.n_atoms
    if w.cell_kind == "cubic":
        pos = np.concatenate([make_structure(w.seed, s, n, w.box, w.cutoff, w.min_dist) for s in range(B)], 0)
        cell = np.tile((np.eye(3) * w.box).astype(np.float32)[None], (B, 1, 1))
    else:
        cell = np.stack([make_lattice(w, s) for s in range(B)])
        pos = np.concatenate([make_structure_general(w.seed, s, n, cell[s], w.box, w.cutoff, w.min_dist) for s in range(B)], 0)
    species = draw_species(w.seed, N, w.n_species, w.species_dist)
    struct_ptr = (np.arange(B + 1, dtype=np.int64) * n).astype(np.int32)
    E_ref = normal(w.seed, STREAM_EREF, 0, B).astype(np.float32)
    F_ref = (0.1 * normal(w.seed, STREAM_FREF, 0, 3 * N)).astype(np.float32).reshape(N, 3)
    stage: Dict[str, np.ndarray] = {}
    if w.kind == KIND_STAGE:
        C = w.channels
        stage["h_in"] = normal(w.seed, STREAM_H_IN, 0, N * C).astype(np.float32).reshape(N, C)
        stage["g_out"] = normal(w.seed, STREAM_G_OUT, 0, N * C).astype(np.float32).reshape(N, C)
        stage["hdot_in"] = normal(w.seed, STREAM_HDOT_IN, 0, N * C).astype(np.float32).reshape(N, C)
        stage["v"] = normal(w.seed, STREAM_V, 0, N * 3).astype(np.float32).reshape(N, 3)
        stage["lam_out"] = normal(w.seed, STREAM_LAM_OUT, 0, N * C).astype(np.float32).reshape(N, C)
    alpha = None
    if w.n_experts > 0:
        # stands in for a router's output: positive coefficients, one set per structure, summing to 1
        a = np.exp(normal(w.seed, STREAM_ALPHA, 0, B * w.n_experts).reshape(B, w.n_experts))
        alpha = (a / a.sum(axis=1, keepdims=True)).astype(np.float32)
    return Inputs(w, pos, species, struct_ptr, cell, draw_params(w), E_ref, F_ref, stage, alpha)


# ----------------------------------------------------------------------------- graph sizes

def draw_graph_sizes(seed: int, total_atoms: int = 12800, median: float = 53.0, mean: float = 85.0,
                     max_size: int = 905) -> np.ndarray:
    """Atom counts of the graphs of one global batch: log-normal with the median and mean of the
    paper's mixed dataset (Appendix A.1, Table 3: mean 85, P50 53, max 905), truncated to
    [1, max_size], drawn until the batch holds total_atoms atoms (12,800 in Sec. 5.1)."""
    sigma = np.sqrt(2.0 * np.log(mean / median))
    out, tot, ctr = [], 0, 0
    while tot < total_atoms:
        z = normal(seed, 11, ctr, 64)
        ctr += 64
        for s in np.clip(np.rint(median * np.exp(sigma * z)), 1, max_size).astype(np.int64):
            out.append(int(s))
            tot += int(s)
            if tot >= total_atoms:
                break
    return np.array(out, dtype=np.int32)
