"""Two pins that stand on nothing the oracle computes itself:

* radius_graph_rows (the per-receiver form of the neighbour definition, used to check rows of a
  system too large for the full pair loop) against radius_graph row by row and against a k-d
  tree, on batches with several structures, multi-image cells, a sheared cell and a molecule;
* one equivariant interaction layer evaluated by explicit loops over edges, channels, paths and
  (m1, m2, m3), with the coupling tensors integrated in closed form from the harmonics'
  polynomials (monomial means on the sphere) -- a different method from the oracle's quadrature --
  and numpy basis functions and envelope, against the oracle's layer output.
"""
import itertools
import math

import numpy as np
import pytest
import torch
from scipy.spatial import cKDTree

from oracle import mlip_oracle as O
from paper_2605_18404_amd import synth


# ------------------------------------------------------------------ rows of the neighbour list

def _batch(cell_kind, box, n=30, n_structs=3, cutoff=4.0):
    w = synth.shrink(synth.WORKLOADS[1], n_structs=n_structs, atoms_per_struct=n, box=box, cutoff=cutoff,
                     cell_kind=cell_kind)
    return w, synth.make_inputs(w)


@pytest.mark.parametrize("cell_kind,box", [("cubic", 9.0), ("cubic", 4.6), ("triclinic", 9.0), ("free", 9.0)])
def test_rows_equal_the_full_list_row_by_row(cell_kind, box):
    # box 4.6 < 2 r_c: the same pair appears under several shifts
    w, inp = _batch(cell_kind, box, n=12 if box < 5 else 30)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    rows = np.arange(w.n_atoms)  # every receiver, in all three structures (offsets a > 0 included)
    got = O.radius_graph_rows(inp.pos, inp.struct_ptr, inp.cell, w.cutoff, rows)
    assert len(got) == w.n_atoms
    n_repeated = 0
    for i, (snd, sh) in zip(rows, got):
        a, b = g["row_ptr"][i], g["row_ptr"][i + 1]
        assert np.array_equal(snd, g["sender"][a:b]), i
        assert np.array_equal(sh, g["shift"][a:b]), i
        assert snd.dtype == np.int32 and sh.dtype == np.int32
        # the atom itself is never its own neighbour (its images are at least a cell height >= r_c away)
        assert not np.any(snd == i), i
        n_repeated += len(snd) - len(np.unique(snd))
    assert (n_repeated > 0) == (box < 5)
    # a subset in arbitrary order gives the same rows
    pick = np.array([w.n_atoms - 1, 0, w.atoms_per_struct, w.atoms_per_struct + 3])
    for i, (snd, sh) in zip(pick, O.radius_graph_rows(inp.pos, inp.struct_ptr, inp.cell, w.cutoff, pick)):
        a, b = g["row_ptr"][i], g["row_ptr"][i + 1]
        assert np.array_equal(snd, g["sender"][a:b]) and np.array_equal(sh, g["shift"][a:b])


def test_rows_against_a_kdtree():
    # independent of radius_graph: minimum-image k-d tree per structure (box >= 2 r_c)
    w, inp = _batch("cubic", 9.0, n=40, n_structs=2)
    n = w.atoms_per_struct
    rows = np.array([0, 7, n - 1, n, n + 11, 2 * n - 1])
    got = O.radius_graph_rows(inp.pos, inp.struct_ptr, inp.cell, w.cutoff, rows)
    for i, (snd, sh) in zip(rows, got):
        s = i // n
        x = inp.pos[s * n:(s + 1) * n].astype(np.float64)
        tree = cKDTree(x, boxsize=w.box)
        want = sorted(j + s * n for j in tree.query_ball_point(x[i - s * n], w.cutoff * (1 - 1e-12)) if j + s * n != i)
        assert snd.tolist() == want  # sorted by sender; one image per pair
        d = inp.pos[snd].astype(np.float64) + sh * w.box - inp.pos[i].astype(np.float64)
        assert np.all((d * d).sum(1) < w.cutoff ** 2) and np.all(np.abs(d) <= w.box / 2 + 1e-9)


def test_rows_of_a_hand_countable_case():
    # two atoms 5 apart along x in a box of 10, cutoff 6: each sees the other at +5 and at -5 (shifts 0 and
    # -1 or +1), never itself; in code order the lower shift comes first
    pos = np.array([[1.0, 2.0, 3.0], [6.0, 2.0, 3.0]])
    cell = (np.eye(3) * 10.0)[None]
    (s0, h0), (s1, h1) = O.radius_graph_rows(pos, np.array([0, 2], np.int32), cell, 6.0, np.array([0, 1]))
    assert s0.tolist() == [1, 1] and h0.tolist() == [[-1, 0, 0], [0, 0, 0]]
    assert s1.tolist() == [0, 0] and h1.tolist() == [[0, 0, 0], [1, 0, 0]]


# ------------------------------------------------------------------ one equivariant layer by hand

def _dfact(n):  # double factorial with (-1)!! = 1
    return 1 if n <= 0 else n * _dfact(n - 2)


def _mono_mean(a, b, c):
    """Mean of x^a y^b z^c over the unit sphere."""
    if a % 2 or b % 2 or c % 2:
        return 0.0
    return _dfact(a - 1) * _dfact(b - 1) * _dfact(c - 1) / _dfact(a + b + c + 1)


def _harmonic_polys():
    """The nine real harmonics (component normalisation, m = -l..l) as {(a, b, c): coefficient} in x^a y^b z^c,
    typed from their textbook forms: 1; sqrt3 (y, z, x); sqrt15 xy, sqrt15 yz, (sqrt5/2)(3 z^2 - 1), sqrt15 xz,
    (sqrt15/2)(x^2 - y^2)."""
    s3, s15, s5 = math.sqrt(3), math.sqrt(15), math.sqrt(5)
    return [
        {(0, 0, 0): 1.0},
        {(0, 1, 0): s3}, {(0, 0, 1): s3}, {(1, 0, 0): s3},
        {(1, 1, 0): s15}, {(0, 1, 1): s15}, {(0, 0, 2): 1.5 * s5, (0, 0, 0): -0.5 * s5}, {(1, 0, 1): s15},
        {(2, 0, 0): 0.5 * s15, (0, 2, 0): -0.5 * s15},
    ]


def _poly_eval(p, x, y, z):
    return sum(co * x ** a * y ** b * z ** c for (a, b, c), co in p.items())


def _hand_couplings():
    """{(l1, l2, l3): T[m1][m2][m3]}: sphere means of triple products of the harmonics' polynomials, each path
    scaled by a positive factor to sum of squares 2 l3 + 1."""
    Y = _harmonic_polys()
    off = [0, 1, 4]
    out = {}
    for l1, l2, l3 in itertools.product(range(3), repeat=3):
        if not (abs(l1 - l2) <= l3 <= l1 + l2) or (l1 + l2 + l3) % 2:
            continue
        T = np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1))
        for m1, m2, m3 in np.ndindex(*T.shape):
            tot = 0.0
            for (e1, c1), (e2, c2), (e3, c3) in itertools.product(Y[off[l1] + m1].items(), Y[off[l2] + m2].items(),
                                                                  Y[off[l3] + m3].items()):
                tot += c1 * c2 * c3 * _mono_mean(e1[0] + e2[0] + e3[0], e1[1] + e2[1] + e3[1], e1[2] + e2[2] + e3[2])
            T[m1, m2, m3] = tot
        out[(l1, l2, l3)] = T * math.sqrt((2 * l3 + 1) / (T ** 2).sum())
    return out


def _layer_setup(gate=0):
    w = synth.shrink(synth.WORKLOADS[2], n_structs=1, atoms_per_struct=3, box=5.0, cutoff=3.0, n_rbf=5, channels=2,
                     edge_hidden=3, n_layers=1, n_species=2, gate=gate)
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    pos = np.array([[0.4, 0.9, 1.1], [2.2, 1.4, 0.3], [4.5, 0.2, 4.6]])  # 0-1 direct; 2 reaches 0 and 1 through the faces
    g = O.radius_graph(pos, inp.struct_ptr, inp.cell, w.cutoff)
    rng = np.random.default_rng(11)
    h = rng.normal(size=(3, w.channels, 9))  # all nine components populated: every path contributes
    return w, inp, cfg, pos, g, h


def _oracle_layer(w, inp, cfg, pos, g, h):
    P = O.unpack_params(torch.tensor(inp.params, dtype=torch.float64), cfg)
    lin = O._Lin(P)
    sid = torch.zeros(3, dtype=torch.long)
    lin.sid = sid
    snd, rcv, rv, r = O.edge_vectors(torch.tensor(pos), g, torch.tensor(inp.cell, dtype=torch.float64), sid)
    return O.equivariant_layer(torch.tensor(h), 0, lin, cfg, snd, rcv, rv, r).numpy()


def _hand_layer(w, inp, pos, g, h, drop_path=None, no_envelope=False):
    C, H, K, rc = w.channels, w.edge_hidden, w.n_rbf, w.cutoff
    P = {k: inp.params[o:o + int(np.prod(s))].reshape(s).astype(np.float64) for k, (o, s) in synth.param_slices(w).items()}
    T = _hand_couplings()
    paths = sorted(T)  # ordered by (l1, l2, l3): row p * C + c of W2 belongs to path p
    assert len(paths) == 11
    Ypoly = _harmonic_polys()
    off = [0, 1, 4]
    sil = lambda t: t / (1.0 + np.exp(-t))
    cell = inp.cell[0].astype(np.float64)
    a = np.zeros((3, C, 9))
    for e in range(len(g["sender"])):
        i, j, S = int(g["receiver"][e]), int(g["sender"][e]), g["shift"][e].astype(np.float64)
        rv = pos[j] + S @ cell - pos[i]
        r = math.sqrt(rv @ rv)
        u = rv / r
        Y = [_poly_eval(p, *u) for p in Ypoly]
        phi = np.array([math.exp(-0.5 * ((r - k * rc / (K - 1)) / (rc / (K - 1))) ** 2) for k in range(K)])
        fc = 1.0 if no_envelope else 0.5 * (1.0 + math.cos(math.pi * r / rc))
        R = (P["l0.W2"] @ sil(P["l0.W1"] @ phi)).reshape(11, C)
        for c in range(C):
            for p, (l1, l2, l3) in enumerate(paths):
                if p == drop_path:
                    continue
                for m1, m2, m3 in np.ndindex(2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1):
                    a[i, c, off[l3] + m3] += fc * R[p, c] * T[(l1, l2, l3)][m1, m2, m3] * h[j, c, off[l1] + m1] * Y[off[l2] + m2]
    out = h.copy()
    for i in range(3):
        for l in range(3):
            Wl = P[f"l0.Wl{l}"]
            for m in range(2 * l + 1):
                out[i, :, off[l] + m] += Wl @ a[i, :, off[l] + m]
    return out


def test_hand_couplings_agree_with_the_quadrature():
    T = _hand_couplings()
    G = O.gaunt_tensors()
    assert sorted(T) == O.PATHS
    for p, key in enumerate(O.PATHS):
        assert np.allclose(G[p].numpy(), T[key], atol=1e-12), key
    # typed value: the (1,1,0) coupling is proportional to delta_{m1 m2}; scaled to unit sum of squares, delta / sqrt3
    assert np.allclose(T[(1, 1, 0)][:, :, 0], np.eye(3) / math.sqrt(3), atol=1e-14)


def test_single_equivariant_layer_by_hand():
    w, inp, cfg, pos, g, h = _layer_setup()
    assert len(g["sender"]) >= 6 and np.abs(g["shift"]).max() == 1  # direct and image edges
    want = _hand_layer(w, inp, pos, g, h)
    got = _oracle_layer(w, inp, cfg, pos, g, h)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-14)
    # the check has teeth: leaving out the envelope, or any single path, moves the result far beyond that
    scale = np.abs(want - h).max()
    assert np.abs(_hand_layer(w, inp, pos, g, h, no_envelope=True) - want).max() > 1e-3 * scale
    for p in range(11):
        assert np.abs(_hand_layer(w, inp, pos, g, h, drop_path=p) - want).max() > 1e-4 * scale, p


def test_single_gated_layer_by_hand():
    # the gated update on top of the hand-evaluated pre-activations u = W^(l) a (hand layer minus h):
    # h_0 += silu(u_0), h_lm += sigmoid(u_0) u_lm for l = 1, 2
    w, inp, cfg, pos, g, h = _layer_setup(gate=1)
    u = _hand_layer(w, inp, pos, g, h) - h
    s = 1.0 / (1.0 + np.exp(-u[:, :, 0]))
    want = h.copy()
    want[:, :, 0] += u[:, :, 0] * s
    want[:, :, 1:] += s[:, :, None] * u[:, :, 1:]
    got = _oracle_layer(w, inp, cfg, pos, g, h)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-14)
    assert np.abs(got - (h + u)).max() > 1e-3 * np.abs(u).max()  # and it differs from the linear update
