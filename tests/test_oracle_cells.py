"""Pins for the oracle on general (triclinic) cells and on molecules in vacuum (zero cell):
a k-d tree over explicitly replicated images, textbook coordination numbers of lattices given by
their primitive cells, two descriptions of one lattice giving one energy, a molecule in vacuum
against the same molecule in a huge periodic box, and full rotation invariance."""
import numpy as np
import pytest
from scipy.spatial import cKDTree

from oracle import mlip_oracle as O
from paper_2605_18404_amd import synth


def tiny(kind_index=1, **kw):
    d = dict(n_structs=2, atoms_per_struct=24, box=9.0, cutoff=4.0, n_rbf=6, channels=4, edge_hidden=5, n_layers=2,
             n_species=3)
    d.update(kw)
    return synth.shrink(synth.WORKLOADS[kind_index], **d)


def energy(w, inp, pos=None, cell=None):
    return O.energy_only(O.cfg_from_workload(w), inp.pos if pos is None else pos, inp.species, inp.struct_ptr,
                         inp.cell if cell is None else cell, inp.params)


def test_triclinic_graph_matches_kdtree_over_replicated_images():
    w = tiny(cell_kind="triclinic", atoms_per_struct=40)
    inp = synth.make_inputs(w)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    got = set(zip(g["receiver"].tolist(), g["sender"].tolist(), map(tuple, g["shift"].tolist())))
    assert len(got) == len(g["sender"])
    want = set()
    n = w.atoms_per_struct
    shifts = [(a, b, c) for a in (-2, -1, 0, 1, 2) for b in (-2, -1, 0, 1, 2) for c in (-2, -1, 0, 1, 2)]
    for s in range(w.n_structs):
        x = inp.pos[s * n:(s + 1) * n].astype(np.float64)
        lat = inp.cell[s].astype(np.float64)
        rep = np.concatenate([x + np.array(S, dtype=np.float64) @ lat for S in shifts])  # 125 images: more than needed
        tree = cKDTree(rep)
        for i in range(n):
            for k in tree.query_ball_point(x[i], w.cutoff * (1 - 1e-12)):
                S, j = shifts[k // n], k % n
                if j == i and S == (0, 0, 0):
                    continue
                want.add((i + s * n, j + s * n, S))
    assert got == want  # in particular no neighbour needs an image beyond +-1
    assert any(abs(S[0]) + abs(S[1]) + abs(S[2]) >= 2 for _, _, S in got)  # edge and corner images occur
    # symmetry
    rev = g["rev"]
    assert np.array_equal(rev[rev], np.arange(len(rev))) and np.array_equal(g["shift"][rev], -g["shift"])


@pytest.mark.parametrize("name,lat,basis,reps,rc,coord", [
    # fcc from its primitive rhombohedral cell, cube edge 4: 12 neighbours at 4 / sqrt(2)
    ("fcc_primitive", np.array([[0, 2, 2], [2, 0, 2], [2, 2, 0]], float), [[0, 0, 0]], 4, 3.0, 12),
    # bcc from its primitive cell, cube edge 3: 8 at 2.598 and 6 at 3
    ("bcc_primitive", np.array([[-1.5, 1.5, 1.5], [1.5, -1.5, 1.5], [1.5, 1.5, -1.5]]), [[0, 0, 0]], 4, 3.1, 14),
    # hexagonal layers (a = 2, 120 degree cell) far apart: 6 in-plane neighbours
    ("hex_layers", np.array([[2, 0, 0], [-1, 3 ** 0.5, 0], [0, 0, 9.0]]), [[0, 0, 0]], 3, 2.1, 6),
    # hcp with the ideal c/a: 12 nearest neighbours
    ("hcp", np.array([[2, 0, 0], [-1, 3 ** 0.5, 0], [0, 0, 2 * (8 / 3) ** 0.5]]), [[0, 0, 0], [1 / 3, 2 / 3, 0.5]], 3, 2.1, 12),
])
def test_lattice_coordination_numbers_from_primitive_cells(name, lat, basis, reps, rc, coord):
    reps3 = (reps, reps, 1) if name == "hex_layers" else (reps, reps, reps)
    frac = np.array([[i + b[0], j + b[1], k + b[2]] for i in range(reps3[0]) for j in range(reps3[1])
                     for k in range(reps3[2]) for b in basis], dtype=np.float64)
    pos = frac @ lat
    cell = (np.array(reps3, dtype=np.float64)[:, None] * lat)[None]
    g = O.radius_graph(pos, np.array([0, len(pos)], np.int32), cell, rc)
    assert np.all(np.diff(g["row_ptr"]) == coord)


def test_cutoff_is_limited_by_the_cell_heights_not_the_edge_lengths():
    lat = np.array([[10.0, 0, 0], [9.0, 4.0, 0], [0, 0, 10.0]])  # edges 10, 9.85, 10; height along b is 4
    one = np.array([[0.5, 0.5, 0.5]])
    O.radius_graph(one, np.array([0, 1], np.int32), lat[None], 3.9)
    with pytest.raises(AssertionError):
        O.radius_graph(one, np.array([0, 1], np.int32), lat[None], 4.5)
    with pytest.raises(AssertionError):
        O.radius_graph(one, np.array([0, 1], np.int32), np.array([[[1.0, 0, 0], [2.0, 0, 0], [0, 0, 1.0]]]), 0.5)


@pytest.mark.parametrize("kind_index", [1, 2])
def test_two_descriptions_of_one_lattice_give_one_energy(kind_index):
    """A cube and the same cube sheared by a whole lattice vector generate the same lattice;
    after wrapping the atoms into the new cell nothing physical has changed."""
    w = tiny(kind_index, box=10.0, cutoff=3.5, **({"channels": 3, "edge_hidden": 4} if kind_index == 2 else {}))
    inp = synth.make_inputs(w)
    E0 = energy(w, inp)
    g0 = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    lat = inp.cell.astype(np.float64).copy()
    lat[:, 1] += lat[:, 0]      # a2' = a2 + a1
    lat[:, 2] -= lat[:, 1]      # a3' = a3 - a2'
    pos = inp.pos.astype(np.float64).copy()
    n = w.atoms_per_struct
    for s in range(w.n_structs):
        f = pos[s * n:(s + 1) * n] @ np.linalg.inv(lat[s])
        pos[s * n:(s + 1) * n] = (f - np.floor(f)) @ lat[s]
    g1 = O.radius_graph(pos, inp.struct_ptr, lat, w.cutoff)
    assert np.array_equal(g0["row_ptr"], g1["row_ptr"]) and not np.array_equal(g0["shift"], g1["shift"])
    E1 = energy(w, inp, pos=pos, cell=lat)
    np.testing.assert_allclose(E1, E0, rtol=1e-11)


def test_triclinic_forces_against_finite_differences_and_rotation():
    w = tiny(2, cell_kind="triclinic", atoms_per_struct=12, n_structs=1, channels=3, edge_hidden=4)
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    r = O.train_step(cfg, inp.pos, inp.species, inp.struct_ptr, inp.cell, inp.params, inp.E_ref, inp.F_ref)
    pos = inp.pos.astype(np.float64)
    for (i, a) in ((0, 0), (5, 1), (11, 2)):
        h = 1e-5
        pp, pm = pos.copy(), pos.copy()
        pp[i, a] += h
        pm[i, a] -= h
        fd = -(energy(w, inp, pos=pp)[0] - energy(w, inp, pos=pm)[0]) / (2 * h)
        assert abs(fd - r["F"][i, a]) <= 1e-6 * max(1.0, abs(fd))
    # rotating atoms and lattice together changes nothing
    q, _ = np.linalg.qr(np.random.default_rng(3).normal(size=(3, 3)))
    q *= np.sign(np.linalg.det(q))
    np.testing.assert_allclose(energy(w, inp, pos=pos @ q.T, cell=inp.cell.astype(np.float64) @ q.T), r["E"], rtol=1e-10)


def test_molecule_graph_matches_kdtree_and_has_no_images():
    w = tiny(cell_kind="free", atoms_per_struct=50, box=9.0)
    inp = synth.make_inputs(w)
    assert not inp.cell.any()
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    assert not g["shift"].any()
    got = set(zip(g["receiver"].tolist(), g["sender"].tolist()))
    want = set()
    n = w.atoms_per_struct
    for s in range(w.n_structs):
        for i, j in cKDTree(inp.pos[s * n:(s + 1) * n].astype(np.float64)).query_pairs(w.cutoff * (1 - 1e-12)):
            want.add((i + s * n, j + s * n))
            want.add((j + s * n, i + s * n))
    assert got == want and len(got) == len(g["sender"])
    # atoms near the faces of the bounding cube have fewer neighbours than a periodic box would give them
    wp = synth.shrink(w, cell_kind="cubic")
    ip = synth.make_inputs(wp)
    assert len(g["sender"]) < len(O.radius_graph(ip.pos, ip.struct_ptr, ip.cell, w.cutoff)["sender"])


@pytest.mark.parametrize("kind_index", [1, 2])
def test_molecule_equals_the_same_atoms_in_a_huge_periodic_box_and_rotates_freely(kind_index):
    w = tiny(kind_index, cell_kind="free", atoms_per_struct=14, box=6.0, **({"channels": 3, "edge_hidden": 4} if kind_index == 2 else {}))
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    r = O.train_step(cfg, inp.pos, inp.species, inp.struct_ptr, inp.cell, inp.params, inp.E_ref, inp.F_ref)
    # a periodic box so large that no image is within the cutoff (the oracle does not need the atoms inside it)
    big = np.tile((np.eye(3) * 100.0)[None], (w.n_structs, 1, 1))
    rb = O.train_step(cfg, inp.pos, inp.species, inp.struct_ptr, big, inp.params, inp.E_ref, inp.F_ref)
    for k in ("E", "F", "grad"):
        np.testing.assert_allclose(r[k], rb[k], rtol=1e-12, atol=1e-14)
    # rigid motion of the whole molecule: E invariant, F rotates, parameter gradient with rotated force labels invariant
    q, _ = np.linalg.qr(np.random.default_rng(5).normal(size=(3, 3)))
    q *= np.sign(np.linalg.det(q))
    pos = inp.pos.astype(np.float64) @ q.T + np.array([3.0, -7.0, 0.5])
    rr = O.train_step(cfg, pos, inp.species, inp.struct_ptr, inp.cell, inp.params, inp.E_ref, inp.F_ref.astype(np.float64) @ q.T)
    np.testing.assert_allclose(rr["E"], r["E"], rtol=1e-10)
    np.testing.assert_allclose(rr["F"], r["F"] @ q.T, rtol=1e-8, atol=1e-11)
    np.testing.assert_allclose(rr["grad"], r["grad"], rtol=1e-7, atol=1e-11)


@pytest.mark.parametrize("kind", ["triclinic", "free"])
def test_generators_keep_atoms_inside_and_pairs_off_the_cutoff_shell(kind):
    w = tiny(cell_kind=kind, atoms_per_struct=60, box=11.0, cutoff=5.0)
    inp = synth.make_inputs(w)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff + 2e-4)
    sid = np.repeat(np.arange(w.n_structs), w.atoms_per_struct)
    off = np.einsum("ea,eab->eb", g["shift"].astype(np.float64), inp.cell.astype(np.float64)[sid[g["receiver"]]])
    d = inp.pos.astype(np.float64)[g["sender"]] + off - inp.pos.astype(np.float64)[g["receiver"]]
    rr = np.sqrt((d * d).sum(1))
    assert rr.min() >= w.min_dist and np.all(np.abs(rr - w.cutoff) >= 1e-4)
    if kind == "triclinic":
        for s in range(w.n_structs):
            inv = np.linalg.inv(inp.cell[s].astype(np.float64)).astype(np.float32)
            x = inp.pos[sid == s]
            f = (x[:, 0:1] * inv[0] + x[:, 1:2] * inv[1]) + x[:, 2:3] * inv[2]  # float32 throughout
            assert f.dtype == np.float32 and f.min() > 5e-4 and f.max() < 1 - 5e-4
        assert np.abs(inp.cell[:, 1, 0]).max() > 0.5  # really sheared
