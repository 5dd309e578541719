"""Pins for the oracle's model, forces, loss gradient, BF/BE split and stage protocol.

Everything here is checked against something other than the oracle's own differentiation:
closed forms, symmetries of the physics, central finite differences of scalar outputs,
and the composition of pipeline stages (the paper's "Correctness Validation": running the
layers as stages must not change the result)."""
import math

import numpy as np
import pytest
import torch
from scipy.spatial.transform import Rotation

from oracle import mlip_oracle as O
from paper_2605_18404_amd import synth

KINDS = {"invariant": 1, "equivariant": 2, "invariant3": 3}


def tiny(which, **kw):
    """A few atoms, a few channels: same recipe as the real workloads."""
    base = synth.WORKLOADS[KINDS[which]]
    d = dict(n_structs=2, atoms_per_struct=10, box=7.2, cutoff=3.5, n_rbf=6, channels=4, edge_hidden=5,
             n_layers=2, n_species=3)
    if which == "equivariant":
        d.update(channels=3, edge_hidden=4)
    if which == "invariant3":
        d.update(kind=synth.KIND_INVARIANT)
    d.update(kw)
    return synth.shrink(base, **d)


def run(w, inp=None, **kw):
    inp = inp or synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    return O.train_step(cfg, inp.pos, inp.species, inp.struct_ptr, inp.cell, inp.params, inp.E_ref, inp.F_ref, **kw)


def energy(w, inp, pos=None, params=None, cell=None, species=None, struct_ptr=None):
    cfg = O.cfg_from_workload(w)
    return O.energy_only(cfg, inp.pos if pos is None else pos, inp.species if species is None else species,
                         inp.struct_ptr if struct_ptr is None else struct_ptr,
                         inp.cell if cell is None else cell, inp.params if params is None else params)


@pytest.mark.parametrize("which", ["invariant", "equivariant", "invariant3"])
def test_energy_symmetries(which):
    w = tiny(which)
    inp = synth.make_inputs(w)
    E0 = energy(w, inp)
    assert E0.shape == (2,) and np.all(np.abs(E0) > 1e-6)
    R = Rotation.from_rotvec([0.4, 0.9, -0.5]).as_matrix()
    pos = inp.pos.astype(np.float64)
    # rotation of positions and lattice
    E1 = energy(w, inp, pos=pos @ R.T, cell=inp.cell.astype(np.float64) @ R.T)
    assert np.allclose(E1, E0, rtol=1e-11, atol=1e-13)
    # improper rotation (reflection): even-parity couplings only, so E is unchanged
    M = np.diag([1.0, -1.0, 1.0])
    E1 = energy(w, inp, pos=pos @ M.T, cell=inp.cell.astype(np.float64) @ M.T)
    assert np.allclose(E1, E0, rtol=1e-11, atol=1e-13)
    # translation (atoms may leave the cell: the oracle does not wrap)
    E1 = energy(w, inp, pos=pos + np.array([0.3, -0.2, 0.9]))
    assert np.allclose(E1, E0, rtol=1e-11, atol=1e-13)
    # permutation of atoms inside a structure
    perm = np.arange(w.n_atoms)
    perm[:10] = np.random.default_rng(0).permutation(10)
    E1 = energy(w, inp, pos=pos[perm], species=inp.species[perm])
    assert np.allclose(E1, E0, rtol=1e-11, atol=1e-13)
    # additivity: each structure alone
    for s in range(2):
        sl = slice(10 * s, 10 * s + 10)
        Es = energy(w, inp, pos=pos[sl], species=inp.species[sl], struct_ptr=np.array([0, 10], np.int32),
                    cell=inp.cell[s:s + 1])
        assert np.allclose(Es[0], E0[s], rtol=1e-12)


@pytest.mark.parametrize("which", ["invariant", "equivariant"])
def test_isolated_atoms_closed_form(which):
    # no edges: h stays the embedding, E = sum_i w_o . silu(U emb[z_i])
    w = tiny(which, n_structs=1, atoms_per_struct=3, box=20.0, min_dist=6.0)
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    assert len(g["sender"]) == 0
    P = {k: inp.params[o:o + int(np.prod(s))].reshape(s).astype(np.float64) for k, (o, s) in synth.param_slices(w).items()}
    y = P["emb"][inp.species] @ P["U"].T
    want = ((y / (1 + np.exp(-y))) @ P["w_o"]).sum()
    assert np.allclose(energy(w, inp)[0], want, rtol=1e-13)
    r = O.train_step(cfg, inp.pos, inp.species, inp.struct_ptr, inp.cell, inp.params, inp.E_ref, inp.F_ref)
    assert np.all(r["F"] == 0.0)


def test_single_invariant_layer_by_hand():
    # 2 atoms, 1 layer, written out with numpy from the model definition
    w = tiny("invariant", n_structs=1, atoms_per_struct=2, n_layers=1, box=8.0, cutoff=3.0, min_dist=1.0)
    inp = synth.make_inputs(w)
    pos = np.array([[1.0, 1.0, 1.0], [2.0, 2.5, 1.5]], np.float32)
    P = {k: inp.params[o:o + int(np.prod(s))].reshape(s).astype(np.float64) for k, (o, s) in synth.param_slices(w).items()}
    sil = lambda t: t / (1 + np.exp(-t))
    r = math.sqrt(1.0 + 2.25 + 0.25)
    mu = np.arange(w.n_rbf) * w.cutoff / (w.n_rbf - 1)
    phi = np.exp(-0.5 * ((r - mu) / (w.cutoff / (w.n_rbf - 1))) ** 2)
    filt = 0.5 * (1 + math.cos(math.pi * r / w.cutoff)) * (P["l0.W2"] @ sil(P["l0.W1"] @ phi))
    h0 = P["emb"][inp.species[:2]]
    a = np.stack([filt * h0[1], filt * h0[0]])
    h1 = h0 + sil(a @ P["l0.V1"].T) @ P["l0.V2"].T
    want = (sil(h1 @ P["U"].T) @ P["w_o"]).sum()
    got = energy(w, inp, pos=pos, species=inp.species[:2])
    assert np.allclose(got[0], want, rtol=1e-13)


def _fd_forces(w, inp, h=1e-4):
    pos = inp.pos.astype(np.float64)
    F = np.zeros_like(pos)
    for i in range(pos.shape[0]):
        for a in range(3):
            p = pos.copy(); p[i, a] += h
            m = pos.copy(); m[i, a] -= h
            F[i, a] = -(energy(w, inp, pos=p).sum() - energy(w, inp, pos=m).sum()) / (2 * h)
    return F


@pytest.mark.parametrize("which,box", [("invariant", 7.2), ("equivariant", 7.2), ("invariant3", 7.2),
                                       ("invariant", 4.6), ("equivariant", 4.6)])  # 4.6 < 2 r_c: several images per pair
def test_forces(which, box):
    w = tiny(which, atoms_per_struct=8, box=box)
    inp = synth.make_inputs(w)
    r = run(w, inp)
    F = r["F"]
    Ffd = _fd_forces(w, inp)
    assert np.linalg.norm(F - Ffd) / np.linalg.norm(Ffd) < 1e-7
    # zero net force per structure (translation invariance)
    for s in range(2):
        assert np.abs(F[8 * s:8 * s + 8].sum(0)).max() < 1e-13 * max(1.0, np.abs(F).max()) + 1e-15
    # equivariance F(Rx) = R F(x)
    R = Rotation.from_rotvec([-0.7, 0.2, 1.3]).as_matrix()
    cfg = O.cfg_from_workload(w)
    r2 = O.train_step(cfg, inp.pos.astype(np.float64) @ R.T, inp.species, inp.struct_ptr,
                      inp.cell.astype(np.float64) @ R.T, inp.params, inp.E_ref, inp.F_ref)
    assert np.allclose(r2["F"], F @ R.T, rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("which", ["invariant", "equivariant"])
def test_pair_force_is_central(which):
    w = tiny(which, n_structs=1, atoms_per_struct=2, box=9.0, cutoff=4.0)
    inp = synth.make_inputs(w)
    pos = np.array([[2.0, 2.0, 2.0], [3.1, 3.4, 1.2]])
    d = pos[1] - pos[0]
    rr = np.linalg.norm(d)
    cfg = O.cfg_from_workload(w)
    r = O.train_step(cfg, pos, inp.species[:2], inp.struct_ptr, inp.cell, inp.params, inp.E_ref, inp.F_ref[:2])
    # along the bond, equal and opposite, magnitude -dE/dr by central difference in r
    h = 1e-5
    Ep = energy(w, inp, pos=np.stack([pos[0], pos[0] + d * (rr + h) / rr]), species=inp.species[:2])[0]
    Em = energy(w, inp, pos=np.stack([pos[0], pos[0] + d * (rr - h) / rr]), species=inp.species[:2])[0]
    dEdr = (Ep - Em) / (2 * h)
    assert np.allclose(r["F"][1], -dEdr * d / rr, rtol=1e-7, atol=1e-12)
    assert np.allclose(r["F"][0], -r["F"][1], rtol=1e-12, atol=1e-15)


def test_loss_value():
    w = tiny("invariant")
    inp = synth.make_inputs(w)
    r = run(w, inp)
    want = np.mean((r["E"] - inp.E_ref.astype(np.float64)) ** 2) + 10.0 * np.mean((r["F"] - inp.F_ref.astype(np.float64)) ** 2)
    assert abs(r["loss"] - want) < 1e-13 * abs(want)


@pytest.mark.parametrize("which", ["invariant", "equivariant", "invariant3"])
def test_loss_gradient_by_finite_differences(which):
    w = tiny(which, atoms_per_struct=6, box=7.2)
    inp = synth.make_inputs(w)
    r = run(w, inp)
    g = r["grad"]
    theta = inp.params.astype(np.float64)
    gfd = np.zeros_like(theta)
    cfg = O.cfg_from_workload(w)
    graph = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)

    def loss_at(th):
        # loss from E and finite-difference-free forces: uses the oracle's F (pinned by test_forces)
        rr = O.train_step(cfg, inp.pos, inp.species, inp.struct_ptr, inp.cell, th, inp.E_ref, inp.F_ref, graph)
        return rr["loss"]

    h = 1e-5
    for k in range(theta.size):
        p = theta.copy(); p[k] += h
        m = theta.copy(); m[k] -= h
        gfd[k] = (loss_at(p) - loss_at(m)) / (2 * h)
    assert np.linalg.norm(g - gfd) / np.linalg.norm(gfd) < 1e-7
    # every parameter tensor individually
    for name, (off, shp) in synth.param_slices(w).items():
        n = int(np.prod(shp))
        a, b = g[off:off + n], gfd[off:off + n]
        assert np.linalg.norm(a - b) <= 1e-6 * np.linalg.norm(b) + 1e-12, name


@pytest.mark.parametrize("which", ["invariant", "equivariant", "invariant3"])
def test_bf_be_split(which):
    w = tiny(which)
    inp = synth.make_inputs(w)
    total = run(w, inp)["grad"]                      # plain ops, no weight copies
    sp = run(w, inp, split=True)
    assert np.allclose(sp["grad_bf"] + sp["grad_be"], total, rtol=1e-11, atol=1e-14)
    assert np.linalg.norm(sp["grad_bf"]) > 1e-3 * np.linalg.norm(total)
    sl = synth.param_slices(w)
    # the embedding is never used by the differentiated graph: no second-order share
    o, s = sl["emb"]
    assert np.all(sp["grad_bf"][o:o + int(np.prod(s))] == 0.0)
    # w_o enters E linearly, so all of dL_F/dw_o is second-order and BE keeps only dL_E/dw_o
    o, s = sl["w_o"]
    cfg = O.cfg_from_workload(w)
    w0 = synth.shrink(w, force_weight=0.0)
    only_E = run(w0, inp)["grad"]
    assert np.allclose(sp["grad_be"][o:o + s[0]], only_E[o:o + s[0]], rtol=1e-11, atol=1e-14)
    # BF's share is linear in the force-loss cotangent: it vanishes when F_ref = F ...
    r0 = run(w, inp)
    inp2 = synth.make_inputs(w)
    inp2.F_ref = r0["F"]
    sp2 = O.train_step(cfg, inp2.pos, inp2.species, inp2.struct_ptr, inp2.cell, inp2.params, inp2.E_ref,
                       inp2.F_ref, split=True)
    assert np.abs(sp2["grad_bf"]).max() < 1e-13
    assert np.allclose(sp2["grad_be"], only_E, rtol=1e-10, atol=1e-13)
    # ... and doubles when the force weight doubles (same F, same F_ref)
    w2 = synth.shrink(w, force_weight=20.0)
    sp3 = run(w2, inp, split=True)
    assert np.allclose(sp3["grad_bf"], 2.0 * sp["grad_bf"], rtol=1e-11, atol=1e-14)


# ------------------------------------------------------------------------------ stage

def _stage_inputs(n_layers=2, **kw):
    w = tiny("invariant3", **kw)
    w = synth.shrink(w, kind=synth.KIND_STAGE, n_layers=n_layers, n_species=1)
    return w, synth.make_inputs(w)


def test_stage_outputs_by_finite_differences():
    w, inp = _stage_inputs(atoms_per_struct=5)
    cfg = O.cfg_from_workload(w)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    st = {k: v.astype(np.float64) for k, v in inp.stage.items()}
    out = O.stage_step(cfg, inp.pos, inp.struct_ptr, inp.cell, inp.params, st["h_in"], st["g_out"],
                       st["hdot_in"], st["v"], st["lam_out"], g)

    def phi(params=None, **over):
        a = dict(st); a.update(over)
        return O.stage_phi(cfg, inp.pos, inp.struct_ptr, inp.cell, inp.params if params is None else params,
                           a["h_in"], a["g_out"], a["hdot_in"], a["v"], a["lam_out"], g)

    h = 1e-5
    theta = inp.params.astype(np.float64)
    gfd = np.zeros_like(theta)
    for k in range(theta.size):
        p = theta.copy(); p[k] += h
        m = theta.copy(); m[k] -= h
        gfd[k] = (phi(p) - phi(m)) / (2 * h)
    assert np.linalg.norm(out["grad"] - gfd) / np.linalg.norm(gfd) < 1e-7
    for name, key in (("g_out", "hdot_out"), ("h_in", "lam_in")):
        base = st[name]
        fd = np.zeros_like(base)
        for idx in np.ndindex(*base.shape):
            p = base.copy(); p[idx] += h
            m = base.copy(); m[idx] -= h
            fd[idx] = (phi(**{name: p}) - phi(**{name: m})) / (2 * h)
        assert np.linalg.norm(out[key] - fd) / np.linalg.norm(fd) < 1e-7, key


def test_stage_identity_phi():
    # <hdot_in, g_in> + <v, p> = <g_out, hdot_out>  (both are the tangent of h_out paired with g_out)
    w, inp = _stage_inputs()
    cfg = O.cfg_from_workload(w)
    st = {k: v.astype(np.float64) for k, v in inp.stage.items()}
    out = O.stage_step(cfg, inp.pos, inp.struct_ptr, inp.cell, inp.params, st["h_in"], st["g_out"],
                       st["hdot_in"], st["v"], st["lam_out"])
    lhs = (st["hdot_in"] * out["g_in"]).sum() + (st["v"] * out["p"]).sum()
    rhs = (st["g_out"] * out["hdot_out"]).sum()
    assert abs(lhs - rhs) < 1e-11 * abs(lhs)


def test_two_chained_stages_equal_one():
    # Table 2's protocol: h forward (SAE), dE/dh backward (SAF), dL_F/d(dE/dh) forward (SGF), dL/dh backward (SGE)
    w4, inp = _stage_inputs(n_layers=4)
    cfg4 = O.cfg_from_workload(w4)
    w2 = synth.shrink(w4, n_layers=2)
    cfg2 = O.cfg_from_workload(w2)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w4.cutoff)
    st = {k: v.astype(np.float64) for k, v in inp.stage.items()}
    whole = O.stage_step(cfg4, inp.pos, inp.struct_ptr, inp.cell, inp.params, st["h_in"], st["g_out"],
                         st["hdot_in"], st["v"], st["lam_out"], g)
    half = synth.param_count(w2)
    thA, thB = inp.params[:half], inp.params[half:]
    z = np.zeros_like(st["h_in"])
    # FE: A then B
    A0 = O.stage_step(cfg2, inp.pos, inp.struct_ptr, inp.cell, thA, st["h_in"], z, z, st["v"], z, g)
    h_mid = A0["h_out"]
    # FF: B then A
    B1 = O.stage_step(cfg2, inp.pos, inp.struct_ptr, inp.cell, thB, h_mid, st["g_out"], z, st["v"], z, g)
    g_mid = B1["g_in"]
    A1 = O.stage_step(cfg2, inp.pos, inp.struct_ptr, inp.cell, thA, st["h_in"], g_mid, st["hdot_in"], st["v"], z, g)
    # BF: A then B
    hdot_mid = A1["hdot_out"]
    B2 = O.stage_step(cfg2, inp.pos, inp.struct_ptr, inp.cell, thB, h_mid, st["g_out"], hdot_mid, st["v"], st["lam_out"], g)
    # BE: B then A
    lam_mid = B2["lam_in"]
    A2 = O.stage_step(cfg2, inp.pos, inp.struct_ptr, inp.cell, thA, st["h_in"], g_mid, st["hdot_in"], st["v"], lam_mid, g)
    assert np.allclose(B1["h_out"], whole["h_out"], rtol=1e-12)
    assert np.allclose(A1["g_in"], whole["g_in"], rtol=1e-11, atol=1e-13)
    assert np.allclose(A1["p"] + B1["p"], whole["p"], rtol=1e-11, atol=1e-13)
    assert np.allclose(B2["hdot_out"], whole["hdot_out"], rtol=1e-11, atol=1e-13)
    assert np.allclose(A2["lam_in"], whole["lam_in"], rtol=1e-10, atol=1e-12)
    for key in ("grad", "grad_bf", "grad_be"):
        assert np.allclose(np.concatenate([A2[key], B2[key]]), whole[key], rtol=1e-10, atol=1e-12), key


def test_stage_chain_reproduces_whole_model():
    """Embedding -> one stage holding all layers -> readout gives the whole model's F and layer gradients."""
    w = tiny("invariant3")
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    full = run(w, inp, split=True)
    sl = synth.param_slices(w)
    C = w.channels
    th = torch.tensor(inp.params, dtype=torch.float64)
    emb = th[sl["emb"][0]:sl["emb"][0] + w.n_species * C].reshape(w.n_species, C)
    U = th[sl["U"][0]:sl["U"][0] + C * C].reshape(C, C)
    wo = th[sl["w_o"][0]:sl["w_o"][0] + C]
    lo = sl["l0.W1"][0]
    hi = sl["U"][0]
    ws = synth.shrink(w, kind=synth.KIND_STAGE)
    cfgs = O.cfg_from_workload(ws)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    h_in = emb[torch.as_tensor(inp.species, dtype=torch.long)].numpy()
    z = np.zeros_like(h_in)
    z3 = np.zeros((w.n_atoms, 3))
    fe = O.stage_step(cfgs, inp.pos, inp.struct_ptr, inp.cell, inp.params[lo:hi], h_in, z, z, z3, z, g)
    hL = torch.tensor(fe["h_out"], requires_grad=True)
    sid = torch.repeat_interleave(torch.arange(w.n_structs), w.atoms_per_struct)

    def readout(h):
        y = h @ U.t()
        return torch.zeros(w.n_structs, dtype=torch.float64).index_add(0, sid, (y * torch.sigmoid(y)) @ wo)

    E = readout(hL)
    assert np.allclose(E.detach().numpy(), full["E"], rtol=1e-12)
    (g_out,) = torch.autograd.grad(E.sum(), hL, create_graph=True)
    ff = O.stage_step(cfgs, inp.pos, inp.struct_ptr, inp.cell, inp.params[lo:hi], h_in, g_out.detach().numpy(), z, z3, z, g)
    F = -ff["p"]
    assert np.allclose(F, full["F"], rtol=1e-10, atol=1e-13)
    v = -(2.0 * w.force_weight / (3 * w.n_atoms)) * (F - inp.F_ref.astype(np.float64))
    Ebar = 2.0 / w.n_structs * (full["E"] - inp.E_ref.astype(np.float64))
    bf = O.stage_step(cfgs, inp.pos, inp.struct_ptr, inp.cell, inp.params[lo:hi], h_in, g_out.detach().numpy(), z, v, z, g)
    hdot = torch.tensor(bf["hdot_out"])
    # readout part of Psi = sum_s Ebar_s E_s + <dE/dh^L, hdot^L>, differentiated w.r.t. h^L
    Psi = (torch.tensor(Ebar) * E).sum() + (g_out * hdot).sum()
    (lam_out,) = torch.autograd.grad(Psi, hL)
    be = O.stage_step(cfgs, inp.pos, inp.struct_ptr, inp.cell, inp.params[lo:hi], h_in, g_out.detach().numpy(), z, v,
                      lam_out.numpy(), g)
    for key in ("grad", "grad_bf", "grad_be"):
        assert np.allclose(be[key], full[key][lo:hi], rtol=1e-9, atol=1e-12), key
    # embedding gradient = scatter of lam_in over species
    gemb = np.zeros((w.n_species, C))
    np.add.at(gemb, inp.species, be["lam_in"])
    o = sl["emb"][0]
    assert np.allclose(gemb.reshape(-1), full["grad"][o:o + w.n_species * C], rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("which", ["invariant", "equivariant", "invariant3"])
def test_streamed_energy_equals_plain_energy(which):
    """The edge-block accumulation used for systems too large for one pass changes nothing but the
    summation order; block sizes that do not divide the edge count, one edge per block, one block."""
    w = tiny(which)
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    E0 = O.energy_only(cfg, inp.pos, inp.species, inp.struct_ptr, inp.cell, inp.params, g)
    n_edges = len(g["sender"])
    assert n_edges > 50
    for chunk in (1, 7, n_edges - 1, n_edges, 10 * n_edges):
        E1 = O.energy_streamed(cfg, inp.pos, inp.species, inp.struct_ptr, inp.cell, inp.params, g, edge_chunk=chunk)
        assert np.allclose(E1, E0, rtol=1e-12, atol=1e-14), chunk
    # and it is an energy of the same positions: moving one atom changes it as the plain one does
    pos = inp.pos.astype(np.float64).copy()
    pos[3] += [0.01, -0.02, 0.015]
    dE0 = O.energy_only(cfg, pos, inp.species, inp.struct_ptr, inp.cell, inp.params, g) - E0
    dE1 = O.energy_streamed(cfg, pos, inp.species, inp.struct_ptr, inp.cell, inp.params, g, edge_chunk=13) - E0
    assert np.allclose(dE1, dE0, rtol=1e-9, atol=1e-14) and np.abs(dE0).max() > 0


# ------------------------------------------------------------------------------ dL/dx

@pytest.mark.parametrize("which,box", [("invariant", 7.2), ("equivariant", 7.2), ("invariant3", 7.2), ("equivariant", 4.6)])
def test_loss_position_gradient_by_finite_differences(which, box):
    """dL/dx against central differences of the loss in every coordinate (the loss is evaluated with the
    oracle's forces, which test_forces pins), and its closed relation to the Hessian-vector product:
    dL/dx = -Ebar F - d/d(eps) F(x + eps v) with v = -dL/dF."""
    w = tiny(which, atoms_per_struct=6, box=box)
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    graph = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    r = O.train_step(cfg, inp.pos, inp.species, inp.struct_ptr, inp.cell, inp.params, inp.E_ref, inp.F_ref, graph, grad_pos=True)
    pos = inp.pos.astype(np.float64)

    def at(x):
        return O.train_step(cfg, x, inp.species, inp.struct_ptr, inp.cell, inp.params, inp.E_ref, inp.F_ref, graph)

    h = 1e-5
    fd = np.zeros_like(pos)
    for i in range(pos.shape[0]):
        for a in range(3):
            p = pos.copy(); p[i, a] += h
            m = pos.copy(); m[i, a] -= h
            fd[i, a] = (at(p)["loss"] - at(m)["loss"]) / (2 * h)
    assert np.linalg.norm(r["grad_pos"] - fd) / np.linalg.norm(fd) < 1e-6
    # zero net derivative per structure: the loss is invariant under a translation of a whole structure
    n = w.atoms_per_struct
    for s in range(w.n_structs):
        assert np.abs(r["grad_pos"][s * n:(s + 1) * n].sum(0)).max() < 1e-12 * max(1.0, np.abs(r["grad_pos"]).max())
    # Hessian-vector form
    Ebar = 2.0 * (r["E"] - inp.E_ref.astype(np.float64)) / w.n_structs
    v = -2.0 * w.force_weight * (r["F"] - inp.F_ref.astype(np.float64)) / (3 * w.n_atoms)
    eps = 1e-5
    dF = (at(pos + eps * v)["F"] - at(pos - eps * v)["F"]) / (2 * eps)
    sid = np.repeat(np.arange(w.n_structs), n)
    assert np.allclose(r["grad_pos"], -Ebar[sid, None] * r["F"] - dF, rtol=1e-6, atol=1e-9 * np.abs(r["grad_pos"]).max())


def test_stage_position_gradient_by_finite_differences():
    w, inp = _stage_inputs(atoms_per_struct=5)
    cfg = O.cfg_from_workload(w)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    st = {k: v.astype(np.float64) for k, v in inp.stage.items()}
    out = O.stage_step(cfg, inp.pos, inp.struct_ptr, inp.cell, inp.params, st["h_in"], st["g_out"], st["hdot_in"], st["v"],
                       st["lam_out"], g, grad_pos=True)
    pos = inp.pos.astype(np.float64)
    phi = lambda x: O.stage_phi(cfg, x, inp.struct_ptr, inp.cell, inp.params, st["h_in"], st["g_out"], st["hdot_in"], st["v"], st["lam_out"], g)
    h = 1e-5
    fd = np.zeros_like(pos)
    for idx in np.ndindex(*pos.shape):
        p = pos.copy(); p[idx] += h
        m = pos.copy(); m[idx] -= h
        fd[idx] = (phi(p) - phi(m)) / (2 * h)
    assert np.linalg.norm(out["grad_pos"] - fd) / np.linalg.norm(fd) < 1e-6
