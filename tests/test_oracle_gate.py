"""Pins for the gated nonlinearity of the equivariant node update (oracle): symmetry of the
energy, an exact reduction to the already pinned linear update, the derivative of the gate itself
by hand, and central differences of E and of the loss."""
import numpy as np
import pytest
from scipy.spatial.transform import Rotation

from oracle import mlip_oracle as O
from paper_2605_18404_amd import synth


def tiny(**kw):
    d = dict(n_structs=2, atoms_per_struct=10, box=7.2, cutoff=3.5, n_rbf=6, channels=3, edge_hidden=4, n_layers=3,
             n_species=3, gate=1)
    d.update(kw)
    return synth.shrink(synth.WORKLOADS[2], **d)


def step(w, inp, params=None, pos=None, **kw):
    return O.train_step(O.cfg_from_workload(w), inp.pos if pos is None else pos, inp.species, inp.struct_ptr, inp.cell,
                        inp.params if params is None else params, inp.E_ref, inp.F_ref, **kw)


def energy(w, inp, pos=None, params=None, cell=None):
    return O.energy_only(O.cfg_from_workload(w), inp.pos if pos is None else pos, inp.species, inp.struct_ptr,
                         inp.cell if cell is None else cell, inp.params if params is None else params)


def test_gate_changes_the_model_and_keeps_its_symmetries():
    w = tiny()
    inp = synth.make_inputs(w)
    E0 = energy(w, inp)
    assert np.abs(E0 - energy(synth.shrink(w, gate=0), inp)).min() > 1e-6
    pos = inp.pos.astype(np.float64)
    for R in (Rotation.from_rotvec([0.4, 0.9, -0.5]).as_matrix(), np.diag([1.0, -1.0, 1.0])):
        E1 = energy(w, inp, pos=pos @ R.T, cell=inp.cell.astype(np.float64) @ R.T)
        np.testing.assert_allclose(E1, E0, rtol=1e-11, atol=1e-13)
    r = step(w, inp)
    R = Rotation.from_rotvec([-0.7, 0.2, 0.3]).as_matrix()
    rr = O.train_step(O.cfg_from_workload(w), pos @ R.T, inp.species, inp.struct_ptr, inp.cell.astype(np.float64) @ R.T,
                      inp.params, inp.E_ref, inp.F_ref.astype(np.float64) @ R.T)
    np.testing.assert_allclose(rr["F"], r["F"] @ R.T, rtol=1e-8, atol=1e-11)     # forces rotate with the frame
    np.testing.assert_allclose(rr["grad"], r["grad"], rtol=1e-7, atol=1e-11)


def test_vanishing_gate_scalars_reduce_to_the_linear_update_with_halved_matrices():
    """With every scalar mixing matrix zero the gate scalars are u_0 = 0: silu(0) = 0 and sigmoid(0) = 1/2,
    so the gated model equals the linear one whose vector and tensor mixing matrices are halved."""
    w = tiny()
    inp = synth.make_inputs(w)
    sl = synth.param_slices(w)
    p_gate, p_lin = inp.params.astype(np.float64).copy(), inp.params.astype(np.float64).copy()
    for l in range(w.n_layers):
        off, shape = sl[f"l{l}.Wl0"]
        p_gate[off:off + int(np.prod(shape))] = 0.0
        p_lin[off:off + int(np.prod(shape))] = 0.0
        for k in (1, 2):
            off, shape = sl[f"l{l}.Wl{k}"]
            p_lin[off:off + int(np.prod(shape))] *= 0.5
    a = step(w, inp, params=p_gate)
    b = step(synth.shrink(w, gate=0), inp, params=p_lin)
    np.testing.assert_allclose(a["E"], b["E"], rtol=1e-12)
    np.testing.assert_allclose(a["F"], b["F"], rtol=1e-10, atol=1e-14)
    # and is a different function as soon as the scalars are switched on
    assert np.abs(step(w, inp)["E"] - a["E"]).min() > 1e-6


def test_single_layer_gate_by_hand():
    """One atom pair, one layer: rebuild h^1 from the linear model's pre-activation u (its h^1 - h^0) and
    apply the gate by hand; the readout of that equals the gated model's energy."""
    import torch
    w = tiny(n_layers=1, n_structs=1, atoms_per_struct=4, box=6.0)
    inp = synth.make_inputs(w)
    cfg_lin = O.cfg_from_workload(synth.shrink(w, gate=0))
    P = O.unpack_params(torch.tensor(inp.params, dtype=torch.float64), cfg_lin)
    lin = O._Lin(P)
    x = torch.tensor(inp.pos, dtype=torch.float64)
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff)
    sid = torch.zeros(4, dtype=torch.long)
    lin.sid = sid
    snd, rcv, rv, r = O.edge_vectors(x, g, torch.tensor(inp.cell, dtype=torch.float64), sid)
    emb = P["emb"][torch.as_tensor(inp.species, dtype=torch.long)]
    h0 = torch.cat([emb[:, :, None], torch.zeros(4, w.channels, 8, dtype=torch.float64)], dim=2)
    u = O.equivariant_layer(h0, 0, lin, cfg_lin, snd, rcv, rv, r) - h0
    s = 1.0 / (1.0 + torch.exp(-u[:, :, 0]))
    h1_scalar = h0[:, :, 0] + u[:, :, 0] * s            # only l = 0 is read out
    y = h1_scalar @ P["U"].T
    eps = (y / (1.0 + torch.exp(-y))) @ P["w_o"].reshape(-1)
    np.testing.assert_allclose(energy(w, inp)[0], float(eps.sum()), rtol=1e-12)
    # the gated vector part: sigmoid(u_0) u_1m, checked on the layer output directly
    h1 = O.equivariant_layer(h0, 0, lin, O.cfg_from_workload(w), snd, rcv, rv, r)
    np.testing.assert_allclose((h1 - h0)[:, :, 1:].numpy(), (s[:, :, None] * u[:, :, 1:]).numpy(), rtol=1e-13, atol=1e-15)


def test_forces_and_gradient_against_central_differences_and_split():
    w = tiny()
    inp = synth.make_inputs(w)
    r = step(w, inp, split=True)
    np.testing.assert_allclose(r["grad_bf"] + r["grad_be"], r["grad"], rtol=1e-12, atol=1e-15)
    pos = inp.pos.astype(np.float64)
    for (i, a) in ((0, 0), (7, 1), (15, 2)):
        h = 1e-5
        pp, pm = pos.copy(), pos.copy()
        pp[i, a] += h
        pm[i, a] -= h
        s = int(i >= 10)
        fd = -(energy(w, inp, pos=pp)[s] - energy(w, inp, pos=pm)[s]) / (2 * h)
        assert abs(fd - r["F"][i, a]) <= 1e-6 * max(1.0, abs(fd))
    p64 = inp.params.astype(np.float64)
    sl = synth.param_slices(w)
    rng = np.random.default_rng(1)
    for name in ("l0.Wl0", "l1.Wl1", "l0.Wl2", "l1.W2", "emb"):
        off, shape = sl[name]
        for idx in rng.choice(int(np.prod(shape)), 2, replace=False):
            i = off + int(idx)
            h = 1e-5
            pp, pm = p64.copy(), p64.copy()
            pp[i] += h
            pm[i] -= h
            fd = (step(w, inp, params=pp)["loss"] - step(w, inp, params=pm)["loss"]) / (2 * h)
            assert abs(fd - r["grad"][i]) <= 2e-6 * max(1.0, abs(fd)), (name, fd, r["grad"][i])
    # the gate puts second-order weight in the mixing matrices of every l
    for name in ("l0.Wl0", "l0.Wl1", "l0.Wl2"):
        off, shape = sl[name]
        assert np.abs(r["grad_bf"][off:off + int(np.prod(shape))]).max() > 0
