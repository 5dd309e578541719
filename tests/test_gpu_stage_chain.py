"""Stage composition on the GPU: an 8-layer model run as two chained 4-layer pipeline stages must give
the update of the unsplit model (the paper's "Correctness Validation": pipelined and non-pipelined runs
of the same step agree up to floating-point summation order).

The tensors that cross the stage boundary are those of Table 2: activations h forward in FE (SAE), dE/dh
backward in FF (SAF), dL_F/d(dE/dh) forward in BF (SGF), dL/dh backward in BE (SGE).  The two stages are
two MLIP_MODEL_STAGE contexts; what sits outside the stages' layers (embedding lookup, readout, loss
cotangents) is evaluated by the test in float64 with plain tensor operations, as a pipeline's first and
last stage would around their layers.  The chained result is compared with the whole-model context's
mlip_train_step (same kernels, unsplit) and with the oracle's.
"""
import numpy as np
import pytest
import torch

from paper_2605_18404_amd import synth
from paper_2605_18404_amd.binding import Mlip

from gpu_common import DEV, DevInputs, dev, oracle_train_step, rel

pytestmark = pytest.mark.gpu


def _chain_case(bf16):
    return synth.shrink(synth.WORKLOADS[1], n_structs=3, atoms_per_struct=40, box=(40 / 0.08) ** (1 / 3), n_layers=8,
                        edge_depth=3, channels=64, edge_hidden=96, gemm_bf16=bf16)


@pytest.mark.parametrize("bf16", [False, True])
def test_two_chained_stages_reproduce_the_whole_model(bf16):
    tol = 2e-2 if bf16 else 1e-4
    w = _chain_case(bf16)
    inp = synth.make_inputs(w)
    d = DevInputs(inp)
    N, B, C, L = w.n_atoms, w.n_structs, w.channels, w.n_layers
    sl = synth.param_slices(w)
    lo, mid, hi = sl["l0.W1"][0], sl[f"l{L // 2}.W1"][0], sl["U"][0]

    # the unsplit model, one context
    whole = Mlip.for_workload(w)
    out = whole.mlip_train_step(d.pos, d.species, d.struct_ptr, d.cell, w.cutoff, d.params, d.E_ref, d.F_ref)
    torch.cuda.synchronize()
    E_w, F_w, g_w = out["E"].cpu().numpy(), out["F"].cpu().numpy(), out["grad"].cpu().numpy()
    n_edges = whole.n_edges
    whole.close()

    # two stage contexts with the layer blocks 0..3 and 4..7 of the same parameter vector
    ws = synth.shrink(w, kind=synth.KIND_STAGE, n_layers=L // 2)
    A, Bst = Mlip.for_workload(ws), Mlip.for_workload(ws)
    thA, thB = dev(inp.params[lo:mid]), dev(inp.params[mid:hi])
    for m in (A, Bst):
        assert m.mlip_graph_build(d.pos, d.struct_ptr, d.cell, w.cutoff) == n_edges

    th = torch.tensor(inp.params, dtype=torch.float64)
    emb = th[sl["emb"][0]:sl["emb"][0] + w.n_species * C].reshape(w.n_species, C)
    U = th[sl["U"][0]:sl["U"][0] + C * C].reshape(C, C).clone().requires_grad_(True)
    wo = th[sl["w_o"][0]:sl["w_o"][0] + C].clone().requires_grad_(True)
    sid = torch.repeat_interleave(torch.arange(B), w.atoms_per_struct)
    species = torch.as_tensor(inp.species, dtype=torch.long)
    f32 = lambda t: t.detach().to(torch.float32).contiguous().to(DEV)

    # FE: embedding -> A -> (SAE) -> B -> readout
    h_in = f32(emb[species])
    h_mid = A.mlip_forward_energy(d.pos, None, thA, h_in=h_in)
    h_L = Bst.mlip_forward_energy(d.pos, None, thB, h_in=h_mid)
    hL = h_L.cpu().double().requires_grad_(True)

    def readout(h):
        y = h @ U.t()
        return torch.zeros(B, dtype=torch.float64).index_add(0, sid, (y * torch.sigmoid(y)) @ wo)

    E = readout(hL)
    (g_out,) = torch.autograd.grad(E.sum(), hL, create_graph=True)
    # FF: readout -> B -> (SAF) -> A; each stage adds its share of dE/dx
    pB, g_mid = Bst.mlip_forward_force(g_out=f32(g_out))
    pA, g_in = A.mlip_forward_force(g_out=g_mid)
    F = -(pA + pB).cpu().double()
    # loss cotangents
    E_ref, F_ref = torch.tensor(inp.E_ref, dtype=torch.float64), torch.tensor(inp.F_ref, dtype=torch.float64)
    Ebar = 2.0 * (E.detach() - E_ref) / B
    v = -2.0 * w.force_weight * (F - F_ref) / (3 * N)
    # BF: A -> (SGF) -> B -> readout
    gA_bf, gB_bf = torch.zeros(mid - lo, device=DEV), torch.zeros(hi - mid, device=DEV)
    hdot_mid = A.mlip_backward_force(f32(v), gA_bf, hdot_in=None)
    hdot_L = Bst.mlip_backward_force(f32(v), gB_bf, hdot_in=hdot_mid)
    # the readout's part of Psi = sum_s Ebar_s E_s + <dE/dh^L, hdot^L>: its gradients w.r.t. h^L, U, w_o
    Psi = (Ebar * E).sum() + (g_out * hdot_L.cpu().double()).sum()
    lam_out, gU, gwo = torch.autograd.grad(Psi, [hL, U, wo])
    # BE: readout -> B -> (SGE) -> A -> embedding
    gA_be, gB_be = torch.zeros_like(gA_bf), torch.zeros_like(gB_bf)
    lam_mid = Bst.mlip_backward_energy(gB_be, lam_out=f32(lam_out))
    lam_in = A.mlip_backward_energy(gA_be, lam_out=lam_mid)
    torch.cuda.synchronize()
    gemb = torch.zeros(w.n_species, C, dtype=torch.float64).index_add(0, species, lam_in.cpu().double())
    g_chain = np.concatenate([gemb.reshape(-1).numpy(), (gA_bf + gA_be).cpu().numpy(), (gB_bf + gB_be).cpu().numpy(),
                              gU.reshape(-1).numpy(), gwo.numpy()])
    A.close()
    Bst.close()

    # chained = unsplit (same kernels: only the readout's precision differs, so far inside the tolerance)
    tight = tol / 2 if bf16 else tol / 4  # bf16: the unsplit model's readout product is a bf16 product, the test's is float64
    assert rel(E.detach().numpy(), E_w) < tight
    assert rel(F.numpy(), F_w) < tight
    assert rel(g_chain, g_w) < tight
    for name, (off, shape) in sl.items():
        n = int(np.prod(shape))
        assert rel(g_chain[off:off + n], g_w[off:off + n]) < 3 * tight, name
    # and both equal the oracle
    ref = oracle_train_step(w, inp)
    assert rel(E.detach().numpy(), ref["E"]) < tol and rel(F.numpy(), ref["F"]) < tol
    assert rel(g_chain, ref["grad"]) < tol
    for name, (off, shape) in sl.items():
        n = int(np.prod(shape))
        assert rel(g_chain[off:off + n], ref["grad"][off:off + n]) < 3 * tol, name
