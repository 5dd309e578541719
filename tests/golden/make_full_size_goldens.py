"""Writes the stored oracle summaries the full-size GPU tests compare against.  Calls only the
oracle, the seeded input generator and the probe definitions; never the HIP path.

    python tests/golden/make_full_size_goldens.py cfg2 cfg2_lmax3 cfg3 cfg4

cfg2 (16 x 256 atoms, equivariant; cfg2_lmax3: the same batch with features up to degree 3) and cfg3 (64 x 128 atoms, pipeline stage at width 512): the
oracle runs every structure of the batch (structures do not interact); stored are E, the loss, and
probes.summarise() of the parameter gradient (cfg3: of BF's and BE's shares separately).  Minutes of
CPU time -- too long for a GPU test, hence stored.

cfg4 (one cell of 20,000 atoms, 1.8 M edges): reverse-mode differentiation of the oracle does not
fit in memory, so the stored values are ones its streamed energy evaluation gives:
  E                       the energy itself;
  dE[k] = D_{d_k} E       directional derivatives in the positions (= -F . d_k), by central differences,
                          for a dense direction (every atom moves) and one confined to 64 atoms;
  dPsi[k] = D_{t_k} Psi   directional derivatives in the parameters of Psi = Ebar E + D_v E for seeded
                          cotangents Ebar, v -- what BF + BE return for those cotangents, projected on t_k;
                          nested central differences (inner in x along v, outer in theta along t_k).
Directions and cotangents come from cfg4_directions() below, which the GPU test calls too.
"""
from __future__ import annotations

import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import probes  # noqa: E402
from oracle import mlip_oracle as O  # noqa: E402
from paper_2605_18404_amd import synth  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
STREAM_DIR = 23


def cfg4_directions(w, n_params):
    """Seeded directions and cotangents of the cfg4 check (numbers only):
    d[0]: every atom moves, +-1 per component, scaled to unit length; d[1]: 64 seeded atoms move, unit length;
    v: N(0,1) per component scaled to length 1e-2 (the size of a force-loss cotangent), Ebar: 0.37;
    t[0]: +-1 on every parameter, scaled per tensor to 1e-3 of ... unit length overall; t[1]: +-1 on the second
    edge-MLP matrix of the middle layer only, unit length."""
    N = w.n_atoms
    u = synth.uniform(w.seed, STREAM_DIR, 0, 3 * N)
    d0 = np.where(u < 0.5, -1.0, 1.0).reshape(N, 3) / np.sqrt(3.0 * N)
    atoms = np.unique(np.minimum((synth.uniform(w.seed, STREAM_DIR + 1, 0, 64) * N).astype(np.int64), N - 1))
    d1 = np.zeros((N, 3))
    d1[atoms] = synth.normal(w.seed, STREAM_DIR + 2, 0, 3 * len(atoms)).reshape(-1, 3)
    d1 /= np.linalg.norm(d1)
    v = synth.normal(w.seed, STREAM_DIR + 3, 0, 3 * N).reshape(N, 3)
    v *= 1e-2 / np.linalg.norm(v)
    ut = synth.uniform(w.seed, STREAM_DIR + 4, 0, n_params)
    t0 = np.where(ut < 0.5, -1.0, 1.0) / np.sqrt(n_params)
    t1 = np.zeros(n_params)
    off, shape = synth.param_slices(w)[f"l{w.n_layers // 2}.W2"]
    n = int(np.prod(shape))
    t1[off:off + n] = np.where(synth.uniform(w.seed, STREAM_DIR + 5, 0, n) < 0.5, -1.0, 1.0) / np.sqrt(n)
    return dict(d=[d0, d1], v=v, Ebar=0.37, t=[t0, t1])


def _write(name, obj):
    path = os.path.join(HERE, name)
    with open(path, "w") as f:
        json.dump(obj, f, indent=0)
        f.write("\n")
    print("wrote", path, os.path.getsize(path), "bytes", flush=True)


def make_cfg2(l_max=2):
    w = synth.WORKLOADS[2] if l_max == 2 else synth.shrink(synth.WORKLOADS[2], l_max=l_max)
    tag = "cfg2" if l_max == 2 else "cfg2_lmax%d" % l_max
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    B, N = w.n_structs, w.n_atoms
    E, F, loss, grad = np.zeros(B), np.zeros((N, 3)), 0.0, np.zeros(inp.params.shape[0])
    for s in range(B):
        t0 = time.time()
        a, b = int(inp.struct_ptr[s]), int(inp.struct_ptr[s + 1])
        sub = dict(cfg)
        # the batch loss is mean_s + fw * mean over all 3N components: per-structure terms rescaled to sum to it
        sub["force_weight"] = cfg["force_weight"] * ((b - a) / N) * B
        r = O.train_step(sub, inp.pos[a:b], inp.species[a:b], np.array([0, b - a], np.int32), inp.cell[s:s + 1], inp.params,
                         inp.E_ref[s:s + 1], inp.F_ref[a:b])
        E[s], F[a:b] = r["E"][0], r["F"]
        loss += r["loss"] / B
        grad += r["grad"] / B
        print(tag, "structure", s, f"{time.time() - t0:.1f} s", flush=True)
    _write("full_size_%s.json" % tag, dict(
        what="oracle (float64) on the whole cfg2 batch%s, seed %d: E per structure, loss, per-structure force norms, "
             "probes.summarise of dL/dtheta" % ("" if l_max == 2 else " with features up to degree %d" % l_max, w.seed),
        E=E.tolist(), loss=loss, F_norm=[float(np.linalg.norm(F[inp.struct_ptr[s]:inp.struct_ptr[s + 1]])) for s in range(B)],
        grad=probes.summarise(w.seed, grad, synth.param_slices(w))))


def make_cfg3():
    w = synth.WORKLOADS[3]
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    st = inp.stage
    g_bf, g_be = np.zeros(inp.params.shape[0]), np.zeros(inp.params.shape[0])
    for s in range(w.n_structs):
        t0 = time.time()
        a, b = int(inp.struct_ptr[s]), int(inp.struct_ptr[s + 1])
        r = O.stage_step(cfg, inp.pos[a:b], np.array([0, b - a], np.int32), inp.cell[s:s + 1], inp.params, st["h_in"][a:b],
                         st["g_out"][a:b], st["hdot_in"][a:b], st["v"][a:b], st["lam_out"][a:b], split=True)
        g_bf += r["grad_bf"]  # Phi is a plain sum over structures
        g_be += r["grad_be"]
        print("cfg3 structure", s, f"{time.time() - t0:.1f} s", flush=True)
    sl = synth.param_slices(w)
    _write("full_size_cfg3.json", dict(
        what="oracle (float64) on the whole cfg3 stage batch, seed %d: probes.summarise of BF's and BE's shares of "
             "dPhi/dtheta (Eq. 2 split) and of their sum" % w.seed,
        grad_bf=probes.summarise(w.seed, g_bf, sl), grad_be=probes.summarise(w.seed, g_be, sl),
        grad=probes.summarise(w.seed, g_bf + g_be, sl)))


def make_cfg4():
    w = synth.WORKLOADS[4]
    inp = synth.make_inputs(w)
    cfg = O.cfg_from_workload(w)
    t0 = time.time()
    g = O.radius_graph(inp.pos, inp.struct_ptr, inp.cell, w.cutoff, chunk=16)
    print("cfg4 graph", len(g["sender"]), "edges", f"{time.time() - t0:.0f} s", flush=True)
    pos, theta = inp.pos.astype(np.float64), inp.params.astype(np.float64)
    D = cfg4_directions(w, theta.shape[0])

    def energy(x, th):
        t1 = time.time()
        e = float(O.energy_streamed(cfg, x, inp.species, inp.struct_ptr, inp.cell, th, g)[0])
        print(f"  energy evaluation {time.time() - t1:.0f} s -> {e!r}", flush=True)
        return e

    out = dict(what="oracle (float64, streamed energy) on the cfg4 cell, seed %d; see this script's docstring" % w.seed,
               n_edges=int(len(g["sender"])))
    out["E"] = energy(pos, theta)
    hx = 2e-3  # positions: step along unit-length directions (per-atom displacements are far smaller)
    out["dE"] = [(energy(pos + hx * d, theta) - energy(pos - hx * d, theta)) / (2 * hx) for d in D["d"]]
    _write("full_size_cfg4.json", out)  # partial result first: the rest takes longest
    vlen = float(np.linalg.norm(D["v"]))
    vhat = D["v"] / vlen

    def psi(th):  # Ebar E + D_v E
        ep, em = energy(pos + hx * vhat, th), energy(pos - hx * vhat, th)
        # E itself from the two displaced values (second-order accurate, like the difference)
        return D["Ebar"] * 0.5 * (ep + em) + vlen * (ep - em) / (2 * hx)

    ht = 2e-3  # parameters: step along unit-length directions
    out["dPsi"] = [(psi(theta + ht * t) - psi(theta - ht * t)) / (2 * ht) for t in D["t"]]
    out["steps"] = dict(hx=hx, ht=ht)
    _write("full_size_cfg4.json", out)


if __name__ == "__main__":
    for name in sys.argv[1:]:
        {"cfg2": make_cfg2, "cfg2_lmax3": lambda: make_cfg2(3), "cfg3": make_cfg3, "cfg4": make_cfg4}[name]()
