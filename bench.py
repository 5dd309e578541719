"""Benchmark of the whole hot path (graph build + FE + FF + loss + BF + BE) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--others cfg0,cfg1,cfg2,cfg3,cfg2_lmax3]
                    [--no-others] [--no-cpu-baseline] [--copy-probe]

Prints ONE JSON line.  The headline (`value`, `ms_per_step`, `phase_ms`, `roofline`) is the largest
single-GPU workload, cfg4: one periodic cell of 20,000 atoms (1.8 M edges) under the l <= 2 equivariant
model with bf16 matrix products -- the stand-in, at this build's scale, for the paper's 400-atom
micro-batches.  `per_workload` carries the same measurements (shorter runs) for the other four
workloads, so that one default run reports all five.  Per workload:
  * atoms/s and edges/s of the full training step, inputs resident in HBM, graph build included;
  * per-phase milliseconds from HIP events (graph, FE, FF + loss, BF, BE);
  * every instrumented kernel's average launch time, measured live with HIP-event pairs recorded by the
    library on the stream it launches on (mlip_kernel_timer_select / _read);
  * the roofline figures of the kernel that takes the most time per step (during the timed steps the
    library's event pairs bracket that kernel's launches): matrix products against the MFMA peak of
    their operand type; the invariant gather kernels against the HBM peak; the equivariant
    tensor-product kernels, which are bound by plain fp32 vector arithmetic, against the fp32 vector
    peak (`bound: "alu"`), with their HBM figures beside it -- both the bytes this build actually
    streams (materialised filter jets) and the floor of an implementation that would stream none.
The float64 CPU oracle is timed on a bounded sample of the headline workload (`cpu_baseline`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_FP32_VALU_TFLOPS = 157.3   # 256 CUs x 128 fp32 FMA lanes x 2 flop x 2.4 GHz
PEAK_BF16_MFMA_TFLOPS = 2500.0
# per l_max of the equivariant model: (non-zero entries of the real coupling tensors, counted from the generated table;
# coupling paths; components of a feature vector; path values per channel as stored)
COUPLINGS = {2: (83, 11, 9, 12), 3: (353, 23, 16, 24)}


def kernel_table(w, E, N):
    """Kernel ids of include/mlip.h -> (name, bound, algorithmic work per launch, extra figures).
    Matrix products: flop = 2 x rows x inner x out, with one row (one jet of two rows) per edge PAIR: opposite edges have
    the same length, so the edge MLP, its filter jets and their adjoints exist once per pair (E / 2).  Invariant gather kernels: HBM bytes, every edge tensor
    and node table touched once, indices and geometry included.  Equivariant tensor-product kernels: fp32
    vector flop = 2 (nnz(T) + components * paths) per edge, channel and evaluation of the trilinear form (1 in FE, 2 in
    FF, 3 in BF, 4 in BE; 83 + 9 * 11 for l <= 2, 353 + 16 * 23 for l <= 3), with two HBM byte counts beside it:
    `hbm_streamed` = what this build moves (the materialised filter jets, 12 (24) values per channel and row, and their
    adjoints, and every node table touched once) and `hbm_floor` = node tables once plus 20 bytes per edge, what an
    implementation that recomputed the filters would move.
    The first layer's input has its l = 0 component only and the readout takes only the l = 0 component of the last
    layer's output, so the method itself needs just l_max + 1 paths in each of these two layers -- (0, l, l) and (l, l, 0),
    (l_max + 1)^2 coupling entries, 4 stored values per channel, node tables of one component where only one is live: all
    per-launch figures of the equivariant model are averages over the layers' launches, each layer counted at its own size."""
    C, H, K = w.channels, w.edge_hidden, w.n_rbf
    eqv = w.l_max >= 2
    nnz, n_paths, n_comp, n_stored = COUPLINGS[w.l_max] if eqv else (0, 1, 1, 1)
    L = w.n_layers
    f4 = 4
    fj = 2 if (w.gemm_bf16 and not getattr(w, "filter_fp32", 0)) else 4   # filter jets
    fx = 2 if w.gemm_bf16 else 4                                           # their adjoints (matrix-product operands)
    geo = 16 + 4                       # unit vector + length, sender index
    tab = N * C * f4                   # one component of a node table
    M = n_comp
    # per layer kind: paths, stored values per channel, coupling entries, node-table components touched by FE, FF, BF, BE
    general = (n_paths, n_stored, nnz, (2 * M, 4 * M, 4 * M, 6 * M))
    if eqv:
        lp = w.l_max + 1
        first = (lp, 4, lp * lp, (1 + M, 1 + M, 1 + 2 * M, 3 + 2 * M))
        last = (lp, 4, lp * lp, (M + 1, 2 + 2 * M, 2 + 2 * M, 3 + 3 * M))
        layers = [first] + [general] * (L - 2) + ([last] if L >= 2 else [])
    else:
        layers = [general] * L
    avg = lambda f: sum(f(x) for x in layers) / len(layers)
    Co = avg(lambda x: x[0]) * C       # width of the radial filter per edge
    Eu = E // 2                        # edge pairs: the rows (jets) of every product of the edge MLP
    t = {
        1: ("fe_hidden_gemm", "mfma", 2.0 * (2 * Eu) * K * H, {}),
        2: ("fe_filter_gemm", "mfma", 2.0 * (2 * Eu) * H * Co, {}),
        7: ("bf_dgrad_gemm", "mfma", 2.0 * Eu * Co * H, {}),
        8: ("be_dgrad_gemm", "mfma", 2.0 * Eu * Co * H, {}),
        9: ("bf_wgrad_gemm", "mfma", 2.0 * Eu * Co * H, {}),
        10: ("be_wgrad_gemm", "mfma", 2.0 * Eu * Co * H, {}),
    }
    jets = {3: 1, 4: 2, 5: 2, 6: 2}    # filter-jet rows read per edge
    adj = {3: 0, 4: 0, 5: 1, 6: 1}     # adjoint rows written per edge
    extra = {3: 0, 4: 0, 5: 8, 6: 8}   # envelope pair
    names = {3: "msg_fe", 4: "msg_ff", 5: "msg_bf", 6: "msg_be"}
    for kid in (3, 4, 5, 6):
        streamed = avg(lambda x: E * x[1] * C * (jets[kid] * fj + adj[kid] * fx) + x[3][kid - 3] * tab) + E * (geo + extra[kid])
        if eqv:
            flop = 2.0 * avg(lambda x: x[2] + M * x[0]) * C * E * (kid - 2)
            floor = avg(lambda x: x[3][kid - 3] * tab) + 20 * E
            t[kid] = (names[kid], "alu", flop, {"hbm_streamed_bytes": streamed, "hbm_floor_bytes": floor})
        else:
            t[kid] = (names[kid], "hbm", streamed, {})
    return dict(sorted(t.items()))


def load_traffic(workload, kernel):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if one exists."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f)[workload][kernel]["bytes_per_launch"]
    except Exception:
        return None


def cpu_baseline(w, inp, budget_s=20.0):
    """Times the oracle as it stands on a bounded sample: whole structures of the batch, one
    after the other (graph build + all four phases each), until about budget_s seconds of CPU
    work have been spent.  A single-structure workload too large for the oracle is sampled by a
    smaller cell of the same density and model (stated in `sample` and in `stand_in`)."""
    import numpy as np
    import torch

    from oracle import mlip_oracle as O
    from paper_2605_18404_amd import synth
    note, stand_in = "", None
    if w.n_structs == 1 and w.atoms_per_struct > 1000:
        n = 300
        stand_in = {"atoms": n, "reason": "the oracle's reverse-mode pass over the 20,000-atom cell does not fit in host memory; "
                                          "same density, same model, periodic cell of 300 atoms"}
        w = synth.shrink(w, atoms_per_struct=n, box=w.box * (n / w.atoms_per_struct) ** (1.0 / 3.0))
        inp = synth.make_inputs(w)
        note = f"a {n}-atom cell of the same density and model stands in for the large cell; "
    cfg = O.cfg_from_workload(w)
    done_atoms, t_used, n_done, passes = 0, 0.0, 0, 0
    # whole passes over the batch until about 12 s are spent (at most 10 passes), never beyond budget_s
    while t_used < 12.0 and passes < 10:
        for s in range(w.n_structs):
            a, b = int(inp.struct_ptr[s]), int(inp.struct_ptr[s + 1])
            sp = np.array([0, b - a], np.int32)
            t0 = time.perf_counter()
            if w.kind == synth.KIND_STAGE:
                st = {k: v[a:b] for k, v in inp.stage.items()}
                O.stage_step(cfg, inp.pos[a:b], sp, inp.cell[s:s + 1], inp.params, st["h_in"], st["g_out"], st["hdot_in"],
                             st["v"], st["lam_out"])
            else:
                O.train_step(cfg, inp.pos[a:b], inp.species[a:b], sp, inp.cell[s:s + 1], inp.params, inp.E_ref[s:s + 1],
                             inp.F_ref[a:b], alpha=None if inp.alpha is None else inp.alpha[s:s + 1])
            t_used += time.perf_counter() - t0
            done_atoms += b - a
            n_done += 1
            if t_used > budget_s:
                break
        passes += 1
        if t_used > budget_s:
            break
    out = {"value": done_atoms / t_used, "unit": "atoms/s", "cores": torch.get_num_threads(), "kind": "oracle",
           "sample": f"{note}{n_done} structure steps ({passes} pass(es) over the batch's {w.n_structs} structures, {done_atoms} atoms), "
                     f"graph build + full step each, {t_used:.1f} s of CPU time"}
    if stand_in:
        out["stand_in"] = stand_in
    return out


WORKLOAD_INDEX = {"cfg0": 0, "cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4": 4, "cfg1_mole128": 1, "cfg2_lmax3": 2}


def make_workload(name):
    from paper_2605_18404_amd import synth
    w = synth.WORKLOADS[WORKLOAD_INDEX[name]]
    if name == "cfg1_mole128":  # the invariant batch with UMA's 128-expert banks in the update MLP (Table 4)
        w = synth.shrink(w, n_experts=128, name="cfg1_invariant_batch_mole128")
    if name == "cfg2_lmax3":    # the equivariant batch with features up to degree 3 (16 components, 23 coupling paths)
        w = synth.shrink(w, l_max=3, name="cfg2_equivariant_batch_lmax3")
    return w


def measure(name, steps, warmup, copy_probe=False):
    """All measurements of one workload: (result dict, workload, inputs)."""
    import numpy as np
    import torch

    from paper_2605_18404_amd import synth
    from paper_2605_18404_amd.binding import Mlip

    w = make_workload(name)
    inp = synth.make_inputs(w)
    dev = "cuda:0"
    t = lambda a: torch.as_tensor(np.ascontiguousarray(a)).to(dev)
    m = Mlip.for_workload(w, device=dev)
    d = dict(pos=t(inp.pos), species=t(inp.species), struct_ptr=t(inp.struct_ptr), cell=t(inp.cell),
             params=t(inp.params), E_ref=t(inp.E_ref), F_ref=t(inp.F_ref))
    st = {k: t(v) for k, v in inp.stage.items()}
    if w.n_experts > 0:
        m.mlip_set_expert_weights(t(inp.alpha))
        grad_alpha = torch.zeros(w.n_structs, w.n_experts, device=dev)
        m.mlip_set_expert_weight_grad(grad_alpha)  # the step then also yields the router's gradient dL/dalpha
    out = None
    grad = torch.zeros(m.mlip_param_count(), device=dev)

    def step(timed=False):
        """One pass of the whole hot path.  A pipeline stage has no loss: its step is graph
        build + FE + FF + BF + BE on the seeded boundary tensors."""
        nonlocal out
        if w.kind != synth.KIND_STAGE:
            out = m.mlip_train_step(d["pos"], d["species"], d["struct_ptr"], d["cell"], w.cutoff, d["params"],
                                    d["E_ref"], d["F_ref"], out=out, timed=timed)
            return out
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)] if timed else None
        mark = (lambda k: ev[k].record()) if timed else (lambda k: None)
        mark(0)
        m.mlip_graph_build(d["pos"], d["struct_ptr"], d["cell"], w.cutoff)
        mark(1)
        m.mlip_forward_energy(d["pos"], None, d["params"], h_in=st["h_in"])
        mark(2)
        m.mlip_forward_force(g_out=st["g_out"])
        mark(3)
        grad.zero_()
        m.mlip_backward_force(st["v"], grad, hdot_in=st["hdot_in"])
        mark(4)
        m.mlip_backward_energy(grad, lam_out=st["lam_out"])
        mark(5)
        res = {}
        if timed:
            torch.cuda.synchronize()
            res["phase_ms"] = [ev[k].elapsed_time(ev[k + 1]) for k in range(5)]
        return res

    for _ in range(warmup):
        step()
    if copy_probe:
        src = torch.ones(64 * 1024 * 1024, device=dev, dtype=torch.float32)
        m.mlip_copy_probe(torch.empty_like(src), src)
    torch.cuda.synchronize()
    E_edges, N = m.n_edges, w.n_atoms
    table = kernel_table(w, E_edges, N)
    # which kernel dominates: one untimed step per candidate with the library's event timer
    per_kernel = {}
    for kid, (kname, _, _, _) in table.items():
        m.mlip_kernel_timer_select(kid)
        step()
        n, tot = m.mlip_kernel_timer_read()
        per_kernel[kname] = {"launches_per_step": n, "avg_us": (tot / n * 1e3) if n else 0.0, "ms_per_step": tot}
    dom = max(table, key=lambda k: per_kernel[table[k][0]]["ms_per_step"])
    m.mlip_kernel_timer_select(dom)  # event pairs around its launches during the timed steps

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / steps
    n_launch, tot_ms = m.mlip_kernel_timer_read()
    m.mlip_kernel_timer_select(0)

    def figures(kid, avg_s):
        kname, bound, work, extra = table[kid]
        if bound == "mfma":
            peak, unit = (PEAK_BF16_MFMA_TFLOPS if w.gemm_bf16 else PEAK_FP32_MFMA_TFLOPS), "TFLOP/s"
            achieved = work / avg_s / 1e12
        elif bound == "alu":
            peak, unit = PEAK_FP32_VALU_TFLOPS, "TFLOP/s"
            achieved = work / avg_s / 1e12
        else:
            peak, unit = PEAK_HBM_GBS, "GB/s"
            achieved = work / avg_s / 1e9
        r = {"kernel": kname, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
             "traffic": load_traffic(w.name, kname), "avg_launch_us": avg_s * 1e6, "algorithmic_work_per_launch": work}
        for k, b in extra.items():  # the tensor-product kernels' HBM figures beside their arithmetic ones
            r[k] = b
            r[k.replace("_bytes", "_GBs")] = b / avg_s / 1e9
            r[k.replace("_bytes", "_frac_of_hbm_peak")] = b / avg_s / 1e9 / PEAK_HBM_GBS
        return r

    roof = figures(dom, tot_ms * 1e-3 / max(n_launch, 1))
    roof["launches_timed"] = n_launch
    # every instrumented kernel against its own roofline (from the selection pass: one step each)
    for kid, (kname, _, _, _) in table.items():
        if per_kernel[kname]["launches_per_step"]:
            f = figures(kid, per_kernel[kname]["avg_us"] * 1e-6)
            per_kernel[kname].update({k: f[k] for k in f if k not in ("kernel", "avg_launch_us")})
    roof["per_kernel"] = per_kernel
    # per-phase times from HIP events (a separate, synchronous pass: it does not enter `value`)
    ph = np.zeros(5)
    n_ph = max(3, min(20, steps))
    for _ in range(n_ph):
        ph += np.array(step(timed=True)["phase_ms"])
    ph /= n_ph
    res = {
        "value": w.n_atoms / (ms * 1e-3), "ms_per_step": ms, "steps": steps, "warmup": warmup,
        "dtype": "bf16" if w.gemm_bf16 else "f32",
        "config": {"workload": w.name, "atoms": w.n_atoms, "structures": w.n_structs, "edges": E_edges,
                   "channels": w.channels, "layers": w.n_layers, "n_rbf": w.n_rbf, "cutoff": w.cutoff,
                   "l_max": w.l_max, "edge_mlp_depth": w.edge_depth, "n_experts": w.n_experts, "includes_graph_build": True,
                   "workspace_GB": m.mlip_workspace_bytes() / 1e9},
        "edges_per_s": E_edges / (ms * 1e-3),
        "phase_ms": {"graph": ph[0], "FE": ph[1], "FF": ph[2], "BF": ph[3], "BE": ph[4]},
        "roofline": roof,
    }
    if w.kind == synth.KIND_STAGE:
        # the stage's measured phase times in the paper's closed-form bubble model (Sec. 4.2)
        from paper_2605_18404_amd import wavek_model
        fe, ff, bf, be = ph[1], ph[2], ph[3], ph[4]
        res["wavek_bubble_model_ms"] = {
            "naive_per_microbatch": wavek_model.naive_bubble(fe, ff, bf, be),
            **{f"P{P}_Nmb32_k{k}": wavek_model.wavek_bubbles(fe, ff, bf, be, P, 32, k) for P in (4, 8) for k in (P, 2 * P, 32)}}
    m.close()
    del m, d, st, grad, out
    torch.cuda.empty_cache()
    return res, w, inp


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg4", choices=sorted(WORKLOAD_INDEX))
    ap.add_argument("--others", default="cfg0,cfg1,cfg2,cfg3,cfg2_lmax3",
                    help="workloads measured with shorter runs and reported under per_workload")
    ap.add_argument("--no-others", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch the library's 256 MiB copy kernel once (calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    head, w, inp = measure(args.workload, args.steps, args.warmup, copy_probe=args.copy_probe)
    line = {
        "metric": "atoms/s per FE+FF+BF+BE train step", "value": head["value"], "unit": "atoms/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": head["config"], "edges_per_s": head["edges_per_s"], "phase_ms": head["phase_ms"], "roofline": head["roofline"],
    }
    if "wavek_bubble_model_ms" in head:
        line["wavek_bubble_model_ms"] = head["wavek_bubble_model_ms"]
    if not args.no_others:
        line["per_workload"] = {}
        for name in [n for n in args.others.split(",") if n and n != args.workload]:
            r, _, _ = measure(name, max(5, min(30, args.steps)), max(2, min(5, args.warmup)))
            roof = r["roofline"]
            line["per_workload"][name] = {
                "workload": r["config"]["workload"], "atoms_per_s": r["value"], "edges_per_s": r["edges_per_s"],
                "ms_per_step": r["ms_per_step"], "steps": r["steps"], "dtype": r["dtype"], "phase_ms": r["phase_ms"],
                "atoms": r["config"]["atoms"], "edges": r["config"]["edges"], "workspace_GB": r["config"]["workspace_GB"],
                "dominant_kernel": {k: roof[k] for k in roof if k != "per_kernel"},
                "per_kernel": roof["per_kernel"],
                **({"wavek_bubble_model_ms": r["wavek_bubble_model_ms"]} if "wavek_bubble_model_ms" in r else {}),
            }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, inp)
        if "stand_in" in line["cpu_baseline"]:
            line["config"]["cpu_baseline_stand_in"] = line["cpu_baseline"]["stand_in"]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
