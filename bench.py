"""Benchmark of the whole hot path (graph build + FE + FF + loss + BF + BE) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1] [--no-cpu-baseline]

Prints ONE JSON line: atoms/s of the full training step on the synthetic workload that stands
in for the paper's 400-atom micro-batches, per-phase milliseconds, the roofline figures of the
dominant kernel (timed live with HIP events through the library's own kernel-timing entry
point) and the float64 CPU oracle timed on a bounded sample of the same workload.
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
PEAK_BF16_MFMA_TFLOPS = 2500.0


# Kernel ids of include/mlip.h and the algorithmic work of one launch (E edges, N atoms):
# GEMMs in flop (2 x rows x inner x out), gather kernels in HBM bytes (each edge tensor and each
# node table touched once, indices and geometry included).
def kernel_table(w, E, N):
    C, H, K = w.channels, w.edge_hidden, w.n_rbf
    eqv = w.l_max == 2
    Co = 11 * C if eqv else C          # width of the radial filter per edge
    f4 = 4
    fj = 2 if w.gemm_bf16 else 4       # filter jets and their adjoints are held in the operand precision
    node = (9 if eqv else 1) * N * C * f4
    geo = 16 + 4                       # unit vector + length, sender index
    return {
        1: ("fe_hidden_gemm", "mfma", 2.0 * (2 * E) * K * H),
        2: ("fe_filter_gemm", "mfma", 2.0 * (2 * E) * H * Co),
        3: ("msg_fe", "hbm", E * Co * fj + 2 * node + E * geo),
        4: ("msg_ff", "hbm", 2 * E * Co * fj + 4 * node + E * geo),
        5: ("msg_bf", "hbm", 3 * E * Co * fj + 4 * node + E * (geo + 8)),
        6: ("msg_be", "hbm", 3 * E * Co * fj + 6 * node + E * (geo + 8)),
        7: ("bf_dgrad_gemm", "mfma", 2.0 * E * Co * H),
        8: ("be_dgrad_gemm", "mfma", 2.0 * E * Co * H),
        9: ("bf_wgrad_gemm", "mfma", 2.0 * E * Co * H),
        10: ("be_wgrad_gemm", "mfma", 2.0 * E * Co * H),
    }


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
    smaller cell of the same density and model (stated in `sample`)."""
    import numpy as np
    import torch

    from oracle import mlip_oracle as O
    from paper_2605_18404_amd import synth
    note = ""
    if w.n_structs == 1 and w.atoms_per_struct > 1000:
        n = 300
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
    return {"value": done_atoms / t_used, "unit": "atoms/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"{note}{n_done} structure steps ({passes} pass(es) over the batch's {w.n_structs} structures, {done_atoms} atoms), "
                      f"graph build + full step each, {t_used:.1f} s of CPU time"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch the library's 256 MiB copy kernel once (calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2605_18404_amd import synth
    from paper_2605_18404_amd.binding import Mlip

    idx = {"cfg0": 0, "cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4": 4, "cfg1_mole128": 1}[args.workload]
    w = synth.WORKLOADS[idx]
    if args.workload == "cfg1_mole128":  # the bench batch with UMA's 128-expert banks in the update MLP (Table 4)
        w = synth.shrink(w, n_experts=128, name="cfg1_invariant_batch_mole128")
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

    for _ in range(args.warmup):
        step()
    if args.copy_probe:
        src = torch.ones(64 * 1024 * 1024, device=dev, dtype=torch.float32)
        m.mlip_copy_probe(torch.empty_like(src), src)
    torch.cuda.synchronize()
    E_edges, N = m.n_edges, w.n_atoms
    table = kernel_table(w, E_edges, N)
    # which kernel dominates: one untimed step per candidate with the library's event timer
    per_kernel_us = {}
    for kid, (name, _, _) in table.items():
        m.mlip_kernel_timer_select(kid)
        step()
        n, tot = m.mlip_kernel_timer_read()
        per_kernel_us[name] = {"launches_per_step": n, "avg_us": (tot / n * 1e3) if n else 0.0, "ms_per_step": tot}
    dom = max(table, key=lambda k: per_kernel_us[table[k][0]]["ms_per_step"])
    m.mlip_kernel_timer_select(dom)  # event pairs around its launches during the timed steps

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / args.steps
    n_launch, tot_ms = m.mlip_kernel_timer_read()
    m.mlip_kernel_timer_select(0)
    name, bound, work = table[dom]
    avg_s = tot_ms * 1e-3 / max(n_launch, 1)
    if bound == "mfma":
        peak, unit = (PEAK_BF16_MFMA_TFLOPS if w.gemm_bf16 else PEAK_FP32_MFMA_TFLOPS), "TFLOP/s"
        achieved = work / avg_s / 1e12
    else:
        peak, unit = PEAK_HBM_GBS, "GB/s"
        achieved = work / avg_s / 1e9
    roof = {"kernel": name, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
            "traffic": load_traffic(w.name, name), "avg_launch_us": avg_s * 1e6, "launches_timed": n_launch,
            "algorithmic_work_per_launch": work, "per_kernel": per_kernel_us}
    # per-phase times from HIP events (a separate, synchronous pass: it does not enter `value`)
    ph = np.zeros(5)
    n_ph = max(3, min(20, args.steps))
    for _ in range(n_ph):
        ph += np.array(step(timed=True)["phase_ms"])
    ph /= n_ph

    line = {
        "metric": "atoms/s per FE+FF+BF+BE train step", "value": w.n_atoms / (ms * 1e-3), "unit": "atoms/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if w.gemm_bf16 else "f32", "data": "synthetic",
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
        line["wavek_bubble_model_ms"] = {
            "naive_per_microbatch": wavek_model.naive_bubble(fe, ff, bf, be),
            **{f"P{P}_Nmb32_k{k}": wavek_model.wavek_bubbles(fe, ff, bf, be, P, 32, k) for P in (4, 8) for k in (P, 2 * P, 32)}}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
