"""Thin ctypes binding over libmlip.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/mlip.h).  Tensors are
torch CUDA (ROCm) tensors used as device memory; their data pointers and the current
stream handle are what crosses the boundary.  There is no CPU path: if the library is
missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmlip.so")
_lib = None

MODEL_INVARIANT, MODEL_EQUIVARIANT, MODEL_STAGE = 0, 1, 2
STATUS = {0: "MLIP_OK", -1: "MLIP_E_INVALID", -2: "MLIP_E_CAPACITY", -3: "MLIP_E_UNSUPPORTED",
          -4: "MLIP_E_STATE", -5: "MLIP_E_HIP", -6: "MLIP_E_POSITION"}


class MlipError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


class mlip_config(C.Structure):
    _fields_ = [("model_kind", C.c_int32), ("n_species", C.c_int32), ("channels", C.c_int32),
                ("n_layers", C.c_int32), ("n_rbf", C.c_int32), ("edge_hidden", C.c_int32),
                ("edge_mlp_depth", C.c_int32), ("l_max", C.c_int32), ("gemm_dtype", C.c_int32),
                ("n_experts", C.c_int32), ("gate", C.c_int32), ("filter_fp32", C.c_int32), ("position_grad", C.c_int32), ("cutoff", C.c_float), ("force_weight", C.c_float),
                ("max_atoms", C.c_int64), ("max_structs", C.c_int64), ("max_edges", C.c_int64)]


class mlip_adamw(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("grad_scale", C.c_float)]


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Loads libmlip.so (once).  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} not found: build it with __graft_entry__.build() "
                           "(python paper_2605_18404_amd/build.py); there is no CPU fallback")
    lib = C.CDLL(_LIB_PATH)
    P, I64, I32, F = C.c_void_p, C.c_int64, C.c_int32, C.c_float
    lib.mlip_create.argtypes = [C.POINTER(mlip_config), P, C.POINTER(P)]
    lib.mlip_destroy.argtypes = [P]
    lib.mlip_param_count.argtypes = [P]
    lib.mlip_param_count.restype = I64
    lib.mlip_workspace_bytes.argtypes = [P]
    lib.mlip_workspace_bytes.restype = I64
    lib.mlip_last_error.argtypes = [P]
    lib.mlip_last_error.restype = C.c_char_p
    lib.mlip_graph_build.argtypes = [P, I64, I32, P, P, P, F, C.POINTER(I64)]
    lib.mlip_graph_export.argtypes = [P, P, P, P, P]
    lib.mlip_graph_export_pairs.argtypes = [P, P, P]
    lib.mlip_graph_sizes.argtypes = [P, C.POINTER(I64), C.POINTER(I64), C.POINTER(I64)]
    lib.mlip_kernel_timer_select.argtypes = [P, I32]
    lib.mlip_kernel_timer_read.argtypes = [P, C.POINTER(I64), C.POINTER(C.c_float)]
    lib.mlip_copy_probe.argtypes = [P, P, P, I64]
    lib.mlip_gars_pack.argtypes = [P, I64, I32, I32, C.c_uint64, P, P, P]
    lib.mlip_set_expert_weights.argtypes = [P, P, I32]
    lib.mlip_set_expert_weight_grad.argtypes = [P, P, I32]
    lib.mlip_input_status.argtypes = [P]
    lib.mlip_set_position_grad.argtypes = [P, P]
    lib.mlip_graph_build_static.argtypes = [I64, I32, P, P, P, F, P, I64, P, P, P, P, C.POINTER(I64)]
    lib.mlip_graph_build_static_error.argtypes = []
    lib.mlip_graph_build_static_error.restype = C.c_char_p
    lib.mlip_optimizer_step.argtypes = [P, I64, P, P, P, P, I32, C.POINTER(mlip_adamw)]
    lib.mlip_forward_energy.argtypes = [P, P, P, P, P, P, P]
    lib.mlip_forward_force.argtypes = [P, P, P, P]
    lib.mlip_loss.argtypes = [P, P, P, P, P, P, P, P]
    lib.mlip_backward_force.argtypes = [P, P, P, P, P]
    lib.mlip_backward_energy.argtypes = [P, P, P, P, P]
    lib.mlip_train_step.argtypes = [P, I64, I32, P, P, P, P, F, P, P, P, P, P, P, P, C.POINTER(C.c_float)]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def mlip_gars_pack(sizes, n_mb: int, d_gp: int, seed: int):
    """Host routine (no GPU): sizes = int32 numpy array of atom counts.
    Returns (mb_ptr [n_mb+1], order [M], type [n_mb]) as int32 numpy arrays."""
    import numpy as np
    lib = load()
    sizes = np.ascontiguousarray(sizes, dtype=np.int32)
    M = sizes.shape[0]
    mb_ptr = np.zeros(n_mb + 1, np.int32)
    order = np.zeros(max(M, 1), np.int32)
    typ = np.zeros(n_mb, np.int32)
    s = lib.mlip_gars_pack(sizes.ctypes.data, M, n_mb, d_gp, C.c_uint64(seed), mb_ptr.ctypes.data, order.ctypes.data,
                           typ.ctypes.data)
    if s != 0:
        raise MlipError(s, "mlip_gars_pack: invalid argument")
    return mb_ptr, order[:M], typ


def mlip_graph_build_static(pos, struct_ptr, cell, cutoff: float, row_ptr, sender, shift, rev, stream=None) -> int:
    """Context-free radius graph into the caller's preallocated device tensors (row_ptr [N+1], sender [cap],
    shift [cap,3], rev [cap], int32).  Allocates nothing on the device.  Returns the edge count."""
    lib = load()
    n = C.c_int64(0)
    st = stream if stream is not None else torch.cuda.current_stream(pos.device)
    cap = min(sender.shape[0], shift.shape[0], rev.shape[0])
    s = lib.mlip_graph_build_static(pos.shape[0], struct_ptr.shape[0] - 1, _ptr(pos, torch.float32),
                                    _ptr(struct_ptr, torch.int32), _ptr(cell, torch.float32), cutoff,
                                    C.c_void_p(st.cuda_stream), cap, _ptr(row_ptr, torch.int32), _ptr(sender, torch.int32),
                                    _ptr(shift, torch.int32), _ptr(rev, torch.int32), C.byref(n))
    if s != 0:
        e = MlipError(s, lib.mlip_graph_build_static_error().decode())
        e.n_edges = int(n.value)
        raise e
    return int(n.value)


class Mlip:
    """One context: model shape + workspace for given capacities, bound to a device stream."""

    def __init__(self, *, model_kind: int, channels: int, n_layers: int, n_rbf: int, edge_hidden: int,
                 edge_mlp_depth: int = 2, l_max: int = 0, n_species: int = 1, gemm_bf16: bool = False,
                 n_experts: int = 0, gate: int = 0, filter_fp32: int = 0, position_grad: int = 0, cutoff: float, force_weight: float = 10.0, max_atoms: int, max_structs: int, max_edges: int,
                 device: str = "cuda:0", stream: Optional[torch.cuda.Stream] = None):
        self.lib = load()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.cfg = mlip_config(model_kind, n_species, channels, n_layers, n_rbf, edge_hidden, edge_mlp_depth, l_max,
                               1 if gemm_bf16 else 0, n_experts, gate, filter_fp32, position_grad, cutoff, force_weight, max_atoms, max_structs, max_edges)
        self.ctx = C.c_void_p()
        s = self.lib.mlip_create(C.byref(self.cfg), C.c_void_p(self.stream.cuda_stream), C.byref(self.ctx))
        if s != 0:
            self.ctx = C.c_void_p()
            raise MlipError(s, "mlip_create failed (bad configuration or out of device memory)")
        self.n_atoms = 0
        self.n_structs = 0
        self.n_edges = 0

    @classmethod
    def for_workload(cls, w, max_edges: Optional[int] = None, **kw) -> "Mlip":
        """Context sized for a synth.Workload (edge capacity from its mean degree, with slack)."""
        import math
        if max_edges is None:
            rho = w.atoms_per_struct / w.box ** 3
            deg = rho * 4.0 / 3.0 * math.pi * w.cutoff ** 3
            max_edges = int(w.n_atoms * (deg * 1.15 + 8))
        args = dict(model_kind=w.kind, channels=w.channels, n_layers=w.n_layers, n_rbf=w.n_rbf,
                    edge_hidden=w.edge_hidden, edge_mlp_depth=w.edge_depth, l_max=w.l_max, n_species=w.n_species,
                    gemm_bf16=w.gemm_bf16, n_experts=getattr(w, "n_experts", 0), gate=getattr(w, "gate", 0), filter_fp32=getattr(w, "filter_fp32", 0), cutoff=w.cutoff, force_weight=w.force_weight, max_atoms=w.n_atoms,
                    max_structs=w.n_structs, max_edges=max_edges)
        args.update(kw)
        return cls(**args)

    def close(self):
        if getattr(self, "ctx", None) is not None and self.ctx.value:
            self.lib.mlip_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, s: int):
        if s != 0:
            raise MlipError(s, self.lib.mlip_last_error(self.ctx).decode())

    # ------------------------------------------------------------------ C entry points
    def mlip_param_count(self) -> int:
        return int(self.lib.mlip_param_count(self.ctx))

    def mlip_workspace_bytes(self) -> int:
        return int(self.lib.mlip_workspace_bytes(self.ctx))

    def mlip_graph_build(self, pos: torch.Tensor, struct_ptr: torch.Tensor, cell: torch.Tensor, cutoff: float) -> int:
        n = C.c_int64(0)
        N, B = pos.shape[0], struct_ptr.shape[0] - 1
        s = self.lib.mlip_graph_build(self.ctx, N, B, _ptr(pos, torch.float32), _ptr(struct_ptr, torch.int32),
                                      _ptr(cell, torch.float32), cutoff, C.byref(n))
        self.n_edges = int(n.value)
        self._check(s)
        self.n_atoms, self.n_structs = N, B
        return self.n_edges

    def mlip_graph_sizes(self):
        a, b, e = C.c_int64(0), C.c_int64(0), C.c_int64(0)
        self._check(self.lib.mlip_graph_sizes(self.ctx, C.byref(a), C.byref(b), C.byref(e)))
        return int(a.value), int(b.value), int(e.value)

    def mlip_set_position_grad(self, grad_pos):
        """grad_pos: device tensor [N,3] float32 that mlip_backward_energy then overwrites with dL/dx, or None."""
        self._check(self.lib.mlip_set_position_grad(self.ctx, _ptr(grad_pos, torch.float32)))
        self._grad_pos = grad_pos  # keep the tensor alive while the library holds its address

    def mlip_input_status(self):
        """Synchronous: raises MlipError if a kernel met a bad species index or coincident atoms."""
        self._check(self.lib.mlip_input_status(self.ctx))

    def mlip_kernel_timer_select(self, kernel_id: int):
        self._check(self.lib.mlip_kernel_timer_select(self.ctx, kernel_id))

    def mlip_kernel_timer_read(self):
        """(launches, total milliseconds) of the selected kernel since it was selected."""
        n, ms = C.c_int64(0), C.c_float(0.0)
        self._check(self.lib.mlip_kernel_timer_read(self.ctx, C.byref(n), C.byref(ms)))
        return int(n.value), float(ms.value)

    def mlip_copy_probe(self, dst, src):
        self._check(self.lib.mlip_copy_probe(self.ctx, _ptr(dst, torch.float32), _ptr(src, torch.float32), src.numel()))

    def mlip_graph_export(self):
        E, N = self.n_edges, self.n_atoms
        o = dict(device=self.device, dtype=torch.int32)
        row_ptr, sender = torch.empty(N + 1, **o), torch.empty(E, **o)
        shift, rev = torch.empty(E, 3, **o), torch.empty(E, **o)
        self._check(self.lib.mlip_graph_export(self.ctx, _ptr(row_ptr), _ptr(sender), _ptr(shift), _ptr(rev)))
        return row_ptr, sender, shift, rev

    def mlip_graph_export_pairs(self):
        E = self.n_edges
        o = dict(device=self.device, dtype=torch.int32)
        slot, pair_edge = torch.empty(E, **o), torch.empty(E // 2, **o)
        self._check(self.lib.mlip_graph_export_pairs(self.ctx, _ptr(slot), _ptr(pair_edge)))
        return slot, pair_edge

    def mlip_set_expert_weights(self, alpha):
        """alpha: device tensor [n_structs, n_experts] float32."""
        self._check(self.lib.mlip_set_expert_weights(self.ctx, _ptr(alpha, torch.float32), int(alpha.shape[0])))

    def mlip_set_expert_weight_grad(self, grad_alpha):
        """grad_alpha: device tensor [n_structs, n_experts] float32 that BF and BE add dL/dalpha to, or None."""
        n = 0 if grad_alpha is None else int(grad_alpha.shape[0])
        self._check(self.lib.mlip_set_expert_weight_grad(self.ctx, _ptr(grad_alpha, torch.float32), n))
        self._grad_alpha = grad_alpha  # keep the tensor alive while the library holds its address

    def mlip_optimizer_step(self, params, grad, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
                            grad_scale=1.0):
        """In-place AdamW update of device float32 vectors params, m, v from grad."""
        n = params.numel()
        if not (grad.numel() == n and m.numel() == n and v.numel() == n):
            raise ValueError("params, grad, m and v must have the same number of elements")
        h = mlip_adamw(lr, beta1, beta2, eps, weight_decay, grad_scale)
        self._check(self.lib.mlip_optimizer_step(self.ctx, n, _ptr(params, torch.float32), _ptr(grad, torch.float32),
                                                 _ptr(m, torch.float32), _ptr(v, torch.float32), int(step), C.byref(h)))

    def mlip_forward_energy(self, pos, species, params, h_in=None):
        f = dict(device=self.device, dtype=torch.float32)
        stage = self.cfg.model_kind == MODEL_STAGE
        E = None if stage else torch.empty(self.n_structs, **f)
        h_out = torch.empty(self.n_atoms, self.cfg.channels, **f) if stage else None
        self._check(self.lib.mlip_forward_energy(self.ctx, _ptr(pos, torch.float32), _ptr(species, torch.int32),
                                                 _ptr(params, torch.float32), _ptr(h_in, torch.float32), _ptr(E), _ptr(h_out)))
        return h_out if stage else E

    def mlip_forward_force(self, g_out=None):
        f = dict(device=self.device, dtype=torch.float32)
        stage = self.cfg.model_kind == MODEL_STAGE
        F = torch.empty(self.n_atoms, 3, **f)
        g_in = torch.empty(self.n_atoms, self.cfg.channels, **f) if stage else None
        self._check(self.lib.mlip_forward_force(self.ctx, _ptr(g_out, torch.float32), _ptr(F), _ptr(g_in)))
        return (F, g_in) if stage else F

    def mlip_loss(self, E, F, E_ref, F_ref):
        f = dict(device=self.device, dtype=torch.float32)
        loss, Ebar, v = torch.empty(1, **f), torch.empty(self.n_structs, **f), torch.empty(self.n_atoms, 3, **f)
        self._check(self.lib.mlip_loss(self.ctx, _ptr(E, torch.float32), _ptr(F, torch.float32), _ptr(E_ref, torch.float32),
                                       _ptr(F_ref, torch.float32), _ptr(loss), _ptr(Ebar), _ptr(v)))
        return loss, Ebar, v

    def mlip_backward_force(self, v, grad_params, hdot_in=None):
        stage = self.cfg.model_kind == MODEL_STAGE
        hdot_out = torch.empty(self.n_atoms, self.cfg.channels, device=self.device, dtype=torch.float32) if stage else None
        self._check(self.lib.mlip_backward_force(self.ctx, _ptr(v, torch.float32), _ptr(hdot_in, torch.float32),
                                                 _ptr(grad_params, torch.float32), _ptr(hdot_out)))
        return hdot_out

    def mlip_backward_energy(self, grad_params, Ebar=None, lam_out=None):
        stage = self.cfg.model_kind == MODEL_STAGE
        lam_in = torch.empty(self.n_atoms, self.cfg.channels, device=self.device, dtype=torch.float32) if stage else None
        self._check(self.lib.mlip_backward_energy(self.ctx, _ptr(Ebar, torch.float32), _ptr(lam_out, torch.float32),
                                                  _ptr(grad_params, torch.float32), _ptr(lam_in)))
        return lam_in

    def mlip_train_step(self, pos, species, struct_ptr, cell, cutoff, params, E_ref, F_ref, out=None, timed=False):
        """out: optional dict of preallocated loss [1], E [B], F [N,3], grad [n_params]."""
        f = dict(device=self.device, dtype=torch.float32)
        N, B = pos.shape[0], struct_ptr.shape[0] - 1
        if out is None:
            out = dict(loss=torch.empty(1, **f), E=torch.empty(B, **f), F=torch.empty(N, 3, **f),
                       grad=torch.empty(self.mlip_param_count(), **f))
        ms = (C.c_float * 5)() if timed else None
        s = self.lib.mlip_train_step(self.ctx, N, B, _ptr(pos, torch.float32), _ptr(species, torch.int32),
                                     _ptr(struct_ptr, torch.int32), _ptr(cell, torch.float32), cutoff,
                                     _ptr(params, torch.float32), _ptr(E_ref, torch.float32), _ptr(F_ref, torch.float32),
                                     _ptr(out["loss"]), _ptr(out["E"]), _ptr(out["F"]), _ptr(out["grad"]), ms)
        self._check(s)
        self.n_atoms, self.n_structs, self.n_edges = self.mlip_graph_sizes()
        if timed:
            out["phase_ms"] = list(ms)
        return out
