"""CPU float64 oracle for the four-phase training step of a conservative message-passing
interatomic potential.  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the CPU
baseline leg of the benchmark may call it; the product (HIP) path never does, and the two
share no code.

What is computed follows the paper's description of a training iteration (Sec. 2,
"Training MLIPs with Four Phases"): FE predicts the energy E, FF takes F = -dE/dx by
differentiating FE, and the parameter gradient of L_total = L_E + L_F (Sec. 4.1, Pass 1,
Rule 2) needs a backward pass through FF (BF, the double backward) and one through FE
(BE).  The oracle is that definition written out: E is evaluated with plain tensor ops,
F and dL/dtheta are obtained by reverse-mode differentiation of those ops (PyTorch
autograd used as a library routine, in float64), with no hand-derived adjoint anywhere.

The split of the gradient between BF and BE is the one of Eq. 2 (Sec. 4.1): BF keeps only
the second-order term -- the dependence of the differentiated graph (FF) on the weights
it uses directly -- and BE collects every first-order term (from L_E and from L_F).  The
oracle realises it by giving each linear map two copies of its weight, one used by the
forward product and one used by the product in its backward rule; the gradient with
respect to the first copy is BE's share, with respect to the second BF's share.

The paper gives no model equations (it trains third-party UMA / eSEN models); the models
here are the invariant and the equivariant (l <= 2, optionally l <= 3) message-passing potentials defined in the
docstrings below, and the readings taken where the benchmark spec leaves a choice are
listed with each function.

Pins (tests/test_oracle_*.py): neighbour list vs a k-d tree and lattice coordination
numbers; spherical harmonics vs scipy; Gaunt tensors vs selection rules and rotation
equivariance; E invariances and closed forms (the gated update also against the linear one
with halved matrices when its gate scalars vanish); F vs central differences of E; dL/dtheta
vs central differences of L; BF+BE = total; stage outputs vs central differences of the
stage scalar and vs the unsplit model; radius_graph_rows row by row vs radius_graph and a k-d tree;
one equivariant layer vs explicit loops with couplings integrated from the harmonics' polynomials;
energy_streamed vs energy_only; the l_max = 3 extension: degree-3 harmonics vs scipy and the addition theorem,
all 23 couplings vs sphere means of typed polynomials, one layer by explicit loops, F and dL/dtheta by central
differences.  No function here is left unpinned.
"""
from __future__ import annotations

import math
from typing import Callable, Dict, List, Optional, Tuple

import numpy as np
import torch

DT = torch.float64

def paths_of(l_max: int) -> List[Tuple[int, int, int]]:
    """The coupling paths (l1, l2, l3) with every degree <= l_max that satisfy the triangle rule and have even
    l1 + l2 + l3, ordered by (l1, l2, l3): 11 paths for l_max = 2, 23 for l_max = 3."""
    return [(l1, l2, l3)
            for l1 in range(l_max + 1) for l2 in range(l_max + 1) for l3 in range(l_max + 1)
            if abs(l1 - l2) <= l3 <= l1 + l2 and (l1 + l2 + l3) % 2 == 0]


PATHS: List[Tuple[int, int, int]] = paths_of(2)
# components of degree l inside the (l_max + 1)^2-vector of node features / harmonics
SL = [slice(0, 1), slice(1, 4), slice(4, 9), slice(9, 16)]


def lmax_of(cfg: Dict) -> int:
    """Highest degree of the equivariant model's features (2 unless the model description says 3)."""
    return int(cfg.get("l_max", 2) or 2)


# ============================================================================ neighbour list

def lattice_images(lat: np.ndarray, cutoff: float) -> np.ndarray:
    """Image shifts S (integer triples, in shift-code order) that a radius graph of one structure
    has to visit.  A structure whose cell matrix is all zeros is a molecule in vacuum: only
    S = 0.  Otherwise the rows of `lat` are the lattice vectors of a general (triclinic) cell
    and the 27 nearest images suffice as long as the cutoff does not exceed any of the three
    perpendicular heights V / |a_b x a_c| of the cell (for a diagonal cell: its edges)."""
    lat = np.asarray(lat, dtype=np.float64)
    if not lat.any():
        return np.zeros((1, 3))
    vol = abs(np.linalg.det(lat))
    assert vol > 0.0, "singular cell"
    heights = [vol / np.linalg.norm(np.cross(lat[(a + 1) % 3], lat[(a + 2) % 3])) for a in range(3)]
    assert cutoff <= min(heights) + 1e-12, "cutoff longer than a cell height"
    rng = np.array([-1.0, 0.0, 1.0])
    return np.stack(np.meshgrid(rng, rng, rng, indexing="ij"), -1).reshape(27, 3)  # code order


def radius_graph(pos: np.ndarray, struct_ptr: np.ndarray, cell: np.ndarray, cutoff: float,
                 chunk: int = 64) -> Dict[str, np.ndarray]:
    """Radius graph by brute force over all atom pairs of a structure and the images
    lattice_images() lists (27 for a periodic cell, general lattice; 1 for a molecule).

    Edge (i <- j, S) exists iff |x_j + S.cell - x_i| < cutoff and (j, S) != (i, 0), i and j
    in the same structure.  Edges are grouped by receiver i (global atom index) and ordered
    inside a row by (sender j, then shift code (Sx+1)*9 + (Sy+1)*3 + (Sz+1)); that order is
    unique.  Returns row_ptr [N+1], sender [E], shift [E,3], receiver [E], rev [E] with
    rev[e] the index of the opposite edge (j <- i, -S).
    """
    pos = np.asarray(pos, dtype=np.float64)
    N = pos.shape[0]
    recv_l, send_l, shift_l = [], [], []
    for s in range(len(struct_ptr) - 1):
        a, b = int(struct_ptr[s]), int(struct_ptr[s + 1])
        lat = np.asarray(cell[s], dtype=np.float64)
        S = lattice_images(lat, cutoff)
        zero = int(np.nonzero((S == 0).all(1))[0][0])
        off = S @ lat  # [n_images,3]
        x = pos[a:b]
        for i0 in range(0, b - a, chunk):
            xi = x[i0:i0 + chunk]
            d = x[None, :, None, :] + off[None, None, :, :] - xi[:, None, None, :]  # [ci, n, images, 3]
            r2 = d[..., 0] * d[..., 0] + d[..., 1] * d[..., 1] + d[..., 2] * d[..., 2]
            ok = r2 < cutoff * cutoff
            ii = np.arange(xi.shape[0])
            ok[ii, ii + i0, zero] = False  # the atom itself, zero shift
            ri, rj, rs = np.nonzero(ok)  # C order: i, then j, then code -> already canonical
            recv_l.append(ri + i0 + a)
            send_l.append(rj + a)
            shift_l.append(S[rs].astype(np.int32))
    receiver = np.concatenate(recv_l).astype(np.int32) if recv_l else np.zeros(0, np.int32)
    sender = np.concatenate(send_l).astype(np.int32) if send_l else np.zeros(0, np.int32)
    shift = np.concatenate(shift_l).astype(np.int32) if shift_l else np.zeros((0, 3), np.int32)
    row_ptr = np.zeros(N + 1, dtype=np.int32)
    np.cumsum(np.bincount(receiver, minlength=N), out=row_ptr[1:])
    # opposite edge: key (receiver, sender, code) <-> (sender, receiver, 26 - code)
    code = (shift[:, 0] + 1) * 9 + (shift[:, 1] + 1) * 3 + (shift[:, 2] + 1)
    key = (receiver.astype(np.int64) * N + sender) * 27 + code
    key_rev = (sender.astype(np.int64) * N + receiver) * 27 + (26 - code)
    rev = np.searchsorted(key, key_rev).astype(np.int32)
    assert np.array_equal(key[rev], key_rev), "graph is not symmetric"
    return dict(row_ptr=row_ptr, sender=sender, shift=shift, receiver=receiver, rev=rev)


def radius_graph_rows(pos: np.ndarray, struct_ptr: np.ndarray, cell: np.ndarray, cutoff: float,
                      rows: np.ndarray) -> List[Tuple[np.ndarray, np.ndarray]]:
    """The same definition as radius_graph, for chosen receivers only (so that rows of a system
    too large for the full pair loop can still be checked one by one).  Returns, per requested
    receiver, (sender [d], shift [d,3]) in the canonical in-row order."""
    pos = np.asarray(pos, dtype=np.float64)
    out = []
    for i in rows:
        s = int(np.searchsorted(struct_ptr, i, side="right") - 1)
        a, b = int(struct_ptr[s]), int(struct_ptr[s + 1])
        lat = np.asarray(cell[s], dtype=np.float64)
        S = lattice_images(lat, cutoff)
        off = S @ lat
        d = pos[a:b, None, :] + off[None, :, :] - pos[i][None, None, :]   # [n, images, 3]
        r2 = d[..., 0] * d[..., 0] + d[..., 1] * d[..., 1] + d[..., 2] * d[..., 2]
        ok = r2 < cutoff * cutoff
        ok[i - a, int(np.nonzero((S == 0).all(1))[0][0])] = False
        rj, rs = np.nonzero(ok)
        out.append(((rj + a).astype(np.int32), S[rs].astype(np.int32)))
    return out


# ============================================================================ edge features

def rbf(r: torch.Tensor, n_rbf: int, cutoff: float) -> torch.Tensor:
    """Gaussian radial basis: phi_k(r) = exp(-gamma (r - mu_k)^2), centres mu_k = k r_c/(K-1)
    on [0, r_c], width equal to the centre spacing: gamma = 1/2 ((K-1)/r_c)^2."""
    mu = torch.arange(n_rbf, dtype=DT) * (cutoff / (n_rbf - 1))
    gamma = 0.5 * ((n_rbf - 1) / cutoff) ** 2
    return torch.exp(-gamma * (r[:, None] - mu[None, :]) ** 2)


def envelope(r: torch.Tensor, cutoff: float) -> torch.Tensor:
    """Cosine cutoff f_c(r) = 1/2 (1 + cos(pi r / r_c)) (edges always have r < r_c)."""
    return 0.5 * (1.0 + torch.cos(math.pi * r / cutoff))


def real_sph_harm(u: torch.Tensor, l_max: int = 2) -> torch.Tensor:
    """Real spherical harmonics l = 0..l_max (2 or 3) of unit vectors u [.., 3] -> [.., (l_max + 1)^2].

    Component normalisation (mean of Y^2 over the sphere is 1, so sum_m Y_lm^2 = 2l+1);
    order inside l is m = -l..l, which for l = 1 is (y, z, x).
    """
    x, y, z = u[..., 0], u[..., 1], u[..., 2]
    s3, s15, s5 = math.sqrt(3.0), math.sqrt(15.0), math.sqrt(5.0)
    comps = [
        torch.ones_like(x),
        s3 * y, s3 * z, s3 * x,
        s15 * x * y, s15 * y * z, 0.5 * s5 * (3.0 * z * z - 1.0), s15 * x * z, 0.5 * s15 * (x * x - y * y),
    ]
    if l_max >= 3:
        a, b, c, d = math.sqrt(35.0 / 8.0), math.sqrt(105.0), math.sqrt(21.0 / 8.0), 0.5 * math.sqrt(7.0)
        comps += [
            a * y * (3.0 * x * x - y * y), b * x * y * z, c * y * (5.0 * z * z - 1.0), d * z * (5.0 * z * z - 3.0),
            c * x * (5.0 * z * z - 1.0), 0.5 * b * z * (x * x - y * y), a * x * (x * x - 3.0 * y * y),
        ]
    return torch.stack(comps, dim=-1)


_GAUNT_CACHE: Dict[int, List[torch.Tensor]] = {}


def gaunt_tensors(l_max: int = 2) -> List[torch.Tensor]:
    """T^p[m1, m2, m3] for the paths p = (l1, l2, l3) of paths_of(l_max): the real Gaunt integral
    (1/4pi) Int Y_l1m1 Y_l2m2 Y_l3m3 dOmega, evaluated by a quadrature that is exact for the
    integrand of degree <= 9 (Gauss-Legendre in cos(theta) x uniform in the azimuth), then scaled
    by a positive factor per path so that the sum of squares is 2 l3 + 1."""
    if l_max in _GAUNT_CACHE:
        return _GAUNT_CACHE[l_max]
    ct, wt = np.polynomial.legendre.leggauss(8)
    nphi = 16
    ph = (np.arange(nphi) + 0.5) * (2.0 * math.pi / nphi)
    CT, PH = np.meshgrid(ct, ph, indexing="ij")
    W = np.repeat(wt[:, None], nphi, 1) * (2.0 * math.pi / nphi) / (4.0 * math.pi)
    st = np.sqrt(1.0 - CT * CT)
    u = torch.tensor(np.stack([st * np.cos(PH), st * np.sin(PH), CT], -1).reshape(-1, 3), dtype=DT)
    Y = real_sph_harm(u, l_max)
    w = torch.tensor(W.reshape(-1), dtype=DT)
    out = []
    for (l1, l2, l3) in paths_of(l_max):
        G = torch.einsum("q,qa,qb,qc->abc", w, Y[:, SL[l1]], Y[:, SL[l2]], Y[:, SL[l3]])
        G = torch.where(G.abs() < 1e-13, torch.zeros_like(G), G)
        out.append(G * math.sqrt((2 * l3 + 1) / float((G * G).sum())))
    _GAUNT_CACHE[l_max] = out
    return out


# ============================================================================ parameters

def unpack_params(flat: torch.Tensor, cfg: Dict) -> Dict[str, torch.Tensor]:
    """Views into the flat float vector.  Layout (row-major [out, in], concatenated):
    whole models start with emb[S,C] and end with U[C,C], w_o[C]; each layer holds
    invariant  W1[H,K], W2[C,H]  (depth 3: W1[H,K], W2[H,H], W3[C,H]),  V1[C,C], V2[C,C]
    (with n_experts > 0: expert banks V1[n_experts,C,C], V2[n_experts,C,C]);
    equivariant W1[H,K], W2[n_paths C,H] (row = path*C + channel; 11 paths, 23 with l_max = 3), Wl0 .. Wl{l_max} [C,C]
    (with n_experts > 0: banks [n_experts,C,C]);
    a stage holds the layer blocks only."""
    C, H, K, S = cfg["channels"], cfg["edge_hidden"], cfg["n_rbf"], cfg["n_species"]
    kind = cfg["kind"]
    names: List[Tuple[str, Tuple[int, ...]]] = []
    if kind != "stage":
        names.append(("emb", (S, C)))
    for l in range(cfg["n_layers"]):
        names.append((f"l{l}.W1", (H, K)))
        if kind == "equivariant":
            names.append((f"l{l}.W2", (len(paths_of(lmax_of(cfg))) * C, H)))
            wshape = (cfg["n_experts"], C, C) if cfg.get("n_experts", 0) > 0 else (C, C)
            names += [(f"l{l}.Wl{k}", wshape) for k in range(lmax_of(cfg) + 1)]
        else:
            if cfg["edge_depth"] == 3:
                names += [(f"l{l}.W2", (H, H)), (f"l{l}.W3", (C, H))]
            else:
                names.append((f"l{l}.W2", (C, H)))
            vshape = (cfg["n_experts"], C, C) if cfg.get("n_experts", 0) > 0 else (C, C)
            names += [(f"l{l}.V1", vshape), (f"l{l}.V2", vshape)]
    if kind != "stage":
        names += [("U", (C, C)), ("w_o", (C,))]
    out, off = {}, 0
    for n, shp in names:
        cnt = int(np.prod(shp))
        out[n] = flat[off:off + cnt].reshape(shp)
        off += cnt
    assert off == flat.numel(), (off, flat.numel())
    return out


class _SplitLinear(torch.autograd.Function):
    """y = x W_fe^T whose backward rule uses a second copy W_ff for the data gradient.
    With W_fe == W_ff numerically this is an ordinary linear map; the two copies only make
    it possible to ask where a weight was used (Eq. 1-2, Sec. 4.1)."""

    @staticmethod
    def forward(ctx, x, w_fe, w_ff):
        ctx.save_for_backward(x, w_ff)
        return x @ w_fe.t()

    @staticmethod
    def backward(ctx, gy):
        x, w_ff = ctx.saved_tensors
        gx = gy @ w_ff
        gw_fe = gy.reshape(-1, gy.shape[-1]).t() @ x.reshape(-1, x.shape[-1])
        return gx, gw_fe, None


class _Lin:
    """Applies named weights; in split mode every linear map goes through _SplitLinear."""

    def __init__(self, P: Dict[str, torch.Tensor], P_ff: Optional[Dict[str, torch.Tensor]] = None,
                 alpha: Optional[torch.Tensor] = None):
        self.P, self.P_ff, self.alpha = P, P_ff, alpha
        self.sid: Optional[torch.Tensor] = None  # structure of each atom (set by the model functions)

    def mole(self, x: torch.Tensor, name: str) -> torch.Tensor:
        """Mixture of linear experts (Sec. 5.1, "Models"): for every structure s the expert matrices of
        the bank are averaged with that structure's coefficients, W_s = sum_k alpha[s,k] W_k, and the
        temporary W_s is applied to the structure's atoms like any dense matrix."""
        B = self.alpha.shape[0]
        W = torch.einsum("bk,kij->bij", self.alpha, self.P[name])
        Wf = None if self.P_ff is None else torch.einsum("bk,kij->bij", self.alpha, self.P_ff[name])
        out = []
        for b in range(B):
            xb = x[self.sid == b]
            out.append(xb @ W[b].t() if Wf is None else _SplitLinear.apply(xb, W[b], Wf[b]))
        return torch.cat(out, dim=0)  # atoms are stored structure by structure

    def node(self, x: torch.Tensor, name: str) -> torch.Tensor:
        """The update MLP's matrices: expert banks when coefficients were given, else dense."""
        return self.mole(x, name) if self.alpha is not None else self(x, name)

    def __call__(self, x: torch.Tensor, name: str) -> torch.Tensor:
        W = self.P[name]
        W2 = W if W.dim() == 2 else W[None, :]
        if self.P_ff is None:
            return x @ W2.t()
        Wf = self.P_ff[name]
        Wf2 = Wf if Wf.dim() == 2 else Wf[None, :]
        return _SplitLinear.apply(x, W2, Wf2)


def silu(x: torch.Tensor) -> torch.Tensor:
    return x * torch.sigmoid(x)


# ============================================================================ models

def edge_vectors(x: torch.Tensor, graph: Dict, cell: torch.Tensor, struct_of_atom: torch.Tensor):
    """r_vec_e = x_j + S_e . cell - x_i, r_e = |r_vec_e| for every edge e = (i <- j, S)."""
    snd = torch.as_tensor(graph["sender"], dtype=torch.long)
    rcv = torch.as_tensor(graph["receiver"], dtype=torch.long)
    S = torch.as_tensor(graph["shift"], dtype=DT)
    off = torch.einsum("ea,eab->eb", S, cell[struct_of_atom[rcv]])
    rv = x[snd] + off - x[rcv]
    r = torch.sqrt((rv * rv).sum(-1))
    return snd, rcv, rv, r


def invariant_messages(h, l, lin: _Lin, cfg, snd, rcv, r):
    """a_i = sum_{e: i<-j} f_c(r_e) * w_e (.) h_j over the given edges,
    w_e = W2 silu(W1 phi(r_e))  (depth 3: W3 silu(W2 silu(W1 phi))).  No biases."""
    phi = rbf(r, cfg["n_rbf"], cfg["cutoff"])
    t = silu(lin(phi, f"l{l}.W1"))
    if cfg["edge_depth"] == 3:
        t = silu(lin(t, f"l{l}.W2"))
        w = lin(t, f"l{l}.W3")
    else:
        w = lin(t, f"l{l}.W2")
    m = envelope(r, cfg["cutoff"])[:, None] * w * h[snd]
    return torch.zeros_like(h).index_add(0, rcv, m)


def invariant_update(h, a, l, lin: _Lin, cfg):
    """h_i <- h_i + V2 silu(V1 a_i)."""
    return h + lin.node(silu(lin.node(a, f"l{l}.V1")), f"l{l}.V2")


def invariant_layer(h, l, lin: _Lin, cfg, snd, rcv, r):
    """One interaction layer: aggregate the messages of all edges, then update the node features."""
    return invariant_update(h, invariant_messages(h, l, lin, cfg, snd, rcv, r), l, lin, cfg)


def equivariant_messages(h, l, lin: _Lin, cfg, snd, rcv, rv, r):
    """h [N, C, (l_max + 1)^2].  a_i = sum_e m_e over the given edges with
    m_e[c; l3 m3] = f_c(r_e) sum_p R_e[p, c] sum_{m1 m2} T^p[m1 m2 m3] h_j[c; l1 m1] Y_{l2 m2}(r_e / r_e),
    R_e = W2 silu(W1 phi(r_e)) reshaped [n_paths, C]."""
    C = cfg["channels"]
    lm = lmax_of(cfg)
    paths = paths_of(lm)
    phi = rbf(r, cfg["n_rbf"], cfg["cutoff"])
    R = lin(silu(lin(phi, f"l{l}.W1")), f"l{l}.W2").reshape(-1, len(paths), C)
    Y = real_sph_harm(rv / r[:, None], lm)
    hj = h[snd]
    T = gaunt_tensors(lm)
    parts = [torch.zeros(hj.shape[0], C, 2 * k + 1, dtype=DT) for k in range(lm + 1)]
    for p, (l1, l2, l3) in enumerate(paths):
        tp = torch.einsum("abk,eca,eb->eck", T[p], hj[:, :, SL[l1]], Y[:, SL[l2]])
        parts[l3] = parts[l3] + R[:, p, :, None] * tp
    m = envelope(r, cfg["cutoff"])[:, None, None] * torch.cat(parts, dim=2)
    return torch.zeros_like(h).index_add(0, rcv, m)


def equivariant_update(h, a, l, lin: _Lin, cfg):
    """h_i[:, l] <- h_i[:, l] + W^(l) a_i[:, l] (one C x C matrix per l, shared over m); with cfg["gate"] the
    gated form h_0 += silu(u_0), h_lm += sigmoid(u_0) u_lm (l >= 1) of u = W^(l) a."""
    upd = [lin.node(a[:, :, SL[k]].transpose(1, 2), f"l{l}.Wl{k}").transpose(1, 2) for k in range(lmax_of(cfg) + 1)]
    if cfg.get("gate", 0):
        u0 = upd[0]
        upd = [silu(u0)] + [torch.sigmoid(u0) * uk for uk in upd[1:]]
    return h + torch.cat(upd, dim=2)


def equivariant_layer(h, l, lin: _Lin, cfg, snd, rcv, rv, r):
    """One interaction layer: aggregate the messages of all edges, then update the node features."""
    return equivariant_update(h, equivariant_messages(h, l, lin, cfg, snd, rcv, rv, r), l, lin, cfg)


def energy(x, species, graph, cell, struct_ptr, lin: _Lin, cfg) -> torch.Tensor:
    """Per-structure energies E_s = sum_{i in s} w_o . silu(U h_i^L) of the whole model
    (h^0 = emb[species]; the equivariant model embeds into l = 0 and reads out from l = 0)."""
    N = x.shape[0]
    B = len(struct_ptr) - 1
    sid = torch.repeat_interleave(torch.arange(B), torch.as_tensor(np.diff(struct_ptr), dtype=torch.long))
    lin.sid = sid
    snd, rcv, rv, r = edge_vectors(x, graph, cell, sid)
    emb = lin.P["emb"][torch.as_tensor(species, dtype=torch.long)]
    if cfg["kind"] == "equivariant":
        h = torch.cat([emb[:, :, None], torch.zeros(N, cfg["channels"], (lmax_of(cfg) + 1) ** 2 - 1, dtype=DT)], dim=2)
        for l in range(cfg["n_layers"]):
            h = equivariant_layer(h, l, lin, cfg, snd, rcv, rv, r)
        h = h[:, :, 0]
    else:
        h = emb
        for l in range(cfg["n_layers"]):
            h = invariant_layer(h, l, lin, cfg, snd, rcv, r)
    eps = lin(silu(lin(h, "U")), "w_o")[:, 0]
    return torch.zeros(B, dtype=DT).index_add(0, sid, eps)


def loss_fn(E, F, E_ref, F_ref, force_weight):
    """L = mean_s (E_s - E_ref,s)^2 + force_weight * mean_{i,alpha} (F - F_ref)^2."""
    return ((E - E_ref) ** 2).mean() + force_weight * ((F - F_ref) ** 2).mean()


def _t(a, grad=False):
    return torch.tensor(np.asarray(a), dtype=DT, requires_grad=grad)


def train_step(cfg: Dict, pos, species, struct_ptr, cell, params, E_ref, F_ref,
               graph: Optional[Dict] = None, split: bool = False, alpha=None, grad_pos: bool = False) -> Dict[str, np.ndarray]:
    """One training step of the whole model: returns loss, E [B], F [N,3], grad [n_params]
    (= dL/dtheta), and with split=True also grad_bf / grad_be, the BF and BE shares.
    alpha [B, n_experts]: mixing coefficients of the expert banks (cfg["n_experts"] > 0); then
    grad_alpha = dL/dalpha is returned too.  grad_pos=True adds grad_pos [N,3] = dL/dx, the derivative of
    the loss with respect to the positions (it differentiates the forces once more in x, so it brings in
    the second derivatives of every edge feature)."""
    if graph is None:
        graph = radius_graph(pos, struct_ptr, cell, cfg["cutoff"])
    x = _t(pos, True)
    cellt = _t(cell)
    theta = _t(params, True)
    P = unpack_params(theta, cfg)
    al = None if alpha is None else _t(alpha, True)
    if split:
        theta_ff = _t(params, True)
        lin = _Lin(P, unpack_params(theta_ff, cfg), alpha=al)
    else:
        lin = _Lin(P, alpha=al)
    E = energy(x, species, graph, cellt, struct_ptr, lin, cfg)
    (dEdx,) = torch.autograd.grad(E.sum(), x, create_graph=True)
    F = -dEdx
    L = loss_fn(E, F, _t(E_ref), _t(F_ref), cfg["force_weight"])
    out = dict(E=E.detach().numpy(), F=F.detach().numpy(), loss=float(L.detach()))
    wrt = [theta] + ([theta_ff] if split else []) + ([al] if al is not None else []) + ([x] if grad_pos else [])
    gs = list(torch.autograd.grad(L, wrt, allow_unused=True))
    if grad_pos:
        gx = gs.pop()
        out["grad_pos"] = np.zeros_like(out["F"]) if gx is None else gx.numpy()
    if al is not None:  # dL/dalpha [B, n_experts]: what a router producing the coefficients would receive
        out["grad_alpha"] = gs.pop().numpy()
    if split:
        g_be, g_bf = gs
        g_bf = torch.zeros_like(theta) if g_bf is None else g_bf
        out["grad_be"], out["grad_bf"] = g_be.numpy(), g_bf.numpy()
        out["grad"] = out["grad_be"] + out["grad_bf"]
    else:
        out["grad"] = gs[0].numpy()
    return out


def energy_only(cfg, pos, species, struct_ptr, cell, params, graph=None, alpha=None) -> np.ndarray:
    if graph is None:
        graph = radius_graph(pos, struct_ptr, cell, cfg["cutoff"])
    with torch.no_grad():
        lin = _Lin(unpack_params(_t(params), cfg), alpha=None if alpha is None else _t(alpha))
        return energy(_t(pos), species, graph, _t(cell), struct_ptr, lin, cfg).numpy()


def energy_streamed(cfg, pos, species, struct_ptr, cell, params, graph, edge_chunk: int = 32768) -> np.ndarray:
    """The same per-structure energies as energy_only, for systems whose per-edge tensors do not fit in
    memory at once: every layer's aggregate a_i = sum_e m_e is accumulated over consecutive blocks of
    edges (the sum over edges is the only place where edges meet), then the layer's node update is applied
    once.  Values only, no derivatives; callers take directional derivatives by central differences."""
    with torch.no_grad():
        lin = _Lin(unpack_params(_t(params), cfg))
        x, cellt = _t(pos), _t(cell)
        N, B = x.shape[0], len(struct_ptr) - 1
        sid = torch.repeat_interleave(torch.arange(B), torch.as_tensor(np.diff(struct_ptr), dtype=torch.long))
        lin.sid = sid
        n_edges = len(graph["sender"])
        emb = lin.P["emb"][torch.as_tensor(species, dtype=torch.long)]
        eqv = cfg["kind"] == "equivariant"
        h = torch.cat([emb[:, :, None], torch.zeros(N, cfg["channels"], (lmax_of(cfg) + 1) ** 2 - 1, dtype=DT)], dim=2) if eqv else emb
        for l in range(cfg["n_layers"]):
            a = torch.zeros_like(h)
            for e0 in range(0, n_edges, edge_chunk):
                part = {k: graph[k][e0:e0 + edge_chunk] for k in ("sender", "receiver", "shift")}
                snd, rcv, rv, r = edge_vectors(x, part, cellt, sid)
                a += (equivariant_messages(h, l, lin, cfg, snd, rcv, rv, r) if eqv
                      else invariant_messages(h, l, lin, cfg, snd, rcv, r))
            h = equivariant_update(h, a, l, lin, cfg) if eqv else invariant_update(h, a, l, lin, cfg)
        if eqv:
            h = h[:, :, 0]
        eps = lin(silu(lin(h, "U")), "w_o")[:, 0]
        return torch.zeros(B, dtype=DT).index_add(0, sid, eps).numpy()


# ============================================================================ pipeline stage

def stage_forward(h_in, x, graph, cell, struct_ptr, lin: _Lin, cfg) -> torch.Tensor:
    """h_out = H(h_in, x; theta): the stage's consecutive invariant layers, nothing else."""
    B = len(struct_ptr) - 1
    sid = torch.repeat_interleave(torch.arange(B), torch.as_tensor(np.diff(struct_ptr), dtype=torch.long))
    snd, rcv, rv, r = edge_vectors(x, graph, cell, sid)
    h = h_in
    for l in range(cfg["n_layers"]):
        h = invariant_layer(h, l, lin, cfg, snd, rcv, r)
    return h


def stage_step(cfg: Dict, pos, struct_ptr, cell, params, h_in, g_out, hdot_in, v, lam_out,
               graph: Optional[Dict] = None, split: bool = True, grad_pos: bool = False) -> Dict[str, np.ndarray]:
    """The four phases for one pipeline stage, with the tensors that cross stage boundaries
    (Table 2: activations h, dE/dh, dL_F/d(dE/dh), dL/dh) supplied by the caller.

    FE: h_out = H(h_in, x).   FF: g_in = (dH/dh_in)^T g_out, p = (dH/dx)^T g_out.
    With Phi = <lam_out, h_out> + <hdot_in, g_in> + <v, p> (lam_out, hdot_in, v constants):
    BF returns hdot_out = dPhi/dg_out and the second-order share of dPhi/dtheta,
    BE returns lam_in = dPhi/dh_in and the first-order share of dPhi/dtheta.
    grad_pos=True adds grad_pos = dPhi/dx, this stage's share of the loss's position derivative.
    """
    if graph is None:
        graph = radius_graph(pos, struct_ptr, cell, cfg["cutoff"])
    x = _t(pos, True)
    hin = _t(h_in, True)
    gout = _t(g_out, True)
    theta = _t(params, True)
    theta_ff = _t(params, True) if split else None
    lin = _Lin(unpack_params(theta, cfg), unpack_params(theta_ff, cfg) if split else None)
    h_out = stage_forward(hin, x, graph, _t(cell), struct_ptr, lin, cfg)
    g_in, p = torch.autograd.grad((h_out * gout).sum(), [hin, x], create_graph=True)
    Phi = (_t(lam_out) * h_out).sum() + (_t(hdot_in) * g_in).sum() + (_t(v) * p).sum()
    wrt = [theta, gout, hin] + ([theta_ff] if split else []) + ([x] if grad_pos else [])
    gs = list(torch.autograd.grad(Phi, wrt, allow_unused=True))
    gx = gs.pop() if grad_pos else None
    out = dict(h_out=h_out.detach().numpy(), g_in=g_in.detach().numpy(), p=p.detach().numpy(),
               Phi=float(Phi.detach()), hdot_out=gs[1].numpy(), lam_in=gs[2].numpy())
    if grad_pos:
        out["grad_pos"] = gx.numpy()
    if split:
        out["grad_be"] = gs[0].numpy()
        out["grad_bf"] = gs[3].numpy()
        out["grad"] = out["grad_be"] + out["grad_bf"]
    else:
        out["grad"] = gs[0].numpy()
    return out


def stage_phi(cfg, pos, struct_ptr, cell, params, h_in, g_out, hdot_in, v, lam_out, graph) -> float:
    """The stage scalar Phi alone (FE + FF only); used for finite-difference pins."""
    x = _t(pos, True)
    hin = _t(h_in, True)
    lin = _Lin(unpack_params(_t(params), cfg))
    h_out = stage_forward(hin, x, graph, _t(cell), struct_ptr, lin, cfg)
    g_in, p = torch.autograd.grad((h_out * _t(g_out)).sum(), [hin, x])
    Phi = (_t(lam_out) * h_out).sum() + (_t(hdot_in) * g_in).sum() + (_t(v) * p).sum()
    return float(Phi.detach())


def cfg_from_workload(w) -> Dict:
    """Plain-dict model description from any object with the workload's attribute names."""
    kind = {0: "invariant", 1: "equivariant", 2: "stage"}[int(w.kind)]
    return dict(kind=kind, channels=w.channels, edge_hidden=w.edge_hidden, n_rbf=w.n_rbf,
                n_species=w.n_species, n_layers=w.n_layers, edge_depth=w.edge_depth,
                cutoff=float(w.cutoff), force_weight=float(w.force_weight),
                n_experts=int(getattr(w, "n_experts", 0)), gate=int(getattr(w, "gate", 0)),
                l_max=int(getattr(w, "l_max", 0)))
