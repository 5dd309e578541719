"""Pins for the oracle's edge features: closed-form values of the radial basis and the
envelope, scipy's spherical harmonics, and for the coupling tensors the selection rules,
hand-integrated entries and rotation equivariance."""
import math

import numpy as np
import torch
from scipy.special import sph_harm_y

from oracle import mlip_oracle as O


def _rand_unit(n, seed=0):
    rng = np.random.default_rng(seed)
    v = rng.normal(size=(n, 3))
    return v / np.linalg.norm(v, axis=1, keepdims=True)


def test_rbf_closed_form_values():
    K, rc = 16, 5.0
    dx = rc / (K - 1)
    mu = np.arange(K) * dx
    phi = O.rbf(torch.tensor(mu), K, rc).numpy()
    assert np.allclose(np.diag(phi), 1.0)
    # one spacing away: exp(-1/2); two: exp(-2)
    assert np.allclose(np.diag(phi, 1), math.exp(-0.5))
    assert np.allclose(np.diag(phi, 2), math.exp(-2.0))
    assert mu[0] == 0.0 and abs(mu[-1] - rc) < 1e-15


def test_envelope_closed_form_values():
    rc = 6.0
    f = O.envelope(torch.tensor([0.0, rc / 3, rc / 2, rc]), rc).numpy()
    assert np.allclose(f, [1.0, 0.75, 0.5, 0.0], atol=1e-15)


def test_sph_harm_matches_scipy():
    u = _rand_unit(50)
    theta = np.arccos(u[:, 2])
    phi = np.arctan2(u[:, 1], u[:, 0])
    got = O.real_sph_harm(torch.tensor(u)).numpy()
    col = 0
    for l in range(3):
        for m in range(-l, l + 1):
            Yc = sph_harm_y(l, abs(m), theta, phi)  # orthonormal, Condon-Shortley phase
            if m == 0:
                ref = Yc.real
            elif m > 0:
                ref = math.sqrt(2) * (-1) ** m * Yc.real
            else:
                ref = math.sqrt(2) * (-1) ** m * Yc.imag
            assert np.allclose(got[:, col], math.sqrt(4 * math.pi) * ref, atol=1e-13), (l, m)
            col += 1


def test_sph_harm_norm_and_l1_direction():
    u = _rand_unit(20, 1)
    Y = O.real_sph_harm(torch.tensor(u)).numpy()
    for l, sl in enumerate(O.SL[:3]):
        assert np.allclose((Y[:, sl] ** 2).sum(1), 2 * l + 1)
    assert np.allclose(Y[:, 1:4], math.sqrt(3) * u[:, [1, 2, 0]])


def test_paths_and_selection_rules():
    assert len(O.PATHS) == 11
    assert O.PATHS == sorted(O.PATHS)
    T = O.gaunt_tensors()
    for p, (l1, l2, l3) in enumerate(O.PATHS):
        assert T[p].shape == (2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1)
        assert abs(float((T[p] ** 2).sum()) - (2 * l3 + 1)) < 1e-12
    for l in range(3):
        # coupling with the constant harmonic is the identity (orthonormality)
        t = T[O.PATHS.index((0, l, l))][0].numpy()
        assert np.allclose(t, np.eye(2 * l + 1), atol=1e-12)
        t = T[O.PATHS.index((l, 0, l))][:, 0, :].numpy()
        assert np.allclose(t, np.eye(2 * l + 1), atol=1e-12)
        t = T[O.PATHS.index((l, l, 0))][:, :, 0].numpy()
        assert np.allclose(t, np.eye(2 * l + 1) / math.sqrt(2 * l + 1), atol=1e-12)


def test_gaunt_entries_integrated_by_hand():
    # (1/4pi) Int 3 z^2 (sqrt5/2)(3 z^2 - 1) = 2/sqrt5 ; with x^2 instead of z^2: -1/sqrt5 ;
    # (1/4pi) Int (sqrt3 x)(sqrt3 y)(sqrt15 x y) = 3 sqrt15 <x^2 y^2> = 3 sqrt15/15 = sqrt(3/5)
    t = O.gaunt_tensors()[O.PATHS.index((1, 1, 2))].numpy()
    raw = np.array([2 / math.sqrt(5), -1 / math.sqrt(5), math.sqrt(3 / 5)])
    got = np.array([t[1, 1, 2], t[2, 2, 2], t[2, 0, 0]])  # l=1 order (y,z,x); l=2 order (xy,yz,z2,xz,x2-y2)
    assert np.allclose(got / got[0], raw / raw[0], atol=1e-12)
    assert got[0] > 0
    # symmetric and traceless in the two l=1 indices
    assert np.allclose(t, t.transpose(1, 0, 2), atol=1e-12)
    assert np.allclose(np.einsum("aak->k", t), 0.0, atol=1e-12)
    # (2,2,2): (1/4pi) Int [(sqrt5/2)(3z^2-1)]^3 = (5 sqrt5/8)(16/35) = 2 sqrt5/7, and
    # (1/4pi) Int (sqrt15 x y)^2 (sqrt5/2)(3z^2-1) = (15 sqrt5/2)(3/105 - 1/15) = -2 sqrt5/7
    t222 = O.gaunt_tensors()[O.PATHS.index((2, 2, 2))].numpy()
    assert t222[2, 2, 2] > 0
    assert abs(t222[0, 0, 2] / t222[2, 2, 2] + 1.0) < 1e-12


def _wigner(l, R, n=40):
    """D with Y_l(R u) = D Y_l(u), by least squares on sampled directions."""
    u = _rand_unit(n, 5)
    A = O.real_sph_harm(torch.tensor(u)).numpy()[:, O.SL[l]]
    Bm = O.real_sph_harm(torch.tensor(u @ R.T)).numpy()[:, O.SL[l]]
    D = np.linalg.lstsq(A, Bm, rcond=None)[0].T
    assert np.allclose(A @ D.T, Bm, atol=1e-11)
    return D


def test_tensor_product_is_rotation_equivariant():
    from scipy.spatial.transform import Rotation
    R = Rotation.from_rotvec([0.3, -1.1, 0.7]).as_matrix()
    D = [_wigner(l, R) for l in range(3)]
    rng = np.random.default_rng(3)
    T = O.gaunt_tensors()
    for p, (l1, l2, l3) in enumerate(O.PATHS):
        a = rng.normal(size=2 * l1 + 1)
        b = rng.normal(size=2 * l2 + 1)
        t = T[p].numpy()
        out = np.einsum("abk,a,b->k", t, a, b)
        out_rot = np.einsum("abk,a,b->k", t, D[l1] @ a, D[l2] @ b)
        assert np.allclose(out_rot, D[l3] @ out, atol=1e-10), (l1, l2, l3)
