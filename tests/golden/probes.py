"""Seeded probes of large result vectors, shared by the script that writes the stored oracle
summaries (make_full_size_goldens.py) and the GPU tests that read them.  A result too large to
store whole (millions of gradient entries) is summarised per tensor by

  * its Euclidean norm,
  * N_SAMPLES entries at seeded positions (an element-by-element check on a sample), and
  * N_PROJ inner products with seeded vectors of +-1 entries: for a difference d between two
    results, the mean of (r . d)^2 over such vectors r is |d|^2, so the projections of both
    results bound the normwise error of the WHOLE tensor, not only of the sample.

No model arithmetic here: numbers are drawn with the input generator's counter-based stream.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np

from paper_2605_18404_amd import synth

N_PROJ, N_SAMPLES = 8, 64
STREAM_PROBE = 21


def signs(seed: int, tensor_index: int, n: int) -> np.ndarray:
    """[N_PROJ, n] entries +-1 for tensor number tensor_index."""
    u = synth.uniform(seed, STREAM_PROBE, tensor_index * (1 << 36), N_PROJ * n).reshape(N_PROJ, n)
    return np.where(u < 0.5, -1.0, 1.0)


def sample_positions(seed: int, tensor_index: int, n: int) -> np.ndarray:
    u = synth.uniform(seed, STREAM_PROBE + 1, tensor_index * (1 << 20), N_SAMPLES)
    return np.minimum((u * n).astype(np.int64), n - 1)


def summarise(seed: int, vec: np.ndarray, slices: Dict[str, Tuple[int, Tuple[int, ...]]]) -> Dict[str, Dict]:
    """Per named tensor of the flat vector: norm, sampled entries, sign projections (float64)."""
    vec = np.asarray(vec, dtype=np.float64).ravel()
    out = {}
    for k, (name, (off, shape)) in enumerate(slices.items()):
        n = int(np.prod(shape))
        t = vec[off:off + n]
        out[name] = dict(norm=float(np.linalg.norm(t)), samples=t[sample_positions(seed, k, n)].tolist(),
                         proj=(signs(seed, k, n) @ t).tolist())
    return out


def compare(got: Dict[str, Dict], want: Dict[str, Dict]) -> Dict[str, float]:
    """Error measures of `got` against the stored `want`: per tensor the normwise error of the sample
    and the error estimated from the projections (root mean square of the projection differences over
    the stored norm), and the same estimate for the whole vector ("flat")."""
    res, num, den = {}, 0.0, 0.0
    for name, w in want.items():
        g = got[name]
        ws, gs = np.array(w["samples"]), np.array(g["samples"])
        d2 = float(np.mean((np.array(g["proj"]) - np.array(w["proj"])) ** 2))
        res[name + ":samples"] = float(np.linalg.norm(gs - ws) / max(np.linalg.norm(ws), 1e-300))
        res[name + ":proj"] = float(np.sqrt(d2) / max(w["norm"], 1e-300))
        num += d2
        den += w["norm"] ** 2
    res["flat"] = float(np.sqrt(num / max(den, 1e-300)))
    return res
