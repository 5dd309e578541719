"""Closed-form pipeline-bubble model of WaveK (paper, Sec. 4.2 "Bubble Analysis" and "Offline
Tuning"), evaluated on per-phase times such as the ones bench.py measures for a pipeline stage.

All times in the same unit.  t = (t_FE, t_FF, t_BF, t_BE) per micro-batch and stage."""
from __future__ import annotations

from typing import Dict, List


def naive_bubble(t_fe: float, t_ff: float, t_bf: float, t_be: float) -> float:
    """Uncovered bubble per micro-batch when a first-order schedule is applied naively
    (Sec. 3, Observation 2): (t_FF + t_BF) - (t_BE + t_FE)."""
    return (t_ff + t_bf) - (t_be + t_fe)


def wavek_bubbles(t_fe: float, t_ff: float, t_bf: float, t_be: float, P: int, n_mb: int, k: int) -> Dict[str, float]:
    """Intra-unit, inter-unit and stage-doubled steady-state bubble sizes for N_mb/k WaveK units."""
    units = n_mb / k
    intra = (t_be - t_ff) * P * units
    inter = (t_bf - t_fe) * P * (units - 1.0)
    doubled = (t_bf + t_be - t_ff - t_fe) * P * n_mb / (2.0 * k) - 0.5 * P * (t_bf - t_fe)
    return {"intra_unit": intra, "inter_unit": inter, "stage_doubled": doubled}


def k_candidates(P: int, n_mb: int, m_mem: float, m_static: float, m_activation: float) -> List[int]:
    """Search space of the offline tuning: k_min = P, k_max = floor((M_mem - M_static) / M_activation),
    preferring values that divide N_mb (all values if none divides)."""
    k_max = int((m_mem - m_static) // m_activation)
    ks = [k for k in range(P, min(k_max, n_mb) + 1)]
    div = [k for k in ks if n_mb % k == 0]
    return div if div else ks
