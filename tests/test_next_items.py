"""The two 'next' items built beyond the hot path: GARS Algorithm 1 (host routine in the
library vs its plain-Python oracle, plus pins of the oracle) and the WaveK bubble model."""
import itertools
import os

import numpy as np
import pytest

from oracle import gars_oracle as G
from paper_2605_18404_amd import synth, wavek_model as W

LIB = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2605_18404_amd", "libmlip.so")


# ------------------------------------------------------------------ oracle pins
def test_gars_oracle_worked_example():
    # sizes 9 7 6 5 4 2 into 2 micro-batches: 9->A, 7->B, 6->B(7<9), 5->A(9<13), 4->B(13<14), 2->A(14<17)
    mbs, tags = G.gars_pack([9, 7, 6, 5, 4, 2], 2, 2, seed=1)
    assert sorted(mbs[0]) == [0, 3, 5] and sorted(mbs[1]) == [1, 2, 4]
    # loads 16 and 17; d_gp = 2: budgets 8 and 8.5 -> 9 > 8 dist, 7 <= 8.5 comm_free
    assert tags == ["dist", "comm_free"]


def test_gars_oracle_properties():
    sizes = synth.draw_graph_sizes(5).tolist()
    n_mb = 32
    mbs, tags = G.gars_pack(sizes, n_mb, 4, seed=3)
    flat = sorted(g for mb in mbs for g in mb)
    assert flat == list(range(len(sizes)))                      # every graph exactly once
    loads = [sum(sizes[g] for g in mb) for mb in mbs]
    assert max(loads) - min(loads) <= max(sizes)                # longest-first placement
    for mb, tag in zip(mbs, tags):                              # tag rule, evaluated directly
        want = "comm_free" if max(sizes[g] for g in mb) * 4 <= sum(sizes[g] for g in mb) else "dist"
        assert tag == want
    # the shuffle only permutes: same sets as the unshuffled packing, and it does permute something
    plain, _ = G.gars_pack(sizes, n_mb, 4, seed=3)
    other, _ = G.gars_pack(sizes, n_mb, 4, seed=4)
    assert [sorted(a) for a in plain] == [sorted(b) for b in other]
    assert plain != other


def test_gars_oracle_within_textbook_bound_of_optimum():
    rng = np.random.default_rng(0)
    for _ in range(20):
        sizes = rng.integers(1, 30, size=7).tolist()
        m = 3
        mbs, _ = G.gars_pack(sizes, m, 1, seed=0)
        got = max(sum(sizes[g] for g in mb) for mb in mbs)
        best = min(max(sum(s for s, a in zip(sizes, assign) if a == j) for j in range(m))
                   for assign in itertools.product(range(m), repeat=len(sizes)))
        assert got <= (4.0 / 3.0 - 1.0 / (3 * m)) * best + 1e-9


# ------------------------------------------------------------------ library routine vs oracle
@pytest.mark.skipif(not os.path.exists(LIB), reason="libmlip.so not built")
@pytest.mark.parametrize("seed,n_mb,d_gp", [(1, 32, 2), (2, 8, 4), (3, 1, 1), (4, 200, 2)])
def test_gars_library_matches_oracle(seed, n_mb, d_gp):
    from paper_2605_18404_amd.binding import mlip_gars_pack
    sizes = synth.draw_graph_sizes(seed)
    mb_ptr, order, typ = mlip_gars_pack(sizes, n_mb, d_gp, seed)
    mbs, tags = G.gars_pack(sizes.tolist(), n_mb, d_gp, seed)
    assert mb_ptr[0] == 0 and mb_ptr[-1] == len(sizes)
    for j in range(n_mb):
        assert order[mb_ptr[j]:mb_ptr[j + 1]].tolist() == mbs[j]          # bit-exact, order included
        assert ("comm_free", "dist")[typ[j]] == tags[j]


@pytest.mark.skipif(not os.path.exists(LIB), reason="libmlip.so not built")
def test_gars_library_edge_cases():
    from paper_2605_18404_amd.binding import MlipError, mlip_gars_pack
    mb_ptr, order, typ = mlip_gars_pack(np.zeros(0, np.int32), 3, 2, 0)       # empty batch
    assert mb_ptr.tolist() == [0, 0, 0, 0] and len(order) == 0 and typ.tolist() == [0, 0, 0]
    with pytest.raises(MlipError):
        mlip_gars_pack(np.array([3, -1], np.int32), 2, 2, 0)
    with pytest.raises(MlipError):
        mlip_gars_pack(np.array([3, 1], np.int32), 0, 2, 0)


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_graph_size_recipe_matches_table_3():
    """The log-normal recipe against the statistics the paper prints for its mixed dataset (Table 3):
    median and mean are matched by construction, the tail of a three-dataset mixture only roughly."""
    t3 = {k: float(v) for k, v in golden_rows("table3_graph_sizes.txt")}
    s = np.concatenate([synth.draw_graph_sizes(k, total_atoms=200000) for k in range(3)])
    assert abs(np.median(s) - t3["p50"]) < 4 and abs(s.mean() - t3["mean"]) < 6
    assert s.max() <= t3["max"] and s.min() >= 1
    assert abs(np.percentile(s, 90) - t3["p90"]) < 0.2 * t3["p90"]
    assert abs(np.percentile(s, 99) - t3["p99"]) < 0.25 * t3["p99"]


def test_bubble_model_on_every_row_of_table_5():
    """The printed phase profile (Table 5): the ratios in parentheses follow from the milliseconds, the
    partial order t_FE < t_FF < t_BE < t_BF holds, the naive schedule's bubble (Sec. 3) is positive, and the
    three closed forms of Sec. 4.2 are mutually consistent (stage-doubled = half of intra + inter) and shrink
    with the unit size k."""
    rows = golden_rows("table5_phase_times.txt")
    assert [r[0] for r in rows] == ["eSEN-220M", "eSEN-100M", "UMA-2.3B", "UMA-1.2B"]
    for r in rows:
        fe, ff, be, bf, rff, rbe, rbf = map(float, r[1:])
        assert abs(ff / fe - rff) < 0.006 and abs(be / fe - rbe) < 0.006 and abs(bf / fe - rbf) < 0.006
        assert fe < ff < be < bf
        assert W.naive_bubble(fe, ff, bf, be) > 0
        prev = None
        for k in (8, 16, 32):
            b = W.wavek_bubbles(fe, ff, bf, be, P=8, n_mb=32, k=k)
            assert abs(b["stage_doubled"] - 0.5 * (b["intra_unit"] + b["inter_unit"])) < 1e-9
            assert all(v >= -1e-12 for v in b.values())
            if prev is not None:
                assert all(b[key] < prev[key] for key in b)
            prev = b
        assert W.wavek_bubbles(fe, ff, bf, be, P=8, n_mb=32, k=32)["inter_unit"] == 0.0  # a single unit has no successor


# ------------------------------------------------------------------ WaveK bubble model
def test_bubble_model_hand_values_and_identity():
    # eSEN-220M row of the phase profile (Appendix "Four Phase Profiler"): FE 24.96, FF 57.67, BE 64.30, BF 118.92
    fe, ff, be, bf = 24.96, 57.67, 64.30, 118.92
    assert abs(W.naive_bubble(fe, ff, bf, be) - ((57.67 + 118.92) - (64.30 + 24.96))) < 1e-12
    b = W.wavek_bubbles(fe, ff, bf, be, P=8, n_mb=32, k=8)
    assert abs(b["intra_unit"] - (64.30 - 57.67) * 8 * 4) < 1e-9          # 212.16
    assert abs(b["inter_unit"] - (118.92 - 24.96) * 8 * 3) < 1e-9         # 2255.04
    # the stage-doubled expression is half the sum of the two (phase times halve when stages double)
    assert abs(b["stage_doubled"] - 0.5 * (b["intra_unit"] + b["inter_unit"])) < 1e-9
    # a larger unit size reduces every term
    b2 = W.wavek_bubbles(fe, ff, bf, be, P=8, n_mb=32, k=16)
    assert all(b2[key] < b[key] for key in b)


def test_k_search_space():
    # k_min = P; k_max = floor((M_mem - M_static) / M_act); divisors of N_mb preferred
    assert W.k_candidates(P=4, n_mb=32, m_mem=40.96, m_static=10.0, m_activation=3.0) == [4, 8]
    assert W.k_candidates(P=4, n_mb=12, m_mem=100.0, m_static=0.0, m_activation=1.0) == [4, 6, 12]
    assert W.k_candidates(P=5, n_mb=12, m_mem=11.0, m_static=0.0, m_activation=1.0) == [6]
    assert W.k_candidates(P=7, n_mb=12, m_mem=11.0, m_static=0.0, m_activation=1.0) == [7, 8, 9, 10, 11]
