"""The algorithmic work per launch that bench.py divides by the measured launch times, evaluated by hand for small
layer counts: a drift of these figures would silently change every reported roofline fraction.  CPU only."""
import bench
from paper_2605_18404_amd import synth


def test_matrix_products_count_one_row_per_edge_pair():
    w = synth.WORKLOADS[1]  # invariant, C = H = 128, K = 32
    E, N = 1000, 50
    t = bench.kernel_table(w, E, N)
    C, H, K = w.channels, w.edge_hidden, w.n_rbf
    assert t[1][2] == 2.0 * E * K * H            # jets of E / 2 pairs = E rows
    assert t[2][2] == 2.0 * E * H * C
    for kid in (7, 8, 9, 10):
        assert t[kid][2] == 2.0 * (E // 2) * C * H
    # gather kernels: filter jets and adjoints per directed edge, node tables once, geometry and indices
    f = 4
    assert t[3][1] == "hbm" and t[3][2] == E * C * f + 2 * N * C * f + E * 20
    assert t[6][2] == 2 * E * C * f + E * C * f + 6 * N * C * f + E * 28


def test_equivariant_layers_are_counted_at_their_own_size():
    E, N = 1200, 40
    nnz, paths, M = 83, 11, 9
    for L in (1, 2, 4):
        w = synth.shrink(synth.WORKLOADS[2], n_layers=L)
        C = w.channels
        t = bench.kernel_table(w, E, N)
        small = 9 + M * 3        # (l_max + 1)^2 entries, l_max + 1 paths: first and last layer
        full = nnz + M * paths
        per_layer = {1: [small], 2: [small, small], 4: [small, full, full, small]}[L]
        want = 2.0 * sum(per_layer) / L * C * E
        for kid, evals in ((3, 1), (4, 2), (5, 3), (6, 4)):
            assert t[kid][1] == "alu"
            assert abs(t[kid][2] - want * evals) < 1e-6 * want
        widths = {1: [3], 2: [3, 3], 4: [3, 11, 11, 3]}[L]
        assert abs(t[2][2] - 2.0 * E * w.edge_hidden * C * sum(widths) / L) < 1e-3


def test_lmax3_counts():
    w = synth.shrink(synth.WORKLOADS[2], l_max=3, n_layers=3)
    t = bench.kernel_table(w, 100, 10)
    want = 2.0 * ((16 + 16 * 4) * 2 + (353 + 16 * 23)) / 3 * w.channels * 100
    assert abs(t[3][2] - want) < 1e-6 * want
