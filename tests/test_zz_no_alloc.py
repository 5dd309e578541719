"""The allocation-free radius graph (mlip_graph_build_static) against the context-based one
(mlip_graph_build + mlip_graph_export): bit-exact, on two calls in a row that share the library's
static work array, the second with a smaller input; then its limits."""
import numpy as np
import pytest
import torch

from paper_2605_18404_amd import synth
from paper_2605_18404_amd.binding import Mlip, MlipError, mlip_graph_build_static

from gpu_common import DEV, DevInputs

pytestmark = pytest.mark.gpu


def _with_context(w, d):
    m = Mlip.for_workload(w)
    n = m.mlip_graph_build(d.pos, d.struct_ptr, d.cell, w.cutoff)
    out = [t.clone() for t in m.mlip_graph_export()]
    torch.cuda.synchronize()
    m.close()
    return n, out


def _static(w, d, cap):
    o = dict(device=DEV, dtype=torch.int32)
    row_ptr, sender = torch.full((w.n_atoms + 1,), -7, **o), torch.full((cap,), -7, **o)
    shift, rev = torch.full((cap, 3), -7, **o), torch.full((cap,), -7, **o)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    n = mlip_graph_build_static(d.pos, d.struct_ptr, d.cell, w.cutoff, row_ptr, sender, shift, rev)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before  # nothing went through torch's allocator either
    return n, (row_ptr, sender, shift, rev)


def test_static_graph_build_matches_context_build_twice():
    W = synth.WORKLOADS
    big = synth.shrink(W[1], n_structs=6)                                  # 1152 atoms, ~83 k edges, several bins
    small = synth.shrink(W[0], atoms_per_struct=50, n_structs=3, box=9.0)  # then a smaller batch on the same scratch
    mixed = synth.shrink(W[1], n_structs=3, cell_kind="free")             # molecules: the bounding-box path
    for w in (big, small, mixed, big):
        d = DevInputs(synth.make_inputs(w))
        n_ref, ref = _with_context(w, d)
        cap = n_ref + 1000
        n, got = _static(w, d, cap)
        assert n == n_ref and n > 0
        assert torch.equal(got[0], ref[0])
        for g, r in zip(got[1:], ref[1:]):
            assert torch.equal(g[:n], r)
            assert bool((g[n:] == -7).all())  # nothing written beyond the edge count


def test_static_graph_build_limits():
    w = synth.shrink(synth.WORKLOADS[0], atoms_per_struct=50, n_structs=2, box=9.0)
    d = DevInputs(synth.make_inputs(w))
    n_ref, _ = _with_context(w, d)
    with pytest.raises(MlipError) as e:  # output buffers too small: reports the count that is needed
        _static(w, d, n_ref - 1)
    assert e.value.code == -2 and e.value.n_edges == n_ref
    o = dict(device=DEV, dtype=torch.int32)
    N = 16385  # one atom more than the static work array is laid out for: refused before anything runs
    pos = torch.zeros(N, 3, device=DEV)
    sp = torch.tensor([0, N], **o)
    with pytest.raises(MlipError) as e:
        mlip_graph_build_static(pos, sp, d.cell[:1].contiguous(), w.cutoff, torch.zeros(N + 1, **o), torch.zeros(8, **o),
                                torch.zeros(8, 3, **o), torch.zeros(8, **o))
    assert e.value.code == -2 and "16384" in str(e.value)
    with pytest.raises(MlipError) as e:  # errors of the ordinary build come through: cutoff beyond the box
        mlip_graph_build_static(d.pos, d.struct_ptr, d.cell, 50.0, *[torch.zeros(s, **o) for s in ((w.n_atoms + 1,), (8,), (8, 3), (8,))])
    assert e.value.code == -1
    n, _ = _static(w, d, n_ref)  # and the next call is unaffected
    assert n == n_ref
