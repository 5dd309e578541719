"""CPU-side checks of the boundary: the library builds, loads and exports every symbol the
header declares, and the generator's parameter layout matches the documented one."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_18404_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2605_18404_amd", "libmlip.so")


def _declared():
    src = open(os.path.join(ROOT, "include", "mlip.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(mlip_[a-z_]+)\s*\(", src)))


def test_header_declares_the_entry_points():
    names = _declared()
    for n in ["mlip_graph_build", "mlip_forward_energy", "mlip_forward_force", "mlip_backward_force",
              "mlip_backward_energy", "mlip_train_step", "mlip_create", "mlip_destroy"]:
        assert n in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.skip("libmlip.so not built (run __graft_entry__.build())")
    lib = ctypes.CDLL(LIB)
    for n in _declared():
        assert hasattr(lib, n), n


def test_binding_fails_loudly_without_the_library(monkeypatch):
    from paper_2605_18404_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libmlip.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_param_layout_counts():
    # emb S*C + L*(H*K + C*H + 2*C*C) + C*C + C
    w = synth.WORKLOADS[0]
    assert synth.param_count(w) == 2 * 32 + 2 * (32 * 16 + 32 * 32 + 2 * 32 * 32) + 32 * 32 + 32
    w = synth.WORKLOADS[3]
    assert synth.param_count(w) == 4 * (512 * 32 + 2 * 512 * 512 + 2 * 512 * 512)
    w = synth.WORKLOADS[2]
    assert synth.param_count(w) == 8 * 64 + 4 * (64 * 32 + 11 * 64 * 64 + 3 * 64 * 64) + 64 * 64 + 64


def test_generator_is_deterministic_and_bounded():
    w = synth.WORKLOADS[0]
    a, b = synth.make_inputs(w), synth.make_inputs(w)
    for k in ("pos", "species", "params", "E_ref", "F_ref"):
        assert np.array_equal(getattr(a, k), getattr(b, k))
    assert a.pos.min() >= 0 and a.pos.max() < w.box
    assert set(np.unique(a.species)) <= set(range(w.n_species))
    n = synth.normal(1, 2, 0, 20000)
    assert abs(n.mean()) < 0.03 and abs(n.std() - 1) < 0.03


def test_header_is_plain_c_and_matches_the_binding_structs(tmp_path):
    """The header compiles as C99 on its own, and the ctypes mirrors of its structs have the C
    compiler's sizes and field offsets."""
    import shutil
    import subprocess
    from paper_2605_18404_amd import binding
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    fields = {"mlip_config": [f[0] for f in binding.mlip_config._fields_],
              "mlip_adamw": [f[0] for f in binding.mlip_adamw._fields_]}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "mlip.h"', 'int main(void) {']
    for st, fs in fields.items():
        lines.append(f'  printf("{st} %zu\\n", sizeof({st}));')
        for f in fs:
            lines.append(f'  printf("{st}.{f} %zu\\n", offsetof({st}, {f}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "probe.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "probe"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True, capture_output=True)
    out = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for st, cls in (("mlip_config", binding.mlip_config), ("mlip_adamw", binding.mlip_adamw)):
        assert int(out[st]) == ctypes.sizeof(cls)
        for f in fields[st]:
            assert int(out[f"{st}.{f}"]) == getattr(cls, f).offset, (st, f)
