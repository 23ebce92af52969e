"""CPU-side checks of the boundary: the library loads, exports what include/saga.h declares,
and its struct layouts match the header (no compute calls: no GPU here)."""
import ctypes
import os
import re

import paper_1810_08403_amd as saga
from paper_1810_08403_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "saga.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(saga_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_entry_point():
    names = _declared_functions()
    assert "saga_layer_forward" in names and len(names) >= 12
    lib = saga.load_library()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in saga.h but not exported"
    assert sorted(saga.EXPORTS) == names


def test_version_string():
    assert "gfx950" in saga.version()


def test_struct_sizes_match_the_header_layout():
    assert ctypes.sizeof(binding.Tensor) == 8 + 3 * 8 + 2 * 4
    assert ctypes.sizeof(binding.EdgeParams) == 7 * 8
    assert ctypes.sizeof(binding.VertexParams) == 4 * 8
    assert ctypes.sizeof(binding.LayerGrads) == 9 * 8
    assert ctypes.sizeof(binding.Timings) == 8 + 5 * 8 + 3 * 8 + 8 + 3 * 4 + 4 + 2 * 8 + 8 + 4 * 8


def test_null_arguments_are_rejected_without_a_gpu():
    lib = saga.load_library()
    assert lib.saga_destroy(None) == 1
    assert lib.saga_graph_destroy(None) == 1
    assert lib.saga_create(None, 0, None, 0) == 1
    assert lib.saga_last_error(None) == b"null context"
    assert lib.saga_peak_device_bytes(None) == 0


def test_header_is_plain_c_and_its_layouts_are_the_binding_s(tmp_path):
    """include/saga.h must compile as C99 on its own (a C caller has nothing else), and the struct sizes and member
    offsets a C compiler gives are the ones the ctypes binding marshals to."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    assert gcc, "gcc is part of the image"
    inc = os.path.join(ROOT, "include")
    members = {
        "saga_tensor": (binding.Tensor, ["data", "rows", "cols", "ld", "dtype", "mem"]),
        "saga_edge_params": (binding.EdgeParams, ["op", "edge_weight", "W_gate", "b_gate", "W_msg", "W_pool", "b_pool"]),
        "saga_vertex_params": (binding.VertexParams, ["W", "bias", "act", "W_self"]),
        "saga_layer_grads": (binding.LayerGrads, ["dX", "dW", "dbias", "dW_self", "dW_gate", "db_gate", "dW_msg", "dW_pool", "db_pool"]),
    }
    lines = ['#include "saga.h"', "#include <stddef.h>", "#include <stdio.h>", "int main(void) {"]
    for name, (_, fields) in members.items():
        lines.append(f'  printf("{name} %zu\\n", sizeof({name}));')
        for f in fields:
            lines.append(f'  printf("{name}.{f} %zu\\n", offsetof({name}, {f}));')
    lines.append('  printf("saga_timings %zu\\n", sizeof(saga_timings));')
    lines += ["  return 0;", "}"]
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, str(src), "-o", str(exe)], check=True)
    got = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for name, (cls, fields) in members.items():
        assert int(got[name]) == ctypes.sizeof(cls), name
        names = [f[0] for f in cls._fields_ if not f[0].startswith(("reserved", "pad"))]   # explicit padding in the binding
        assert names == fields, (name, names)
        for f in fields:
            assert int(got[f"{name}.{f}"]) == getattr(cls, f).offset, (name, f)
    assert int(got["saga_timings"]) == ctypes.sizeof(binding.Timings)


def test_every_option_of_saga_set_option_is_documented_in_the_header():
    src = open(os.path.join(ROOT, "paper_1810_08403_amd", "csrc", "saga_api.hip")).read()
    names = set(re.findall(r'!strcmp\(name, "([a-z_0-9]+)"\)', src))
    assert len(names) >= 10
    header = open(os.path.join(ROOT, "include", "saga.h")).read()
    missing = [n for n in sorted(names) if f'"{n}"' not in header]
    assert not missing, f"options without a line in saga.h: {missing}"
