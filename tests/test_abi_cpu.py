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
    assert ctypes.sizeof(binding.Timings) == 8 + 5 * 8 + 3 * 8 + 8 + 3 * 4 + 4 + 2 * 8


def test_null_arguments_are_rejected_without_a_gpu():
    lib = saga.load_library()
    assert lib.saga_destroy(None) == 1
    assert lib.saga_graph_destroy(None) == 1
    assert lib.saga_create(None, 0, None, 0) == 1
    assert lib.saga_last_error(None) == b"null context"
    assert lib.saga_peak_device_bytes(None) == 0
