"""The C-ABI library loads and exports every symbol include/bita.h declares (CPU only:
no compute call is made)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "bita.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bita_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2401_12522_amd import build, binding
    if not os.path.exists(build.LIB_PATH):
        build.build_library()
    lib = ctypes.CDLL(build.LIB_PATH)
    names = _declared_symbols()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_host_side_errors_without_gpu_work():
    """Argument validation happens before any device call."""
    from paper_2401_12522_amd import binding
    L = binding.lib()
    assert L.bita_packed_bytes(32, 688) == 2 * 11 * 2048
    assert L.bita_packed_bytes(0, 5) == 0
    assert L.bita_build_tree(None, None, None, 0, 0, None, None, 1, None, None) == -1
    assert b"bita_build_tree" in L.bita_last_error()
    assert L.bita_accept(None, None, None, 1, None, None, None, None, None, None, None) == -1
    assert L.bita_workspace_bytes(None, 1, 1) == 0
    assert L.bita_tree_template_info(None, 0) == -1
