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


def test_build_report_shows_no_register_spill_in_the_gemm():
    """The build writes every kernel's register and scratch use next to the objects (and refuses
    to link a skinny GEMM that spills).  Where the report of the library's build is at hand (it
    does not travel with the library), the GEMM instantiations use no scratch and the two
    attention forms that are known to spill a few registers outside their loop stay within that."""
    import json
    import pytest
    from paper_2401_12522_amd import build
    path = os.path.join(build.PKG_DIR, "_build", "libbita_kernel_resources.json")
    if not os.path.exists(path):
        pytest.skip("no build report beside the library")
    res = json.load(open(path))
    gemm = {k: v for k, v in res.items() if "gemm_skinny_kernel" in k}
    assert len(gemm) >= 100
    assert all(v["scratch"] == 0 for v in gemm.values())
    spilling = {k: v["scratch"] for k, v in res.items() if v.get("scratch", 0) > 0}
    assert all("tree_attn_kernelILi128ELi2E" in k and s <= 64 for k, s in spilling.items()), spilling


def test_resource_remarks_are_parsed():
    from paper_2401_12522_amd import build
    tag = "[-Rpass-analysis=kernel-resource-usage]"
    remarks = [f"a.hip:1:1: remark: Function Name: _Zk1 {tag}", f"a.hip:1:1: remark:     VGPRs: 20 {tag}",
               f"a.hip:1:1: remark:     ScratchSize [bytes/lane]: 8 {tag}", f"a.hip:1:1: remark:     Occupancy [waves/SIMD]: 4 {tag}",
               f"a.hip:9:1: remark: Function Name: _Zk2 {tag}", f"a.hip:9:1: remark:     AGPRs: 3 {tag}"]
    assert build._kernel_resources(remarks) == {"_Zk1": {"vgprs": 20, "scratch": 8, "occupancy": 4}, "_Zk2": {"agprs": 3}}
    lines = ["x.hip:3:1: warning: something", remarks[0], "    1 | code", "      | ^", "real error"]
    assert build._without_remarks(lines) == ["x.hip:3:1: warning: something", "real error"]
