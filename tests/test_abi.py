"""The C-ABI library loads and exports every symbol include/sttm.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sttm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sttm_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2507_07990_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in sttm.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_host_side_geometry_helpers():
    from paper_2507_07990_amd import binding as b
    assert b.sttm_nodes_per_frame(16, 16, 1) == 256 + 64 + 16 + 4 + 1
    assert b.sttm_nodes_per_frame(13, 13, 1) == 341          # tables are laid out on the padded grid
    assert b.sttm_nodes_per_frame(14, 14, 4) == 256 + 64 + 16
    assert b.sttm_nodes_per_frame(27, 27, 1) == 1024 + 256 + 64 + 16 + 4 + 1
    assert b.sttm_nodes_per_frame(33, 8, 1) == 0 and b.sttm_nodes_per_frame(8, 8, 3) == 0
    assert b.sttm_node_index(16, 16, 1, 0, 3, 5) == 3 * 16 + 5
    assert b.sttm_node_index(16, 16, 1, 4, 0, 0) == 340
    assert b.sttm_node_index(16, 16, 1, 5, 0, 0) == -1
    assert b.sttm_workspace_bytes(1, 8, 8, 8, 64, b.STTM_F32, 1) > 0
    assert b.sttm_workspace_bytes(1, 8, 8, 8, 60, b.STTM_F32, 1) == 0     # D % 8
    assert b.sttm_workspace_bytes(1, 8, 8, 8, 64, 7, 1) == 0
