"""The C-ABI library loads and exports every function include/mlip.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "mlip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mlip_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_all_declared_symbols():
    import __graft_entry__ as ge
    lib_path = os.path.join(ROOT, "paper_2506_02023_amd", "libmlip.so")
    if not os.path.exists(lib_path):
        ge.build()
    lib = ctypes.CDLL(lib_path)
    names = _declared()
    assert {"mlip_build_graph", "mlip_forward", "mlip_graph_destroy", "mlip_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    lib.mlip_version.restype = ctypes.c_char_p
    assert b"gfx950" in lib.mlip_version()


def test_profile_groups_of_the_binding_match_the_header():
    """mlip_profile_read fills MLIP_PROF_COUNT entries: the binding's arrays are sized by its list of group names, which
    must therefore name every group of the header, in the header's order."""
    from paper_2506_02023_amd import binding as B
    text = open(os.path.join(ROOT, "include", "mlip.h")).read()
    groups = {name: int(value) for name, value in re.findall(r"\bMLIP_PROF_([A-Z_]+)\s*=\s*(\d+)", text)}
    count = groups.pop("COUNT")
    assert sorted(groups.values()) == list(range(count))
    by_index = [name.lower() for name, _ in sorted(groups.items(), key=lambda kv: kv[1])]
    assert list(B.PROF_GROUPS) == by_index


def test_argument_errors_without_gpu():
    """Error paths that are decided before any HIP call."""
    from paper_2506_02023_amd import binding as B
    L = B.lib()
    h = ctypes.c_void_p(None)
    cell = (ctypes.c_double * 9)(*[1, 0, 0, 0, 1, 0, 0, 0, 1])
    dummy = ctypes.c_void_p(16)
    assert L.mlip_build_graph(None, cell, dummy, 4, 1.0, 1, None, ctypes.byref(h)) == -1
    assert L.mlip_build_graph(dummy, cell, dummy, 0, 1.0, 1, None, ctypes.byref(h)) == -1
    assert L.mlip_build_graph(dummy, cell, dummy, 4, -1.0, 1, None, ctypes.byref(h)) == -1
    assert L.mlip_build_graph(dummy, cell, dummy, 4, 1.0, 0, None, ctypes.byref(h)) == -1
    assert L.mlip_build_graph(dummy, cell, dummy, 4, 1.0, 65, None, ctypes.byref(h)) == -1
    assert h.value is None
    assert b"n_slabs" in L.mlip_last_error()
    assert L.mlip_forward(None, None, 0, None, None, None) == -1
