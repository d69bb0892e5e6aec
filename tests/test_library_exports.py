"""The C-ABI library loads and exports every symbol include/leoam.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "leoam.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_][a-z0-9_]*)\s*\(", text)) - {"defined"})


def test_library_exports_every_declared_symbol():
    from paper_2506_20187_amd import build as b
    if b.needs_build():
        b.build_library(verbose=False)
    lib = ctypes.CDLL(b.LIB)
    names = declared_functions()
    assert {"kv_chunk_abstract_build", "chunk_score", "chunk_topk_select", "sparse_chunk_attention_decode"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"libleoam.so does not export {n}"


def test_binding_names_match_header():
    import paper_2506_20187_amd as L
    for n in declared_functions():
        assert n in L.binding.EXPORTS
    assert L.version() >= 100
    assert L.status_string(0) == "ok"


def test_host_side_argument_checks_without_gpu():
    # shape faults are refused before any HIP call, so this runs on a CPU-only box
    import paper_2506_20187_amd as L
    s = L.make_shape(1, 32, 8, 128, 131072, 8192, 256, 2)
    assert L.leoam_workspace_bytes(s, 4096) > 0
    assert L.leoam_workspace_bytes(L.make_shape(1, 32, 8, 64, 131072, 8192, 256, 2), 4096) == 0
    lib = L.binding._lib
    assert lib.chunk_score(ctypes.byref(s), None, None, None, None, None, None) == -1
    bad = L.make_shape(1, 32, 8, 128, 131072, 8192, 9000, 2)
    assert lib.chunk_score(ctypes.byref(bad), None, None, None, None, None, None) == -1
