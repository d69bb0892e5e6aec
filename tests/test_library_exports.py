"""The C-ABI library loads and exports every symbol include/leoam.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

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
    # q, K, V and the abstract are read with 16-byte loads: a misaligned address is refused
    ok, odd = ctypes.c_void_p(4096), ctypes.c_void_p(4096 + 8)
    assert lib.chunk_score(ctypes.byref(s), odd, ok, ok, ok, None, None) == -1
    assert lib.chunk_score(ctypes.byref(s), ok, odd, ok, ok, None, None) == -1
    assert lib.kv_chunk_abstract_build(ctypes.byref(s), odd, None, ok, ok, ok, None) == -1
    assert lib.sparse_chunk_attention_decode(ctypes.byref(s), ok, ok, odd, None, ok, ok, ok, ok, ctypes.c_float(1.0), ok, None,
                                             ok, 1 << 30, None) == -1


def test_host_side_checks_of_the_later_entry_points():
    """Workspace sizes and argument refusals of the one-call step, the abstract maintenance and the tree
    refinement are host arithmetic: no GPU needed."""
    import paper_2506_20187_amd as L
    lib = L.binding._lib
    s = L.make_shape(16, 32, 8, 128, 131072, 4096, 256, 2)
    fused, plain = L.leoam_fused_workspace_bytes(s, 4096), L.leoam_workspace_bytes(s, 4096)
    assert fused >= plain + 16 * 8 * 4                     # arrival counters in front of the partials
    assert L.leoam_fused_workspace_bytes(L.make_shape(16, 32, 8, 64, 131072, 4096, 256, 2), 4096) == 0
    # tree refinement: node_cap below the initial chunk count, k outside [1, n_ctx], compressed store
    t = L.make_shape(1, 4, 1, 128, 4096, 64, 1, 2)
    assert L.leoam_tree_workspace_bytes(t, 1000) == 1 * 1 * (1000 * 2 * 16 + 500 * 16)
    args = [None] * 3
    def refine(shape, cs, k, rounds, cap):
        return lib.chunk_tree_refine(ctypes.byref(shape), None, None, None, cs, k, rounds, cap, None, None, None, None,
                                     None, None, 0, None)
    assert refine(t, 64, 100, 10, 63) == -1                # 64 initial chunks do not fit 63 nodes
    assert refine(t, 64, 0, 10, 128) == -1 and refine(t, 64, 4097, 10, 128) == -1
    assert refine(t, 32, 100, 10, 256) == -1               # 128 initial chunks but the abstract has room for 64
    assert refine(t, 64, 100, -1, 128) == -1
    assert refine(L.make_shape(1, 4, 1, 128, 4096, 64, 1, 3), 64, 100, 10, 128) == -3
    assert refine(t, 64, 100, 10, 128) == -1               # shape fine: null pointers are refused next
    # abstract maintenance
    assert lib.kv_chunk_abstract_append(ctypes.byref(t), None, None, None, 64, None, None, None) == -1
    assert lib.kv_chunk_abstract_append(ctypes.byref(L.make_shape(1, 4, 1, 128, 4096, 64, 1, 3)), None, None, None, 64,
                                        None, None, None) in (-1, -3)
    assert lib.leoam_workspace_init(None, 16, None) == -1


def test_host_side_checks_of_the_compression_entry_points():
    """Argument refusals of kv_chunk_compress and the compressed share theta (Sec. 4.4) are host arithmetic."""
    import paper_2506_20187_amd as L
    lib = L.binding._lib
    s = L.make_shape(2, 8, 2, 128, 1000, 64, 16, 1)
    assert L.leoam_compressed_bytes_bound(s) == 2 * 2 * 1000 * 128
    none = [None] * 3

    def compress(shape, blob_bytes, ptr=None):
        return lib.kv_chunk_compress(ctypes.byref(shape), ptr, ptr, ptr, ptr, ptr, ptr, ptr, blob_bytes, ptr, None, None)
    assert compress(s, 1 << 20) == -1                                        # null pointers
    fake = ctypes.c_void_p(4096)
    assert compress(L.make_shape(2, 8, 2, 128, 1000, 64, 16, 0), 1 << 20, fake) == -3      # fp32 source
    assert compress(s, 2 * 2 * 1000 * 128 - 1, fake) == -4                   # blobs below the bound
    # theta: equal sides inside (0, 1); the formula's two sides are written out here
    D, ratio, bw, t0, tc, rate = 64e6, 0.25, 16e9, 0.3e-3, 2.0e-3, 200e9
    th = L.leoam_compression_share(D, ratio, bw, t0, tc, rate)
    assert 0 < th < 1
    assert abs((t0 + D * (1 - th + th * ratio) / bw) - (tc + D * th / rate)) < 1e-12
    assert L.leoam_compression_share(D, ratio, bw, 0.0, 10e-3, rate) == 0.0
    assert L.leoam_compression_share(D, ratio, 1e9, t0, 1e-3, rate) == 1.0
    import oracle
    for args in ((D, ratio, bw, t0, tc, rate), (1e9, 0.5, 50e9, 0.0, 5e-3, 1e12), (3e8, 0.27, 25e9, 1e-3, 4e-3, 3e11)):
        assert abs(L.leoam_compression_share(*args) - oracle.compression_share(*args)) <= 1e-15
    with pytest.raises(L.LeoamError):
        L.leoam_compression_share(D, 1.5, bw, t0, tc, rate)
    with pytest.raises(L.LeoamError):
        L.leoam_compression_share(-1.0, ratio, bw, t0, tc, rate)
