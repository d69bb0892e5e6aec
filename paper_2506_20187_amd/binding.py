"""Thin ctypes binding of libleoam.so: same names as the C entry points.

Argument marshalling only.  Tensors are torch CUDA tensors (device memory and
the current HIP stream come from torch; nothing else does).  If the library
has not been built, importing this module raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libleoam.so")

F32, F16, BF16, Q8Q4 = 0, 1, 2, 3
_DTYPE_TAG = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}

OK = 0
E_INVALID_ARG, E_BAD_BOUNDARIES, E_UNSUPPORTED, E_WORKSPACE, E_HIP = -1, -2, -3, -4, -6


class LeoamError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("batch", "n_q_heads", "n_kv_heads", "head_dim", "n_ctx", "c_max",
                                                "k_max", "kv_dtype", "abstract_dtype")]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2506_20187_amd/build.py) first")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    sp = ctypes.POINTER(Shape)
    lib.kv_chunk_abstract_build.argtypes = [sp, vp, vp, vp, vp, vp, vp]
    lib.chunk_score.argtypes = [sp, vp, vp, vp, vp, vp, vp]
    lib.chunk_score_pin.argtypes = [sp, vp, i32, i32, vp, vp]
    lib.kv_chunk_abstract_append.argtypes = [sp, vp, vp, vp, i32, vp, vp, vp]
    lib.chunk_tree_refine.argtypes = [sp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.leoam_tree_workspace_bytes.argtypes = [sp, i32]
    lib.leoam_tree_workspace_bytes.restype = sz
    lib.leoam_tree_evaluations.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_double]
    lib.leoam_tree_evaluations.restype = ctypes.c_double
    lib.chunk_topk_select.argtypes = [sp, vp, vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.sparse_chunk_attention_decode.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, vp, sz, vp]
    lib.chunk_select_attention_decode.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, i32, i32, ctypes.c_float, vp, vp, vp,
                                                  vp, vp, vp, sz, vp]
    lib.chunk_select_attention_decode_static.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, i32, i32, ctypes.c_float, vp, vp,
                                                         vp, vp, vp, vp]
    lib.kv_chunk_compress.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp]
    lib.kv_chunk_recompress.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp]
    lib.chunk_compression_tags.argtypes = [sp, vp, vp, vp, vp, vp]
    lib.leoam_compressed_bytes_bound.argtypes = [sp]
    lib.leoam_compressed_bytes_bound.restype = sz
    lib.leoam_compression_share.argtypes = [ctypes.c_double] * 6
    lib.leoam_compression_share.restype = ctypes.c_double
    lib.leoam_workspace_bytes.argtypes = [sp, i32]
    lib.leoam_workspace_bytes.restype = sz
    lib.leoam_fused_workspace_bytes.argtypes = [sp, i32]
    lib.leoam_fused_workspace_bytes.restype = sz
    lib.leoam_fused_control_bytes.argtypes = [sp]
    lib.leoam_fused_control_bytes.restype = sz
    lib.leoam_workspace_init.argtypes = [vp, sz, vp]
    lib.leoam_validate_boundaries.argtypes = [sp, vp, vp, vp]
    lib.leoam_copy_probe.argtypes = [vp, vp, sz, vp]
    lib.leoam_read_probe.argtypes = [vp, sz, vp, vp]
    lib.leoam_status_string.argtypes = [ctypes.c_int]
    lib.leoam_status_string.restype = ctypes.c_char_p
    lib.leoam_version.restype = ctypes.c_int
    for name in ("kv_chunk_abstract_build", "chunk_score", "chunk_score_pin", "chunk_topk_select", "sparse_chunk_attention_decode",
                 "chunk_select_attention_decode", "chunk_select_attention_decode_static", "kv_chunk_abstract_append", "chunk_tree_refine",
                 "kv_chunk_compress", "kv_chunk_recompress", "chunk_compression_tags", "leoam_workspace_init",
                 "leoam_validate_boundaries", "leoam_copy_probe", "leoam_read_probe"):
        getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()

EXPORTS = ("kv_chunk_abstract_build", "chunk_score", "chunk_score_pin", "chunk_topk_select", "sparse_chunk_attention_decode",
           "chunk_select_attention_decode", "chunk_select_attention_decode_static", "leoam_fused_workspace_bytes",
           "leoam_fused_control_bytes",
           "leoam_workspace_init",
           "kv_chunk_abstract_append", "leoam_tree_evaluations", "chunk_tree_refine", "leoam_tree_workspace_bytes",
           "kv_chunk_compress", "kv_chunk_recompress", "chunk_compression_tags", "leoam_compressed_bytes_bound", "leoam_compression_share",
           "leoam_workspace_bytes", "leoam_validate_boundaries", "leoam_copy_probe", "leoam_read_probe", "leoam_status_string",
           "leoam_version")


def status_string(status: int) -> str:
    return _lib.leoam_status_string(int(status)).decode()


def version() -> int:
    return int(_lib.leoam_version())


def make_shape(batch, n_q_heads, n_kv_heads, head_dim, n_ctx, c_max, k_max, dtype) -> Shape:
    """dtype: a torch dtype, or Q8Q4 for the compressed store (q and abstract are then fp16)."""
    tag = _DTYPE_TAG[dtype] if isinstance(dtype, torch.dtype) else int(dtype)
    return Shape(batch, n_q_heads, n_kv_heads, head_dim, n_ctx, c_max, k_max, tag, F16 if tag == Q8Q4 else tag)


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status: int, where: str) -> None:
    if status != OK:
        raise LeoamError(status, where)


def kv_chunk_abstract_build(shape: Shape, K, chunk_off, n_chunks, abstract, stream=None, qmeta=None) -> None:
    _check(_lib.kv_chunk_abstract_build(ctypes.byref(shape), _p(K), _p(qmeta), _p(chunk_off), _p(n_chunks), _p(abstract),
                                        _stream(stream)), "kv_chunk_abstract_build")


def kv_chunk_abstract_append(shape: Shape, K, chunk_off, n_chunks, chunk_size: int, abstract, status=None,
                             stream=None) -> None:
    _check(_lib.kv_chunk_abstract_append(ctypes.byref(shape), _p(K), _p(chunk_off), _p(n_chunks), int(chunk_size),
                                         _p(abstract), _p(status), _stream(stream)), "kv_chunk_abstract_append")


def chunk_tree_refine(shape: Shape, q, K, abstract, chunk_size: int, k_tokens: int, max_rounds: int, node_cap: int,
                      ref_off, ref_score, ref_count, ref_evals, ref_status, workspace, stream=None) -> None:
    nbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(_lib.chunk_tree_refine(ctypes.byref(shape), _p(q), _p(K), _p(abstract), int(chunk_size), int(k_tokens),
                                  int(max_rounds), int(node_cap), _p(ref_off), _p(ref_score), _p(ref_count),
                                  _p(ref_evals), _p(ref_status), _p(workspace), nbytes, _stream(stream)),
           "chunk_tree_refine")


def chunk_score_pin(shape: Shape, n_chunks, sink_chunks: int, tail_chunks: int, score_ub, stream=None) -> None:
    _check(_lib.chunk_score_pin(ctypes.byref(shape), _p(n_chunks), int(sink_chunks), int(tail_chunks), _p(score_ub),
                                _stream(stream)), "chunk_score_pin")


def kv_chunk_compress(shape: Shape, K, V, chunk_off, n_chunks, four_bit, kblob, vblob, qmeta, total_bytes=None,
                      stream=None) -> None:
    """K, V fp16 / bf16 -> the 8-bit / 4-bit store (kblob, vblob uint8; qmeta int32 [B,Hkv,c_max,8])."""
    if kblob.numel() * kblob.element_size() != vblob.numel() * vblob.element_size():
        raise ValueError("kblob and vblob must have the same size")
    _check(_lib.kv_chunk_compress(ctypes.byref(shape), _p(K), _p(V), _p(chunk_off), _p(n_chunks), _p(four_bit), _p(kblob),
                                  _p(vblob), kblob.numel() * kblob.element_size(), _p(qmeta), _p(total_bytes),
                                  _stream(stream)), "kv_chunk_compress")


def kv_chunk_recompress(shape: Shape, K, V, chunk_off, n_chunks, four_bit_old, four_bit_new, kblob, vblob, qmeta,
                        used_bytes, info, stream=None) -> None:
    """A store written under four_bit_old brought to four_bit_new: only the chunks whose tag changed are encoded again.
    used_bytes: int64[1] (in / out), info: int64[3] (out)."""
    if kblob.numel() * kblob.element_size() != vblob.numel() * vblob.element_size():
        raise ValueError("kblob and vblob must have the same size")
    _check(_lib.kv_chunk_recompress(ctypes.byref(shape), _p(K), _p(V), _p(chunk_off), _p(n_chunks), _p(four_bit_old),
                                    _p(four_bit_new), _p(kblob), _p(vblob), kblob.numel() * kblob.element_size(),
                                    _p(qmeta), _p(used_bytes), _p(info), _stream(stream)), "kv_chunk_recompress")


def chunk_compression_tags(shape: Shape, n_chunks, sel_idx, sel_count, four_bit, stream=None) -> None:
    _check(_lib.chunk_compression_tags(ctypes.byref(shape), _p(n_chunks), _p(sel_idx), _p(sel_count), _p(four_bit),
                                       _stream(stream)), "chunk_compression_tags")


def leoam_compressed_bytes_bound(shape: Shape) -> int:
    return int(_lib.leoam_compressed_bytes_bound(ctypes.byref(shape)))


def leoam_compression_share(n_bytes: float, ratio: float, bandwidth: float, t_other: float, t_compute: float,
                            decompress_rate: float) -> float:
    th = float(_lib.leoam_compression_share(float(n_bytes), float(ratio), float(bandwidth), float(t_other),
                                            float(t_compute), float(decompress_rate)))
    if th < 0:
        raise LeoamError(E_INVALID_ARG, "leoam_compression_share")
    return th


def leoam_tree_workspace_bytes(shape: Shape, node_cap: int) -> int:
    return int(_lib.leoam_tree_workspace_bytes(ctypes.byref(shape), int(node_cap)))


def leoam_tree_evaluations(n_tokens: int, n_chunks: int, rho: float) -> float:
    return float(_lib.leoam_tree_evaluations(int(n_tokens), int(n_chunks), float(rho)))


def chunk_score(shape: Shape, q, abstract, n_chunks, score_ub, score_lb=None, stream=None) -> None:
    _check(_lib.chunk_score(ctypes.byref(shape), _p(q), _p(abstract), _p(n_chunks), _p(score_ub), _p(score_lb),
                            _stream(stream)), "chunk_score")


def chunk_topk_select(shape: Shape, score_ub, chunk_off, n_chunks, max_chunks: int, token_budget: int, sel_idx,
                      sel_count, sel_tokens=None, workspace=None, stream=None) -> None:
    nbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(_lib.chunk_topk_select(ctypes.byref(shape), _p(score_ub), _p(chunk_off), _p(n_chunks), int(max_chunks),
                                  int(token_budget), _p(sel_idx), _p(sel_count), _p(sel_tokens), _p(workspace),
                                  nbytes, _stream(stream)), "chunk_topk_select")


def sparse_chunk_attention_decode(shape: Shape, q, K, V, chunk_off, n_chunks, sel_idx, sel_count, softmax_scale,
                                  out, lse, workspace, stream=None, qmeta=None) -> None:
    nbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(_lib.sparse_chunk_attention_decode(ctypes.byref(shape), _p(q), _p(K), _p(V), _p(qmeta), _p(chunk_off), _p(n_chunks),
                                              _p(sel_idx), _p(sel_count), ctypes.c_float(softmax_scale), _p(out),
                                              _p(lse), _p(workspace), nbytes, _stream(stream)),
           "sparse_chunk_attention_decode")


def chunk_select_attention_decode(shape: Shape, score_ub, q, K, V, chunk_off, n_chunks, max_chunks: int,
                                  token_budget: int, softmax_scale, sel_idx, sel_count, sel_tokens, out, lse, workspace,
                                  stream=None, qmeta=None) -> None:
    nbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(_lib.chunk_select_attention_decode(ctypes.byref(shape), _p(score_ub), _p(q), _p(K), _p(V), _p(qmeta),
                                              _p(chunk_off), _p(n_chunks), int(max_chunks), int(token_budget),
                                              ctypes.c_float(softmax_scale), _p(sel_idx), _p(sel_count), _p(sel_tokens),
                                              _p(out), _p(lse), _p(workspace), nbytes, _stream(stream)),
           "chunk_select_attention_decode")


STATIC_SCRATCH_BYTES = 4 << 20


def chunk_select_attention_decode_static(shape: Shape, score_ub, q, K, V, chunk_off, n_chunks, max_chunks: int,
                                         token_budget: int, softmax_scale, sel_idx, sel_count, sel_tokens, out, lse,
                                         stream=None, qmeta=None) -> None:
    """chunk_select_attention_decode with the library's own static workspace (allocates nothing)."""
    _check(_lib.chunk_select_attention_decode_static(ctypes.byref(shape), _p(score_ub), _p(q), _p(K), _p(V), _p(qmeta),
                                                     _p(chunk_off), _p(n_chunks), int(max_chunks), int(token_budget),
                                                     ctypes.c_float(softmax_scale), _p(sel_idx), _p(sel_count),
                                                     _p(sel_tokens), _p(out), _p(lse), _stream(stream)),
           "chunk_select_attention_decode_static")


def leoam_fused_workspace_bytes(shape: Shape, max_tokens: int) -> int:
    return int(_lib.leoam_fused_workspace_bytes(ctypes.byref(shape), int(max_tokens)))


def leoam_fused_control_bytes(shape: Shape) -> int:
    return int(_lib.leoam_fused_control_bytes(ctypes.byref(shape)))


def leoam_workspace_init(workspace, stream=None) -> None:
    nbytes = workspace.numel() * workspace.element_size()
    _check(_lib.leoam_workspace_init(_p(workspace), nbytes, _stream(stream)), "leoam_workspace_init")


def leoam_workspace_bytes(shape: Shape, max_tokens: int) -> int:
    return int(_lib.leoam_workspace_bytes(ctypes.byref(shape), int(max_tokens)))


def leoam_validate_boundaries(shape: Shape, chunk_off, n_chunks, stream=None) -> int:
    return int(_lib.leoam_validate_boundaries(ctypes.byref(shape), _p(chunk_off), _p(n_chunks), _stream(stream)))


def leoam_copy_probe(dst, src, nbytes: int, stream=None) -> None:
    _check(_lib.leoam_copy_probe(_p(dst), _p(src), int(nbytes), _stream(stream)), "leoam_copy_probe")


def leoam_read_probe(src, nbytes: int, sink, stream=None) -> None:
    _check(_lib.leoam_read_probe(_p(src), int(nbytes), _p(sink), _stream(stream)), "leoam_read_probe")


def default_scale(head_dim: int) -> float:
    return 1.0 / math.sqrt(head_dim)
