"""ctypes front end of the float64 CPU oracle (oracle/leoam_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports it and it never
imports the product package.

Inputs are numpy arrays or CPU torch tensors in their stored dtype (fp32, fp16,
bf16); they are widened exactly to double inside the C code.  Outputs are numpy
arrays: doubles for attention, float32 scores (the double sum rounded once, the
precision the selection is taken in), int32 selections.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "leoam_oracle.c")
_LIB = os.path.join(_HERE, "libleoam_oracle.so")
_lib = None

F32, F16, BF16, F64 = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over (sequence, head))."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11", _SRC, "-lm", "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_threads(n: int) -> None:
    _load().orc_set_threads(ctypes.c_int(n))


def _as_numpy(x) -> Tuple[np.ndarray, int]:
    """Return (contiguous numpy view of the stored bits, dtype tag)."""
    try:
        import torch
        if isinstance(x, torch.Tensor):
            x = x.detach().cpu().contiguous()
            if x.dtype == torch.bfloat16:
                return x.view(torch.int16).numpy().view(np.uint16), BF16
            x = x.numpy()
    except ImportError:  # pragma: no cover
        pass
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        return x, F32
    if x.dtype == np.float16:
        return x.view(np.uint16), F16
    if x.dtype == np.float64:
        return x, F64
    raise TypeError(f"unsupported dtype {x.dtype}")


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i32(x) -> np.ndarray:
    try:
        import torch
        if isinstance(x, torch.Tensor):
            x = x.detach().cpu().numpy()
    except ImportError:  # pragma: no cover
        pass
    return np.ascontiguousarray(x, dtype=np.int32)


def widen(x) -> np.ndarray:
    """Exact float64 copy of a stored fp32/fp16/bf16 array."""
    a, tag = _as_numpy(x)
    out = np.empty(a.shape, dtype=np.float64)
    _load().orc_widen(_ptr(a), ctypes.c_int(tag), ctypes.c_size_t(0), ctypes.c_size_t(a.size), _ptr(out))
    return out


def abstract_build(K, chunk_off, n_chunks, full: bool = True) -> np.ndarray:
    """Sec. 4.3 abstract: float64 [B,Hkv,c_max,2,D]; [..,0,:]=kmax, [..,1,:]=kmin.
    Rows of unused chunks are NaN.  full=False: the chunks may stop before N (a
    cache that is still being filled)."""
    a, tag = _as_numpy(K)
    B, Hkv, N, D = a.shape
    off = _i32(chunk_off)
    nc = _i32(n_chunks)
    c_max = off.shape[1] - 1
    _check_boundaries(off, nc, N, full)
    out = np.full((B, Hkv, c_max, 2, D), np.nan, dtype=np.float64)
    rc = _load().orc_abstract_build(tag, B, Hkv, N, D, _ptr(a), _ptr(off), _ptr(nc), c_max, _ptr(out))
    assert rc == 0
    return out


def _check_boundaries(off: np.ndarray, nc: np.ndarray, N: int, full: bool = True) -> None:
    for b in range(off.shape[0]):
        row = off[b, : nc[b] + 1]
        if row[0] != 0 or (row[-1] != N if full else row[-1] > N) or np.any(np.diff(row) <= 0):
            raise ValueError(f"chunk boundaries of sequence {b} do not tile [0,{N})")


def abstract_append(K, chunk_off, n_chunks, chunk_size: int, abstract):
    """One decode step of abstract maintenance (Sec. 4.3 abstract, Sec. 2.1 token-by-token
    decoding): the key at index chunk_off[b][n_chunks[b]] joins the last chunk, or opens a
    new one once the last chunk holds chunk_size tokens.  Returns new copies
    (chunk_off, n_chunks, abstract float64, status int32 [B])."""
    a, tag = _as_numpy(K)
    B, Hkv, N, D = a.shape
    off = _i32(chunk_off).copy()
    nc = _i32(n_chunks).copy()
    c_max = off.shape[1] - 1
    _check_boundaries(off, nc, N, full=False)
    ab = np.array(abstract, dtype=np.float64, copy=True, order="C")
    assert ab.shape == (B, Hkv, c_max, 2, D)
    status = np.zeros(B, dtype=np.int32)
    rc = _load().orc_abstract_append(tag, B, Hkv, N, D, _ptr(a), _ptr(off), _ptr(nc), c_max, int(chunk_size), _ptr(ab),
                                     _ptr(status))
    assert rc == 0
    return off, nc, ab, status


def tree_evaluations(n_tokens: int, n_chunks: int, rho: float) -> float:
    """Sec. 4.2 "Dynamic chunk resizing": f(m) = m * sum_{i=0}^{log2(n/m)-1} (2 rho)^i, summed
    term by term in the order printed."""
    size = n_tokens // n_chunks
    levels = int(round(np.log2(size)))
    assert n_chunks * size == n_tokens and (1 << levels) == size
    total = 0.0
    for i in range(levels):
        total += (2.0 * rho) ** i
    return n_chunks * total


def chunk_score(q, abstract, n_chunks, want_lower: bool = False, want_f64: bool = False):
    """Sec. 4.1/4.3 bounds.  q [B,Hq,D]; abstract float64 [B,Hkv,c_max,2,D].
    Returns ub float32 [B,Hkv,c_max] (and lb, ub64, lb64 on request)."""
    qd = widen(q) if not (isinstance(q, np.ndarray) and q.dtype == np.float64) else np.ascontiguousarray(q)
    ab = np.ascontiguousarray(abstract, dtype=np.float64)
    B, Hq, D = qd.shape
    _, Hkv, c_max, two, D2 = ab.shape
    assert two == 2 and D2 == D and Hq % Hkv == 0
    nc = _i32(n_chunks)
    ub = np.empty((B, Hkv, c_max), dtype=np.float32)
    lb = np.empty((B, Hkv, c_max), dtype=np.float32)
    ub64 = np.empty((B, Hkv, c_max), dtype=np.float64)
    lb64 = np.empty((B, Hkv, c_max), dtype=np.float64)
    rc = _load().orc_chunk_score(B, Hq, Hkv, D, _ptr(qd), _ptr(ab), _ptr(nc), c_max, _ptr(ub), _ptr(lb),
                                 _ptr(ub64), _ptr(lb64))
    assert rc == 0
    res = [ub]
    if want_lower:
        res.append(lb)
    if want_f64:
        res += [ub64, lb64] if want_lower else [ub64]
    return res[0] if len(res) == 1 else tuple(res)


def topk_select(score, chunk_off, n_chunks, max_chunks: int, token_budget: int, k_max: int,
                want_margin: bool = False):
    """Sec. 4.2/6.1 selection.  Returns (sel_idx [B,Hkv,k_max], sel_count, sel_tokens[, margin])."""
    s = np.ascontiguousarray(score, dtype=np.float32)
    B, Hkv, c_max = s.shape
    off = _i32(chunk_off)
    nc = _i32(n_chunks)
    assert off.shape == (B, c_max + 1)
    sel = np.empty((B, Hkv, k_max), dtype=np.int32)
    cnt = np.empty((B, Hkv), dtype=np.int32)
    tok = np.empty((B, Hkv), dtype=np.int32)
    mar = np.empty((B, Hkv), dtype=np.float64)
    rc = _load().orc_topk_select(B, Hkv, _ptr(s), _ptr(off), _ptr(nc), c_max, int(max_chunks), int(token_budget),
                                 int(k_max), _ptr(sel), _ptr(cnt), _ptr(tok), _ptr(mar))
    if rc != 0:
        raise ValueError("k_max too small for the selection")
    return (sel, cnt, tok, mar) if want_margin else (sel, cnt, tok)


def sparse_attention(q, K, V, chunk_off, sel_idx, sel_count, scale: Optional[float] = None):
    """Eq. (1) over the selected chunks.  Returns (out float64 [B,Hq,D], lse float64 [B,Hq])."""
    ka, tag = _as_numpy(K)
    va, tag_v = _as_numpy(V)
    assert tag == tag_v and ka.shape == va.shape
    B, Hkv, N, D = ka.shape
    qd = widen(q) if not (isinstance(q, np.ndarray) and q.dtype == np.float64) else np.ascontiguousarray(q)
    Hq = qd.shape[1]
    off = _i32(chunk_off)
    c_max = off.shape[1] - 1
    sel = _i32(sel_idx)
    cnt = _i32(sel_count)
    k_max = sel.shape[2]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    fn = _load().orc_sparse_attention
    rc = fn(tag, B, Hq, Hkv, N, D, _ptr(qd), _ptr(ka), _ptr(va), _ptr(off), c_max, _ptr(sel), _ptr(cnt), k_max,
            ctypes.c_double(scale), _ptr(out), _ptr(lse))
    assert rc == 0
    return out, lse


def decode_step(q, K, V, chunk_off, n_chunks, max_chunks, token_budget, k_max, abstract=None):
    """The whole per-step path in the paper's order: (abstract) -> score -> select -> attention."""
    if abstract is None:
        abstract = abstract_build(K, chunk_off, n_chunks)
    ub = chunk_score(q, abstract, n_chunks)
    sel, cnt, tok = topk_select(ub, chunk_off, n_chunks, max_chunks, token_budget, k_max)
    out, lse = sparse_attention(q, K, V, chunk_off, sel, cnt)
    return dict(abstract=abstract, score=ub, sel_idx=sel, sel_count=cnt, sel_tokens=tok, out=out, lse=lse)


# ---------------------------------------------------------------------------
# compressed KV store (8-bit / 4-bit codes per chunk)
# ---------------------------------------------------------------------------
QCHUNK_DTYPE = np.dtype([("byte_off", "<i8"), ("bits", "<i4"), ("scale_k", "<f4"), ("zero_k", "<f4"),
                         ("scale_v", "<f4"), ("zero_v", "<f4"), ("reserved", "<i4")])
assert QCHUNK_DTYPE.itemsize == 32


def _u8(x) -> np.ndarray:
    try:
        import torch
        if isinstance(x, torch.Tensor):
            x = x.detach().cpu().numpy()
    except ImportError:  # pragma: no cover
        pass
    return np.ascontiguousarray(x).view(np.uint8).reshape(-1)


def _qmeta(x) -> np.ndarray:
    """[B,Hkv,c_max] records: accepts the structured array or its int32 [B,Hkv,c_max,8] image."""
    try:
        import torch
        if isinstance(x, torch.Tensor):
            x = x.detach().cpu().numpy()
    except ImportError:  # pragma: no cover
        pass
    x = np.ascontiguousarray(x)
    if x.dtype != QCHUNK_DTYPE:
        x = x.view(QCHUNK_DTYPE).reshape(x.shape[:-1])
    return x


def half_ceil(x: float) -> float:
    fn = _load().orc_half_ceil
    fn.restype = ctypes.c_double
    return float(fn(ctypes.c_double(x)))


def half_floor(x: float) -> float:
    fn = _load().orc_half_floor
    fn.restype = ctypes.c_double
    return float(fn(ctypes.c_double(x)))


def dequant(blob, qmeta, chunk_off, n_chunks, n_ctx: int, head_dim: int, which: str = "k") -> np.ndarray:
    """Stored values scale*code+zero of the whole store: float64 [B,Hkv,N,D]."""
    qm = _qmeta(qmeta)
    B, Hkv, c_max = qm.shape
    off, nc = _i32(chunk_off), _i32(n_chunks)
    out = np.zeros((B, Hkv, n_ctx, head_dim), dtype=np.float64)
    bl = _u8(blob)
    rc = _load().orc_dequant(B, Hkv, n_ctx, head_dim, _ptr(bl), _ptr(qm), 1 if which == "v" else 0, _ptr(off),
                             _ptr(nc), c_max, _ptr(out))
    assert rc == 0
    return out


def abstract_build_q(kblob, qmeta, chunk_off, n_chunks, head_dim: int = 128) -> np.ndarray:
    """Sec. 4.3 abstract of the stored values, rounded outward to binary16: float64 [B,Hkv,c_max,2,D]."""
    qm = _qmeta(qmeta)
    B, Hkv, c_max = qm.shape
    off, nc = _i32(chunk_off), _i32(n_chunks)
    out = np.full((B, Hkv, c_max, 2, head_dim), np.nan, dtype=np.float64)
    bl = _u8(kblob)
    rc = _load().orc_abstract_build_q(B, Hkv, head_dim, _ptr(bl), _ptr(qm), _ptr(off), _ptr(nc), c_max, _ptr(out))
    assert rc == 0
    return out


def sparse_attention_q(q, kblob, vblob, qmeta, chunk_off, sel_idx, sel_count, scale: Optional[float] = None):
    """Eq. (1) over the kept chunks of the compressed store."""
    qm = _qmeta(qmeta)
    B, Hkv, c_max = qm.shape
    qd = widen(q) if not (isinstance(q, np.ndarray) and q.dtype == np.float64) else np.ascontiguousarray(q)
    Hq, D = qd.shape[1], qd.shape[2]
    off = _i32(chunk_off)
    sel, cnt = _i32(sel_idx), _i32(sel_count)
    k_max = sel.shape[2]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    kb, vb = _u8(kblob), _u8(vblob)
    rc = _load().orc_sparse_attention_q(B, Hq, Hkv, D, _ptr(qd), _ptr(kb), _ptr(vb), _ptr(qm), _ptr(off), c_max,
                                        _ptr(sel), _ptr(cnt), k_max, ctypes.c_double(scale), _ptr(out), _ptr(lse))
    assert rc == 0
    return out, lse


def tree_refine(q, K, chunk_size: int, k_tokens: int, max_rounds: int, node_cap: int):
    """Sec. 4.2 tree-structured chunk refinement (see leoam_oracle.c).  Returns
    (ref_off int32 [B,Hkv,node_cap+1], ref_score float32 [B,Hkv,node_cap], ref_count [B,Hkv],
    evaluations [B,Hkv], status [B,Hkv])."""
    ka, tag = _as_numpy(K)
    B, Hkv, N, D = ka.shape
    qd = widen(q) if not (isinstance(q, np.ndarray) and q.dtype == np.float64) else np.ascontiguousarray(q)
    Hq = qd.shape[1]
    off = np.zeros((B, Hkv, node_cap + 1), dtype=np.int32)
    score = np.full((B, Hkv, node_cap), -np.inf, dtype=np.float32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    evals = np.zeros((B, Hkv), dtype=np.int32)
    status = np.zeros((B, Hkv), dtype=np.int32)
    rc = _load().orc_tree_refine(tag, B, Hq, Hkv, N, D, _ptr(ka), _ptr(qd), int(chunk_size), int(k_tokens), int(max_rounds),
                                 int(node_cap), _ptr(off), _ptr(score), _ptr(cnt), _ptr(evals), _ptr(status))
    if rc != 0:
        raise ValueError("tree_refine: node_cap below the initial chunk count, or k_tokens outside [1, N]")
    return off, score, cnt, evals, status


def chunk_compress(K, V, chunk_off, n_chunks, four_bit):
    """Sec. 4.4 / 6.1 compressed store of K, V [B,Hkv,N,D] (see leoam_oracle.c).  `four_bit` [B,c_max]
    tags the 4-bit chunks.  Returns (kblob uint8, vblob uint8, qmeta records [B,Hkv,c_max])."""
    ka, tag = _as_numpy(K)
    va, tag_v = _as_numpy(V)
    assert tag == tag_v and ka.shape == va.shape
    B, Hkv, N, D = ka.shape
    off, nc = _i32(chunk_off), _i32(n_chunks)
    c_max = off.shape[1] - 1
    _check_boundaries(off, nc, N)
    fb = np.ascontiguousarray(np.asarray(four_bit).astype(np.uint8))
    assert fb.shape == (B, c_max)
    cap = B * Hkv * (N * D + 16 * c_max)
    kblob = np.zeros(cap, dtype=np.uint8)
    vblob = np.zeros(cap, dtype=np.uint8)
    qm = np.zeros((B, Hkv, c_max), dtype=QCHUNK_DTYPE)
    total = np.zeros(1, dtype=np.int64)
    rc = _load().orc_chunk_compress(tag, B, Hkv, N, D, _ptr(ka), _ptr(va), _ptr(off), _ptr(nc), c_max, _ptr(fb),
                                    _ptr(kblob), _ptr(vblob), ctypes.c_int64(cap), _ptr(qm), _ptr(total))
    assert rc == 0
    n = int(total[0])
    return kblob[:n].copy(), vblob[:n].copy(), qm


def chunk_recompress(K, V, chunk_off, n_chunks, four_old, four_new, kblob, vblob, qmeta, used_bytes: int):
    """A store built under the tags `four_old` brought to `four_new` by re-encoding only the chunks whose
    tag changed (see leoam_oracle.c).  kblob / vblob: uint8 arrays of the full capacity (modified in place,
    as is qmeta).  Returns (status, used_bytes, chunks re-encoded); status 1 = no room, nothing changed."""
    ka, tag = _as_numpy(K)
    va, tag_v = _as_numpy(V)
    assert tag == tag_v and ka.shape == va.shape
    B, Hkv, N, D = ka.shape
    off, nc = _i32(chunk_off), _i32(n_chunks)
    c_max = off.shape[1] - 1
    _check_boundaries(off, nc, N)
    fo = np.ascontiguousarray(np.asarray(four_old).astype(np.uint8))
    fn = np.ascontiguousarray(np.asarray(four_new).astype(np.uint8))
    assert fo.shape == (B, c_max) and fn.shape == (B, c_max)
    assert kblob.dtype == np.uint8 and vblob.dtype == np.uint8 and kblob.flags.c_contiguous and vblob.flags.c_contiguous
    assert kblob.shape == vblob.shape and qmeta.dtype == QCHUNK_DTYPE and qmeta.shape == (B, Hkv, c_max)
    used = np.asarray([used_bytes], dtype=np.int64)
    changed = np.zeros(1, dtype=np.int64)
    rc = _load().orc_chunk_recompress(tag, B, Hkv, N, D, _ptr(ka), _ptr(va), _ptr(off), _ptr(nc), c_max, _ptr(fo),
                                      _ptr(fn), _ptr(kblob), _ptr(vblob), ctypes.c_int64(kblob.size), _ptr(qmeta),
                                      _ptr(used), _ptr(changed))
    return int(rc), int(used[0]), int(changed[0])


def compression_share(n_bytes: float, ratio: float, bandwidth: float, t_other: float, t_compute: float,
                      decompress_rate: float) -> float:
    """Sec. 4.4: the share theta of the transmitted bytes that is sent compressed (see leoam_oracle.c)."""
    fn = _load().orc_compression_share
    fn.restype = ctypes.c_double
    return float(fn(*(ctypes.c_double(float(x)) for x in (n_bytes, ratio, bandwidth, t_other, t_compute, decompress_rate))))


def compression_tags(n_chunks, sel_idx, sel_count, c_max: int) -> np.ndarray:
    """Sec. 4.4: which chunks form the compressed share, given a selection of the chunks that matter most
    (Sec. 4.2 order).  A chunk of a sequence is stored 4-bit unless some kv head keeps it: uint8 [B, c_max],
    1 = 4-bit, 0 for kept chunks and for slots >= n_chunks[b].  Plain loops."""
    nc, sel, cnt = _i32(n_chunks), _i32(sel_idx), _i32(sel_count)
    B, Hkv, _ = sel.shape
    out = np.zeros((B, c_max), dtype=np.uint8)
    for b in range(B):
        for c in range(min(int(nc[b]), c_max)):
            kept = False
            for h in range(Hkv):
                for i in range(int(cnt[b, h])):
                    if int(sel[b, h, i]) == c:
                        kept = True
            out[b, c] = 0 if kept else 1
    return out


def score_pin(score, n_chunks, sink_chunks: int, tail_chunks: int) -> np.ndarray:
    """Always-kept chunks (the paper forces none; Sec. 2.1 decoding appends to the tail chunk): a copy of the
    score rows [B,Hkv,c_max] with the first `sink_chunks` and the last `tail_chunks` chunks of every sequence
    set to the largest float, which the Sec. 4.2 order then reads first."""
    out = np.array(score, dtype=np.float32, copy=True)
    nc = _i32(n_chunks)
    big = np.finfo(np.float32).max
    for b in range(out.shape[0]):
        n = min(int(nc[b]), out.shape[2])
        for c in range(n):
            if c < sink_chunks or c >= n - tail_chunks:
                out[b, :, c] = big
    return out
