"""Builds the compressed KV store (input preparation for the int8/int4 workload).

Per (sequence, kv head, chunk, tensor) asymmetric affine quantisation with one
scale and one zero point: code = round((x - zero) / scale), zero = min over the
chunk, scale = (max - min) / levels with levels = 255 (8-bit codes 0..255) or 15 (4-bit codes 0..15).  8-bit chunks keep one byte per
element; 4-bit chunks pack two codes per byte (even channel in the low nibble).
K and V blobs share the per-chunk byte offsets.  Which chunks are 4-bit is
given by `four_bit[b, c]` (the paper chooses a share from a latency model,
Sec. 4.4; here the tag is an input).
"""
from __future__ import annotations

from typing import Tuple

import numpy as np
import torch

QCHUNK_WORDS = 8      # int32 words per chunk record (32 bytes)


def quantize_store(K: torch.Tensor, V: torch.Tensor, chunk_off: np.ndarray, n_chunks: np.ndarray,
                   four_bit: np.ndarray) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """K, V [B,Hkv,N,D] (any float dtype, any device) -> (kblob uint8, vblob uint8, qmeta int32 [B,Hkv,c_max,8]).

    qmeta rows are the 32-byte records {int64 byte_off, int32 bits, float scale_k, zero_k, scale_v, zero_v, int32 0}.
    """
    B, Hkv, N, D = K.shape
    dev = K.device
    c_max = chunk_off.shape[1] - 1
    # byte layout: chunks of (b,h) in order, (b,h) pairs in order; rows are D (8-bit) or D/2 (4-bit) bytes
    row_bytes = np.where(four_bit, D // 2, D).astype(np.int64)                       # [B, c_max]
    sizes = np.diff(chunk_off.astype(np.int64), axis=1)                              # [B, c_max]
    valid = np.arange(c_max)[None, :] < n_chunks[:, None]
    chunk_bytes = np.where(valid, sizes * row_bytes, 0)
    chunk_bytes = (chunk_bytes + 15) // 16 * 16
    per_b = chunk_bytes.sum(axis=1)                                                  # bytes of one head of sequence b
    total = int((per_b * Hkv).sum())
    kblob = torch.zeros(max(16, total), dtype=torch.uint8, device=dev)
    vblob = torch.zeros(max(16, total), dtype=torch.uint8, device=dev)
    meta = np.zeros((B, Hkv, c_max), dtype=np.dtype([("byte_off", "<i8"), ("bits", "<i4"), ("scale_k", "<f4"),
                                                    ("zero_k", "<f4"), ("scale_v", "<f4"), ("zero_v", "<f4"),
                                                    ("reserved", "<i4")]))
    base = 0
    for b in range(B):
        within = np.concatenate([[0], np.cumsum(chunk_bytes[b])[:-1]])
        n = int(n_chunks[b])
        off = chunk_off[b].astype(np.int64)
        seg_id = torch.from_numpy(np.repeat(np.arange(n), sizes[b, :n])).to(dev)     # token -> chunk
        for h in range(Hkv):
            head_base = base + h * int(per_b[b])
            meta["byte_off"][b, h, :] = head_base + within
            meta["bits"][b, h, :] = np.where(four_bit[b], 4, 8)
            for name, X, blob in (("k", K, kblob), ("v", V, vblob)):
                x = X[b, h].to(torch.float32)                                        # [N, D]
                # per-chunk min / max over all elements of the chunk
                row_min, row_max = x.min(dim=1).values, x.max(dim=1).values
                cmin = torch.full((n,), float("inf"), device=dev).scatter_reduce(0, seg_id, row_min, "amin")
                cmax = torch.full((n,), float("-inf"), device=dev).scatter_reduce(0, seg_id, row_max, "amax")
                levels = torch.from_numpy(np.where(four_bit[b, :n], 15.0, 255.0).astype(np.float32)).to(dev)
                scale = (cmax - cmin) / levels
                zero = cmin
                meta["scale_" + name][b, h, :n] = scale.cpu().numpy()
                meta["zero_" + name][b, h, :n] = zero.cpu().numpy()
                s_tok, z_tok, l_tok = scale[seg_id], zero[seg_id], levels[seg_id]
                safe = torch.where(s_tok > 0, s_tok, torch.ones_like(s_tok))
                codes = torch.clamp(torch.round((x - z_tok[:, None]) / safe[:, None]), min=0).minimum(l_tok[:, None])
                codes = torch.where((s_tok > 0)[:, None], codes, torch.zeros_like(codes)).to(torch.uint8)
                # scatter the rows of each format into the blob
                fb_tok = torch.from_numpy(np.repeat(four_bit[b, :n], sizes[b, :n])).to(dev)
                tok_in_chunk = torch.arange(N, device=dev) - torch.from_numpy(off[:n]).to(dev)[seg_id]
                row_b = torch.where(fb_tok, D // 2, D)
                row_start = torch.from_numpy(head_base + within[:n]).to(dev)[seg_id] + tok_in_chunk * row_b
                idx8 = torch.nonzero(~fb_tok).flatten()
                if idx8.numel():
                    dst = row_start[idx8][:, None] + torch.arange(D, device=dev)[None, :]
                    blob[dst.reshape(-1)] = codes[idx8].reshape(-1)
                idx4 = torch.nonzero(fb_tok).flatten()
                if idx4.numel():
                    c4 = codes[idx4]
                    packed = (c4[:, 0::2] | (c4[:, 1::2] << 4)).to(torch.uint8)
                    dst = row_start[idx4][:, None] + torch.arange(D // 2, device=dev)[None, :]
                    blob[dst.reshape(-1)] = packed.reshape(-1)
        base += int(per_b[b]) * Hkv
    qmeta = torch.from_numpy(meta.view(np.int32).reshape(B, Hkv, c_max, QCHUNK_WORDS).copy()).to(dev)
    return kblob, vblob, qmeta


def tag_four_bit(chunk_off: np.ndarray, n_chunks: np.ndarray, heavy_tokens: np.ndarray, share: float = 0.5) -> np.ndarray:
    """four_bit[b, c]: chunks without heavy tokens first, until `share` of the chunks are tagged."""
    B, c1 = chunk_off.shape
    c_max = c1 - 1
    out = np.zeros((B, c_max), dtype=bool)
    for b in range(B):
        n = int(n_chunks[b])
        has_heavy = np.add.reduceat(heavy_tokens[b].astype(np.int64), chunk_off[b, :n]) > 0
        order = np.argsort(has_heavy, kind="stable")              # light chunks first
        out[b, order[: int(share * n)]] = True
    return out


class QuantCase:
    """A dense case (its fp16 query is kept) plus its compressed store."""

    def __init__(self, case, kblob, vblob, qmeta, four_bit):
        self.case, self.kblob, self.vblob, self.qmeta, self.four_bit = case, kblob, vblob, qmeta, four_bit


def make_quant_case(config: str = "c4", layer: int = 0, four_bit_share: float = 0.5, **kw) -> QuantCase:
    """Config `config` generated as usual, then stored as 8-bit chunks with the
    `four_bit_share` of chunks that hold no heavy token stored as 4-bit; q is fp16."""
    from .workloads import make_case
    case = make_case(config, layer=layer, **kw)
    case.q = case.q.to(torch.float16)
    off = case.chunk_off.cpu().numpy()
    nc = case.n_chunks.cpu().numpy()
    fb = tag_four_bit(off, nc, case.extra["heavy"], four_bit_share)
    kblob, vblob, qmeta = quantize_store(case.K, case.V, off, nc, fb)
    return QuantCase(case, kblob, vblob, qmeta, fb)
