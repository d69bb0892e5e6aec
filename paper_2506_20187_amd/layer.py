"""Buffer holder for one layer's decode step (allocation + call order only)."""
from __future__ import annotations

import torch

from . import binding as B


class DecodeLayer:
    """Owns abstract / score / selection / output / workspace buffers of one
    layer and calls the entry points in the paper's order.  All arithmetic
    happens inside libleoam.so."""

    def __init__(self, K: torch.Tensor, V: torch.Tensor, chunk_off: torch.Tensor, n_chunks: torch.Tensor,
                 n_q_heads: int, k_max: int, max_chunks: int, token_budget: int, qmeta: torch.Tensor = None,
                 n_kv_heads: int = None, n_ctx: int = None, head_dim: int = 128):
        """Dense store: K, V [B,Hkv,N,D].  Compressed store: K, V are the byte blobs, qmeta the
        [B,Hkv,c_max,8] int32 chunk records, and n_kv_heads / n_ctx must be given."""
        self.qmeta = qmeta
        if qmeta is None:
            batch, hkv, n_ctx, d = K.shape
            dtype, adtype = K.dtype, K.dtype
        else:
            batch, hkv, d = chunk_off.shape[0], int(n_kv_heads), int(head_dim)
            dtype, adtype = B.Q8Q4, torch.float16
        self.K, self.V, self.chunk_off, self.n_chunks = K, V, chunk_off, n_chunks
        self.max_chunks, self.token_budget = int(max_chunks), int(token_budget)
        c_max = chunk_off.shape[1] - 1
        self.shape = B.make_shape(batch, n_q_heads, hkv, d, int(n_ctx), c_max, k_max, dtype)
        dev = K.device
        self.abstract = torch.empty(batch, hkv, c_max, 2, d, dtype=adtype, device=dev)
        self.score = torch.empty(batch, hkv, c_max, dtype=torch.float32, device=dev)
        self.sel_idx = torch.empty(batch, hkv, k_max, dtype=torch.int32, device=dev)
        self.sel_count = torch.empty(batch, hkv, dtype=torch.int32, device=dev)
        self.sel_tokens = torch.empty(batch, hkv, dtype=torch.int32, device=dev)
        self.out = torch.empty(batch, n_q_heads, d, dtype=torch.float32, device=dev)
        self.lse = torch.empty(batch, n_q_heads, dtype=torch.float32, device=dev)
        pad16 = lambda n: (max(16, n) + 15) // 16 * 16
        # workspace of the one-launch select + attention: starts with arrival counters, zeroed once
        self.workspace = torch.empty(pad16(B.leoam_fused_workspace_bytes(self.shape, token_budget)), dtype=torch.uint8,
                                     device=dev)
        B.leoam_workspace_init(self.workspace)
        # workspace of the separate attention call (contents irrelevant)
        self.att_workspace = torch.empty(pad16(B.leoam_workspace_bytes(self.shape, token_budget)), dtype=torch.uint8,
                                         device=dev)
        self.scale = B.default_scale(d)

    def build_abstract(self, stream=None) -> None:
        B.kv_chunk_abstract_build(self.shape, self.K, self.chunk_off, self.n_chunks, self.abstract, stream, self.qmeta)

    def step(self, q: torch.Tensor, stream=None) -> torch.Tensor:
        """score, then selection + attention in one call."""
        s = self.shape
        B.chunk_score(s, q, self.abstract, self.n_chunks, self.score, None, stream)
        B.chunk_select_attention_decode(s, self.score, q, self.K, self.V, self.chunk_off, self.n_chunks, self.max_chunks,
                                        self.token_budget, self.scale, self.sel_idx, self.sel_count, self.sel_tokens,
                                        self.out, self.lse, self.workspace, stream, self.qmeta)
        return self.out

    def step_separate(self, q: torch.Tensor, stream=None) -> torch.Tensor:
        """The same step through the three separate entry points."""
        s = self.shape
        B.chunk_score(s, q, self.abstract, self.n_chunks, self.score, None, stream)
        B.chunk_topk_select(s, self.score, self.chunk_off, self.n_chunks, self.max_chunks, self.token_budget,
                            self.sel_idx, self.sel_count, self.sel_tokens, None, stream)
        B.sparse_chunk_attention_decode(s, q, self.K, self.V, self.chunk_off, self.n_chunks, self.sel_idx,
                                        self.sel_count, self.scale, self.out, self.lse, self.att_workspace, stream, self.qmeta)
        return self.out
