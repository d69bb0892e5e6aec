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
                 n_kv_heads: int = None, n_ctx: int = None, head_dim: int = 128, buffers: dict = None):
        """Dense store: K, V [B,Hkv,N,D].  Compressed store: K, V are the byte blobs, qmeta the
        [B,Hkv,c_max,8] int32 chunk records, and n_kv_heads / n_ctx must be given.  `buffers` may bring
        abstract / score / sel_idx / sel_count / sel_tokens / out / lse tensors of the right shapes (a
        DecodeStack passes slices of its stacked tensors); what it does not bring is allocated here."""
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
        bufs = buffers or {}

        def buf(name, shape, dtype):
            t = bufs.get(name)
            if t is None:
                return torch.empty(*shape, dtype=dtype, device=dev)
            assert tuple(t.shape) == tuple(shape) and t.dtype == dtype and t.is_contiguous(), name
            return t
        self.abstract = buf("abstract", (batch, hkv, c_max, 2, d), adtype)
        self.score = buf("score", (batch, hkv, c_max), torch.float32)
        self.sel_idx = buf("sel_idx", (batch, hkv, k_max), torch.int32)
        self.sel_count = buf("sel_count", (batch, hkv), torch.int32)
        self.sel_tokens = buf("sel_tokens", (batch, hkv), torch.int32)
        self.out = buf("out", (batch, n_q_heads, d), torch.float32)
        self.lse = buf("lse", (batch, n_q_heads), torch.float32)
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

    def attend_given(self, q: torch.Tensor, stream=None) -> torch.Tensor:
        """Attention over kept lists that are already in sel_idx / sel_count (one kernel, in-launch merge)."""
        B.chunk_select_attention_decode(self.shape, None, q, self.K, self.V, self.chunk_off, self.n_chunks, self.max_chunks,
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


class DecodeStack:
    """The layers of one model as slices of stacked tensors, and the schedules of a decode step over them.

    Sec. 4.4 of the paper evaluates (and fetches) the next layer's KV while the current layer computes.
    With every tier in one GPU's HBM the fetch is gone and what is left to move ahead is the evaluation
    itself; it needs the next layer's query before that layer runs, i.e. a query supplied up front (the
    previous step's, or a speculated one).  Because the per-chunk arrays of all layers are rows of one
    [layers * batch, ...] tensor with a common `c_max`, "ahead" can be taken to its end: ONE chunk_score
    call (and, if wanted, one chunk_topk_select call) evaluates every layer of the step, which is also what
    fills the chip when the batch is small.  Only buffer ownership and call order live here; every step of
    the path runs in libleoam.so.

      step_sequential      per layer: chunk_score, chunk_select_attention_decode            (the reference order)
      step_layer_ahead     the same calls, chunk_score of layer l+1 on a second stream
                           (same priority) while layer l selects and attends
      step_scores_ahead    one chunk_score over all layers, then per layer chunk_select_attention_decode
      step_select_ahead    one chunk_score and one chunk_topk_select over all layers, then per layer
                           chunk_select_attention_decode with the kept lists given (it only attends, in
                           one kernel)
    `q_eval` [layers, B, Hq, D] are the queries the evaluation uses, `q` the ones attention uses; with
    q_eval == q every schedule returns exactly what step_sequential returns.
    """

    def __init__(self, Ks, Vs, chunk_offs, n_chunks, n_q_heads: int, k_max: int, max_chunks: int, token_budget: int,
                 qmetas=None, n_kv_heads: int = None, n_ctx: int = None, head_dim: int = 128):
        """Dense stores: Ks, Vs are per-layer [B,Hkv,N,D] tensors.  Compressed stores: Ks, Vs are the per-layer byte
        blobs, `qmetas` the per-layer [B,Hkv,c_max_l,8] int32 chunk records, and n_kv_heads / n_ctx must be given
        (the records are copied into rows of the common capacity; queries and abstracts are fp16)."""
        self.n_layers = len(Ks)
        quant = qmetas is not None
        if quant:
            batch, hkv, d = int(chunk_offs[0].shape[0]), int(n_kv_heads), int(head_dim)
            dev, dtype, adtype = Ks[0].device, B.Q8Q4, torch.float16
        else:
            batch, hkv, n_ctx, d = Ks[0].shape
            dev, dtype, adtype = Ks[0].device, Ks[0].dtype, Ks[0].dtype
        self.batch = batch
        c_max = max(int(co.shape[1]) - 1 for co in chunk_offs)
        rows = self.n_layers * batch
        # boundary rows padded to the common capacity (entries past n_chunks are ignored by the library)
        self.chunk_off = torch.full((rows, c_max + 1), int(n_ctx), dtype=torch.int32, device=dev)
        for l, co in enumerate(chunk_offs):
            self.chunk_off[l * batch:(l + 1) * batch, : co.shape[1]] = co
        self.n_chunks = torch.cat([nc.reshape(batch) for nc in n_chunks]).to(torch.int32).contiguous()
        self.abstract = torch.empty(rows, hkv, c_max, 2, d, dtype=adtype, device=dev)
        self.score = torch.empty(rows, hkv, c_max, dtype=torch.float32, device=dev)
        self.sel_idx = torch.empty(rows, hkv, k_max, dtype=torch.int32, device=dev)
        self.sel_count = torch.empty(rows, hkv, dtype=torch.int32, device=dev)
        self.sel_tokens = torch.empty(rows, hkv, dtype=torch.int32, device=dev)
        self.out = torch.empty(rows, n_q_heads, d, dtype=torch.float32, device=dev)
        self.lse = torch.empty(rows, n_q_heads, dtype=torch.float32, device=dev)
        self.shape_all = B.make_shape(rows, n_q_heads, hkv, d, int(n_ctx), c_max, k_max, dtype)
        self.max_chunks, self.token_budget = int(max_chunks), int(token_budget)
        self.qmeta = None
        if quant:
            self.qmeta = torch.zeros(rows, hkv, c_max, 8, dtype=torch.int32, device=dev)
            for l, qm in enumerate(qmetas):
                self.qmeta[l * batch:(l + 1) * batch, :, : qm.shape[2]] = qm
        self.layers = []
        for l in range(self.n_layers):
            sl = slice(l * batch, (l + 1) * batch)
            bufs = {n: getattr(self, n)[sl] for n in ("abstract", "score", "sel_idx", "sel_count", "sel_tokens", "out", "lse")}
            if quant:
                self.layers.append(DecodeLayer(Ks[l], Vs[l], self.chunk_off[sl], self.n_chunks[sl], n_q_heads, k_max,
                                               max_chunks, token_budget, qmeta=self.qmeta[sl], n_kv_heads=hkv,
                                               n_ctx=int(n_ctx), head_dim=d, buffers=bufs))
            else:
                self.layers.append(DecodeLayer(Ks[l], Vs[l], self.chunk_off[sl], self.n_chunks[sl], n_q_heads, k_max,
                                               max_chunks, token_budget, buffers=bufs))
        self.side = torch.cuda.Stream(device=dev)          # default priority, as the main stream
        self.scored = [torch.cuda.Event() for _ in range(self.n_layers)]

    def build_abstract(self) -> None:
        for lay in self.layers:
            lay.build_abstract()

    def _q_rows(self, q: torch.Tensor) -> torch.Tensor:
        return q.reshape(self.n_layers * self.batch, q.shape[-2], q.shape[-1])

    def score_all(self, q_eval: torch.Tensor, stream=None) -> None:
        B.chunk_score(self.shape_all, self._q_rows(q_eval), self.abstract, self.n_chunks, self.score, None, stream)

    def select_all(self, stream=None) -> None:
        B.chunk_topk_select(self.shape_all, self.score, self.chunk_off, self.n_chunks, self.max_chunks, self.token_budget,
                            self.sel_idx, self.sel_count, self.sel_tokens, None, stream)

    def step_sequential(self, q: torch.Tensor, q_eval: torch.Tensor = None) -> torch.Tensor:
        q_eval = q if q_eval is None else q_eval
        for l, lay in enumerate(self.layers):
            s = lay.shape
            B.chunk_score(s, q_eval[l], lay.abstract, lay.n_chunks, lay.score, None)
            B.chunk_select_attention_decode(s, lay.score, q[l], lay.K, lay.V, lay.chunk_off, lay.n_chunks, lay.max_chunks,
                                            lay.token_budget, lay.scale, lay.sel_idx, lay.sel_count, lay.sel_tokens,
                                            lay.out, lay.lse, lay.workspace, None, lay.qmeta)
        return self.out

    def step_layer_ahead(self, q: torch.Tensor, q_eval: torch.Tensor = None) -> torch.Tensor:
        q_eval = q if q_eval is None else q_eval
        main = torch.cuda.current_stream()
        self.side.wait_stream(main)                    # the previous step's selections have read the score rows
        for l, lay in enumerate(self.layers):
            # evaluation of layer l on the side stream; it runs while layer l-1 selects and attends
            B.chunk_score(lay.shape, q_eval[l], lay.abstract, lay.n_chunks, lay.score, None, self.side)
            self.scored[l].record(self.side)
            main.wait_event(self.scored[l])
            B.chunk_select_attention_decode(lay.shape, lay.score, q[l], lay.K, lay.V, lay.chunk_off, lay.n_chunks,
                                            lay.max_chunks, lay.token_budget, lay.scale, lay.sel_idx, lay.sel_count,
                                            lay.sel_tokens, lay.out, lay.lse, lay.workspace, main, lay.qmeta)
        return self.out

    def step_scores_ahead(self, q: torch.Tensor, q_eval: torch.Tensor = None) -> torch.Tensor:
        self.score_all(q if q_eval is None else q_eval)
        for l, lay in enumerate(self.layers):
            B.chunk_select_attention_decode(lay.shape, lay.score, q[l], lay.K, lay.V, lay.chunk_off, lay.n_chunks,
                                            lay.max_chunks, lay.token_budget, lay.scale, lay.sel_idx, lay.sel_count,
                                            lay.sel_tokens, lay.out, lay.lse, lay.workspace, None, lay.qmeta)
        return self.out

    def step_select_ahead(self, q: torch.Tensor, q_eval: torch.Tensor = None) -> torch.Tensor:
        self.score_all(q if q_eval is None else q_eval)
        self.select_all()
        for l, lay in enumerate(self.layers):
            B.chunk_select_attention_decode(lay.shape, None, q[l], lay.K, lay.V, lay.chunk_off, lay.n_chunks,
                                            lay.max_chunks, lay.token_budget, lay.scale, lay.sel_idx, lay.sel_count,
                                            lay.sel_tokens, lay.out, lay.lse, lay.workspace, None, lay.qmeta)
        return self.out

