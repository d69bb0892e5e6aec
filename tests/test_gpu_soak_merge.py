"""Soak of the in-launch merge of attention splits.

Workgroups that share a (sequence, kv head) publish their partial (m, l, acc[128]) with agent-scope relaxed
atomic stores, wait for the stores to be acknowledged, and take a ticket; the workgroup that draws the last
ticket reads every partial back with agent-scope atomic loads and combines them in split order.  That
exchange has no release / acquire fence (on this multi-XCD part a fence is an L2 write-back and invalidate), so
it rests on the hardware's ordering of acknowledged write-through stores, not on the HIP memory model.  A stale
partial would be a silently wrong output, so every configuration is launched many times with the partial area
re-poisoned with a changing pattern before every launch, and every result is compared bit for bit with the
first one (which is checked against the oracle).  The loop stops at the first mismatch.
(Two splits per (sequence, kv head) at batch sizes that reserve exchange words are combined differently - one
atomic exchange per output element carries the value itself - and are soaked the same way.)"""
import os

import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu
LAUNCHES = int(os.environ.get("LEOAM_SOAK_LAUNCHES", "2000"))      # per configuration; a longer soak: set the variable


@pytest.fixture(scope="module")
def L():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2506_20187_amd as lib
    return lib


def soak(L, lay, q, n_splits, launches, want_out):
    s = lay.shape
    head = L.leoam_fused_control_bytes(s)           # arrival counters (+ exchange words): zero between calls
    nbytes = head + n_splits * s.batch * s.n_q_heads * 130 * 4
    ws = torch.zeros((nbytes + 15) // 16 * 16, dtype=torch.uint8, device="cuda")

    def launch():
        L.chunk_select_attention_decode(s, lay.score, q, lay.K, lay.V, lay.chunk_off, lay.n_chunks, lay.max_chunks,
                                        lay.token_budget, lay.scale, lay.sel_idx, lay.sel_count, lay.sel_tokens, lay.out,
                                        lay.lse, ws, None, lay.qmeta)
    ws[head:] = 0xFF
    launch()
    torch.cuda.synchronize()
    first_out, first_lse = lay.out.clone(), lay.lse.clone()
    err = np.abs(first_out.cpu().numpy().astype(np.float64) - want_out).max()
    assert err <= 2e-3, f"first launch: max-abs error {err} ({n_splits} splits)"
    for i in range(launches):
        ws[head:] = (i * 37 + 11) % 255 + 1            # a new non-zero byte pattern in every partial
        lay.out.fill_(float("nan"))
        launch()
        ok = torch.equal(lay.out, first_out) and torch.equal(lay.lse, first_lse)     # (synchronises)
        assert ok, f"launch {i} with {n_splits} splits differs from the first launch"
        assert not ws[:head].any(), f"launch {i}: control words not back at zero"


def dense_layer(L, oracle, hq, hkv, dtype_cfg="c2"):
    case = gen.make_case(dtype_cfg, layer=13, n_ctx=65536, hq=hq, hkv=hkv, token_budget=16384, device="cuda")
    lay = L.DecodeLayer(case.K, case.V, case.chunk_off, case.n_chunks, case.hq, case.k_max, case.max_chunks,
                        case.token_budget)
    lay.build_abstract()
    lay.step(case.q)
    torch.cuda.synchronize()
    sel, cnt = lay.sel_idx.cpu().numpy(), lay.sel_count.cpu().numpy()
    want, _ = oracle.sparse_attention(case.q.cpu(), case.K.cpu(), case.V.cpu(), case.chunk_off.cpu(), sel, cnt)
    return case, lay, want


@pytest.mark.parametrize("n_splits", [2, 3, 16, 64])
def test_one_launch_kernel_16bit(L, oracle, n_splits):
    case, lay, want = dense_layer(L, oracle, 16, 4)           # 4 (sequence, kv head) pairs: up to 64 splits each
    soak(L, lay, case.q, n_splits, LAUNCHES, want)


@pytest.mark.parametrize("n_splits", [2, 16])
def test_separate_kernels_merging_in_the_launch(L, oracle, n_splits):
    # group size 8 takes chunk_topk_select + the split attention kernel, whose splits (up to 16) are merged
    # in the launch by the same exchange
    case, lay, want = dense_layer(L, oracle, 32, 4)
    soak(L, lay, case.q, n_splits, LAUNCHES // 2, want)


@pytest.mark.parametrize("n_splits", [2, 3, 16, 64])
def test_one_launch_kernel_compressed_store(L, oracle, n_splits):
    qc = gen.make_quant_case("c4", layer=9, n_ctx=131072, hq=16, hkv=4, token_budget=16384, device="cuda")
    c = qc.case
    lay = L.DecodeLayer(qc.kblob, qc.vblob, c.chunk_off, c.n_chunks, c.hq, c.k_max, c.max_chunks, c.token_budget,
                        qmeta=qc.qmeta, n_kv_heads=c.hkv, n_ctx=c.n_ctx)
    lay.build_abstract()
    lay.step(c.q)
    torch.cuda.synchronize()
    want, _ = oracle.sparse_attention_q(c.q.cpu(), qc.kblob.cpu(), qc.vblob.cpu(), qc.qmeta.cpu(), c.chunk_off.cpu(),
                                        lay.sel_idx.cpu().numpy(), lay.sel_count.cpu().numpy())
    soak(L, lay, c.q, n_splits, LAUNCHES, want)


def test_two_splits_combined_through_exchange_words(L, oracle):
    """Batch sizes between half a workgroup and one workgroup per compute unit (here 16 sequences x 8 kv heads)
    give two splits per (sequence, kv head), which are combined by one atomic exchange per output element
    instead of the ticket: the same soak (the partial area behind the control words is unused, and poisoned)."""
    case = gen.make_case("c3", layer=13, batch=16, n_ctx=4096 + 37, hq=32, hkv=8, token_budget=1024, device="cuda")
    lay = L.DecodeLayer(case.K, case.V, case.chunk_off, case.n_chunks, case.hq, case.k_max, case.max_chunks,
                        case.token_budget)
    lay.build_abstract()
    lay.step(case.q)
    torch.cuda.synchronize()
    assert L.leoam_fused_control_bytes(lay.shape) > 16 * 8 * 4 + 256, "this shape was meant to have exchange words"
    sel, cnt = lay.sel_idx.cpu().numpy(), lay.sel_count.cpu().numpy()
    want, _ = oracle.sparse_attention(case.q.cpu(), case.K.cpu(), case.V.cpu(), case.chunk_off.cpu(), sel, cnt)
    soak(L, lay, case.q, 2, LAUNCHES, want)
