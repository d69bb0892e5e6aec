"""Layer-ahead evaluation (Sec. 4.4 of the paper: the next layer's importance evaluation runs while the current
layer computes).  DecodeStack's schedules -- chunk_score of layer l+1 on a second stream, one chunk_score over all
layers, one chunk_score and one chunk_topk_select over all layers -- must return bit for bit what the sequential
order returns, and with evaluation queries that differ from the attention queries they must equal the oracle's
score(q_eval) -> select -> attention(q)."""
import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu
N_LAYERS = 4


@pytest.fixture(scope="module")
def L():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2506_20187_amd as lib
    return lib


def make_stack(L, cfg, **kw):
    cases = [gen.make_case(cfg, layer=l, device="cuda", **kw) for l in (0, 9, 20, 31)[:N_LAYERS]]
    c = cases[0]
    k_max = max(x.k_max for x in cases)            # (the generator sizes the kept list per layer)
    stack = L.DecodeStack([x.K for x in cases], [x.V for x in cases], [x.chunk_off for x in cases],
                          [x.n_chunks for x in cases], c.hq, k_max, c.max_chunks, c.token_budget)
    stack.build_abstract()
    q = torch.stack([x.q for x in cases]).contiguous()
    return cases, stack, q


def snapshot(stack):
    return [t.clone() for t in (stack.score, stack.sel_idx, stack.sel_count, stack.sel_tokens, stack.out, stack.lse)]


def poison(stack):
    stack.score.fill_(float("nan"))
    stack.out.fill_(float("nan"))
    stack.lse.fill_(float("nan"))
    for t in (stack.sel_idx, stack.sel_count, stack.sel_tokens):
        t.fill_(-7)


@pytest.mark.parametrize("cfg,kw", [("c2", dict(n_ctx=16384 + 5, hq=8, hkv=2, token_budget=2048)),
                                    ("c3", dict(batch=3, n_ctx=8192 + 100, hq=8, hkv=2, token_budget=1024)),
                                    ("c1", dict(n_ctx=8192 + 37, hq=8, hkv=8, token_budget=1024))],
                         ids=["c2_reduced", "c3_reduced", "c1_reduced"])
def test_schedules_equal_the_sequential_order(L, oracle, cfg, kw):
    cases, stack, q = make_stack(L, cfg, **kw)
    # the stack's layers against stand-alone layers (own buffers, own capacity): same bits
    for l, case in enumerate(cases):
        lay = L.DecodeLayer(case.K, case.V, case.chunk_off, case.n_chunks, case.hq, case.k_max, case.max_chunks,
                            case.token_budget)
        lay.build_abstract()
        lay.step(case.q)
        poison(stack)
        stack.step_sequential(q)
        torch.cuda.synchronize()
        sl = slice(l * case.batch, (l + 1) * case.batch)
        n, k = lay.shape.c_max, lay.shape.k_max
        assert torch.equal(stack.score[sl][:, :, :n], lay.score)
        assert torch.equal(stack.sel_idx[sl][:, :, :k], lay.sel_idx) and torch.all(stack.sel_idx[sl][:, :, k:] == -1)
        assert torch.equal(stack.sel_count[sl], lay.sel_count) and torch.equal(stack.sel_tokens[sl], lay.sel_tokens)
        assert torch.equal(stack.out[sl], lay.out) and torch.equal(stack.lse[sl], lay.lse)
    poison(stack)
    stack.step_sequential(q)
    torch.cuda.synchronize()
    want = snapshot(stack)
    for name in ("step_layer_ahead", "step_scores_ahead"):
        for rep in range(3):                      # repeated: the second stream must also wait for the previous step
            poison(stack)
            getattr(stack, name)(q)
            torch.cuda.synchronize()
            for what, a, b in zip(("score", "sel_idx", "sel_count", "sel_tokens", "out", "lse"), snapshot(stack), want):
                assert torch.equal(a, b), f"{name}: {what} differs (repetition {rep})"
    # the schedule that also selects ahead attends with the kept lists given: the same tables, the same splits,
    # the same bits as the one-call step; the separate calls give the same scores and kept lists
    poison(stack)
    stack.step_select_ahead(q)
    torch.cuda.synchronize()
    for what, a, b in zip(("score", "sel_idx", "sel_count", "sel_tokens", "out", "lse"), snapshot(stack), want):
        assert torch.equal(a, b), f"step_select_ahead: {what} differs"
    poison(stack)
    for lay, case in zip(stack.layers, cases):
        lay.step_separate(case.q)
    torch.cuda.synchronize()
    for what, a, b in zip(("score", "sel_idx", "sel_count", "sel_tokens"), snapshot(stack), want):
        assert torch.equal(a, b), what


def test_evaluation_with_an_earlier_query(L, oracle):
    """The evaluation runs on queries supplied up front (here: the attention queries plus noise, standing for the
    previous step's); the kept lists then follow q_eval and the attention uses q: every schedule against the oracle."""
    cases, stack, q = make_stack(L, "c2", n_ctx=16384 + 5, hq=8, hkv=2, token_budget=2048)
    g = torch.Generator(device="cuda").manual_seed(5)
    q_eval = (q.float() + 0.5 * torch.randn(q.shape, generator=g, device="cuda")).to(q.dtype)
    want = []
    for l, case in enumerate(cases):
        K, V = case.K.cpu(), case.V.cpu()
        off, nc = case.chunk_off.cpu(), case.n_chunks.cpu()
        ab = oracle.abstract_build(K, off, nc)
        ub = oracle.chunk_score(q_eval[l].cpu(), np.nan_to_num(ab), nc)
        sel, cnt, tok = oracle.topk_select(ub, off, nc, case.max_chunks, case.token_budget, case.k_max)
        out, _ = oracle.sparse_attention(q[l].cpu(), K, V, off, sel, cnt)
        want.append((sel, out))
    differs = False
    for name in ("step_sequential", "step_layer_ahead", "step_scores_ahead", "step_select_ahead"):
        poison(stack)
        getattr(stack, name)(q, q_eval)
        torch.cuda.synchronize()
        for l, (sel, out) in enumerate(want):
            sl = slice(l * stack.batch, (l + 1) * stack.batch)
            got = stack.sel_idx[sl].cpu().numpy()
            assert np.array_equal(got[:, :, : sel.shape[2]], sel) and np.all(got[:, :, sel.shape[2]:] == -1), \
                f"{name}: kept list of layer {l}"
            err = np.abs(stack.out[sl].cpu().numpy().astype(np.float64) - out).max()
            assert err <= 2e-3, f"{name}: attention max-abs error {err}"
    stack.step_sequential(q)
    torch.cuda.synchronize()
    for l, (sel, _) in enumerate(want):
        sl = slice(l * stack.batch, (l + 1) * stack.batch)
        differs |= not np.array_equal(stack.sel_idx[sl].cpu().numpy()[:, :, : sel.shape[2]], sel)
    assert differs, "the evaluation queries were meant to change some kept list"


def test_schedules_on_the_compressed_store(L, oracle):
    """The 8-bit / 4-bit store: every schedule returns what the sequential order returns bit for bit (kept lists,
    scores) and the oracle's attention on the stored codes within 2e-3."""
    qcs = [gen.make_quant_case("c4", layer=l, n_ctx=16384 + 64, hq=8, hkv=2, token_budget=2048) for l in (0, 17, 31)]
    cases = [qc.case for qc in qcs]
    c = cases[0]
    dev = lambda t: t.cuda().contiguous()
    k_max = max(x.k_max for x in cases)
    stack = L.DecodeStack([dev(qc.kblob) for qc in qcs], [dev(qc.vblob) for qc in qcs], [dev(x.chunk_off) for x in cases],
                          [dev(x.n_chunks) for x in cases], c.hq, k_max, c.max_chunks, c.token_budget,
                          qmetas=[dev(qc.qmeta) for qc in qcs], n_kv_heads=c.hkv, n_ctx=c.n_ctx)
    stack.build_abstract()
    q = torch.stack([dev(x.q) for x in cases]).contiguous()
    poison(stack)
    stack.step_sequential(q)
    torch.cuda.synchronize()
    want = snapshot(stack)
    for l, qc in enumerate(qcs):
        x = qc.case
        off, nc = x.chunk_off.cpu(), x.n_chunks.cpu()
        ab = oracle.abstract_build_q(qc.kblob, qc.qmeta, off, nc)
        ub = oracle.chunk_score(x.q.cpu(), np.nan_to_num(ab), nc)
        sel, cnt, tok = oracle.topk_select(ub, off, nc, x.max_chunks, x.token_budget, x.k_max)
        out, _ = oracle.sparse_attention_q(x.q.cpu(), qc.kblob, qc.vblob, qc.qmeta, off, sel, cnt)
        sl = slice(l * stack.batch, (l + 1) * stack.batch)
        got = stack.sel_idx[sl].cpu().numpy()
        assert np.array_equal(got[:, :, : sel.shape[2]], sel) and np.all(got[:, :, sel.shape[2]:] == -1), f"kept list of layer {l}"
        assert np.abs(stack.out[sl].cpu().numpy().astype(np.float64) - out).max() <= 2e-3
    for name in ("step_layer_ahead", "step_scores_ahead"):
        poison(stack)
        getattr(stack, name)(q)
        torch.cuda.synchronize()
        for what, a, b in zip(("score", "sel_idx", "sel_count", "sel_tokens", "out", "lse"), snapshot(stack), want):
            assert torch.equal(a, b), f"{name}: {what} differs"
    poison(stack)
    stack.step_select_ahead(q)
    torch.cuda.synchronize()
    for what, a, b in zip(("score", "sel_idx", "sel_count", "sel_tokens", "out", "lse"), snapshot(stack), want):
        assert torch.equal(a, b), f"step_select_ahead: {what} differs"
