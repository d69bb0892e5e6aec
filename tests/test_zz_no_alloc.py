"""chunk_select_attention_decode_static (the entry point for callers that cannot allocate: its arrival
counters and split partials live in a buffer inside the library image) against chunk_select_attention_decode
on the same inputs: kept lists bit-exact, outputs bit-exact when both run the same number of splits
(the merge order is fixed), and both against the oracle.  Calls in a row with different shapes share the
buffer: a large batch first, then smaller inputs whose counters lie where the first call's partials were."""
import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}


@pytest.fixture(scope="module")
def L():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2506_20187_amd as lib
    return lib


def both_ways(L, oracle, case):
    K, V, q = case.K.cuda(), case.V.cuda(), case.q.cuda()
    lay = L.DecodeLayer(K, V, case.chunk_off.cuda(), case.n_chunks.cuda(), case.hq, case.k_max, case.max_chunks,
                        case.token_budget)
    lay.build_abstract()
    lay.step(q)                                   # chunk_score + chunk_select_attention_decode (caller's workspace)
    torch.cuda.synchronize()
    want = [t.clone() for t in (lay.sel_idx, lay.sel_count, lay.sel_tokens, lay.out, lay.lse)]
    for t in (lay.sel_idx, lay.sel_count, lay.sel_tokens):
        t.fill_(-7)
    lay.out.fill_(float("nan"))
    lay.lse.fill_(float("nan"))
    L.chunk_select_attention_decode_static(lay.shape, lay.score, q, lay.K, lay.V, lay.chunk_off, lay.n_chunks,
                                           lay.max_chunks, lay.token_budget, lay.scale, lay.sel_idx, lay.sel_count,
                                           lay.sel_tokens, lay.out, lay.lse)
    torch.cuda.synchronize()
    got = (lay.sel_idx, lay.sel_count, lay.sel_tokens, lay.out, lay.lse)
    for name, a, b in zip(("sel_idx", "sel_count", "sel_tokens"), got, want):
        assert torch.equal(a, b), name
    same_splits = L.leoam_fused_workspace_bytes(lay.shape, lay.token_budget) <= L.binding.STATIC_SCRATCH_BYTES
    if same_splits:
        assert torch.equal(got[3], want[3]) and torch.equal(got[4], want[4]), "same splits, same merge order: same bits"
    ref = oracle.decode_step(case.q, case.K, case.V, case.chunk_off, case.n_chunks, case.max_chunks, case.token_budget,
                             case.k_max)
    assert np.array_equal(lay.sel_idx.cpu().numpy(), ref["sel_idx"])
    err = np.abs(lay.out.cpu().numpy().astype(np.float64) - ref["out"]).max()
    assert err <= TOL[case.dtype], f"attention max-abs error {err}"
    return same_splits


def test_static_workspace_calls_in_a_row(L, oracle):
    # 48 (sequence, kv head) pairs, two splits each; then one sequence with two kv heads (many splits; its
    # counters and first partials lie where the first call left partials); then the fp32 shape that takes the
    # two-launch path; then the first shape again
    big = gen.make_case("c3", layer=9, batch=6, n_ctx=8192 + 100, hq=32, hkv=8, token_budget=1024)
    small = gen.make_case("c2", layer=17, n_ctx=4096 + 5, hq=8, hkv=2, token_budget=512)
    tiny = gen.make_case("c0")
    for case in (big, small, tiny, big, small):
        assert both_ways(L, oracle, case)


def test_static_workspace_refuses_what_does_not_fit(L):
    t = torch.zeros(64, device="cuda")
    # fp32 takes the two-launch path: its smallest workspace is one partial per (b, q head) = 520 bytes each
    shape = L.make_shape(2048, 8, 8, 128, 4096, 64, 64, torch.float32)
    assert 2048 * 8 * 520 > L.binding.STATIC_SCRATCH_BYTES
    with pytest.raises(L.LeoamError) as e:
        L.chunk_select_attention_decode_static(shape, t, t, t, t, t, t, 0, 0, 1.0, t, t, t, t, None)
    assert e.value.status == -4
    torch.cuda.synchronize()
