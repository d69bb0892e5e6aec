"""GPU parity at the full sizes of the benchmarked configurations, in the launch configuration
bench.py times: every layer of c1 and c2 (all sequences, all heads), and every layer that bench.py
keeps resident of c3 (a stated sample of sequences) and of the compressed-store workload c4 (the whole
layer: it has one sequence).  Same bars as test_gpu_parity.py: abstracts, scores and kept lists bit-exact
against the float64 oracle, attention outputs within 2e-3 max-abs (fp16 / bf16 / compressed store)."""
import numpy as np
import pytest
import torch

import gen
from test_gpu_parity import check_path

pytestmark = pytest.mark.gpu

RESIDENT = [0, 1, 2, 7, 15, 23, 30, 31]          # the layers bench.py keeps resident for c3 and c4


@pytest.fixture(scope="module")
def L():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2506_20187_amd as lib
    return lib


def test_resident_layers_match_the_benchmark():
    import bench
    assert bench.RESIDENT["c3"] == RESIDENT and bench.RESIDENT["c4"] == RESIDENT
    assert bench.RESIDENT["c1"] == list(range(32)) and bench.RESIDENT["c2"] == list(range(32))


@pytest.mark.parametrize("layer", range(32))
@pytest.mark.parametrize("cfg", ["c1", "c2"])
def test_path_every_layer_full_size(L, oracle, cfg, layer):
    """All 32 layers of the Llama-2-7B-shaped (32K, fp16, MHA) and Llama-3-8B-shaped (128K, bf16, GQA)
    configurations at full size, every head, through chunk_score -> chunk_select_attention_decode."""
    case = gen.make_case(cfg, layer=layer, device="cuda")
    check_path(L, oracle, case)
    del case
    torch.cuda.empty_cache()


@pytest.mark.parametrize("layer", RESIDENT)
def test_path_c3_every_resident_layer_sampled(L, oracle, layer):
    """Batch 16 x 128K: the GPU runs the whole layer as bench.py does; the oracle checks three of the sixteen
    sequences end to end (which three moves with the layer, so that the eight layers cover all sequences but one)."""
    case = gen.make_case("c3", layer=layer, device="cuda")
    first = (2 * RESIDENT.index(layer)) % 14
    check_path(L, oracle, case, seqs=slice(first, first + 3))
    del case
    torch.cuda.empty_cache()


@pytest.mark.parametrize("layer", RESIDENT)
def test_path_c4_every_resident_layer(L, oracle, layer):
    """512K context, 8-bit / 4-bit store written by kv_chunk_compress exactly as bench.py writes it (the half of
    the chunks without a heavy token as 4-bit); the oracle works on the stored codes: abstract, scores and kept
    lists bit-exact, attention within 2e-3."""
    B = L.binding
    case = gen.make_case("c4", layer=layer, device="cuda")
    q = case.q.to(torch.float16)
    fb = gen.tag_four_bit(case.chunk_off.cpu().numpy(), case.n_chunks.cpu().numpy(), case.extra["heavy"], 0.5)
    nb, hk, n_ctx = case.K.shape[0], case.K.shape[1], case.K.shape[2]
    c_max = case.chunk_off.shape[1] - 1
    shape = B.make_shape(nb, case.hq, hk, 128, n_ctx, c_max, 1, case.K.dtype)
    cap = B.leoam_compressed_bytes_bound(shape)
    kb = torch.empty(cap, dtype=torch.uint8, device="cuda")
    vb = torch.empty(cap, dtype=torch.uint8, device="cuda")
    qm = torch.empty(nb, hk, c_max, 8, dtype=torch.int32, device="cuda")
    used = torch.zeros(1, dtype=torch.int64, device="cuda")
    fbd = torch.from_numpy(np.ascontiguousarray(fb).astype(np.uint8)).cuda()
    B.kv_chunk_compress(shape, case.K, case.V, case.chunk_off, case.n_chunks, fbd, kb, vb, qm, used)
    torch.cuda.synchronize()
    n = int(used.item())
    kb, vb = kb[:n].clone(), vb[:n].clone()
    case.K = case.V = None
    lay = L.DecodeLayer(kb, vb, case.chunk_off, case.n_chunks, case.hq, case.k_max, case.max_chunks, case.token_budget,
                        qmeta=qm, n_kv_heads=case.hkv, n_ctx=case.n_ctx)
    lay.build_abstract()
    lay.step(q)
    torch.cuda.synchronize()
    off, nc = case.chunk_off.cpu(), case.n_chunks.cpu()
    kbh, vbh, qmh = kb.cpu(), vb.cpu(), qm.cpu()
    ab = oracle.abstract_build_q(kbh, qmh, off, nc)
    got_ab = lay.abstract.cpu().to(torch.float64).numpy()
    for b in range(nb):
        assert np.array_equal(got_ab[b, :, : nc[b]], ab[b, :, : nc[b]]), "abstract"
    ub = oracle.chunk_score(q.cpu(), np.nan_to_num(ab), nc)
    assert np.array_equal(lay.score.cpu().numpy(), ub), "score"
    sel, cnt, tok = oracle.topk_select(ub, off, nc, case.max_chunks, case.token_budget, case.k_max)
    assert np.array_equal(lay.sel_idx.cpu().numpy(), sel), "sel_idx"
    assert np.array_equal(lay.sel_count.cpu().numpy(), cnt) and np.array_equal(lay.sel_tokens.cpu().numpy(), tok)
    out, lse = oracle.sparse_attention_q(q.cpu(), kbh, vbh, qmh, off, sel, cnt)
    err = np.abs(lay.out.cpu().numpy().astype(np.float64) - out).max()
    assert err <= 2e-3, f"attention max-abs error {err}"
    assert np.abs(lay.lse.cpu().numpy().astype(np.float64) - lse).max() <= 1e-3
    del lay, kb, vb, qm, case
    torch.cuda.empty_cache()
