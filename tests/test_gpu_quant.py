"""GPU parity of the compressed-store entry points (8-bit / 4-bit chunks) against
the CPU oracle: abstracts bit-exact (outward-rounded binary16), selections
bit-exact, attention outputs within 2e-3 max-abs."""
import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def L():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2506_20187_amd as lib
    return lib


def run_quant_path(L, qc):
    c = qc.case
    lay = L.DecodeLayer(qc.kblob.cuda(), qc.vblob.cuda(), c.chunk_off.cuda(), c.n_chunks.cuda(), c.hq, c.k_max,
                        c.max_chunks, c.token_budget, qmeta=qc.qmeta.cuda(), n_kv_heads=c.hkv, n_ctx=c.n_ctx)
    lay.build_abstract()
    lay.step(c.q.cuda())
    torch.cuda.synchronize()
    return lay


def check_quant_path(L, oracle, qc):
    c = qc.case
    lay = run_quant_path(L, qc)
    off, nc = c.chunk_off.cpu(), c.n_chunks.cpu()
    kb, vb, qm = qc.kblob.cpu(), qc.vblob.cpu(), qc.qmeta.cpu()
    ab = oracle.abstract_build_q(kb, qm, off, nc)
    got_ab = lay.abstract.cpu().to(torch.float64).numpy()
    for b in range(c.batch):
        assert np.array_equal(got_ab[b, :, : nc[b]], ab[b, :, : nc[b]]), "abstract"
    ub = oracle.chunk_score(c.q.cpu(), np.nan_to_num(ab), nc)
    assert np.array_equal(lay.score.cpu().numpy(), ub), "score"
    sel, cnt, tok = oracle.topk_select(ub, off, nc, c.max_chunks, c.token_budget, c.k_max)
    assert np.array_equal(lay.sel_idx.cpu().numpy(), sel) and np.array_equal(lay.sel_count.cpu().numpy(), cnt)
    assert np.array_equal(lay.sel_tokens.cpu().numpy(), tok)
    out, lse = oracle.sparse_attention_q(c.q.cpu(), kb, vb, qm, off, sel, cnt)
    err = np.abs(lay.out.cpu().numpy().astype(np.float64) - out).max()
    assert err <= TOL, f"attention max-abs error {err}"
    got_lse = lay.lse.cpu().numpy().astype(np.float64)
    assert np.array_equal(np.isneginf(got_lse), np.isneginf(lse)), "lse: -inf exactly where nothing is kept"
    kept = ~np.isneginf(lse)
    assert not kept.any() or np.abs(got_lse[kept] - lse[kept]).max() <= 1e-3, "lse"
    return err


@pytest.mark.parametrize("share", [0.0, 0.5, 1.0])
def test_quant_abstract_and_attention_random_store(L, oracle, share):
    rng = np.random.default_rng(int(share * 10))
    g = torch.Generator().manual_seed(11)
    B, Hkv, G, N = 2, 2, 4, 1500
    K = torch.randn(B, Hkv, N, 128, generator=g) * 2.0
    V = torch.randn(B, Hkv, N, 128, generator=g)
    q = (torch.randn(B, Hkv * G, 128, generator=g) * 1.3).to(torch.float16)
    offs = [gen.make_boundaries(N, rng, sizes=(1, 3, 8, 17, 40)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    fb = rng.random((B, c_max)) < share
    kb, vb, qm = gen.quantize_store(K, V, packed, counts, fb)
    shape = L.make_shape(B, Hkv * G, Hkv, 128, N, c_max, c_max, L.binding.Q8Q4)
    ab = torch.full((B, Hkv, c_max, 2, 128), float("nan"), dtype=torch.float16, device="cuda")
    dpacked, dcounts = torch.from_numpy(packed).cuda(), torch.from_numpy(counts).cuda()
    L.kv_chunk_abstract_build(shape, kb.cuda(), dpacked, dcounts, ab, qmeta=qm.cuda())
    torch.cuda.synchronize()
    want_ab = oracle.abstract_build_q(kb, qm, packed, counts)
    got_ab = ab.cpu().to(torch.float64).numpy()
    for b in range(B):
        assert np.array_equal(got_ab[b, :, : counts[b]], want_ab[b, :, : counts[b]])
        assert np.isnan(got_ab[b, :, counts[b]:]).all()
    sel = np.full((B, Hkv, c_max), -1, dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    for b in range(B):
        for h in range(Hkv):
            n = int(rng.integers(1, counts[b]))
            sel[b, h, :n] = np.sort(rng.choice(counts[b], size=n, replace=False))
            cnt[b, h] = n
    cnt[1, 0] = 0
    want, want_lse = oracle.sparse_attention_q(q, kb, vb, qm, packed, sel, cnt)
    out = torch.full((B, Hkv * G, 128), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, Hkv * G), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(L.leoam_workspace_bytes(shape, 0), dtype=torch.uint8, device="cuda")
    L.sparse_chunk_attention_decode(shape, q.cuda(), kb.cuda(), vb.cuda(), dpacked, dcounts, torch.from_numpy(sel).cuda(),
                                    torch.from_numpy(cnt).cuda(), L.default_scale(128), out, lse, ws, qmeta=qm.cuda())
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.abs(got - want).max() <= TOL
    assert np.all(got[1, 0:G] == 0)
    fin = np.isfinite(want_lse)
    assert np.abs(lse.cpu().numpy().astype(np.float64)[fin] - want_lse[fin]).max() <= 1e-3


@pytest.mark.parametrize("layer,G", [(0, 4), (31, 4), (12, 1), (5, 2), (20, 8)])
def test_quant_path_c4_reduced(L, oracle, layer, G):
    qc = gen.make_quant_case("c4", layer=layer, n_ctx=32768 + 77, hq=2 * G, hkv=2, token_budget=2048)
    check_quant_path(L, oracle, qc)


@pytest.mark.parametrize("seed", list(range(12)))
def test_quant_path_random_shapes(L, oracle, seed):
    """The compressed store on shapes drawn at random (seeded): recipe, batch, heads and group size, ragged context,
    share of 4-bit chunks, token budget and chunk limit; every step against the oracle."""
    rng = np.random.default_rng(3000 + seed)
    config = ("c2", "c3", "c4")[int(rng.integers(3))]
    hkv = int(rng.integers(1, 4))
    g = (1, 2, 4, 8)[int(rng.integers(4))]
    n_ctx = int(rng.integers(600, 9000))
    qc = gen.make_quant_case(config, layer=int(rng.integers(32)), four_bit_share=float(rng.random()), batch=int(rng.integers(1, 4)),
                             n_ctx=n_ctx, hq=hkv * g, hkv=hkv, dtype=("f16", "bf16")[int(rng.integers(2))],
                             token_budget=int(rng.integers(1, n_ctx)), max_chunks=int(rng.integers(0, 40)))
    check_quant_path(L, oracle, qc)


def test_quant_path_c4_full_shape_layer(L, oracle):
    """One layer at the full compressed-KV stress shape (512K context), generated and quantised in HBM."""
    qc = gen.make_quant_case("c4", layer=20, device="cuda")
    check_quant_path(L, oracle, qc)


def test_quant_error_codes(L):
    t = torch.zeros(64, device="cuda")
    shape = L.make_shape(1, 8, 2, 128, 4096, 2000, 2000, L.binding.Q8Q4)
    with pytest.raises(L.LeoamError) as e:       # record table missing
        L.kv_chunk_abstract_build(shape, t, t, t, t)
    assert e.value.status == -1
    ws = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(L.LeoamError) as e:       # more kept chunks than the compressed-store kernel indexes
        L.sparse_chunk_attention_decode(shape, t, t, t, t, t, t, t, 1.0, t, None, ws, qmeta=t)
    assert e.value.status == -3
    torch.cuda.synchronize()


@pytest.mark.parametrize("n_ctx,G", [(32768 + 77, 4), (32768 + 77, 1), (589824, 4), (327680, 2), (786432, 4)])
def test_quant_one_call_equals_separate_calls(L, oracle, n_ctx, G):
    """The one-launch kernel of the compressed store (selection inside the launch, splits merged by the last
    workgroup) against the separate select / attention calls and the oracle; the larger context has more than
    8192 chunks; the contexts are chosen so that the selection runs with 4, 6, 10 and 12 chunks per lane.  The workspace's partials start as garbage, the
    second call must leave the same bits as the first."""
    qc = gen.make_quant_case("c4", layer=9, n_ctx=n_ctx, hq=G, hkv=1, token_budget=4096, device="cuda")
    c = qc.case
    lay = L.DecodeLayer(qc.kblob, qc.vblob, c.chunk_off, c.n_chunks, c.hq, c.k_max, c.max_chunks, c.token_budget,
                        qmeta=qc.qmeta, n_kv_heads=c.hkv, n_ctx=c.n_ctx)
    if n_ctx == 589824:
        assert 8192 < lay.shape.c_max <= 10240          # ten chunks per lane in the selection
    if n_ctx == 327680:
        assert 4096 < lay.shape.c_max <= 6144           # six
    if n_ctx == 786432:
        assert 10240 < lay.shape.c_max <= 12288         # twelve
    lay.build_abstract()
    head = L.leoam_fused_control_bytes(lay.shape)        # control words stay zero, the partials behind them do not matter
    lay.workspace[head:].fill_(0x7f)
    lay.step(c.q)
    torch.cuda.synchronize()
    one = [t.clone() for t in (lay.sel_idx, lay.sel_count, lay.sel_tokens, lay.out, lay.lse)]
    assert not lay.workspace[:head].any()        # counters reset by the merging workgroups
    lay.step(c.q)
    torch.cuda.synchronize()
    for a, b in zip(one, (lay.sel_idx, lay.sel_count, lay.sel_tokens, lay.out, lay.lse)):
        assert torch.equal(a, b)
    lay.step_separate(c.q)
    torch.cuda.synchronize()
    assert torch.equal(one[0], lay.sel_idx) and torch.equal(one[1], lay.sel_count) and torch.equal(one[2], lay.sel_tokens)
    assert (one[3] - lay.out).abs().max().item() <= 1e-4
    off, nc = c.chunk_off.cpu(), c.n_chunks.cpu()
    kb, vb, qm = qc.kblob.cpu(), qc.vblob.cpu(), qc.qmeta.cpu()
    # the kept list of the one-launch kernel against the oracle's own abstract -> score -> selection
    ab = oracle.abstract_build_q(kb, qm, off, nc)
    ub = oracle.chunk_score(c.q.cpu(), np.nan_to_num(ab), nc)
    assert np.array_equal(lay.score.cpu().numpy(), ub), "score"
    sel, cnt, tok = oracle.topk_select(ub, off, nc, c.max_chunks, c.token_budget, c.k_max)
    assert np.array_equal(one[0].cpu().numpy(), sel), "sel_idx"
    assert np.array_equal(one[1].cpu().numpy(), cnt) and np.array_equal(one[2].cpu().numpy(), tok)
    out, lse = oracle.sparse_attention_q(c.q.cpu(), kb, vb, qm, off, sel, cnt)
    assert np.abs(one[3].cpu().numpy().astype(np.float64) - out).max() <= TOL
    assert np.abs(one[4].cpu().numpy().astype(np.float64) - lse).max() <= 1e-3
