"""GPU parity of kv_chunk_compress (Sec. 4.4 dynamic KV compression, Sec. 6.1 INT4)
against the CPU oracle: byte offsets, formats, scales, zero points and every code
byte bit-exact (the code decision is taken in float on both sides)."""
import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def L():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2506_20187_amd as lib
    return lib


def gpu_compress(L, K, V, packed, counts, fb, hq=None, poison=True):
    B, Hkv, N, _ = K.shape
    c_max = packed.shape[1] - 1
    shape = L.make_shape(B, hq or Hkv, Hkv, 128, N, c_max, 1, K.dtype)
    cap = L.leoam_compressed_bytes_bound(shape)
    assert cap == B * Hkv * N * 128
    kb = torch.full((cap,), 0xA5 if poison else 0, dtype=torch.uint8, device="cuda")
    vb = torch.full((cap,), 0x5A if poison else 0, dtype=torch.uint8, device="cuda")
    qm = torch.full((B, Hkv, c_max, 8), -7, dtype=torch.int32, device="cuda")
    total = torch.zeros(1, dtype=torch.int64, device="cuda")
    L.kv_chunk_compress(shape, K.cuda(), V.cuda(), torch.from_numpy(packed).cuda(), torch.from_numpy(counts).cuda(),
                        torch.from_numpy(np.ascontiguousarray(fb).astype(np.uint8)).cuda(), kb, vb, qm, total)
    torch.cuda.synchronize()
    return kb.cpu().numpy(), vb.cpu().numpy(), qm.cpu().numpy(), int(total.item())


def check_against_oracle(oracle, got, K, V, packed, counts, fb):
    kb, vb, qm, total = got
    wk, wv, wq = oracle.chunk_compress(K, V, packed, counts, fb)
    assert total == wk.size == wv.size
    rec = qm.view(oracle.QCHUNK_DTYPE).reshape(wq.shape)
    assert np.array_equal(rec.view(np.uint8), wq.view(np.uint8)), "records (offsets, formats, scales, zero points)"
    assert np.array_equal(kb[:total], wk[:total]), "K codes"
    assert np.array_equal(vb[:total], wv[:total]), "V codes"
    # nothing past the used bytes is touched
    assert (kb[total:] == 0xA5).all() and (vb[total:] == 0x5A).all()


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("share", [0.0, 0.5, 1.0])
def test_compress_exact_ragged_chunks(L, oracle, dtype, share):
    # chunk sizes 1..200: below, at and above the 64 rows a workgroup holds in registers; three tiles of the
    # layout scan would need c_max > 2048, covered by the full-shape test below
    rng = np.random.default_rng(int(share * 10) + (dtype == torch.float16))
    g = torch.Generator().manual_seed(5)
    B, Hkv, N = 2, 3, 3000
    K = (torch.randn(B, Hkv, N, 128, generator=g) * 1.9).to(dtype)
    V = torch.randn(B, Hkv, N, 128, generator=g).to(dtype)
    offs = [gen.make_boundaries(N, rng, sizes=(1, 2, 15, 16, 63, 64, 65, 130, 200)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    assert counts.min() < c_max or B == 1                 # some unused record slots
    fb = rng.random((B, c_max)) < share
    check_against_oracle(oracle, gpu_compress(L, K, V, packed, counts, fb), K, V, packed, counts, fb)


@pytest.mark.parametrize("seed", list(range(8)))
def test_compress_random_shapes(L, oracle, seed):
    """Shapes and value ranges drawn at random (seeded): dtype, batch, heads, ragged context, chunk-size mixes from
    single tokens to 300 rows, magnitudes over five decades, values on a coarse grid (ties at the code boundaries),
    any share of 4-bit chunks."""
    rng = np.random.default_rng(7000 + seed)
    dtype = (torch.float16, torch.bfloat16)[int(rng.integers(2))]
    B, Hkv, N = int(rng.integers(1, 6)), int(rng.integers(1, 4)), int(rng.integers(50, 4000))
    g = torch.Generator().manual_seed(seed)
    K = (torch.randn(B, Hkv, N, 128, generator=g) * float(10 ** rng.uniform(-3, 2))).to(dtype)
    V = (torch.randn(B, Hkv, N, 128, generator=g) * float(10 ** rng.uniform(-2, 1))).to(dtype)
    if rng.integers(3) == 0:
        K = (torch.randint(-8, 9, (B, Hkv, N, 128), generator=g).float() * 0.25).to(dtype)
    sizes = [(1, 2, 15, 16, 63, 64, 65, 130, 200), (1, 3, 16, 40, 70), (32, 64), (1,), (7, 300)][int(rng.integers(5))]
    offs = [gen.make_boundaries(N, rng, sizes=sizes) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    fb = rng.random((B, c_max)) < rng.random()
    check_against_oracle(oracle, gpu_compress(L, K, V, packed, counts, fb), K, V, packed, counts, fb)


def test_compress_many_sequences(L, oracle):
    # more sequences than the layout kernel sums in one round (a wave per earlier sequence, sixteen at a time)
    rng = np.random.default_rng(77)
    g = torch.Generator().manual_seed(6)
    B, Hkv, N = 37, 2, 300
    K = torch.randn(B, Hkv, N, 128, generator=g).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, 128, generator=g).to(torch.bfloat16)
    offs = [gen.make_boundaries(N, rng, sizes=(1, 3, 16, 40, 70)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    fb = rng.random((B, c_max)) < 0.5
    check_against_oracle(oracle, gpu_compress(L, K, V, packed, counts, fb), K, V, packed, counts, fb)


def test_compress_degenerate_values(L, oracle):
    # constant chunks (scale 0), chunks on the code grid with ties, one huge outlier, negative zero
    N, B, Hkv = 256, 1, 2
    g = torch.Generator().manual_seed(9)
    K = torch.randn(B, Hkv, N, 128, generator=g)
    V = torch.randn(B, Hkv, N, 128, generator=g)
    K[:, :, 0:16] = 0.75                                     # constant
    V[:, :, 0:16] = -0.0
    K[:, :, 16:32] = torch.arange(16 * 128).reshape(16, 128).remainder(256).float() * 0.5      # ties at k + 1/2 steps
    K[:, :, 16, 0], K[:, :, 16, 1] = 0.0, 255.0
    V[:, :, 40, 7] = 60000.0                                 # outlier: everything else collapses to code 0
    K, V = K.to(torch.float16), V.to(torch.float16)
    packed = np.array([[0, 16, 32, 48, 256]], dtype=np.int32)
    counts = np.array([4], dtype=np.int32)
    for fb in ([[False, False, False, False]], [[True, True, True, True]], [[False, True, False, True]]):
        fb = np.array(fb)
        check_against_oracle(oracle, gpu_compress(L, K, V, packed, counts, fb), K, V, packed, counts, fb)


def test_compress_then_decode_path(L, oracle):
    """The store written by the GPU feeds the compressed decode path: abstract, score, selection and attention
    equal the oracle's on that store."""
    rng = np.random.default_rng(3)
    g = torch.Generator().manual_seed(3)
    B, Hkv, G, N = 2, 2, 4, 2048
    K = (torch.randn(B, Hkv, N, 128, generator=g) * 1.5).to(torch.float16)
    V = torch.randn(B, Hkv, N, 128, generator=g).to(torch.float16)
    q = (torch.randn(B, Hkv * G, 128, generator=g)).to(torch.float16)
    offs = [gen.make_boundaries(N, rng, sizes=(16, 32, 64, 128)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    fb = rng.random((B, c_max)) < 0.5
    kb, vb, qm, total = gpu_compress(L, K, V, packed, counts, fb, hq=Hkv * G, poison=False)
    lay = L.DecodeLayer(torch.from_numpy(kb).cuda(), torch.from_numpy(vb).cuda(), torch.from_numpy(packed).cuda(),
                        torch.from_numpy(counts).cuda(), Hkv * G, c_max, 0, 512, qmeta=torch.from_numpy(qm).cuda(),
                        n_kv_heads=Hkv, n_ctx=N)
    lay.build_abstract()
    lay.step(q.cuda())
    torch.cuda.synchronize()
    rec = qm.view(oracle.QCHUNK_DTYPE).reshape(B, Hkv, c_max)
    ab = oracle.abstract_build_q(kb, rec, packed, counts)
    ub = oracle.chunk_score(q, np.nan_to_num(ab), counts)
    assert np.array_equal(lay.score.cpu().numpy(), ub)
    sel, cnt, tok = oracle.topk_select(ub, packed, counts, 0, 512, c_max)
    assert np.array_equal(lay.sel_idx.cpu().numpy(), sel) and np.array_equal(lay.sel_count.cpu().numpy(), cnt)
    out, lse = oracle.sparse_attention_q(q, kb, vb, rec, packed, sel, cnt)
    assert np.abs(lay.out.cpu().numpy().astype(np.float64) - out).max() <= 2e-3
    # and the store is close to the cache it came from: half a step per element
    deq = oracle.dequant(kb, rec, packed, counts, N, 128, "k")
    step = np.zeros((B, Hkv, N))
    for b in range(B):
        step[b] = np.repeat(rec["scale_k"][b, :, :counts[b]], np.diff(packed[b, :counts[b] + 1]), axis=1)
    assert (np.abs(deq - K.double().numpy()) <= step[..., None] * (0.5 + 1e-4) + 1e-12).all()


def test_compress_full_shape_sampled(L, oracle):
    """The compressed-store workload at its full shape (512K tokens, 8 kv heads, chunks of 32..512): the layout
    is checked everywhere by its defining sums, sampled chunks against the oracle one by one."""
    case = gen.make_case("c4", layer=3, device="cuda")
    K, V = case.K, case.V
    assert K.dtype in (torch.float16, torch.bfloat16)
    packed, counts = case.chunk_off.cpu().numpy(), case.n_chunks.cpu().numpy()
    B, Hkv, N, _ = K.shape
    c_max = packed.shape[1] - 1
    fb = gen.tag_four_bit(packed, counts, case.extra["heavy"], 0.5)
    shape = L.make_shape(B, case.hq, Hkv, 128, N, c_max, 1, K.dtype)
    cap = L.leoam_compressed_bytes_bound(shape)
    kb = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    vb = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    qm = torch.zeros(B, Hkv, c_max, 8, dtype=torch.int32, device="cuda")
    total = torch.zeros(1, dtype=torch.int64, device="cuda")
    L.kv_chunk_compress(shape, K, V, case.chunk_off, case.n_chunks, torch.from_numpy(fb.astype(np.uint8)).cuda(), kb, vb,
                        qm, total)
    torch.cuda.synchronize()
    rec = qm.cpu().numpy().view(oracle.QCHUNK_DTYPE).reshape(B, Hkv, c_max)
    sizes = np.diff(packed.astype(np.int64), axis=1)
    pos = 0
    for b in range(B):
        n = counts[b]
        nbytes = sizes[b, :n] * np.where(fb[b, :n], 64, 128)
        within = np.concatenate([[0], np.cumsum(nbytes)[:-1]])
        for h in range(Hkv):
            assert np.array_equal(rec["byte_off"][b, h, :n], pos + within)
            assert np.array_equal(rec["bits"][b, h, :n], np.where(fb[b, :n], 4, 8))
            pos += int(nbytes.sum())
        assert not rec[b, :, n:].view(np.uint8).any()
    assert int(total.item()) == pos
    rng = np.random.default_rng(0)
    kb_h, vb_h = kb[:pos].cpu().numpy(), vb[:pos].cpu().numpy()
    picks = [(0, h, int(c)) for h in range(Hkv) for c in rng.choice(counts[0], size=6, replace=False)]
    picks += [(0, 0, 0), (0, Hkv - 1, int(counts[0]) - 1), (0, 3, int(np.argmax(sizes[0, :counts[0]])))]
    for b, h, c in picks:
        t0, t1 = int(packed[b, c]), int(packed[b, c + 1])
        wk, wv, wq = oracle.chunk_compress(K[b:b + 1, h:h + 1, t0:t1].cpu(), V[b:b + 1, h:h + 1, t0:t1].cpu(),
                                           np.array([[0, t1 - t0]], dtype=np.int32), np.array([1], dtype=np.int32),
                                           np.array([[fb[b, c]]]))
        r, w = rec[b, h, c], wq[0, 0, 0]
        for f in ("bits", "scale_k", "zero_k", "scale_v", "zero_v"):
            assert r[f] == w[f], (b, h, c, f)
        o = int(r["byte_off"])
        assert np.array_equal(kb_h[o:o + wk.size], wk) and np.array_equal(vb_h[o:o + wv.size], wv), (b, h, c)


def test_compress_error_codes(L):
    B, Hkv, N, c_max = 1, 2, 64, 4
    K = torch.zeros(B, Hkv, N, 128, dtype=torch.float16, device="cuda")
    off = torch.tensor([[0, 16, 32, 48, 64]], dtype=torch.int32, device="cuda")
    nc = torch.tensor([4], dtype=torch.int32, device="cuda")
    fb = torch.zeros(B, c_max, dtype=torch.uint8, device="cuda")
    qm = torch.zeros(B, Hkv, c_max, 8, dtype=torch.int32, device="cuda")
    shape = L.make_shape(B, Hkv, Hkv, 128, N, c_max, 1, torch.float16)
    small = torch.zeros(B * Hkv * N * 128 - 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(L.LeoamError) as e:
        L.kv_chunk_compress(shape, K, K, off, nc, fb, small, small, qm)
    assert e.value.status == L.binding.E_WORKSPACE
    ok = torch.zeros(B * Hkv * N * 128, dtype=torch.uint8, device="cuda")
    K32 = K.float()
    with pytest.raises(L.LeoamError) as e:
        L.kv_chunk_compress(L.make_shape(B, Hkv, Hkv, 128, N, c_max, 1, torch.float32), K32, K32, off, nc, fb, ok, ok, qm)
    assert e.value.status == L.binding.E_UNSUPPORTED
    L.kv_chunk_compress(shape, K, K, off, nc, fb, ok, ok, qm)       # all-zero cache: scale 0, codes 0
    torch.cuda.synchronize()
    assert not ok.any() and (qm[..., 2] == 8).all() and not qm[..., 3:].any()


def test_compress_bad_boundaries_stay_inside_the_blobs(L, oracle):
    """Boundaries that rise, fall and rise again: every rising step is a chunk inside the context, together
    they hold more rows than the context.  Falling steps take no room, and a chunk that would end past
    blob_bytes is not written."""
    B, Hkv, N, c_max = 1, 2, 256, 5
    g = torch.Generator().manual_seed(11)
    K = torch.randn(B, Hkv, N, 128, generator=g).to(torch.float16)
    V = torch.randn(B, Hkv, N, 128, generator=g).to(torch.float16)
    off = torch.tensor([[0, 256, 0, 256, 100, 90]], dtype=torch.int32, device="cuda")
    nc = torch.tensor([5], dtype=torch.int32, device="cuda")
    fb = torch.zeros(B, c_max, dtype=torch.uint8, device="cuda")
    shape = L.make_shape(B, Hkv, Hkv, 128, N, c_max, 1, torch.float16)
    cap = L.leoam_compressed_bytes_bound(shape)
    guard = 4096
    kbig = torch.full((cap + guard,), 0xEE, dtype=torch.uint8, device="cuda")
    vbig = torch.full((cap + guard,), 0xEE, dtype=torch.uint8, device="cuda")
    qm = torch.zeros(B, Hkv, c_max, 8, dtype=torch.int32, device="cuda")
    total = torch.zeros(1, dtype=torch.int64, device="cuda")
    L.kv_chunk_compress(shape, K.cuda(), V.cuda(), off, nc, fb, kbig[:cap], vbig[:cap], qm, total)
    torch.cuda.synchronize()
    assert (kbig[cap:] == 0xEE).all() and (vbig[cap:] == 0xEE).all(), "nothing is written past blob_bytes"
    # two whole-context chunks per head at 8 bits: twice what a head's share of the blob holds
    assert int(total.item()) == 2 * cap
    # head 0's two chunks fill the blob (the same codes twice), head 1's would lie past it
    packed1 = np.array([[0, N]], dtype=np.int32)
    wk, wv, _ = oracle.chunk_compress(K[:, :1], V[:, :1], packed1, np.array([1], dtype=np.int32), np.zeros((1, 1), dtype=bool))
    half = N * 128
    kb, vb = kbig[:cap].cpu().numpy(), vbig[:cap].cpu().numpy()
    assert np.array_equal(kb[:half], wk) and np.array_equal(kb[half:], wk)
    assert np.array_equal(vb[:half], wv) and np.array_equal(vb[half:], wv)


def test_compression_tags_exact_and_policy_loop(L, oracle):
    """chunk_compression_tags against the oracle on ragged selections, then the whole policy loop on the GPU:
    theta from the latency condition -> token budget (1 - theta) N -> selection by score -> tags -> compressed
    store, every step equal to the oracle's."""
    rng = np.random.default_rng(17)
    g = torch.Generator().manual_seed(17)
    B, Hkv, G, N = 3, 2, 4, 4096
    offs = [gen.make_boundaries(N, rng, sizes=(8, 16, 32, 64)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    shape = L.make_shape(B, Hkv * G, Hkv, 128, N, c_max, c_max, torch.float16)
    d_off, d_nc = torch.from_numpy(packed).cuda(), torch.from_numpy(counts).cuda()
    # (a) hand-made selections: empty rows, everything, duplicates across heads, ids out of range, stale tail entries
    sel = np.full((B, Hkv, c_max), -1, dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    sel[0, 0, :counts[0]] = np.arange(counts[0]); cnt[0, 0] = counts[0]
    sel[1, 0, :5] = [0, 3, 4, c_max + 7, -2]; cnt[1, 0] = 5
    sel[1, 1, :6] = [3, 9, 9, 11, 2, 1]; cnt[1, 1] = 4                  # entries 4, 5 are stale
    tags = torch.full((B, c_max), 9, dtype=torch.uint8, device="cuda")
    L.chunk_compression_tags(shape, d_nc, torch.from_numpy(sel).cuda(), torch.from_numpy(cnt).cuda(), tags)
    torch.cuda.synchronize()
    assert np.array_equal(tags.cpu().numpy(), oracle.compression_tags(counts, sel, cnt, c_max))
    # (b) the loop
    theta = L.leoam_compression_share(2.0 * B * Hkv * N * 256, 0.25, 20e9, 0.2e-3, 0.5e-3, 400e9)
    assert 0 < theta < 1 and abs(theta - oracle.compression_share(2.0 * B * Hkv * N * 256, 0.25, 20e9, 0.2e-3, 0.5e-3, 400e9)) < 1e-15
    budget = int((1 - theta) * N)
    K = (torch.randn(B, Hkv, N, 128, generator=g) * 1.5).to(torch.float16)
    V = torch.randn(B, Hkv, N, 128, generator=g).to(torch.float16)
    q = torch.randn(B, Hkv * G, 128, generator=g).to(torch.float16)
    lay = L.DecodeLayer(K.cuda(), V.cuda(), d_off, d_nc, Hkv * G, c_max, 0, budget)
    lay.build_abstract()
    lay.step_separate(q.cuda())
    L.chunk_compression_tags(shape, d_nc, lay.sel_idx, lay.sel_count, tags)
    torch.cuda.synchronize()
    ab = oracle.abstract_build(K, packed, counts)
    ub = oracle.chunk_score(q, np.nan_to_num(ab), counts)
    osel, ocnt, otok = oracle.topk_select(ub, packed, counts, 0, budget, c_max)
    assert np.array_equal(lay.sel_idx.cpu().numpy(), osel)
    want = oracle.compression_tags(counts, osel, ocnt, c_max)
    got = tags.cpu().numpy()
    assert np.array_equal(got, want)
    # every head keeps at most (1 - theta) N tokens, so at least the share theta - (Hkv - 1)(1 - theta) of the tokens is 4-bit
    sizes = np.diff(packed.astype(np.int64), axis=1)
    for b in range(B):
        four_tokens = int((sizes[b, :counts[b]] * got[b, :counts[b]]).sum())
        assert four_tokens >= N - Hkv * budget
    check_against_oracle(oracle, gpu_compress(L, K, V, packed, counts, got.astype(bool)), K, V, packed, counts, got.astype(bool))


# ---------------------------------------------------------------------------
# kv_chunk_recompress: a live store brought to new tags, only the changed chunks encoded again
# ---------------------------------------------------------------------------
def gpu_store(L, K, V, packed, counts, fb, cap):
    """kv_chunk_compress into blobs of `cap` bytes (poisoned), everything left on the GPU"""
    B, Hkv, N, _ = K.shape
    c_max = packed.shape[1] - 1
    shape = L.make_shape(B, Hkv, Hkv, 128, N, c_max, 1, K.dtype)
    st = dict(shape=shape, K=K.cuda(), V=V.cuda(), off=torch.from_numpy(packed).cuda(), nc=torch.from_numpy(counts).cuda(),
              kb=torch.full((cap,), 0xA5, dtype=torch.uint8, device="cuda"),
              vb=torch.full((cap,), 0x5A, dtype=torch.uint8, device="cuda"),
              qm=torch.full((B, Hkv, c_max, 8), -7, dtype=torch.int32, device="cuda"),
              used=torch.zeros(1, dtype=torch.int64, device="cuda"), info=torch.full((3,), -7, dtype=torch.int64, device="cuda"))
    L.kv_chunk_compress(shape, st["K"], st["V"], st["off"], st["nc"], tags_dev(fb), st["kb"], st["vb"], st["qm"], st["used"])
    torch.cuda.synchronize()
    return st


def tags_dev(fb):
    return torch.from_numpy(np.ascontiguousarray(fb).astype(np.uint8)).cuda()


def oracle_store(oracle, K, V, packed, counts, fb, cap):
    wk, wv, wq = oracle.chunk_compress(K, V, packed, counts, fb)
    kb, vb = np.full(cap, 0xA5, dtype=np.uint8), np.full(cap, 0x5A, dtype=np.uint8)
    kb[: wk.size], vb[: wv.size] = wk, wv
    return kb, vb, wq, wk.size


def assert_same_store(oracle, st, want):
    kb, vb, wq, used = want
    rec = st["qm"].cpu().numpy().view(oracle.QCHUNK_DTYPE).reshape(wq.shape)
    for f in ("byte_off", "bits", "scale_k", "zero_k", "scale_v", "zero_v"):
        assert np.array_equal(rec[f], wq[f]), f
    assert int(st["used"].item()) == used
    assert np.array_equal(st["kb"].cpu().numpy(), kb), "K blob (codes, holes and untouched bytes)"
    assert np.array_equal(st["vb"].cpu().numpy(), vb), "V blob"


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_recompress_exact_chain_of_retags(L, oracle, dtype):
    rng = np.random.default_rng(41 + (dtype == torch.float16))
    g = torch.Generator().manual_seed(6)
    B, Hkv, N = 3, 2, 2500
    K = (torch.randn(B, Hkv, N, 128, generator=g) * 1.9).to(dtype)
    V = torch.randn(B, Hkv, N, 128, generator=g).to(dtype)
    offs = [gen.make_boundaries(N, rng, sizes=(1, 2, 15, 16, 63, 64, 65, 130)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    cap = 3 * B * Hkv * N * 128
    tags = [rng.random((B, c_max)) < s for s in (0.5, 0.5, 0.9, 0.1, 0.1)]        # the last step changes nothing
    st = gpu_store(L, K, V, packed, counts, tags[0], cap)
    kb, vb, wq, used = oracle_store(oracle, K, V, packed, counts, tags[0], cap)
    assert_same_store(oracle, st, (kb, vb, wq, used))
    for old, new in zip(tags, tags[1:]):
        rc, used_new, changed = oracle.chunk_recompress(K, V, packed, counts, old, new, kb, vb, wq, used)
        assert rc == 0
        L.kv_chunk_recompress(st["shape"], st["K"], st["V"], st["off"], st["nc"], tags_dev(old), tags_dev(new), st["kb"],
                              st["vb"], st["qm"], st["used"], st["info"])
        torch.cuda.synchronize()
        assert st["info"].cpu().tolist() == [0, changed, used_new - used]
        used = used_new
        assert_same_store(oracle, st, (kb, vb, wq, used))
    # the kernels that read the store follow the records: attention over the re-tagged store (moved chunks, holes)
    G = 4
    q = (torch.randn(B, Hkv * G, 128, generator=g) * 1.3).to(torch.float16)
    sel = np.full((B, Hkv, c_max), -1, dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    for b in range(B):
        for h in range(Hkv):
            n = int(rng.integers(1, counts[b]))
            sel[b, h, :n] = np.sort(rng.choice(counts[b], size=n, replace=False))
            cnt[b, h] = n
    want, _ = oracle.sparse_attention_q(q, kb, vb, wq, packed, sel, cnt)
    qshape = L.make_shape(B, Hkv * G, Hkv, 128, N, c_max, c_max, L.binding.Q8Q4)
    out = torch.full((B, Hkv * G, 128), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(L.leoam_workspace_bytes(qshape, 0), dtype=torch.uint8, device="cuda")
    L.sparse_chunk_attention_decode(qshape, q.cuda(), st["kb"], st["vb"], st["off"], st["nc"], torch.from_numpy(sel).cuda(),
                                    torch.from_numpy(cnt).cuda(), L.default_scale(128), out, None, ws, qmeta=st["qm"])
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy().astype(np.float64) - want).max() <= 2e-3
    ab = torch.empty(B, Hkv, c_max, 2, 128, dtype=torch.float16, device="cuda")
    L.kv_chunk_abstract_build(qshape, st["kb"], st["off"], st["nc"], ab, qmeta=st["qm"])
    torch.cuda.synchronize()
    want_ab = oracle.abstract_build_q(kb, wq, packed, counts)
    got_ab = ab.cpu().to(torch.float64).numpy()
    for b in range(B):
        assert np.array_equal(got_ab[b, :, : counts[b]], want_ab[b, :, : counts[b]])


def test_recompress_without_room_changes_nothing(L, oracle):
    rng = np.random.default_rng(43)
    g = torch.Generator().manual_seed(7)
    B, Hkv, N = 2, 2, 900
    K = torch.randn(B, Hkv, N, 128, generator=g).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, 128, generator=g).to(torch.bfloat16)
    offs = [gen.make_boundaries(N, rng, sizes=(4, 16, 33)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    cap = B * Hkv * N * 128                      # the bound: a store of 4-bit chunks fills half of it
    old, new = np.ones((B, c_max), dtype=bool), np.zeros((B, c_max), dtype=bool)
    st = gpu_store(L, K, V, packed, counts, old, cap)
    before = [st[k].clone() for k in ("kb", "vb", "qm", "used")]
    new[0, 0] = True                              # every chunk but one would move: twice the room that is left
    L.kv_chunk_recompress(st["shape"], st["K"], st["V"], st["off"], st["nc"], tags_dev(old), tags_dev(new), st["kb"],
                          st["vb"], st["qm"], st["used"], st["info"])
    torch.cuda.synchronize()
    assert st["info"].cpu().tolist() == [1, 0, 0]
    for a, k in zip(before, ("kb", "vb", "qm", "used")):
        assert torch.equal(a, st[k]), k
    # a third of the chunks fits
    new2 = old.copy()
    want = oracle_store(oracle, K, V, packed, counts, old, cap)
    kb, vb, wq, used = want
    for b in range(B):
        new2[b, : counts[b] // 3] = False
    rc, used_new, changed = oracle.chunk_recompress(K, V, packed, counts, old, new2, kb, vb, wq, used)
    assert rc == 0
    L.kv_chunk_recompress(st["shape"], st["K"], st["V"], st["off"], st["nc"], tags_dev(old), tags_dev(new2), st["kb"],
                          st["vb"], st["qm"], st["used"], st["info"])
    torch.cuda.synchronize()
    assert st["info"].cpu().tolist() == [0, changed, used_new - used]
    assert_same_store(oracle, st, (kb, vb, wq, used_new))
