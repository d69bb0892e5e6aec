"""GPU parity: libleoam.so (through its C ABI) against the float64 CPU oracle,
element by element, on the same seeded inputs.

Bars: abstracts, scores, kept chunk ids / counts / token totals bit-exact;
attention outputs within 1e-5 (fp32) and 2e-3 (fp16, bf16) max-abs.
"""
import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}
TDT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@pytest.fixture(scope="module")
def L():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2506_20187_amd as lib
    return lib


def dev(x):
    return x.cuda().contiguous() if isinstance(x, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(x)).cuda()


def host_f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def random_boundaries(rng, B, N, sizes):
    offs = []
    for _ in range(B):
        off = [0]
        while off[-1] < N:
            off.append(min(N, off[-1] + int(rng.choice(sizes))))
        offs.append(np.asarray(off, dtype=np.int32))
    return gen.pack_boundaries(offs, N)


def gpu_abstract(L, K, packed, counts):
    B, Hkv, N, D = K.shape
    c_max = packed.shape[1] - 1
    shape = L.make_shape(B, Hkv, Hkv, D, N, c_max, 1, K.dtype)
    ab = torch.full((B, Hkv, c_max, 2, D), float("nan"), dtype=K.dtype, device="cuda")
    L.kv_chunk_abstract_build(shape, dev(K), dev(packed), dev(counts), ab)
    torch.cuda.synchronize()
    return ab


# ---------------------------------------------------------------------------
# a1 abstract
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_abstract_exact(L, oracle, dtype):
    rng = np.random.default_rng(10)
    B, Hkv, N, D = 2, 3, 1037, 128
    K = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    packed, counts, c_max = random_boundaries(rng, B, N, (1, 2, 3, 7, 16, 33, 70))
    want = oracle.abstract_build(K, packed, counts)
    got = host_f64(gpu_abstract(L, K, packed, counts))
    for b in range(B):
        n = counts[b]
        assert np.array_equal(got[b, :, :n], want[b, :, :n])
        assert np.isnan(got[b, :, n:]).all()        # rows of absent chunks are not written


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_abstract_append_exact(L, oracle, dtype):
    """One new token per sequence and step: boundaries, counts, status and abstract rows follow the oracle bit for bit."""
    rng = np.random.default_rng(77)
    B, Hkv, N, D, cs, c_max = 4, 5, 150, 128, 8, 14
    K = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    off = np.zeros((B, c_max + 1), dtype=np.int32)
    nc = np.asarray([0, 3, 2, 1], dtype=np.int32)
    off[1, :4] = [0, 5, 12, 35]              # last chunk longer than the chunk size: a new chunk opens at once
    off[2, :3] = [0, 70, 146]                # reaches the end of the cache after four steps
    off[3, :2] = [0, 3]                      # runs out of chunk slots
    ab0 = oracle.abstract_build(K, off, nc, full=False)
    shape = L.make_shape(B, Hkv, Hkv, D, N, c_max, 1, TDT[dtype])
    d_off, d_nc = dev(off), dev(nc)
    d_ab = torch.from_numpy(np.nan_to_num(ab0, nan=512.0)).to(TDT[dtype]).cuda()      # unused rows hold a marker
    d_K, d_st = dev(K), torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ab = ab0
    seen = set()
    for step in range(120):
        off, nc, ab, st = oracle.abstract_append(K, off, nc, cs, ab)
        L.kv_chunk_abstract_append(shape, d_K, d_off, d_nc, cs, d_ab, d_st)
        torch.cuda.synchronize()
        assert np.array_equal(d_st.cpu().numpy(), st), f"status, step {step}"
        assert np.array_equal(d_nc.cpu().numpy(), nc), f"n_chunks, step {step}"
        got_off, got_ab = d_off.cpu().numpy(), host_f64(d_ab)
        for b in range(B):
            assert np.array_equal(got_off[b, : nc[b] + 1], off[b, : nc[b] + 1]), f"boundaries, step {step}"
            assert np.array_equal(got_ab[b, :, : nc[b]], ab[b, :, : nc[b]]), f"abstract, step {step}"
            assert np.all(got_ab[b, :, nc[b]:] == 512.0)                              # rows of absent chunks untouched
        seen |= set(st.tolist())
    assert seen == {0, 1, 2}


def test_decode_loop_with_appends(L, oracle):
    """A short decode loop: append the step's key, then score -> select -> attention on the grown cache."""
    case = gen.make_case("c2", layer=11, n_ctx=4096, hq=8, hkv=2, token_budget=512)
    K, V = case.K, case.V
    B, Hkv, N, D = K.shape
    c_max = case.chunk_off.shape[1] - 1 + 8
    # the cache starts 40 tokens short of its capacity: keep the chunks that end before that point
    row = case.chunk_off[0].numpy()
    keep = int(np.searchsorted(row[: int(case.n_chunks[0]) + 1], N - 40, side="right")) - 1
    off = np.zeros((B, c_max + 1), dtype=np.int32)
    off[0, : keep + 1] = row[: keep + 1]
    nc = np.asarray([keep], dtype=np.int32)
    layer = L.DecodeLayer(dev(K), dev(V), dev(off), dev(nc), case.hq, case.k_max, 0, case.token_budget)
    layer.build_abstract()
    ab = oracle.abstract_build(K, off, nc, full=False)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for step in range(12):
        q = (case.q.float() + 0.3 * torch.from_numpy(rng.standard_normal(tuple(case.q.shape)).astype(np.float32))).to(K.dtype)
        off, nc, ab, st = oracle.abstract_append(K, off, nc, 16, ab)
        L.kv_chunk_abstract_append(layer.shape, layer.K, layer.chunk_off, layer.n_chunks, 16, layer.abstract, None)
        layer.step(dev(q))
        torch.cuda.synchronize()
        ub = oracle.chunk_score(q, np.nan_to_num(ab), nc)
        sel, cnt, tok = oracle.topk_select(ub, off, nc, 0, case.token_budget, case.k_max)
        out, _ = oracle.sparse_attention(q, K, V, off, sel, cnt)
        n = int(nc[0])
        assert np.array_equal(layer.n_chunks.cpu().numpy(), nc)
        assert np.array_equal(layer.score[:, :, :n].cpu().numpy(), ub[:, :, :n]), f"score, step {step}"
        assert np.array_equal(layer.sel_idx.cpu().numpy(), sel) and np.array_equal(layer.sel_count.cpu().numpy(), cnt)
        assert np.abs(host_f64(layer.out) - out).max() <= TOL[case.dtype], f"attention, step {step}"


# ---------------------------------------------------------------------------
# a2 score
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,G", [("f32", 1), ("f32", 4), ("f16", 1), ("f16", 2), ("bf16", 4), ("bf16", 8)])
def test_score_exact(L, oracle, dtype, G):
    rng = np.random.default_rng(20 + G)
    B, Hkv, N, D = 2, 2, 3000, 128
    K = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    q = torch.from_numpy(rng.standard_normal((B, Hkv * G, D)).astype(np.float32)).to(TDT[dtype])
    packed, counts, c_max = random_boundaries(rng, B, N, (1, 4, 9, 16, 25))
    ab64 = oracle.abstract_build(K, packed, counts)
    ub, lb = oracle.chunk_score(q, np.nan_to_num(ab64), counts, want_lower=True)
    ab = torch.from_numpy(np.nan_to_num(ab64)).to(TDT[dtype])           # exact: abstract values are key values
    shape = L.make_shape(B, Hkv * G, Hkv, D, N, c_max, 1, TDT[dtype])
    s_ub = torch.empty(B, Hkv, c_max, dtype=torch.float32, device="cuda")
    s_lb = torch.empty_like(s_ub)
    L.chunk_score(shape, dev(q), dev(ab), dev(counts), s_ub, s_lb)
    s_only = torch.empty_like(s_ub)
    L.chunk_score(shape, dev(q), dev(ab), dev(counts), s_only, None)
    torch.cuda.synchronize()
    assert np.array_equal(s_ub.cpu().numpy(), ub)
    assert np.array_equal(s_lb.cpu().numpy(), lb)
    assert np.array_equal(s_only.cpu().numpy(), ub)


@pytest.mark.parametrize("dtype,G,c_max", [("bf16", 4, 301), ("f16", 2, 264), ("bf16", 1, 333), ("f32", 4, 300)])
def test_score_exact_many_heads_odd_capacity(L, oracle, dtype, G, c_max):
    """Enough (sequence, kv head) pairs for the large-launch shapes (pairs of row sets when only the upper
    bound of two to four heads is asked for, else pipelined groups of four sets), with capacities that let
    the abstracts of different pairs start at every offset inside 16 KiB (pairs and groups are cut at
    multiples of their size, so the first one of a (sequence, kv head) is partly skipped), and ragged
    chunk counts."""
    rng = np.random.default_rng(c_max)
    B, Hkv, D = 64, 8, 128
    counts = rng.integers(c_max // 2, c_max + 1, size=B).astype(np.int32)
    counts[:3] = (c_max, 0, 1)
    # abstracts straight from random key values: kmax >= kmin element-wise
    a = rng.standard_normal((B, Hkv, c_max, D)).astype(np.float32)
    b = rng.standard_normal((B, Hkv, c_max, D)).astype(np.float32)
    ab = torch.from_numpy(np.stack([np.maximum(a, b), np.minimum(a, b)], axis=3)).to(TDT[dtype])      # [B,Hkv,c_max,2,D]
    q = torch.from_numpy(rng.standard_normal((B, Hkv * G, D)).astype(np.float32)).to(TDT[dtype])
    ub, lb = oracle.chunk_score(q, ab.to(torch.float64).numpy(), counts, want_lower=True)
    shape = L.make_shape(B, Hkv * G, Hkv, D, 4096, c_max, 1, TDT[dtype])
    abd = dev(ab)
    set_bytes = 16 * D * abd.element_size()                  # sixteen abstract rows
    leads = {((abd.data_ptr() + i * c_max * 2 * D * abd.element_size()) // set_bytes) & 3 for i in range(B * Hkv)}
    assert len(leads) > 1, "the capacities were chosen so that the first groups differ"
    s_ub = torch.empty(B, Hkv, c_max, dtype=torch.float32, device="cuda")
    s_lb = torch.empty_like(s_ub)
    L.chunk_score(shape, dev(q), abd, dev(counts), s_ub, s_lb)
    s_only = torch.empty_like(s_ub)
    L.chunk_score(shape, dev(q), abd, dev(counts), s_only, None)
    torch.cuda.synchronize()
    assert np.array_equal(s_ub.cpu().numpy(), ub)
    assert np.array_equal(s_lb.cpu().numpy(), lb)
    assert np.array_equal(s_only.cpu().numpy(), ub)


@pytest.mark.parametrize("dtype,G,c_max", [("bf16", 4, 5), ("f16", 2, 17), ("bf16", 1, 9)])
def test_score_exact_tiny_capacity_many_sequences(L, oracle, dtype, G, c_max):
    """A large launch (thousands of (sequence, kv head) pairs) whose rows hold only one to three row sets:
    most waves of a workgroup then have nothing of their own to contract, and the abstracts of different
    pairs start at every 512-byte offset."""
    rng = np.random.default_rng(100 + c_max)
    B, Hkv, D = 640, 8, 128
    counts = rng.integers(0, c_max + 1, size=B).astype(np.int32)
    counts[:2] = (c_max, 0)
    a = rng.standard_normal((B, Hkv, c_max, D)).astype(np.float32)
    b = rng.standard_normal((B, Hkv, c_max, D)).astype(np.float32)
    ab = torch.from_numpy(np.stack([np.maximum(a, b), np.minimum(a, b)], axis=3)).to(TDT[dtype])
    q = torch.from_numpy(rng.standard_normal((B, Hkv * G, D)).astype(np.float32)).to(TDT[dtype])
    ub, lb = oracle.chunk_score(q, ab.to(torch.float64).numpy(), counts, want_lower=True)
    shape = L.make_shape(B, Hkv * G, Hkv, D, 4096, c_max, 1, TDT[dtype])
    s_ub = torch.empty(B, Hkv, c_max, dtype=torch.float32, device="cuda")
    s_lb = torch.empty_like(s_ub)
    L.chunk_score(shape, dev(q), dev(ab), dev(counts), s_ub, s_lb)
    s_only = torch.empty_like(s_ub)
    L.chunk_score(shape, dev(q), dev(ab), dev(counts), s_only, None)
    torch.cuda.synchronize()
    assert np.array_equal(s_ub.cpu().numpy(), ub)
    assert np.array_equal(s_lb.cpu().numpy(), lb)
    assert np.array_equal(s_only.cpu().numpy(), ub)


@pytest.mark.parametrize("seed", list(range(10)))
def test_score_exact_random_shapes(L, oracle, seed):
    """Launch shapes drawn at random (seeded): dtype, group size, kv heads, capacity 1 ... 1200 and as many sequences as
    keep the oracle quick (small and large launches, pairs and groups), ragged chunk counts."""
    rng = np.random.default_rng(13000 + seed)
    dtype = ("f32", "f16", "bf16")[int(rng.integers(3))]
    G = (1, 2, 4, 8)[int(rng.integers(4))]
    Hkv, D = int(rng.integers(1, 9)), 128
    c_max = int(rng.integers(1, 1200))
    B = int(rng.integers(1, max(2, min(700, 1_500_000 // (Hkv * c_max)))))
    counts = rng.integers(0, c_max + 1, size=B).astype(np.int32)
    counts[0] = c_max
    a = rng.standard_normal((B, Hkv, c_max, D)).astype(np.float32)
    b = rng.standard_normal((B, Hkv, c_max, D)).astype(np.float32)
    ab = torch.from_numpy(np.stack([np.maximum(a, b), np.minimum(a, b)], axis=3)).to(TDT[dtype])
    q = torch.from_numpy(rng.standard_normal((B, Hkv * G, D)).astype(np.float32)).to(TDT[dtype])
    ub, lb = oracle.chunk_score(q, ab.to(torch.float64).numpy(), counts, want_lower=True)
    shape = L.make_shape(B, Hkv * G, Hkv, D, 4096, c_max, 1, TDT[dtype])
    s_ub = torch.empty(B, Hkv, c_max, dtype=torch.float32, device="cuda")
    s_lb, s_only = torch.empty_like(s_ub), torch.empty_like(s_ub)
    L.chunk_score(shape, dev(q), dev(ab), dev(counts), s_ub, s_lb)
    L.chunk_score(shape, dev(q), dev(ab), dev(counts), s_only, None)
    torch.cuda.synchronize()
    assert np.array_equal(s_ub.cpu().numpy(), ub)
    assert np.array_equal(s_lb.cpu().numpy(), lb)
    assert np.array_equal(s_only.cpu().numpy(), ub)


# ---------------------------------------------------------------------------
# a3 select
# ---------------------------------------------------------------------------
def gpu_select(L, score, packed, counts, max_chunks, budget, k_max, N):
    B, Hkv, c_max = score.shape
    shape = L.make_shape(B, Hkv, Hkv, 128, N, c_max, k_max, torch.float32)
    sel = torch.full((B, Hkv, k_max), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((B, Hkv), -7, dtype=torch.int32, device="cuda")
    tok = torch.full((B, Hkv), -7, dtype=torch.int32, device="cuda")
    L.chunk_topk_select(shape, dev(score), dev(packed), dev(counts), max_chunks, budget, sel, cnt, tok)
    torch.cuda.synchronize()
    return sel.cpu().numpy(), cnt.cpu().numpy(), tok.cpu().numpy()


@pytest.mark.parametrize("C", [5, 130, 1024, 1500, 3000, 5000, 8192, 9000, 11000, 16384])
def test_select_exact(L, oracle, C):
    rng = np.random.default_rng(C)
    B, Hkv = 2, 3
    offs = []
    for b in range(B):
        n = C if b == 0 else max(1, C - int(rng.integers(0, C // 2 + 1)))
        sizes = rng.integers(1, 40, size=n)
        offs.append(np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32))
    N = int(max(o[-1] for o in offs))
    offs = [np.concatenate([o[:-1], [N]]).astype(np.int32) for o in offs]      # both rows end at N
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    flavours = {
        "normal": rng.standard_normal((B, Hkv, c_max)).astype(np.float32) * 30 + 200,
        "ties": rng.integers(-3, 4, size=(B, Hkv, c_max)).astype(np.float32),
        "wide": (rng.standard_normal((B, Hkv, c_max)) * 10.0 ** rng.integers(-20, 20, size=(B, Hkv, c_max))).astype(np.float32),
        "flat": np.full((B, Hkv, c_max), -0.0, dtype=np.float32),
        # scores on both sides of zero: the first pass of the descent (sub-ranges equal in the bit pattern)
        # leaves hundreds of chunks in the cut sub-range, which takes further passes
        "around_zero": rng.standard_normal((B, Hkv, c_max)).astype(np.float32) * 20,
        "uniform_around_zero": ((rng.random((B, Hkv, c_max)) - 0.5) * 100).astype(np.float32),
    }
    flavours["flat"][:, :, ::2] = 0.0
    total = N
    for name, score in flavours.items():
        for max_chunks, budget in ((0, total // 10), (max(1, C // 7), 0), (max(1, C // 3), total // 5), (0, 0), (1, 0),
                                   (0, 1), (0, total)):
            k_max = c_max
            want = oracle.topk_select(score, packed, counts, max_chunks, budget, k_max)
            got = gpu_select(L, score, packed, counts, max_chunks, budget, k_max, N)
            for w, g, what in zip(want, got, ("sel_idx", "sel_count", "sel_tokens")):
                assert np.array_equal(w, g), f"{what} differs: C={C} {name} max_chunks={max_chunks} budget={budget}"


@pytest.mark.parametrize("m", [1, 2, 16, 17, 33, 64, 65, 128, 129, 256, 257, 512, 513, 1024, 1025])
def test_select_cluster_at_the_threshold(L, oracle, m):
    """m chunks with nearly equal (distinct, and a few equal) scores sit where the budget runs out, the
    others far above and far below: after the first histogram pass exactly those m are left to be ranked,
    which takes the pairwise step through every width of its lane groups and, past its limit of 256, through
    further passes of the descent and the scan over equal keys."""
    rng = np.random.default_rng(m)
    B, Hkv, C = 2, 2, m + 300
    sizes = rng.integers(1, 33, size=(B, C))
    offs = [np.concatenate([[0], np.cumsum(sizes[b])]).astype(np.int32) for b in range(B)]
    N = int(max(o[-1] for o in offs))
    offs = [np.concatenate([o[:-1], [N]]).astype(np.int32) for o in offs]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    score = np.empty((B, Hkv, c_max), dtype=np.float32)
    for b in range(B):
        for h in range(Hkv):
            role = rng.permutation(C)
            s = np.empty(C, dtype=np.float32)
            s[role[:100]] = 1000.0 + rng.standard_normal(100) * 50              # far above
            s[role[100:300]] = -1000.0 + rng.standard_normal(200) * 50          # far below
            cluster = 10.0 + np.float32(2e-6) * rng.integers(0, max(2, m // 2), size=m)     # one bin wide, with ties
            s[role[300:]] = cluster.astype(np.float32)
            score[b, h, :C] = s
    for frac in (0.25, 0.5, 0.9):
        # the 100 high chunks hold about 100 * 16.5 tokens; the budget ends part of the way into the cluster
        budget = int(100 * 16.5 + frac * m * 16.5)
        want = oracle.topk_select(score, packed, counts, 0, budget, c_max)
        got = gpu_select(L, score, packed, counts, 0, budget, c_max, N)
        for w, g, what in zip(want, got, ("sel_idx", "sel_count", "sel_tokens")):
            assert np.array_equal(w, g), f"{what} differs: m={m} budget={budget}"
        max_chunks = 100 + int(frac * m)
        want = oracle.topk_select(score, packed, counts, max_chunks, 0, c_max)
        got = gpu_select(L, score, packed, counts, max_chunks, 0, c_max, N)
        for w, g, what in zip(want, got, ("sel_idx", "sel_count", "sel_tokens")):
            assert np.array_equal(w, g), f"{what} differs: m={m} max_chunks={max_chunks}"


def test_select_kmax_caps_the_count(L, oracle):
    rng = np.random.default_rng(3)
    C, N = 200, 200 * 8
    off = gen.uniform_boundaries(N, 8)[None, :]
    score = rng.standard_normal((1, 2, C)).astype(np.float32)
    sel, cnt, tok = gpu_select(L, score, off, np.asarray([C], dtype=np.int32), 0, 0, 10, N)
    want = oracle.topk_select(score, off, [C], 10, 0, 10)
    assert np.array_equal(sel, want[0]) and np.array_equal(cnt, want[1]) and np.array_equal(tok, want[2])


# ---------------------------------------------------------------------------
# a4 attention
# ---------------------------------------------------------------------------
def gpu_attention(L, case_dtype, q, K, V, packed, counts, sel, cnt, k_max, max_tokens=0, n_splits=None):
    B, Hkv, N, D = K.shape
    Hq = q.shape[1]
    c_max = packed.shape[1] - 1
    shape = L.make_shape(B, Hq, Hkv, D, N, c_max, k_max, TDT[case_dtype])
    out = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device="cuda")
    nbytes = L.leoam_workspace_bytes(shape, max_tokens)
    if n_splits is not None:          # smallest workspace (one split) plus room for n_splits - 1 more partials
        nbytes = L.leoam_workspace_bytes(shape, 1) + (n_splits - 1) * B * Hq * (D + 2) * 4
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    L.sparse_chunk_attention_decode(shape, dev(q), dev(K), dev(V), dev(packed), dev(counts), dev(sel), dev(cnt),
                                    L.default_scale(D), out, lse, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("dtype,G", [("f32", 1), ("f32", 2), ("f32", 4), ("f32", 8), ("f16", 1), ("f16", 8), ("bf16", 4),
                                      ("bf16", 2)])
def test_attention_random_selection(L, oracle, dtype, G):
    rng = np.random.default_rng(40 + G)
    B, Hkv, N, D = 2, 2, 2500, 128
    K = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    V = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    q = torch.from_numpy(rng.standard_normal((B, Hkv * G, D)).astype(np.float32) * 1.5).to(TDT[dtype])
    packed, counts, c_max = random_boundaries(rng, B, N, (1, 5, 16, 31, 64))
    k_max = c_max
    sel = np.full((B, Hkv, k_max), -1, dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    for b in range(B):
        for h in range(Hkv):
            n = int(rng.integers(1, counts[b]))
            ids = np.sort(rng.choice(counts[b], size=n, replace=False))
            sel[b, h, :n] = ids
            cnt[b, h] = n
    cnt[1, 1] = 0                                     # one head keeps nothing
    want, want_lse = oracle.sparse_attention(q, K, V, packed, sel, cnt)
    for n_splits in (None, 1, 3, 3):      # default, one split, three splits (twice: the workspace is reusable)
        got, got_lse = gpu_attention(L, dtype, q, K, V, packed, counts, sel, cnt, k_max, n_splits=n_splits)
        assert np.abs(got - want).max() <= TOL[dtype]
        fin = np.isfinite(want_lse)
        assert np.array_equal(np.isneginf(got_lse), np.isneginf(want_lse))
        assert np.abs(got_lse[fin] - want_lse[fin]).max() <= 1e-4
        assert np.all(got[1, G:2 * G] == 0)


def test_attention_select_all_is_dense(L, oracle):
    g = torch.Generator().manual_seed(7)
    B, Hkv, G, N, D = 1, 2, 4, 1111, 128
    K = torch.randn(B, Hkv, N, D, generator=g).to(torch.bfloat16)
    V = torch.randn(B, Hkv, N, D, generator=g).to(torch.bfloat16)
    q = torch.randn(B, Hkv * G, D, generator=g).to(torch.bfloat16)
    rng = np.random.default_rng(1)
    packed, counts, c_max = random_boundaries(rng, B, N, (16, 32, 50))
    sel = np.tile(np.arange(c_max, dtype=np.int32), (B, Hkv, 1))
    cnt = np.tile(counts[:, None], (1, Hkv)).astype(np.int32)
    got, _ = gpu_attention(L, "bf16", q, K, V, packed, counts, sel, cnt, c_max)
    Kd = K.to(torch.float64).repeat_interleave(G, dim=1)
    Vd = V.to(torch.float64).repeat_interleave(G, dim=1)
    p = torch.softmax(torch.einsum("bjd,bjtd->bjt", q.to(torch.float64), Kd) / D ** 0.5, dim=-1)
    dense = torch.einsum("bjt,bjtd->bjd", p, Vd).numpy()
    assert np.abs(got - dense).max() <= TOL["bf16"]


def test_attention_ignores_bad_ids(L, oracle):
    g = torch.Generator().manual_seed(8)
    B, Hkv, N, D = 1, 1, 256, 128
    K = torch.randn(B, Hkv, N, D, generator=g)
    V = torch.randn(B, Hkv, N, D, generator=g)
    q = torch.randn(B, Hkv, D, generator=g)
    off = gen.uniform_boundaries(N, 16)[None, :]
    good = np.asarray([[[2, 5, -1, -1]]], dtype=np.int32)
    bad = np.asarray([[[2, 99, 5, -3]]], dtype=np.int32)       # ids outside [0, 16) add no tokens
    want, _ = oracle.sparse_attention(q, K, V, off, good, np.asarray([[2]], dtype=np.int32))
    got, _ = gpu_attention(L, "f32", q, K, V, off, np.asarray([16], dtype=np.int32), bad, np.asarray([[4]], dtype=np.int32), 4)
    assert np.abs(got - want).max() <= TOL["f32"]


# ---------------------------------------------------------------------------
# whole path on the paper-shaped configs
# ---------------------------------------------------------------------------
def run_path(L, case, separate=False):
    """abstract -> score -> select -> attention through the C ABI; the last two
    steps either in one call (what bench.py times) or as two calls."""
    layer = L.DecodeLayer(dev(case.K), dev(case.V), dev(case.chunk_off), dev(case.n_chunks), case.hq, case.k_max,
                          case.max_chunks, case.token_budget)
    assert L.leoam_validate_boundaries(layer.shape, layer.chunk_off, layer.n_chunks) == 0
    layer.build_abstract()
    for buf in (layer.sel_idx, layer.sel_count, layer.sel_tokens):
        buf.fill_(-7)
    layer.out.fill_(float("nan"))
    layer.lse.fill_(float("nan"))
    (layer.step_separate if separate else layer.step)(dev(case.q))
    torch.cuda.synchronize()
    return layer


def explain_score_mismatch(got, ub, ub64):
    """Which kind of score mismatch this is: the kernel and the oracle add the same exact products in
    different orders, so their float64 sums can differ in the last place and round to different floats
    only when the sum lies at a rounding midpoint of float32 (expected about once in 1e9 scores); anything
    else is an arithmetic error in the kernel."""
    bad = np.argwhere(got != ub)
    lines = [f"{len(bad)} scores differ"]
    for b, h, c in bad[:8]:
        s64, lo = float(ub64[b, h, c]), np.float32(ub64[b, h, c])
        other = np.nextafter(lo, np.float32(np.inf) if s64 > float(lo) else np.float32(-np.inf))
        mid = 0.5 * (float(lo) + float(other))
        rel = abs(s64 - mid) / max(abs(s64), 1e-300)
        kind = "float64 sum at a float32 rounding midpoint (summation order)" if rel < 1e-12 else "NOT a rounding tie: kernel error"
        lines.append(f"  (b={b}, h={h}, chunk={c}): gpu {got[b, h, c]!r} oracle {ub[b, h, c]!r} float64 sum {s64!r}: {kind}")
    return "\n".join(lines)


def explain_selection_mismatch(got_sel, sel, ub, margin):
    """On a kept-list mismatch: the oracle's margin at the cut (score of the last kept chunk minus score of the
    first one left out) per (sequence, kv head), and whether it is a near-tie (< 1e-6 of the score)."""
    lines = []
    for b, h in np.argwhere((got_sel != sel).any(axis=2))[:8]:
        kept = sel[b, h][sel[b, h] >= 0]
        ref = float(np.abs(ub[b, h, kept]).min()) if len(kept) else 0.0
        m = float(margin[b, h])
        kind = "near-tie at the cut" if m < 1e-6 * ref else "clear margin: selection error"
        only_gpu = sorted(set(got_sel[b, h][got_sel[b, h] >= 0].tolist()) - set(kept.tolist()))[:6]
        only_orc = sorted(set(kept.tolist()) - set(got_sel[b, h][got_sel[b, h] >= 0].tolist()))[:6]
        lines.append(f"  (b={b}, h={h}): cut margin {m:.3e} at |score| {ref:.3e}: {kind}; only gpu {only_gpu}, only oracle {only_orc}")
    return "kept lists differ\n" + "\n".join(lines)


def check_path(L, oracle, case, seqs=None, separate=False):
    layer = run_path(L, case, separate)
    sl = slice(None) if seqs is None else seqs
    K, V, q = case.K[sl].cpu(), case.V[sl].cpu(), case.q[sl].cpu()
    off, nc = case.chunk_off[sl].cpu(), case.n_chunks[sl].cpu()
    ab = oracle.abstract_build(K, off, nc)
    got_ab = host_f64(layer.abstract[sl])
    for b in range(ab.shape[0]):
        assert np.array_equal(got_ab[b, :, : nc[b]], ab[b, :, : nc[b]]), "abstract"
    ub, ub64 = oracle.chunk_score(q, np.nan_to_num(ab), nc, want_f64=True)
    got_ub = layer.score[sl].cpu().numpy()
    assert np.array_equal(got_ub, ub), explain_score_mismatch(got_ub, ub, ub64)
    sel, cnt, tok, margin = oracle.topk_select(ub, off, nc, case.max_chunks, case.token_budget, case.k_max, want_margin=True)
    got_sel = layer.sel_idx[sl].cpu().numpy()
    assert np.array_equal(got_sel, sel), explain_selection_mismatch(got_sel, sel, ub, margin)
    assert np.array_equal(layer.sel_count[sl].cpu().numpy(), cnt), "sel_count"
    assert np.array_equal(layer.sel_tokens[sl].cpu().numpy(), tok), "sel_tokens"
    out, lse = oracle.sparse_attention(q, K, V, off, sel, cnt)
    err = np.abs(host_f64(layer.out[sl]) - out).max()
    assert err <= TOL[case.dtype], f"attention max-abs error {err}"
    got_lse = host_f64(layer.lse[sl])
    assert np.array_equal(np.isneginf(got_lse), np.isneginf(lse)), "lse: -inf exactly where nothing is kept"
    kept = ~np.isneginf(lse)
    assert not kept.any() or np.abs(got_lse[kept] - lse[kept]).max() <= 1e-3, "lse"
    return dict(err=err, tokens=tok, margin=margin)


SEPARATE = pytest.mark.parametrize("separate", [False, True], ids=["one_call", "two_calls"])


@SEPARATE
def test_path_c0(L, oracle, separate):
    case = gen.make_case("c0")
    res = check_path(L, oracle, case, separate=separate)
    assert np.all(res["tokens"] == 512)


@SEPARATE
@pytest.mark.parametrize("layer", [0, 31])
def test_path_c1_reduced(L, oracle, layer, separate):
    case = gen.make_case("c1", layer=layer, n_ctx=8192 + 37, hq=8, hkv=8, token_budget=1024)
    check_path(L, oracle, case, separate=separate)


@SEPARATE
@pytest.mark.parametrize("layer", [0, 17, 31])
def test_path_c2_reduced(L, oracle, layer, separate):
    case = gen.make_case("c2", layer=layer, n_ctx=16384 + 5, hq=8, hkv=2, token_budget=2048)
    check_path(L, oracle, case, separate=separate)


@SEPARATE
def test_path_c3_reduced_batch(L, oracle, separate):
    case = gen.make_case("c3", layer=9, batch=3, n_ctx=8192 + 100, hq=8, hkv=2, token_budget=1024)
    check_path(L, oracle, case, separate=separate)


@pytest.mark.parametrize("seed", list(range(24)))
def test_path_random_shapes(L, oracle, seed):
    """Shapes drawn at random (seeded): workload recipe, dtype, batch, heads and group size, ragged context
    length, token budget and chunk limit, one-call or separate entry points; every step against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    config = ("c1", "c2", "c3")[int(rng.integers(3))]
    dtype = ("f32", "f16", "bf16")[int(rng.integers(3))]
    hkv = int(rng.integers(1, 4))
    g = (1, 2, 4, 8)[int(rng.integers(4))]
    batch = int(rng.integers(1, 4))
    n_ctx = int(rng.integers(300, 6000))
    budget = int(rng.integers(1, n_ctx))
    max_chunks = int(rng.integers(0, 40))           # 0: no chunk limit
    case = gen.make_case(config, layer=int(rng.integers(32)), batch=batch, n_ctx=n_ctx, hq=hkv * g, hkv=hkv, dtype=dtype,
                         token_budget=budget, max_chunks=max_chunks)
    check_path(L, oracle, case, separate=bool(rng.integers(2)))


def test_path_two_splits_per_head(L, oracle):
    """16 sequences x 8 kv heads: two workgroups per (sequence, kv head), combined through the exchange words of the
    workspace (one atomic exchange per output element); ragged context, small budget."""
    case = gen.make_case("c3", layer=20, batch=16, n_ctx=4096 + 37, hq=32, hkv=8, token_budget=768)
    check_path(L, oracle, case)
    case = gen.make_case("c3", layer=2, batch=16, n_ctx=2048 + 5, hq=16, hkv=8, token_budget=8)      # nothing fits
    layer = run_path(L, case)
    assert int(layer.sel_count.abs().sum()) == 0 and torch.all(layer.out == 0) and torch.all(torch.isneginf(layer.lse))
    assert not layer.workspace[: L.leoam_fused_control_bytes(layer.shape)].any()


@SEPARATE
def test_path_empty_selection(L, oracle, separate):
    case = gen.make_case("c2", layer=3, n_ctx=4096, hq=4, hkv=1, token_budget=8)     # every chunk has >= 16 tokens
    layer = run_path(L, case, separate)
    assert int(layer.sel_count.abs().sum()) == 0
    assert torch.all(layer.sel_idx == -1)
    assert torch.all(layer.out == 0) and torch.all(torch.isneginf(layer.lse))


@pytest.mark.parametrize("cfg,layer,separate", [("c1", 5, False), ("c2", 0, False), ("c2", 31, False), ("c2", 31, True)])
def test_path_full_size_layer(L, oracle, cfg, layer, separate):
    """One layer at the full shape of the benchmarked configuration, generated in HBM."""
    case = gen.make_case(cfg, layer=layer, device="cuda")
    check_path(L, oracle, case, separate=separate)


@pytest.mark.parametrize("layer", [30, 0])
def test_path_c3_full_shape_sampled(L, oracle, layer):
    """Batch-16 128K layer in the launch configuration bench.py times (a deep layer with about 3K chunks
    per sequence, the first layer with about 4.5K: four and six chunks per lane in the selection); the
    oracle checks two of the sixteen sequences end to end."""
    case = gen.make_case("c3", layer=layer, device="cuda")
    check_path(L, oracle, case, seqs=slice(5, 7))


# ---------------------------------------------------------------------------
# selection + attention in one call
# ---------------------------------------------------------------------------
def gpu_select_attend(L, dtype, score, q, K, V, packed, counts, max_chunks, budget, k_max, ws=None, n_splits=None):
    B, Hkv, N, D = K.shape
    Hq = q.shape[1]
    c_max = packed.shape[1] - 1
    shape = L.make_shape(B, Hq, Hkv, D, N, c_max, k_max, TDT[dtype])
    sel = torch.full((B, Hkv, k_max), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((B, Hkv), -7, dtype=torch.int32, device="cuda")
    tok = torch.full((B, Hkv), -7, dtype=torch.int32, device="cuda")
    out = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device="cuda")
    if ws is None:
        nbytes = L.leoam_fused_workspace_bytes(shape, budget)
        head = L.leoam_fused_control_bytes(shape)
        if n_splits is not None:      # control words + room for exactly n_splits partials
            nbytes = head + n_splits * B * Hq * (D + 2) * 4
        ws = torch.empty((nbytes + 15) // 16 * 16, dtype=torch.uint8, device="cuda")
        L.leoam_workspace_init(ws)
        ws[head:] = 0xFF               # the partials area needs no initialisation: poison it (NaN patterns)
    L.chunk_select_attention_decode(shape, dev(score), dev(q), dev(K), dev(V), dev(packed), dev(counts), max_chunks,
                                    budget, L.default_scale(D), sel, cnt, tok, out, lse, ws)
    torch.cuda.synchronize()
    return (sel.cpu().numpy(), cnt.cpu().numpy(), tok.cpu().numpy(), out.cpu().numpy().astype(np.float64),
            lse.cpu().numpy().astype(np.float64), ws)


@pytest.mark.parametrize("dtype,G,C", [("bf16", 4, 700), ("bf16", 4, 3000), ("f16", 1, 1500), ("f16", 2, 6000),
                                       ("bf16", 2, 300), ("bf16", 1, 40), ("f16", 4, 2047), ("bf16", 4, 4500), ("bf16", 4, 7000),
                                       ("bf16", 8, 900), ("f16", 8, 3000), ("bf16", 8, 5000), ("f32", 2, 900),
                                       ("f32", 4, 1300)])
                                       # (the last five: shapes that take two launches)
def test_select_attention_one_call(L, oracle, dtype, G, C):
    rng = np.random.default_rng(1000 + C + G)
    B, Hkv, D = 2, 2, 128
    offs = []
    for b in range(B):
        n = C if b == 0 else max(1, C - int(rng.integers(0, C // 3 + 1)))
        sizes = rng.integers(1, 9, size=n)
        offs.append(np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32))
    N = int(max(o[-1] for o in offs))
    offs = [np.concatenate([o[:-1], [N]]).astype(np.int32) for o in offs]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    K = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    V = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    q = torch.from_numpy(rng.standard_normal((B, Hkv * G, D)).astype(np.float32) * 1.5).to(TDT[dtype])
    score = (rng.standard_normal((B, Hkv, c_max)) * 20).astype(np.float32)
    score[:, :, ::5] = np.round(score[:, :, ::5])              # some exact ties
    k_max = min(c_max, 2048)
    ws = None
    for max_chunks, budget, n_splits in ((0, N // 8, None), (0, N // 8, 1), (0, N // 3, 3), (0, N // 3, 3),
                                         (max(1, C // 9), 0, 5), (0, 1, None), (0, 0, 2), (1, 0, 2)):
        # the library caps the count at k_max; the oracle takes that cap as max_chunks
        cap = min(max_chunks, k_max) if max_chunks > 0 else k_max
        want_sel, want_cnt, want_tok = oracle.topk_select(score, packed, counts, cap, budget, k_max)
        want_out, want_lse = oracle.sparse_attention(q, K, V, packed, want_sel, want_cnt)
        sel, cnt, tok, out, lse, ws_used = gpu_select_attend(L, dtype, score, q, K, V, packed, counts, max_chunks, budget,
                                                             k_max, n_splits=n_splits)
        tag = f"max_chunks={max_chunks} budget={budget} splits={n_splits}"
        assert np.array_equal(cnt, want_cnt), tag
        assert np.array_equal(sel, want_sel), tag
        assert np.array_equal(tok, want_tok), tag
        assert np.abs(out - want_out).max() <= TOL[dtype], tag
        fin = np.isfinite(want_lse)
        assert np.array_equal(np.isneginf(lse), np.isneginf(want_lse)), tag
        assert np.abs(lse[fin] - want_lse[fin]).max() <= 1e-4 if fin.any() else True
        if ws is None:
            ws = ws_used
    # the same workspace serves call after call without being cleared again, and the result does not
    # depend on which workgroup happens to merge: bit-identical from call to call
    want_sel, want_cnt, want_tok = oracle.topk_select(score, packed, counts, 0, N // 8, k_max)
    want_out, _ = oracle.sparse_attention(q, K, V, packed, want_sel, want_cnt)
    first = None
    for _ in range(4):
        sel, cnt, tok, out, lse, _ = gpu_select_attend(L, dtype, score, q, K, V, packed, counts, 0, N // 8, k_max, ws=ws)
        assert np.array_equal(sel, want_sel) and np.abs(out - want_out).max() <= TOL[dtype]
        first = (out, lse) if first is None else first
        assert np.array_equal(out, first[0]) and np.array_equal(lse, first[1])
    head = L.leoam_fused_control_bytes(L.make_shape(B, Hkv * G, Hkv, D, N, c_max, k_max, TDT[dtype]))
    assert int(ws[:head].to(torch.int32).sum()) == 0           # control words are back at zero


@pytest.mark.parametrize("dtype,G,C", [("bf16", 4, 700), ("bf16", 4, 3000), ("f16", 1, 1500), ("f16", 2, 2047), ("bf16", 2, 40),
                                       ("bf16", 8, 900), ("f32", 2, 900)])
                                       # (the last two: shapes that take the separate attention kernels)
def test_one_call_with_a_given_selection(L, oracle, dtype, G, C):
    """chunk_select_attention_decode with score_ub = NULL: the kept lists are inputs (unsorted, with ids out of
    range and an empty list among them) and the call only attends; against the oracle, for every number of
    splits, and bit-identical from call to call on one workspace."""
    rng = np.random.default_rng(2000 + C + G)
    B, Hkv, D = 2, 2, 128
    offs = []
    for b in range(B):
        n = C if b == 0 else max(2, C - int(rng.integers(0, C // 3 + 1)))
        sizes = rng.integers(1, 9, size=n)
        offs.append(np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32))
    N = int(max(o[-1] for o in offs))
    offs = [np.concatenate([o[:-1], [N]]).astype(np.int32) for o in offs]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    K = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    V = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    q = torch.from_numpy(rng.standard_normal((B, Hkv * G, D)).astype(np.float32) * 1.5).to(TDT[dtype])
    k_max = min(c_max, 2048)
    sel = np.full((B, Hkv, k_max), -1, dtype=np.int32)
    cnt = np.zeros((B, Hkv), dtype=np.int32)
    for b in range(B):
        for h in range(Hkv):
            n = int(rng.integers(1, min(counts[b], k_max)))
            sel[b, h, :n] = rng.permutation(counts[b])[:n]           # any order
            cnt[b, h] = n
    cnt[1, 1] = 0                                     # one head keeps nothing
    clean_sel = sel.copy()
    sel[0, 0, 3] = counts[0] + 5                      # ids outside [0, n_chunks) contribute no tokens
    sel[0, 1, 0] = -4
    for bad in ((0, 0, 3), (0, 1, 0)):
        clean_sel[bad] = -1
    # the oracle takes the list without the bad ids (kept order, shorter count)
    osel = np.full_like(sel, -1)
    ocnt = cnt.copy()
    for b in range(B):
        for h in range(Hkv):
            ids = [i for i in clean_sel[b, h, : cnt[b, h]] if i >= 0]
            osel[b, h, : len(ids)] = ids
            ocnt[b, h] = len(ids)
    want, want_lse = oracle.sparse_attention(q, K, V, packed, osel, ocnt)
    shape = L.make_shape(B, Hkv * G, Hkv, D, N, c_max, k_max, TDT[dtype])
    dq, dK, dV, doff, dnc = dev(q), dev(K), dev(V), dev(packed), dev(counts)
    dsel, dcnt = dev(sel), dev(cnt)
    tok = torch.full((B, Hkv), -7, dtype=torch.int32, device="cuda")
    head = L.leoam_fused_control_bytes(shape)
    for n_splits in (None, 1, 2, 5):
        nbytes = L.leoam_fused_workspace_bytes(shape, 0)
        if n_splits is not None:
            nbytes = max(head + n_splits * B * Hkv * G * (D + 2) * 4, head + 16)
            if dtype == "f32" or G == 8:
                nbytes = max(nbytes, L.leoam_fused_workspace_bytes(shape, 1))
        ws = torch.empty((nbytes + 15) // 16 * 16, dtype=torch.uint8, device="cuda")
        L.leoam_workspace_init(ws)
        ws[head:] = 0xFF
        first = None
        for _ in range(3):
            out = torch.full((B, Hkv * G, D), float("nan"), dtype=torch.float32, device="cuda")
            lse = torch.full((B, Hkv * G), float("nan"), dtype=torch.float32, device="cuda")
            L.chunk_select_attention_decode(shape, None, dq, dK, dV, doff, dnc, 0, 0, L.default_scale(D), dsel, dcnt, tok,
                                            out, lse, ws)
            torch.cuda.synchronize()
            got, got_lse = out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
            assert np.abs(got - want).max() <= TOL[dtype], f"splits={n_splits}"
            fin = np.isfinite(want_lse)
            assert np.array_equal(np.isneginf(got_lse), np.isneginf(want_lse))
            assert np.abs(got_lse[fin] - want_lse[fin]).max() <= 1e-4
            assert np.all(got[1, G:2 * G] == 0)
            first = (got, got_lse) if first is None else first
            assert np.array_equal(got, first[0]) and np.array_equal(got_lse, first[1])
        assert int(ws[:head].to(torch.int32).sum()) == 0           # counters are back at zero
    assert torch.equal(dsel, dev(sel)) and torch.equal(dcnt, dev(cnt)) and int(tok.min()) == -7      # inputs untouched


def test_stream_ordered_merge_switch(L, tmp_path):
    """LEOAM_STREAM_ORDERED_MERGE=1 (read once per process, so a child process) makes the one-call entry point run
    the selection, attention and merge kernels back to back: same kept lists bit for bit, outputs within float
    rounding of a different split of the kept tokens."""
    import os
    import subprocess
    import sys
    code = r"""
import sys, numpy as np, torch
sys.path.insert(0, sys.argv[1])
import gen, paper_2506_20187_amd as L
case = gen.make_case("c3", layer=9, batch=3, n_ctx=8192 + 100, hq=8, hkv=2, token_budget=1024, device="cuda")
lay = L.DecodeLayer(case.K, case.V, case.chunk_off, case.n_chunks, case.hq, case.k_max, case.max_chunks, case.token_budget)
lay.build_abstract()
lay.step(case.q)
torch.cuda.synchronize()
np.savez(sys.argv[2], sel=lay.sel_idx.cpu().numpy(), cnt=lay.sel_count.cpu().numpy(), tok=lay.sel_tokens.cpu().numpy(),
         out=lay.out.cpu().numpy(), lse=lay.lse.cpu().numpy())
"""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = {}
    for tag, val in (("in_launch", "0"), ("stream_ordered", "1")):
        path = str(tmp_path / f"{tag}.npz")
        env = dict(os.environ, LEOAM_STREAM_ORDERED_MERGE=val)
        subprocess.run([sys.executable, "-c", code, root, path], check=True, env=env, timeout=300)
        res[tag] = np.load(path)
    a, b = res["in_launch"], res["stream_ordered"]
    for k in ("sel", "cnt", "tok"):
        assert np.array_equal(a[k], b[k]), k
    assert np.abs(a["out"] - b["out"]).max() <= 1e-4 and np.abs(a["lse"] - b["lse"]).max() <= 1e-4


# ---------------------------------------------------------------------------
# tree-structured chunk refinement (Sec. 4.2)
# ---------------------------------------------------------------------------
def gpu_tree_refine(L, dtype, q, K, cs, k, max_rounds, cap):
    B, Hkv, N, D = K.shape
    Hq = q.shape[1]
    m0 = -(-N // cs)
    off0 = np.minimum(np.arange(m0 + 1, dtype=np.int64) * cs, N).astype(np.int32)
    packed = np.tile(off0, (B, 1))
    counts = np.full(B, m0, dtype=np.int32)
    shape = L.make_shape(B, Hq, Hkv, D, N, m0, 1, TDT[dtype])
    ab = torch.empty(B, Hkv, m0, 2, D, dtype=TDT[dtype], device="cuda")
    L.kv_chunk_abstract_build(shape, dev(K), dev(packed), dev(counts), ab)
    r_off = torch.full((B, Hkv, cap + 1), -7, dtype=torch.int32, device="cuda")
    r_score = torch.full((B, Hkv, cap), float("nan"), dtype=torch.float32, device="cuda")
    r_cnt = torch.full((B, Hkv), -7, dtype=torch.int32, device="cuda")
    r_ev, r_st = torch.full_like(r_cnt, -7), torch.full_like(r_cnt, -7)
    ws = torch.empty(L.leoam_tree_workspace_bytes(shape, cap), dtype=torch.uint8, device="cuda")
    L.chunk_tree_refine(shape, dev(q), dev(K), ab, cs, k, max_rounds, cap, r_off, r_score, r_cnt, r_ev, r_st, ws)
    torch.cuda.synchronize()
    return r_off, r_score, r_cnt, r_ev.cpu().numpy(), r_st.cpu().numpy()


def check_tree(L, oracle, dtype, q, K, cs, k, max_rounds, cap):
    want_off, want_score, want_cnt, want_ev, want_st = oracle.tree_refine(q, K, cs, k, max_rounds, cap)
    r_off, r_score, r_cnt, ev, st = gpu_tree_refine(L, dtype, q, K, cs, k, max_rounds, cap)
    tag = f"cs={cs} k={k} rounds={max_rounds} cap={cap}"
    assert np.array_equal(st, want_st), tag
    assert np.array_equal(r_cnt.cpu().numpy(), want_cnt), tag
    assert np.array_equal(ev, want_ev), tag
    got_off, got_score = r_off.cpu().numpy(), r_score.cpu().numpy()
    B, Hkv = want_cnt.shape
    for b in range(B):
        for h in range(Hkv):
            n = want_cnt[b, h]
            assert np.array_equal(got_off[b, h, : n + 1], want_off[b, h, : n + 1]), tag
            assert np.array_equal(got_score[b, h, :n], want_score[b, h, :n]), tag
    return r_off, r_score, r_cnt, want_ev


@pytest.mark.parametrize("dtype,G,N,cs", [("f32", 1, 256, 16), ("bf16", 4, 1024, 64), ("f16", 2, 300, 32), ("bf16", 1, 2500, 64),
                                          ("f16", 8, 512, 8)])
def test_tree_refine_exact(L, oracle, dtype, G, N, cs):
    rng = np.random.default_rng(N + G)
    B, Hkv, D = 2, 3, 128
    K = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(TDT[dtype])
    q = torch.from_numpy(rng.standard_normal((B, Hkv * G, D)).astype(np.float32)).to(TDT[dtype])
    for k, rounds, cap in ((N // 10, 10 ** 6, N), (1, 10 ** 6, N), (N // 3, 2, N), (N // 10, 0, N), (N, 5, N),
                           (N // 4, 10 ** 6, -(-N // cs) + 5)):
        check_tree(L, oracle, dtype, q, K, cs, max(1, k), rounds, cap)


@pytest.mark.parametrize("seed", list(range(16)))
def test_tree_refine_random_shapes(L, oracle, seed):
    """Shapes and data drawn at random (seeded): dtype, group size, ragged context, initial chunk size, k, round limit,
    node capacity (sometimes too small: reported), Gaussian keys / hot runs in a desert / small-integer keys with
    massive ties."""
    rng = np.random.default_rng(5000 + seed)
    dtype = ("f32", "f16", "bf16")[int(rng.integers(3))]
    G = (1, 2, 4, 8)[int(rng.integers(4))]
    B, Hkv, D = int(rng.integers(1, 3)), int(rng.integers(1, 3)), 128
    N = int(rng.integers(40, 3000))
    cs = (4, 8, 16, 32, 64)[int(rng.integers(5))]
    m0 = -(-N // cs)
    k = int(rng.integers(1, N + 1)) if rng.integers(4) else int(rng.integers(1, max(2, N // 20)))
    rounds = (0, 1, 3, 10 ** 6)[int(rng.integers(4))]
    cap = max(m0, m0 + int(rng.integers(0, N)) if rng.integers(3) else N)
    kind = int(rng.integers(3))
    g = torch.Generator().manual_seed(seed)
    if kind == 0:
        K = torch.randn(B, Hkv, N, D, generator=g)
    elif kind == 1:
        K = torch.randn(B, Hkv, N, D, generator=g) * 0.1
    else:
        K = torch.randint(-2, 3, (B, Hkv, N, D), generator=g).float()
    q = torch.randn(B, Hkv * G, D, generator=g)
    if kind == 1:
        for b in range(B):
            for h in range(Hkv):
                for s0 in rng.integers(0, max(1, N - 20), size=4):
                    K[b, h, s0:s0 + int(rng.integers(1, 20))] += 5.0 * (q[b, h * G] / q[b, h * G].norm())
    if kind == 2:
        q = torch.randint(-2, 3, (B, Hkv * G, D), generator=g).float()
    check_tree(L, oracle, dtype, q.to(TDT[dtype]), K.to(TDT[dtype]), cs, k, rounds, cap)


def test_tree_refine_ties_and_deserts(L, oracle):
    # all tokens equal: the complete tree, ties resolved by index
    K = torch.ones(1, 2, 64, 128)
    q = torch.ones(1, 2, 128)
    check_tree(L, oracle, "f32", q, K, 8, 5, 100, 64)
    check_tree(L, oracle, "f32", q, K, 8, 5, 100, 20)          # node_cap too small: reported, partition still valid
    # clusters of important tokens in a desert
    g = torch.Generator().manual_seed(9)
    N, cs, D = 4096, 64, 128
    K = (torch.randn(1, 1, N, D, generator=g) * 0.1)
    q = torch.randn(1, 1, D, generator=g)
    hot = np.concatenate([np.arange(s, s + 24) for s in (100, 1500, 1540, 3000, 4000)])
    K[0, 0, hot] += 6.0 * (q[0, 0] / q[0, 0].norm())
    K, q = K.to(torch.bfloat16), q.to(torch.bfloat16)
    _, _, _, ev = check_tree(L, oracle, "bf16", q, K, cs, len(hot), 10 ** 6, 512)
    assert ev[0, 0] < N // 8


def test_tree_refine_full_context(L, oracle):
    """128K tokens per head, chunks of 64, k = 4096 (the shape bench.py times): planted runs, and Gaussian keys
    with a round limit (the tree then stops unfinished, which must match too)."""
    K, q, hot = gen.make_desert_keys(1, 2, 4, 131072, clusters=128, cluster_len=(32, 32), dtype="bf16", device="cuda")
    K, q = K.cpu(), q.cpu()
    _, _, r_cnt, ev = check_tree(L, oracle, "bf16", q, K, 64, 4096, 64, 32768)
    assert np.all(r_cnt.cpu().numpy() == 257) and np.all(ev < 131072 // 8)
    case = gen.make_case("c2", layer=20, hkv=1, hq=4)
    check_tree(L, oracle, "bf16", case.q, case.K, 64, 4096, 12, 32768)


def test_tree_refine_feeds_selection_and_attention(L, oracle):
    """refine -> chunk_topk_select with a budget of k tokens -> attention, read as batch * n_kv_heads
    sequences of one kv head: the attention runs over exactly the k most important tokens."""
    rng = np.random.default_rng(31)
    B, Hkv, G, N, D, cs, k = 2, 2, 4, 2048, 128, 64, 200
    K = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(torch.bfloat16)
    V = torch.from_numpy(rng.standard_normal((B, Hkv, N, D)).astype(np.float32)).to(torch.bfloat16)
    q = torch.from_numpy(rng.standard_normal((B, Hkv * G, D)).astype(np.float32)).to(torch.bfloat16)
    cap = N                   # random keys have no deserts: the tree grows close to single tokens
    r_off, r_score, r_cnt, _ = check_tree(L, oracle, "bf16", q, K, cs, k, 10 ** 6, cap)
    shape = L.make_shape(B * Hkv, G, 1, D, N, cap, cap, torch.bfloat16)
    sel = torch.empty(B * Hkv, 1, cap, dtype=torch.int32, device="cuda")
    cnt = torch.empty(B * Hkv, 1, dtype=torch.int32, device="cuda")
    tok = torch.empty_like(cnt)
    out = torch.empty(B * Hkv, G, D, dtype=torch.float32, device="cuda")
    ws = torch.empty(L.leoam_fused_workspace_bytes(shape, k), dtype=torch.uint8, device="cuda")
    L.leoam_workspace_init(ws)
    L.chunk_select_attention_decode(shape, r_score.view(B * Hkv, 1, cap), dev(q), dev(K), dev(V), r_off.view(B * Hkv, cap + 1),
                                    r_cnt.view(B * Hkv), 0, k, L.default_scale(D), sel, cnt, tok, out, None, ws)
    torch.cuda.synchronize()
    assert torch.all(tok == k)
    # token-level reference: softmax attention over the k most important tokens of every (b, kv head)
    Kd, Vd, qd = K.double(), V.double(), q.double().view(B, Hkv, G, D)
    logits = torch.einsum("bhgd,bhtd->bhgt", qd, Kd)
    imp = logits.max(dim=2).values.float()
    want = torch.empty(B, Hkv, G, D, dtype=torch.float64)
    for b in range(B):
        for h in range(Hkv):
            order = np.lexsort((np.arange(N), -imp[b, h].double().numpy()))[:k]
            idx = torch.from_numpy(np.sort(order))
            p = torch.softmax(logits[b, h][:, idx] / D ** 0.5, dim=-1)
            want[b, h] = p @ Vd[b, h, idx]
    assert np.abs(host_f64(out).reshape(B, Hkv, G, D) - want.numpy()).max() <= TOL["bf16"]


# ---------------------------------------------------------------------------
# error paths (host-visible faults are refused before any launch)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("sink,tail", [(0, 0), (1, 1), (4, 2), (10000, 0), (0, 10000)])
def test_score_pin_exact_and_selection(L, oracle, sink, tail):
    """chunk_score_pin against the oracle on ragged sequence lengths, and the selection that follows it."""
    rng = np.random.default_rng(sink * 7 + tail)
    B, Hkv, c_max, N = 3, 2, 1500, 24000
    nc = np.array([1500, 700, 3], dtype=np.int32)
    off = np.zeros((B, c_max + 1), dtype=np.int32)
    for b in range(B):
        cuts = np.sort(rng.choice(np.arange(1, N), size=nc[b] - 1, replace=False))
        off[b, 1:nc[b]] = cuts
        off[b, nc[b]:] = N
    score = rng.standard_normal((B, Hkv, c_max)).astype(np.float32)
    shape = L.make_shape(B, Hkv, Hkv, 128, N, c_max, c_max, torch.float16)
    d_score, d_nc, d_off = torch.from_numpy(score).cuda(), torch.from_numpy(nc).cuda(), torch.from_numpy(off).cuda()
    L.chunk_score_pin(shape, d_nc, sink, tail, d_score)
    torch.cuda.synchronize()
    want = oracle.score_pin(score, nc, sink, tail)
    assert np.array_equal(d_score.cpu().numpy(), want)
    sel = torch.empty(B, Hkv, c_max, dtype=torch.int32, device="cuda")
    cnt = torch.empty(B, Hkv, dtype=torch.int32, device="cuda")
    tok = torch.empty_like(cnt)
    L.chunk_topk_select(shape, d_score, d_off, d_nc, 0, 2048, sel, cnt, tok)
    torch.cuda.synchronize()
    osel, ocnt, otok = oracle.topk_select(want, off, nc, 0, 2048, c_max)
    assert np.array_equal(sel.cpu().numpy(), osel) and np.array_equal(cnt.cpu().numpy(), ocnt)
    assert np.array_equal(tok.cpu().numpy(), otok)


def test_error_codes(L):
    t = torch.zeros(16, device="cuda")
    ok = L.make_shape(1, 8, 8, 128, 64, 4, 4, torch.float32)
    for bad, code in ((L.make_shape(1, 8, 8, 64, 64, 4, 4, torch.float32), -3),
                      (L.make_shape(1, 9, 8, 128, 64, 4, 4, torch.float32), -1),
                      (L.make_shape(1, 24, 8, 128, 64, 4, 4, torch.float32), -3),
                      (L.make_shape(1, 8, 8, 128, 64, 4, 5, torch.float32), -1),
                      (L.make_shape(1, 8, 8, 128, 64, 20000, 4, torch.float32), -3),
                      (L.make_shape(0, 8, 8, 128, 64, 4, 4, torch.float32), -1)):
        with pytest.raises(L.LeoamError) as e:
            L.chunk_score(bad, t, t, t, t)
        assert e.value.status == code
    with pytest.raises(L.LeoamError) as e:
        L.chunk_score(ok, None, t, t, t)
    assert e.value.status == -1
    with pytest.raises(L.LeoamError) as e:
        L.sparse_chunk_attention_decode(ok, t, t, t, t, t, t, t, 1.0, t, None, torch.zeros(8, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -4
    off = torch.tensor([[0, 10, 5, 64, 64]], dtype=torch.int32, device="cuda")
    assert L.leoam_validate_boundaries(ok, off, torch.tensor([3], dtype=torch.int32, device="cuda")) == -2
    torch.cuda.synchronize()
