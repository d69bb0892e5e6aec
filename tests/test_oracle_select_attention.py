"""Pins for the oracle's selection (Sec. 4.2, 6.1) and sparse attention (Eq. 1).

Selection is checked against a repeated-argmax brute force written here, against
textbook top-k in the uniform-size case and against closed-form special cases.
Attention is checked against dense softmax attention computed with torch in
float64, and against invariances that follow from Eq. (1).
"""
import numpy as np
import pytest
import torch

import gen


def brute_select(score_row, sizes, max_chunks, budget):
    """Repeatedly take the largest remaining score (lowest index on ties)
    while both limits hold; stop at the first chunk that does not fit."""
    s = np.asarray(score_row, dtype=np.float64).copy()
    kept, tokens = [], 0
    for _ in range(len(s)):
        c = int(np.argmax(s))            # first occurrence = lowest index
        if max_chunks > 0 and len(kept) + 1 > max_chunks:
            break
        if budget > 0 and tokens + sizes[c] > budget:
            break
        kept.append(c)
        tokens += int(sizes[c])
        s[c] = -np.inf
    return sorted(kept), tokens


@pytest.mark.parametrize("seed", range(6))
def test_select_equals_repeated_argmax(oracle, seed):
    rng = np.random.default_rng(seed)
    B, Hkv = 2, 3
    offs = []
    for _ in range(B):
        sizes = rng.integers(1, 9, size=int(rng.integers(5, 30)))
        offs.append(np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32))
    N = 10_000
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    # few distinct values -> many ties
    score = rng.integers(-2, 3, size=(B, Hkv, c_max)).astype(np.float32)
    for max_chunks, budget in ((0, 20), (4, 0), (5, 17), (0, 0), (1, 1)):
        sel, cnt, tok = oracle.topk_select(score, packed, counts, max_chunks, budget, c_max)
        for b in range(B):
            sizes = np.diff(offs[b])
            for h in range(Hkv):
                want, wtok = brute_select(score[b, h, : counts[b]], sizes, max_chunks, budget)
                assert list(sel[b, h, : cnt[b, h]]) == want
                assert np.all(sel[b, h, cnt[b, h]:] == -1)
                assert tok[b, h] == wtok


def test_select_special_cases(oracle):
    C, s = 40, 8
    off = gen.uniform_boundaries(C * s, s)[None, :]
    rng = np.random.default_rng(11)
    score = rng.standard_normal((1, 2, C)).astype(np.float32)
    # uniform size: exactly min(max_chunks, budget // s) chunks = textbook top-k
    for max_chunks, budget in ((7, 0), (0, 50), (3, 50), (9, 50)):
        k = min(x for x in (max_chunks if max_chunks > 0 else C, budget // s if budget > 0 else C))
        sel, cnt, tok = oracle.topk_select(score, off, [C], max_chunks, budget, C)
        for h in range(2):
            want = np.sort(torch.topk(torch.from_numpy(score[0, h]), k).indices.numpy())
            assert cnt[0, h] == k and tok[0, h] == k * s
            assert np.array_equal(sel[0, h, :k], want)
    # all scores equal: chunks 0,1,2,... until the budget is reached
    flat = np.zeros((1, 1, C), dtype=np.float32)
    sel, cnt, tok = oracle.topk_select(flat, off, [C], 0, 5 * s + 3, C)
    assert cnt[0, 0] == 5 and list(sel[0, 0, :5]) == [0, 1, 2, 3, 4]
    # budget >= N: everything
    sel, cnt, tok = oracle.topk_select(score, off, [C], 0, C * s, C)
    assert np.all(cnt == C) and np.array_equal(sel[0, 0], np.arange(C)) and np.all(tok == C * s)
    # first chunk alone exceeds the budget: nothing
    sel, cnt, tok = oracle.topk_select(score, off, [C], 0, s - 1, C)
    assert np.all(cnt == 0) and np.all(sel == -1) and np.all(tok == 0)
    # -0.0 and +0.0 tie: lowest index first
    z = np.asarray([[[0.0, -0.0, 0.0, -1.0]]], dtype=np.float32)
    o4 = gen.uniform_boundaries(4, 1)[None, :]
    sel, cnt, tok = oracle.topk_select(z, o4, [4], 2, 0, 4)
    assert list(sel[0, 0, :2]) == [0, 1]
    with pytest.raises(ValueError):
        oracle.topk_select(score, off, [C], 0, 0, 3)


def test_prefix_rule_stops_at_first_misfit(oracle):
    # order by score: sizes 4, 10, 2 with budget 8 -> only the first fits; the
    # small third chunk is NOT taken after the misfit
    off = np.asarray([[0, 4, 14, 16]], dtype=np.int32)
    score = np.asarray([[[3.0, 2.0, 1.0]]], dtype=np.float32)
    sel, cnt, tok = oracle.topk_select(score, off, [3], 0, 8, 3)
    assert cnt[0, 0] == 1 and tok[0, 0] == 4 and sel[0, 0, 0] == 0


def dense_reference(q, K, V, G, token_mask=None):
    """softmax(q K^T / sqrt(d)) V with torch float64 library ops."""
    qd = torch.as_tensor(q).to(torch.float64)
    Kd = torch.as_tensor(K).to(torch.float64).repeat_interleave(G, dim=1)
    Vd = torch.as_tensor(V).to(torch.float64).repeat_interleave(G, dim=1)
    z = torch.einsum("bjd,bjtd->bjt", qd, Kd) / Kd.shape[-1] ** 0.5
    if token_mask is not None:
        z = z.masked_fill(~torch.as_tensor(token_mask)[:, None, :].repeat_interleave(1, dim=1), float("-inf"))
    p = torch.softmax(z, dim=-1)
    return torch.einsum("bjt,bjtd->bjd", p, Vd).numpy(), torch.logsumexp(z, dim=-1).numpy(), p.numpy()


@pytest.mark.parametrize("G,dtype", [(1, torch.float32), (4, torch.bfloat16), (2, torch.float16)])
def test_select_all_is_dense_attention(oracle, G, dtype):
    g = torch.Generator().manual_seed(3)
    B, Hkv, N, D = 2, 2, 77, 16
    K = torch.randn(B, Hkv, N, D, generator=g).to(dtype)
    V = torch.randn(B, Hkv, N, D, generator=g).to(dtype)
    q = torch.randn(B, Hkv * G, D, generator=g).to(dtype)
    rng = np.random.default_rng(0)
    offs = [gen.make_boundaries(N, rng, sizes=(3, 5, 8)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    sel = np.tile(np.arange(c_max, dtype=np.int32), (B, Hkv, 1))
    cnt = np.tile(counts[:, None], (1, Hkv)).astype(np.int32)
    out, lse = oracle.sparse_attention(q, K, V, packed, sel, cnt)
    ref, ref_lse, _ = dense_reference(q, K, V, G)
    assert np.allclose(out, ref, rtol=0, atol=1e-12)
    assert np.allclose(lse, ref_lse, rtol=0, atol=1e-12)


def test_partial_selection_matches_masked_dense(oracle):
    g = torch.Generator().manual_seed(4)
    B, Hkv, G, N, D = 1, 2, 2, 64, 8
    K = torch.randn(B, Hkv, N, D, generator=g)
    V = torch.randn(B, Hkv, N, D, generator=g)
    q = torch.randn(B, Hkv * G, D, generator=g)
    off = np.asarray([[0, 5, 9, 20, 33, 40, 64]], dtype=np.int32)
    sel = np.asarray([[[1, 3, 4, -1], [0, 5, -1, -1]]], dtype=np.int32)
    cnt = np.asarray([[3, 2]], dtype=np.int32)
    out, lse = oracle.sparse_attention(q, K, V, off, sel, cnt)
    for h in range(Hkv):
        mask = np.zeros((1, N), dtype=bool)
        for c in sel[0, h, : cnt[0, h]]:
            mask[0, off[0, c]:off[0, c + 1]] = True
        ref, ref_lse, _ = dense_reference(q[:, h * G:(h + 1) * G], K[:, h:h + 1], V[:, h:h + 1], G, mask)
        assert np.allclose(out[:, h * G:(h + 1) * G], ref, atol=1e-12)
        assert np.allclose(lse[:, h * G:(h + 1) * G], ref_lse, atol=1e-12)


def test_attention_invariances(oracle):
    g = torch.Generator().manual_seed(5)
    B, Hkv, G, N, D = 1, 1, 2, 48, 8
    K = torch.randn(B, Hkv, N, D, generator=g)
    V = torch.randn(B, Hkv, N, D, generator=g)
    q = torch.randn(B, Hkv * G, D, generator=g)
    off = gen.uniform_boundaries(N, 8)[None, :]
    sel = np.asarray([[[1, 2, 4]]], dtype=np.int32)
    cnt = np.asarray([[3]], dtype=np.int32)
    base, base_lse = oracle.sparse_attention(q, K, V, off, sel, cnt)
    # order of the kept chunks does not matter
    out, _ = oracle.sparse_attention(q, K, V, off, sel[:, :, ::-1].copy(), cnt)
    assert np.allclose(out, base, atol=1e-13)
    # cutting every chunk in two and keeping both halves changes nothing
    off2 = gen.uniform_boundaries(N, 4)[None, :]
    sel2 = np.asarray([[[2, 3, 4, 5, 8, 9]]], dtype=np.int32)
    out, lse = oracle.sparse_attention(q, K, V, off2, sel2, np.asarray([[6]], dtype=np.int32))
    assert np.allclose(out, base, atol=1e-13) and np.allclose(lse, base_lse, atol=1e-13)
    # a single one-token chunk returns that token's value row
    off1 = gen.uniform_boundaries(N, 1)[None, :]
    out, lse = oracle.sparse_attention(q, K, V, off1, np.asarray([[[17]]], dtype=np.int32), np.asarray([[1]], dtype=np.int32))
    assert np.array_equal(out[0, 0], V[0, 0, 17].to(torch.float64).numpy())
    assert np.array_equal(out[0, 1], V[0, 0, 17].to(torch.float64).numpy())
    # adding a constant to every kept logit (keys shifted along q) moves lse only
    qv = q[0, 0].to(torch.float64)
    K2 = K.to(torch.float64) + 0.25 * qv / (qv @ qv) * D ** 0.5
    out, lse = oracle.sparse_attention(q[:, :1], K2.numpy(), V.to(torch.float64).numpy(), off, sel, cnt)
    assert np.allclose(out[0, 0], base[0, 0], atol=1e-12)
    assert np.allclose(lse[0, 0], base_lse[0, 0] + 0.25, atol=1e-12)
    # nothing kept
    out, lse = oracle.sparse_attention(q, K, V, off, sel, np.asarray([[0]], dtype=np.int32))
    assert np.all(out == 0) and np.all(np.isneginf(lse))


def test_c0_planted_chunks_are_selected_and_output_is_near_dense(oracle):
    case = gen.make_case("c0")
    res = oracle.decode_step(case.q, case.K, case.V, case.chunk_off, case.n_chunks,
                             case.max_chunks, case.token_budget, case.k_max)
    planted_chunks = sorted(set(int(t) // 32 for t in case.planted))
    assert len(planted_chunks) == 16
    # the recipe's precondition: every planted token's true logit beats the
    # loose bound of every chunk without a planted token
    Kd = case.K.to(torch.float64).numpy()
    qd = case.q.to(torch.float64).numpy()
    logits = np.einsum("bhd,bhtd->bht", qd, Kd)
    noise = np.ones(case.c_max, dtype=bool)
    noise[planted_chunks] = False
    assert logits[0][:, case.planted].min(axis=1).min() > res["score"][0][:, noise].max()
    for h in range(case.hkv):
        assert list(res["sel_idx"][0, h]) == planted_chunks
    assert np.all(res["sel_count"] == 16) and np.all(res["sel_tokens"] == 512)
    # closeness to dense attention: |sparse - dense| <= 2 (1 - mu) max|V| with
    # mu the dense softmax mass on the kept tokens
    ref, _, p = dense_reference(case.q, case.K, case.V, 1)
    kept = np.zeros(case.n_ctx, dtype=bool)
    for c in planted_chunks:
        kept[c * 32:(c + 1) * 32] = True
    mu = p[0][:, kept].sum(axis=1)
    vmax = float(case.V.abs().max())
    err = np.abs(res["out"] - ref)[0].max(axis=1)
    assert np.all(err <= 2 * (1 - mu) * vmax + 1e-12)
    assert mu.min() > 0.999


def test_generated_boundaries_tile_the_context():
    rng = np.random.default_rng(9)
    for kw in (dict(sizes=(16, 32, 64, 128)), dict(size_range=(16, 256)), dict(size_range=(32, 512))):
        for n in (4096, 5000, 1 << 15):
            heavy = rng.random(n) < 0.1
            off = gen.make_boundaries(n, rng, heavy=heavy, depth=0.7, **kw)
            assert off[0] == 0 and off[-1] == n and np.all(np.diff(off) > 0)
            lo = min(kw.get("sizes", kw.get("size_range")))
            hi = max(kw.get("sizes", kw.get("size_range")))
            sizes = np.diff(off)
            assert sizes.max() <= hi and np.all(sizes[:-1][sizes[:-1] < lo] >= 0)
