"""CPU pins of the oracle's tree-structured chunk refinement (Sec. 4.2, Fig. 9): the refined
partition, read through the ordinary selection with a budget of k tokens, must give the k most
important tokens of a token-level evaluation; evaluation counts follow closed forms."""
import numpy as np
import pytest
import torch

FMAX = np.float32(3.402823466e+38)


def importance(q, K, G):
    """float32( max over the group's heads of q_j.k_t ), the double sum rounded once: [B,Hkv,N]"""
    Kd, qd = K.to(torch.float64), q.to(torch.float64)
    B, Hkv, N, D = Kd.shape
    z = torch.einsum("bhgd,bhtd->bhgt", qd.view(B, Hkv, G, D), Kd)
    return (z.max(dim=2).values.numpy().astype(np.float32) + np.float32(0.0))


def brute_topk(imp, k):
    """token-level top-k, ties to the lower index: boolean [B,Hkv,N]"""
    B, H, N = imp.shape
    out = np.zeros((B, H, N), dtype=bool)
    for b in range(B):
        for h in range(H):
            order = np.lexsort((np.arange(N), -imp[b, h].astype(np.float64)))
            out[b, h, order[:k]] = True
    return out


def selected_tokens(oracle, off, score, cnt, N, k):
    """tokens of the chunks the ordinary selection keeps from the refined partition with a budget of k"""
    B, H, cap = score.shape
    sel, n_sel, tok = oracle.topk_select(score.reshape(B * H, 1, cap), off.reshape(B * H, cap + 1), cnt.reshape(B * H), 0, k, cap)
    out = np.zeros((B * H, N), dtype=bool)
    o = off.reshape(B * H, cap + 1)
    for i in range(B * H):
        for c in sel[i, 0, : n_sel[i, 0]]:
            out[i, o[i, c]:o[i, c + 1]] = True
    return out.reshape(B, H, N), tok.reshape(B, H)


def check_partition(off, cnt, N):
    for row, n in zip(off.reshape(-1, off.shape[-1]), cnt.reshape(-1)):
        r = row[: n + 1]
        assert r[0] == 0 and r[-1] == N and np.all(np.diff(r) > 0)


@pytest.mark.parametrize("dtype,G,N,cs,k", [(torch.float32, 1, 256, 16, 20), (torch.bfloat16, 4, 512, 64, 51),
                                             (torch.float16, 2, 300, 32, 7), (torch.float32, 1, 128, 8, 128),
                                             (torch.bfloat16, 1, 1024, 64, 1), (torch.float32, 4, 1000, 16, 333)])
def test_refined_selection_is_token_level_topk(oracle, dtype, G, N, cs, k):
    g = torch.Generator().manual_seed(N + k)
    B, Hkv, D = 2, 2, 128
    K = torch.randn(B, Hkv, N, D, generator=g).to(dtype)
    q = torch.randn(B, Hkv * G, D, generator=g).to(dtype)
    off, score, cnt, evals, status = oracle.tree_refine(q, K, cs, k, 10 ** 6, N)
    assert np.all(status == 0)
    check_partition(off, cnt, N)
    want = brute_topk(importance(q, K, G), k)
    got, tok = selected_tokens(oracle, off, score, cnt, N, k)
    assert np.array_equal(got, want)
    assert np.all(tok == k)
    m0 = -(-N // cs)
    assert np.all(evals >= m0) and np.all((evals - m0) % 2 == 0) and np.all(evals <= 2 * N - m0)
    # without ties the confirmed chunks are the runs of important tokens and the chunk count is that of the run-length code
    for b in range(B):
        for h in range(Hkv):
            n = cnt[b, h]
            confirmed = score[b, h, :n] == FMAX
            if k == N:
                assert n == 1 and confirmed[0]
                continue
            runs = 1 + int(np.count_nonzero(np.diff(want[b, h].astype(np.int8))))
            marks = np.zeros(N, dtype=bool)
            for c in np.nonzero(confirmed)[0]:
                marks[off[b, h, c]:off[b, h, c + 1]] = True
            assert np.array_equal(marks, want[b, h])
            assert n >= runs          # unimportant single tokens next to an important one may stay apart from their desert


def test_worked_example_shape(oracle):
    """32 tokens, 8 chunks of 4, 6 important tokens: all four of the last chunk, one in chunk 0, one in chunk 2
    (the situation of the Sec. 4.2 example).  Importance = key channel 0, so the bounds are the chunk's max / min."""
    N = 32
    vals = np.linspace(0.1, 1.0, N)
    np.random.default_rng(0).shuffle(vals)
    vals[28:32] = [10, 11, 12, 13]
    vals[1], vals[9] = 5, 6
    K = torch.zeros(1, 1, N, 128)
    K[0, 0, :, 0] = torch.from_numpy(vals).float()
    q = torch.zeros(1, 1, 128)
    q[0, 0, 0] = 1
    off, score, cnt, evals, status = oracle.tree_refine(q, K, 4, 6, 100, 64)
    n = cnt[0, 0]
    assert list(off[0, 0, : n + 1]) == [0, 1, 2, 9, 10, 28, 32]
    assert list(score[0, 0, :n] == FMAX) == [False, True, False, True, False, True]      # important sizes 1, 1, 4
    # 8 initial evaluations; isolating one token of a chunk of 4 takes two binary splits = 4 evaluations, twice
    assert evals[0, 0] == 8 + 4 + 4
    assert 8 < evals[0, 0] < 32        # between fixed chunks and token-level management
    got, _ = selected_tokens(oracle, off, score, cnt, N, 6)
    assert sorted(np.nonzero(got[0, 0])[0]) == [1, 9, 28, 29, 30, 31]
    # fixed chunks of 4 with the same budget would also take the 3 unimportant neighbours of tokens 1 and 9
    off0, score0, cnt0, evals0, _ = oracle.tree_refine(q, K, 4, 6, 0, 64)
    assert evals0[0, 0] == 8


def test_all_equal_tokens_build_the_complete_tree(oracle):
    N, cs, k = 64, 8, 5
    K = torch.ones(1, 1, N, 128)
    q = torch.ones(1, 1, 128)
    off, score, cnt, evals, status = oracle.tree_refine(q, K, cs, k, 100, N)
    m0 = N // cs
    assert evals[0, 0] == m0 + 2 * (N - m0)            # every chunk is split down to single tokens
    assert cnt[0, 0] == N
    got, _ = selected_tokens(oracle, off, score, cnt, N, k)
    assert list(np.nonzero(got[0, 0])[0]) == [0, 1, 2, 3, 4]     # ties go to the lowest indices


def test_no_rounds_is_the_chunk_level_evaluation(oracle):
    g = torch.Generator().manual_seed(3)
    B, Hkv, N, D, cs = 1, 2, 256, 128, 16
    K = torch.randn(B, Hkv, N, D, generator=g)
    q = torch.randn(B, Hkv, D, generator=g)
    off, score, cnt, evals, status = oracle.tree_refine(q, K, cs, 40, 0, 64)
    assert np.all(evals == N // cs)
    boundaries = np.arange(0, N + 1, cs, dtype=np.int32)[None, :]
    ab = oracle.abstract_build(K, boundaries, [N // cs])
    ub = oracle.chunk_score(q, ab, [N // cs])
    # every chunk of the output is a run of initial chunks and carries the largest upper bound of the run
    for h in range(Hkv):
        n = cnt[0, h]
        assert np.all(off[0, h, : n + 1] % cs == 0)
        for c in range(n):
            lo, hi = off[0, h, c] // cs, off[0, h, c + 1] // cs
            if score[0, h, c] != FMAX:
                assert score[0, h, c] == ub[0, h, lo:hi].max()


def test_sparse_inputs_need_fewer_evaluations_than_tokens(oracle):
    """A few clusters of important tokens in a desert (Sec. 3.5): far fewer evaluations than one per token."""
    g = torch.Generator().manual_seed(9)
    N, cs, D = 4096, 64, 128
    K = torch.randn(1, 1, N, D, generator=g) * 0.1
    q = torch.randn(1, 1, D, generator=g)
    qn = q[0, 0] / q[0, 0].norm()
    hot = np.concatenate([np.arange(s, s + 24) for s in (100, 1500, 1540, 3000, 4000)])
    K[0, 0, hot] += 6.0 * qn
    off, score, cnt, evals, status = oracle.tree_refine(q, K, cs, len(hot), 10 ** 6, N)
    got, _ = selected_tokens(oracle, off, score, cnt, N, len(hot))
    assert sorted(np.nonzero(got[0, 0])[0]) == sorted(hot)
    assert evals[0, 0] < N // 8
    assert cnt[0, 0] < 40


def test_node_cap_overflow_is_reported(oracle):
    K = torch.ones(1, 1, 64, 128)
    q = torch.ones(1, 1, 128)
    off, score, cnt, evals, status = oracle.tree_refine(q, K, 8, 5, 100, 20)      # the complete tree needs 64 nodes
    assert status[0, 0] == 1
    check_partition(off, cnt, 64)
    assert cnt[0, 0] <= 20
    with pytest.raises(ValueError):
        oracle.tree_refine(q, K, 8, 5, 100, 7)
