"""CPU pins of the oracle's abstract maintenance (Sec. 4.3 abstract under token-by-token decoding,
Sec. 2.1) and of the evaluation-count formula of Sec. 4.2 "Dynamic chunk resizing"."""
import numpy as np
import pytest
import torch


def brute_abstract(K, off, nc):
    """numpy max / min over the tokens of every chunk, written from the definition."""
    Kd = K.to(torch.float64).numpy()
    B, H, N, D = Kd.shape
    out = np.full((B, H, off.shape[1] - 1, 2, D), np.nan)
    for b in range(B):
        for c in range(nc[b]):
            seg = Kd[b, :, off[b, c]:off[b, c + 1], :]
            out[b, :, c, 0] = seg.max(axis=1)
            out[b, :, c, 1] = seg.min(axis=1)
    return out


def same(a, b):
    return np.array_equal(np.nan_to_num(a, nan=-12345.0), np.nan_to_num(b, nan=-12345.0))


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
def test_append_equals_rebuild(oracle, dtype):
    g = torch.Generator().manual_seed(11)
    B, H, N, D, cs, c_max = 2, 3, 200, 128, 16, 20
    K = torch.randn(B, H, N, D, generator=g).to(dtype)
    # sequence 0 starts empty, sequence 1 starts with three ragged chunks (the last one longer than cs)
    off = np.zeros((B, c_max + 1), dtype=np.int32)
    nc = np.asarray([0, 3], dtype=np.int32)
    off[1, :4] = [0, 5, 12, 12 + 23]
    ab = brute_abstract(K, off, nc)
    lens = [0, 35]
    for step in range(70):
        off, nc, ab, st = oracle.abstract_append(K, off, nc, cs, ab)
        assert np.all(st == 0)
        lens = [x + 1 for x in lens]
        for b in range(B):
            assert off[b, nc[b]] == lens[b]
        assert same(ab, brute_abstract(K, off, nc)), f"step {step}"
    # closed form of the boundaries: sequence 0 is cut every cs tokens; sequence 1 opened a new chunk at once
    assert list(off[0, :nc[0] + 1]) == [0, 16, 32, 48, 64, 70]
    assert list(off[1, :nc[1] + 1]) == [0, 5, 12, 35, 51, 67, 83, 99, 105]
    # and the library routine agrees on the final state
    assert same(ab, oracle.abstract_build(K, off, nc, full=False))


def test_append_capacity_limits(oracle):
    g = torch.Generator().manual_seed(12)
    B, H, N, D, cs, c_max = 3, 2, 12, 128, 4, 3
    K = torch.randn(B, H, N, D, generator=g)
    off = np.zeros((B, c_max + 1), dtype=np.int32)
    off[0, :4] = [0, 4, 8, 12]          # full cache
    off[1, :4] = [0, 4, 8, 11]          # room in the last chunk
    off[2, :4] = [0, 2, 6, 10]          # last chunk full and no chunk slot left
    nc = np.asarray([3, 3, 3], dtype=np.int32)
    ab = brute_abstract(K, off, nc)
    off2, nc2, ab2, st = oracle.abstract_append(K, off, nc, cs, ab)
    assert list(st) == [1, 0, 2]
    assert np.array_equal(off2[0], off[0]) and np.array_equal(off2[2], off[2]) and list(nc2) == [3, 3, 3]
    assert list(off2[1, :4]) == [0, 4, 8, 12]
    assert same(ab2[0], ab[0]) and same(ab2[2], ab[2])
    assert same(ab2, brute_abstract(K, off2, nc2))


def test_append_one_token_chunks(oracle):
    """chunk_size 1: every token is its own chunk, kmax == kmin == the key."""
    g = torch.Generator().manual_seed(13)
    K = torch.randn(1, 1, 6, 128, generator=g)
    off = np.zeros((1, 7), dtype=np.int32)
    nc = np.zeros(1, dtype=np.int32)
    ab = np.full((1, 1, 6, 2, 128), np.nan)
    for _ in range(6):
        off, nc, ab, st = oracle.abstract_append(K, off, nc, 1, ab)
    assert list(off[0]) == [0, 1, 2, 3, 4, 5, 6] and nc[0] == 6
    assert np.array_equal(ab[0, 0, :, 0], K[0, 0].double().numpy()) and np.array_equal(ab[0, 0, :, 1], K[0, 0].double().numpy())


# ---------------------------------------------------------------------------
# Sec. 4.2 "Dynamic chunk resizing": f(m) = m * sum_{i=0}^{log2(n/m)-1} (2 rho)^i
# ---------------------------------------------------------------------------
def test_tree_evaluations_closed_forms(oracle):
    for n, m in ((32, 8), (4096, 64), (131072, 2048), (64, 64), (64, 1)):
        L = int(np.log2(n // m))
        assert oracle.tree_evaluations(n, m, 0.0) == (m if L > 0 else 0)      # nothing is ever split
        assert oracle.tree_evaluations(n, m, 0.5) == m * L                    # every term is 1
        for rho in (0.1, 0.2, 0.37, 0.8, 1.0):
            r = 2 * rho
            geo = L if r == 1.0 else (1 - r ** L) / (1 - r)                   # geometric series
            assert oracle.tree_evaluations(n, m, rho) == pytest.approx(m * geo, rel=1e-12)
    # full refinement (rho = 1) of n tokens in chunks of s costs m (s - 1) = n - m evaluations
    assert oracle.tree_evaluations(1024, 16, 1.0) == 1024 - 16
    # the worked example of Sec. 4.2 (32 tokens, 8 chunks of 4, 20 % important): between the 8 evaluations of
    # fixed chunks and the 32 of token-level management, and next to the 12 the paper counts for its tree
    f = oracle.tree_evaluations(32, 8, 0.2)
    assert 8 < f < 32 and abs(f - 12) < 1


def test_library_tree_evaluations_matches(oracle):
    import paper_2506_20187_amd as L
    for n, m, rho in ((32, 8, 0.2), (4096, 64, 0.1), (131072, 2048, 0.5), (64, 64, 0.3), (1 << 20, 1 << 14, 0.9)):
        assert L.leoam_tree_evaluations(n, m, rho) == pytest.approx(oracle.tree_evaluations(n, m, rho), rel=1e-13)
    for n, m, rho in ((32, 0, 0.2), (32, 64, 0.2), (30, 4, 0.2), (96, 8, 0.2), (32, 8, -0.1), (32, 8, 1.5)):
        assert L.leoam_tree_evaluations(n, m, rho) == -1.0
