"""Pins for the oracle's abstract (Sec. 4.3) and chunk bounds (Sec. 4.1, 4.3).

Every check compares the oracle with something that is not the oracle: a
numpy reduction written here, a brute-force dot product over the tokens, a
closed form, or a number the paper prints (tests/golden/paper_values.txt).
"""
import os

import numpy as np
import pytest
import torch

import gen

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def paper_values():
    out = {}
    with open(GOLD) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = [s.strip() for s in line.split("=")]
            out[k] = float(v)
    return out


def rand_case(rng, B=2, Hkv=3, G=2, N=97, D=16, dtype=np.float32, sizes=(1, 2, 5, 8, 13)):
    K = rng.standard_normal((B, Hkv, N, D)).astype(dtype)
    q = rng.standard_normal((B, Hkv * G, D)).astype(dtype)
    offs = []
    for _ in range(B):
        off = [0]
        while off[-1] < N:
            off.append(min(N, off[-1] + int(rng.choice(sizes))))
        offs.append(np.asarray(off, dtype=np.int32))
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    return K, q, packed, counts, c_max


def brute_abstract(K, packed, counts):
    B, Hkv, N, D = K.shape
    c_max = packed.shape[1] - 1
    out = np.full((B, Hkv, c_max, 2, D), np.nan)
    for b in range(B):
        for c in range(counts[b]):
            seg = K[b, :, packed[b, c]:packed[b, c + 1], :].astype(np.float64)
            out[b, :, c, 0, :] = seg.max(axis=1)
            out[b, :, c, 1, :] = seg.min(axis=1)
    return out


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_abstract_equals_bruteforce(oracle, dtype):
    rng = np.random.default_rng(1)
    K, q, packed, counts, c_max = rand_case(rng, dtype=dtype)
    got = oracle.abstract_build(K, packed, counts)
    want = brute_abstract(K, packed, counts)
    assert np.array_equal(got, want, equal_nan=True)
    # abstract values are stored key values: representable in the key dtype
    fin = got[np.isfinite(got)]
    assert np.array_equal(fin.astype(dtype).astype(np.float64), fin)


def test_abstract_bf16_and_half_widening(oracle):
    # every fp16 and bf16 bit pattern widens to the value torch gives
    bits = np.arange(65536, dtype=np.uint16)
    for tdt in (torch.float16, torch.bfloat16):
        t = torch.from_numpy(bits.view(np.int16).copy()).view(tdt)
        got = oracle.widen(t)
        want = t.to(torch.float64).numpy()
        assert np.array_equal(got, want, equal_nan=True)
    K = torch.randn(1, 2, 40, 8, dtype=torch.float32).to(torch.bfloat16)
    off = gen.uniform_boundaries(40, 7)[None, :]
    got = oracle.abstract_build(K, off, [len(off[0]) - 1])
    want = brute_abstract(K.to(torch.float64).numpy(), off, [len(off[0]) - 1])
    assert np.array_equal(got, want)


def test_abstract_merge_law(oracle):
    # abstract of the union of two neighbours = elementwise max / min of theirs
    rng = np.random.default_rng(2)
    K = rng.standard_normal((1, 2, 64, 8)).astype(np.float32)
    fine = gen.uniform_boundaries(64, 4)[None, :]
    coarse = gen.uniform_boundaries(64, 8)[None, :]
    a_f = oracle.abstract_build(K, fine, [16])
    a_c = oracle.abstract_build(K, coarse, [8])
    assert np.array_equal(a_c[:, :, :, 0], np.maximum(a_f[:, :, 0::2, 0], a_f[:, :, 1::2, 0]))
    assert np.array_equal(a_c[:, :, :, 1], np.minimum(a_f[:, :, 0::2, 1], a_f[:, :, 1::2, 1]))


def test_boundaries_must_tile(oracle):
    K = np.zeros((1, 1, 10, 4), dtype=np.float32)
    for bad in ([0, 4, 9], [1, 5, 10], [0, 5, 5, 10], [0, 6, 4, 10]):
        with pytest.raises(ValueError):
            oracle.abstract_build(K, np.asarray([bad], dtype=np.int32), [len(bad) - 1])


def test_abstract_size_matches_paper(oracle):
    pv = paper_values()
    # Sec. 6.5: chunk 64 -> abstracts are 1/64 of K+V, under the printed 1.6 %
    s = int(pv["abstract_chunk_size"])
    N, D = 256, 8
    K = np.zeros((1, 1, N, D), dtype=np.float16)
    off = gen.uniform_boundaries(N, s)[None, :]
    ab = oracle.abstract_build(K, off, [N // s])
    abstract_elems = ab.size                      # 2 key vectors per chunk
    kv_elems = 2 * K.size                         # K and V
    assert abstract_elems / kv_elems == pv["abstract_overhead_exact"] == 1.0 / s
    assert abstract_elems / kv_elems < pv["abstract_overhead_bound"]
    # Sec. 4.3: against the keys alone the abstract is 2/n' of the volume
    n1 = int(pv["lka_chunk_size"])
    off = gen.uniform_boundaries(N, n1)[None, :]
    ab = oracle.abstract_build(K, off, [N // n1])
    assert ab.size / K.size == 2.0 / n1
    assert pv["lka_alpha"] + ab.size / K.size == pytest.approx(pv["lka_fraction_formula"], abs=0)


def test_evaluation_counts_of_worked_example(oracle):
    # Sec. 4.2 example: one bound evaluation per chunk (8) vs per token (32)
    pv = paper_values()
    N, s = int(pv["example_tokens"]), int(pv["example_chunk_size"])
    rng = np.random.default_rng(3)
    K = rng.standard_normal((1, 1, N, 8)).astype(np.float32)
    q = rng.standard_normal((1, 1, 8)).astype(np.float32)
    for size, want in ((s, pv["example_chunk_evaluations"]), (1, pv["example_token_evaluations"])):
        off = gen.uniform_boundaries(N, size)[None, :]
        n = off.shape[1] - 1
        ub = oracle.chunk_score(q, oracle.abstract_build(K, off, [n]), [n])
        assert np.isfinite(ub).sum() == want
    assert N // s == pv["example_chunks"]
    assert int(0.2 * N) == pv["example_important_tokens"]


def token_logits(K, q, G):
    """Brute force q.k per (b, q head, token), float64, written with einsum."""
    B, Hkv, N, D = K.shape
    Kd = K.astype(np.float64)
    qd = q.astype(np.float64).reshape(B, Hkv, G, D)
    return np.einsum("bhgd,bhtd->bhgt", qd, Kd)


@pytest.mark.parametrize("G", [1, 4])
def test_bounds_enclose_every_token(oracle, G):
    rng = np.random.default_rng(4)
    K, q, packed, counts, c_max = rand_case(rng, G=G)
    ab = oracle.abstract_build(K, packed, counts)
    ub, lb, ub64, lb64 = oracle.chunk_score(q, ab, counts, want_lower=True, want_f64=True)
    z = token_logits(K, q, G)
    B, Hkv = K.shape[:2]
    tight = 0
    for b in range(B):
        for c in range(counts[b]):
            seg = z[b, :, :, packed[b, c]:packed[b, c + 1]]          # [Hkv,G,s]
            hi = seg.max(axis=(1, 2))
            lo = seg.min(axis=(1, 2))
            assert np.all(ub64[b, :, c] >= hi - 1e-12)
            assert np.all(lb64[b, :, c] <= lo + 1e-12)
            if packed[b, c + 1] - packed[b, c] == 1:
                # one token: the bounds are the dot product itself (per head), so
                # the group score is the max / min over the group's heads
                assert np.allclose(ub64[b, :, c], hi, rtol=0, atol=1e-12)
                assert np.allclose(lb64[b, :, c], lo, rtol=0, atol=1e-12)
                tight += 1
        assert np.all(np.isneginf(ub[b, :, counts[b]:]))
    assert tight > 0
    assert np.array_equal(ub, ub64.astype(np.float32))
    assert np.array_equal(lb, lb64.astype(np.float32))


def test_single_token_chunks_reduce_to_gemv(oracle):
    # s_c = 1 everywhere, one head per group: U = L = K q, a library mat-vec
    rng = np.random.default_rng(5)
    N, D = 50, 32
    K = rng.standard_normal((1, 2, N, D)).astype(np.float32)
    q = rng.standard_normal((1, 2, D)).astype(np.float32)
    off = gen.uniform_boundaries(N, 1)[None, :]
    ab = oracle.abstract_build(K, off, [N])
    ub, lb, ub64, lb64 = oracle.chunk_score(q, ab, [N], want_lower=True, want_f64=True)
    for h in range(2):
        ref = K[0, h].astype(np.float64) @ q[0, h].astype(np.float64)
        assert np.allclose(ub64[0, h], ref, rtol=0, atol=1e-12)
        assert np.allclose(lb64[0, h], ref, rtol=0, atol=1e-12)


def test_sign_special_cases_and_width_identity(oracle):
    rng = np.random.default_rng(6)
    K, q, packed, counts, c_max = rand_case(rng, B=1, Hkv=2, G=1, N=60, D=8)
    ab = oracle.abstract_build(K, packed, counts)
    n = counts[0]
    kmax, kmin = ab[0, :, :n, 0, :], ab[0, :, :n, 1, :]
    qpos = np.abs(q)
    ub64 = oracle.chunk_score(qpos, ab, counts, want_f64=True)[1]
    assert np.allclose(ub64[0, :, :n], np.einsum("hd,hcd->hc", qpos[0].astype(np.float64), kmax), atol=1e-12)
    ub64 = oracle.chunk_score(-qpos, ab, counts, want_f64=True)[1]
    assert np.allclose(ub64[0, :, :n], np.einsum("hd,hcd->hc", -qpos[0].astype(np.float64), kmin), atol=1e-12)
    # U - L = sum_d |q_d| (kmax_d - kmin_d)
    _, _, ub64, lb64 = oracle.chunk_score(q, ab, counts, want_lower=True, want_f64=True)
    width = np.einsum("hd,hcd->hc", np.abs(q[0]).astype(np.float64), kmax - kmin)
    assert np.allclose((ub64 - lb64)[0, :, :n], width, atol=1e-10)


def test_parent_bound_dominates_children(oracle):
    # merging two chunks can only raise the upper bound and lower the lower one
    rng = np.random.default_rng(7)
    K = rng.standard_normal((1, 2, 64, 16)).astype(np.float32)
    q = rng.standard_normal((1, 4, 16)).astype(np.float32)
    fine = gen.uniform_boundaries(64, 4)[None, :]
    coarse = gen.uniform_boundaries(64, 8)[None, :]
    uf, lf = oracle.chunk_score(q, oracle.abstract_build(K, fine, [16]), [16], want_lower=True)
    uc, lc = oracle.chunk_score(q, oracle.abstract_build(K, coarse, [8]), [8], want_lower=True)
    assert np.all(uc >= np.maximum(uf[:, :, 0::2], uf[:, :, 1::2]))
    assert np.all(lc <= np.minimum(lf[:, :, 0::2], lf[:, :, 1::2]))


def test_group_score_is_max_over_group(oracle):
    rng = np.random.default_rng(8)
    K, q, packed, counts, c_max = rand_case(rng, B=1, Hkv=2, G=4, N=40, D=8)
    ab = oracle.abstract_build(K, packed, counts)
    grouped = oracle.chunk_score(q, ab, counts, want_f64=True)[1]
    per_head = []
    for g in range(4):
        qg = q.reshape(1, 2, 4, 8)[:, :, g, :]
        per_head.append(oracle.chunk_score(np.ascontiguousarray(qg), ab, counts, want_f64=True)[1])
    assert np.array_equal(grouped, np.maximum.reduce(per_head))


def test_negative_zero_score_is_canonical(oracle):
    K = np.zeros((1, 1, 4, 4), dtype=np.float32)
    q = -np.ones((1, 1, 4), dtype=np.float32)
    off = gen.uniform_boundaries(4, 2)[None, :]
    ub = oracle.chunk_score(q, oracle.abstract_build(K, off, [2]), [2])
    assert not np.signbit(ub).any()
