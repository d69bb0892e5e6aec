"""Pins for the oracle's compressed-store functions (Sec. 4.4 compression, Sec. 6.1 INT4).

The oracle works on stored codes; these tests tie it to things that are not the
oracle: a numpy dequantisation written here, numpy's own float16 rounding, the
dense oracle functions applied to the dequantised values, and the rounding bound
of an affine quantiser.
"""
import numpy as np
import pytest
import torch

import gen


def small_store(seed=0, B=2, Hkv=2, N=150, share=0.5):
    rng = np.random.default_rng(seed)
    g = torch.Generator().manual_seed(seed)
    K = torch.randn(B, Hkv, N, 128, generator=g) * 1.7
    V = torch.randn(B, Hkv, N, 128, generator=g)
    offs = [gen.make_boundaries(N, rng, sizes=(1, 4, 9, 16)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    fb = rng.random((B, c_max)) < share
    kb, vb, qm = gen.quantize_store(K, V, packed, counts, fb)
    return K, V, packed, counts, c_max, fb, kb, vb, qm


def numpy_dequant(blob, qm_words, packed, counts, N, which):
    """Independent decoding of the byte layout described in include/leoam.h."""
    blob = blob.numpy()
    w = qm_words.numpy()
    B, Hkv, c_max, _ = w.shape
    out = np.zeros((B, Hkv, N, 128))
    for b in range(B):
        for h in range(Hkv):
            for c in range(counts[b]):
                rec = w[b, h, c]
                byte_off = int(rec[0:2].view(np.int64)[0])
                bits = int(rec[2])
                f = rec[3:7].view(np.float32).astype(np.float64)
                s, z = (f[0], f[1]) if which == "k" else (f[2], f[3])
                t0, t1 = packed[b, c], packed[b, c + 1]
                n = t1 - t0
                if bits == 8:
                    codes = blob[byte_off: byte_off + n * 128].reshape(n, 128).astype(np.float64)
                else:
                    raw = blob[byte_off: byte_off + n * 64].reshape(n, 64)
                    codes = np.empty((n, 128))
                    codes[:, 0::2] = raw & 15
                    codes[:, 1::2] = raw >> 4
                out[b, h, t0:t1] = s * codes + z
    return out


def test_dequant_matches_layout_and_rounding_bound(oracle):
    K, V, packed, counts, c_max, fb, kb, vb, qm = small_store()
    N = K.shape[2]
    for which, X, blob in (("k", K, kb), ("v", V, vb)):
        got = oracle.dequant(blob, qm, packed, counts, N, 128, which)
        assert np.array_equal(got, numpy_dequant(blob, qm, packed, counts, N, which))
        # an affine quantiser with rounding is within half a step of the value it stores
        meta = qm.numpy().view(oracle.QCHUNK_DTYPE).reshape(qm.shape[:3])
        scale = meta["scale_" + which].astype(np.float64)
        err = np.abs(got - X.numpy().astype(np.float64))
        for b in range(K.shape[0]):
            for c in range(counts[b]):
                seg = err[b, :, packed[b, c]:packed[b, c + 1]].max(axis=(1, 2))
                assert np.all(seg <= scale[b, :, c] / 2 * (1 + 1e-6) + 1e-7)
    assert set(np.unique(meta["bits"][:, :, : counts.min()])) <= {4, 8}


def test_outward_rounding_to_half(oracle):
    rng = np.random.default_rng(1)
    xs = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-9, 5, 2000), [0.0, 1.0, -1.0, 65504.0, 65505.0,
                         -65505.0, 6e-8, -6e-8, 1e-12]])
    halves = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float64)
    halves = np.sort(halves[np.isfinite(halves)])
    for x in xs:
        up, down = oracle.half_ceil(float(x)), oracle.half_floor(float(x))
        # brute force over every finite half
        ge = halves[halves >= x]
        le = halves[halves <= x]
        assert up == (ge[0] if ge.size else np.inf)
        assert down == (le[-1] if le.size else -np.inf)
        assert down <= x <= up


def test_quant_abstract_is_outward_rounded_abstract_of_stored_values(oracle):
    K, V, packed, counts, c_max, fb, kb, vb, qm = small_store(seed=2)
    N = K.shape[2]
    stored = oracle.dequant(kb, qm, packed, counts, N, 128, "k")           # float64 stored values
    exact = oracle.abstract_build(stored, packed, counts)                   # dense abstract of them (pinned elsewhere)
    got = oracle.abstract_build_q(kb, qm, packed, counts)
    for b in range(K.shape[0]):
        n = counts[b]
        kmax, kmin = got[b, :, :n, 0], got[b, :, :n, 1]
        assert np.all(kmax >= exact[b, :, :n, 0]) and np.all(kmin <= exact[b, :, :n, 1])
        # representable in binary16 and no further than one half step away
        assert np.array_equal(kmax.astype(np.float16).astype(np.float64), kmax)
        assert np.array_equal(kmin.astype(np.float16).astype(np.float64), kmin)
        near = exact[b, :, :n, 0].astype(np.float16).astype(np.float64)     # numpy's round-to-nearest
        step = np.spacing(np.abs(near).astype(np.float16)).astype(np.float64)
        assert np.all(kmax - exact[b, :, :n, 0] <= step)
    # the bound property survives: score from the fp16 abstract encloses every stored key
    g = torch.Generator().manual_seed(5)
    q = torch.randn(K.shape[0], 4, 128, generator=g).to(torch.float16)
    ub, lb, ub64, lb64 = oracle.chunk_score(q, np.nan_to_num(got), counts, want_lower=True, want_f64=True)
    logits = np.einsum("bhgd,bhtd->bhgt", q.to(torch.float64).numpy().reshape(K.shape[0], 2, 2, 128), stored)
    for b in range(K.shape[0]):
        for c in range(counts[b]):
            seg = logits[b, :, :, packed[b, c]:packed[b, c + 1]]
            assert np.all(ub64[b, :, c] >= seg.max(axis=(1, 2)) - 1e-9)
            assert np.all(lb64[b, :, c] <= seg.min(axis=(1, 2)) + 1e-9)


def test_quant_attention_equals_dense_attention_on_stored_values(oracle):
    K, V, packed, counts, c_max, fb, kb, vb, qm = small_store(seed=3)
    N = K.shape[2]
    g = torch.Generator().manual_seed(6)
    q = torch.randn(K.shape[0], 4, 128, generator=g).to(torch.float16)
    rng = np.random.default_rng(3)
    sel = np.full((K.shape[0], 2, c_max), -1, dtype=np.int32)
    cnt = np.zeros((K.shape[0], 2), dtype=np.int32)
    for b in range(K.shape[0]):
        for h in range(2):
            n = int(rng.integers(1, counts[b]))
            sel[b, h, :n] = np.sort(rng.choice(counts[b], size=n, replace=False))
            cnt[b, h] = n
    cnt[0, 1] = 0
    got, got_lse = oracle.sparse_attention_q(q, kb, vb, qm, packed, sel, cnt)
    Ks = oracle.dequant(kb, qm, packed, counts, N, 128, "k")
    Vs = oracle.dequant(vb, qm, packed, counts, N, 128, "v")
    want, want_lse = oracle.sparse_attention(q.to(torch.float64).numpy(), Ks, Vs, packed, sel, cnt)
    assert np.allclose(got, want, rtol=0, atol=1e-12)
    assert np.array_equal(np.isneginf(got_lse), np.isneginf(want_lse))
    fin = np.isfinite(want_lse)
    assert np.allclose(got_lse[fin], want_lse[fin], rtol=0, atol=1e-12)
