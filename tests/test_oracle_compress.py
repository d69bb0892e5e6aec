"""Pins for the oracle's compression step (Sec. 4.4 dynamic KV compression, Sec. 6.1 INT4).

oracle.chunk_compress builds the 8-bit / 4-bit store; these tests tie it to things
that are not that function: data that already lies on the code grid (codes, scale
and zero are then known in closed form), the rounding bound of an affine quantiser
checked through a decoder written here, ties that must round to even, a byte layout
computed by hand, and the generator's torch implementation of the same store.
oracle.compression_share is tied to the two sides of the latency condition written
out here.
"""
import numpy as np
import pytest
import torch

import gen
import oracle


def decode(blob, qm, packed, counts, N, which):
    """Independent decoding of the byte layout: value = scale * code + zero."""
    B, Hkv, c_max = qm.shape
    out = np.zeros((B, Hkv, N, 128))
    codes = np.zeros((B, Hkv, N, 128), dtype=np.int64)
    for b in range(B):
        for h in range(Hkv):
            for c in range(counts[b]):
                rec = qm[b, h, c]
                s, z = float(rec["scale_" + which]), float(rec["zero_" + which])
                t0, t1 = packed[b, c], packed[b, c + 1]
                start = int(rec["byte_off"])
                if rec["bits"] == 8:
                    cd = blob[start:start + (t1 - t0) * 128].reshape(t1 - t0, 128).astype(np.int64)
                else:
                    by = blob[start:start + (t1 - t0) * 64].reshape(t1 - t0, 64).astype(np.int64)
                    cd = np.empty((t1 - t0, 128), dtype=np.int64)
                    cd[:, 0::2] = by & 15
                    cd[:, 1::2] = by >> 4
                codes[b, h, t0:t1] = cd
                out[b, h, t0:t1] = s * cd + z
    return out, codes


def random_case(seed, dtype, B=2, Hkv=2, N=150, share=0.5):
    rng = np.random.default_rng(seed)
    g = torch.Generator().manual_seed(seed)
    K = (torch.randn(B, Hkv, N, 128, generator=g) * 1.7).to(dtype)
    V = torch.randn(B, Hkv, N, 128, generator=g).to(dtype)
    offs = [gen.make_boundaries(N, rng, sizes=(1, 4, 9, 16)) for _ in range(B)]
    packed, counts, c_max = gen.pack_boundaries(offs, N)
    fb = rng.random((B, c_max)) < share
    return K, V, packed, counts, c_max, fb


@pytest.mark.parametrize("bits", [8, 4])
def test_data_on_the_grid_gives_its_own_codes(bits):
    # x = zero + step * k, step a power of two, every k of 0..levels present: zero, scale and the codes are known
    levels = 255 if bits == 8 else 15
    rng = np.random.default_rng(bits)
    N = 24
    k = rng.integers(0, levels + 1, size=(1, 1, N, 128))
    k[0, 0, 0, 0], k[0, 0, 1, 5] = 0, levels
    step, zero = 2.0 ** -4, -3.0
    K = torch.from_numpy(zero + step * k).to(torch.float16)
    assert np.array_equal(K.double().numpy(), zero + step * k)           # representable
    V = torch.from_numpy(1.0 + 2.0 * step * k[..., ::-1].copy()).to(torch.float16)
    packed = np.array([[0, N]], dtype=np.int32)
    counts = np.array([1], dtype=np.int32)
    kb, vb, qm = oracle.chunk_compress(K, V, packed, counts, np.array([[bits == 4]]))
    rec = qm[0, 0, 0]
    assert rec["bits"] == bits and rec["byte_off"] == 0
    assert rec["scale_k"] == np.float32(step) and rec["zero_k"] == np.float32(zero)
    assert rec["scale_v"] == np.float32(2 * step) and rec["zero_v"] == np.float32(1.0)
    _, ck = decode(kb, qm, packed, counts, N, "k")
    _, cv = decode(vb, qm, packed, counts, N, "v")
    assert np.array_equal(ck, k) and np.array_equal(cv, k[..., ::-1])


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16, torch.float32])
def test_round_trip_within_half_a_step_and_extremes_exact(dtype):
    K, V, packed, counts, c_max, fb = random_case(11, dtype)
    kb, vb, qm = oracle.chunk_compress(K, V, packed, counts, fb)
    for X, blob, which in ((K, kb, "k"), (V, vb, "v")):
        x = X.double().numpy()
        deq, codes = decode(blob, qm, packed, counts, x.shape[2], which)
        for b in range(x.shape[0]):
            for h in range(x.shape[1]):
                for c in range(counts[b]):
                    t0, t1 = packed[b, c], packed[b, c + 1]
                    rec = qm[b, h, c]
                    s = float(rec["scale_" + which])
                    levels = 255 if rec["bits"] == 8 else 15
                    seg, cd = x[b, h, t0:t1], codes[b, h, t0:t1]
                    assert float(rec["zero_" + which]) == seg.min()
                    # scale is the float quotient of the float range
                    assert rec["scale_" + which] == np.float32(np.float32(seg.max()) - np.float32(seg.min())) / np.float32(levels)
                    # half a step, plus the float rounding of the quotient (x - zero) / scale <= levels
                    # (a few units of 2^-24 * levels steps) - the decision is taken in float
                    assert np.abs(deq[b, h, t0:t1] - seg).max() <= s * (0.5 + 4 * levels * 2.0 ** -24) + 1e-30
                    assert cd.min() >= 0 and cd.max() <= levels
                    assert cd[np.unravel_index(seg.argmin(), seg.shape)] == 0
                    if s > 0:
                        assert cd[np.unravel_index(seg.argmax(), seg.shape)] == levels


def test_constant_chunk_and_single_token_chunks():
    N = 6
    K = torch.full((1, 1, N, 128), 0.75, dtype=torch.float16)
    V = torch.arange(N * 128, dtype=torch.float32).reshape(1, 1, N, 128).to(torch.float16)
    packed = np.array([[0, 1, 2, 6]], dtype=np.int32)
    counts = np.array([3], dtype=np.int32)
    fb = np.array([[False, True, False]])
    kb, vb, qm = oracle.chunk_compress(K, V, packed, counts, fb)
    assert np.all(qm["scale_k"] == 0) and np.all(qm["zero_k"] == np.float32(0.75))
    dk, ck = decode(kb, qm, packed, counts, N, "k")
    assert np.all(ck == 0) and np.all(dk == 0.75)
    # a single-token 8-bit chunk of 128 consecutive integers: 127 / 255 per level
    dv, cv = decode(vb, qm, packed, counts, N, "v")
    assert np.abs(dv[0, 0, 0] - np.arange(128)).max() <= 0.5 * 127 / 255 * (1 + 1e-6)


def test_ties_round_to_even():
    # zero = 0, scale = 1: the values k + 1/2 sit exactly between two codes
    N = 2
    x = np.zeros((1, 1, N, 128))
    x[0, 0, 0, :8] = [0.5, 1.5, 2.5, 3.5, 4.5, 253.5, 254.5, 255.0]
    K = torch.from_numpy(x).to(torch.float16)
    assert np.array_equal(K.double().numpy(), x)
    packed = np.array([[0, N]], dtype=np.int32)
    kb, vb, qm = oracle.chunk_compress(K, K, packed, np.array([1], dtype=np.int32), np.array([[False]]))
    assert qm[0, 0, 0]["scale_k"] == 1.0 and qm[0, 0, 0]["zero_k"] == 0.0
    _, ck = decode(kb, qm, packed, [1], N, "k")
    assert list(ck[0, 0, 0, :8]) == [0, 2, 2, 4, 4, 254, 254, 255]


def test_byte_layout_by_hand():
    # B=2, Hkv=2; sequence 0: chunks of 3 (8-bit), 5 (4-bit), 2 (8-bit) tokens; sequence 1: one 4-bit chunk of 10, c_max 3
    N = 10
    g = torch.Generator().manual_seed(3)
    K = torch.randn(2, 2, N, 128, generator=g).to(torch.bfloat16)
    V = torch.randn(2, 2, N, 128, generator=g).to(torch.bfloat16)
    packed = np.array([[0, 3, 8, 10], [0, 10, 10, 10]], dtype=np.int32)
    counts = np.array([3, 1], dtype=np.int32)
    fb = np.array([[False, True, False], [True, False, False]])
    kb, vb, qm = oracle.chunk_compress(K, V, packed, counts, fb)
    head0 = 3 * 128 + 5 * 64 + 2 * 128                      # 960 bytes, every chunk already a multiple of 16
    assert list(qm["byte_off"][0, 0]) == [0, 384, 704]
    assert list(qm["byte_off"][0, 1]) == [head0, head0 + 384, head0 + 704]
    assert qm["byte_off"][1, 0, 0] == 2 * head0 and qm["byte_off"][1, 1, 0] == 2 * head0 + 640
    assert list(qm["bits"][0, 0]) == [8, 4, 8] and qm["bits"][1, 0, 0] == 4
    assert kb.size == vb.size == 2 * head0 + 2 * 640
    # records past n_chunks are zero
    assert not np.any(qm[1, :, 1:].view(np.uint8))
    # nibble order: channel 0 in the low nibble.  Put the chunk's max at channel 0 and its min at channel 1 of a token.
    K2 = K.clone()
    K2[1, 0, 4, 0], K2[1, 0, 4, 1] = 100.0, -100.0
    kb2, _, qm2 = oracle.chunk_compress(K2, V, packed, counts, fb)
    assert kb2[int(qm2["byte_off"][1, 0, 0]) + 4 * 64] == 0x0F


def test_total_size_and_alignment():
    # rows are 64 or 128 bytes at D = 128, so a chunk is always a multiple of 16 bytes: the blob is the plain sum
    K, V, packed, counts, c_max, fb = random_case(5, torch.float16)
    kb, vb, qm = oracle.chunk_compress(K, V, packed, counts, fb)
    sizes = np.diff(packed.astype(np.int64), axis=1)
    valid = np.arange(c_max)[None, :] < counts[:, None]
    total = int((np.where(valid, sizes * np.where(fb, 64, 128), 0).sum(axis=1) * K.shape[1]).sum())
    assert kb.size == vb.size == total
    assert np.all(qm["byte_off"] % 16 == 0)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_matches_the_generators_torch_implementation(dtype):
    K, V, packed, counts, c_max, fb = random_case(21, dtype, B=2, Hkv=3, N=130)
    kb, vb, qm = oracle.chunk_compress(K, V, packed, counts, fb)
    gk, gv, gq = gen.quantize_store(K, V, packed, counts, fb)
    assert np.array_equal(kb, gk.numpy()[:kb.size]) and np.array_equal(vb, gv.numpy()[:vb.size])
    gq = gq.numpy().view(oracle.QCHUNK_DTYPE).reshape(qm.shape)
    for b in range(qm.shape[0]):
        n = counts[b]
        for f in ("byte_off", "bits", "scale_k", "zero_k", "scale_v", "zero_v"):
            assert np.array_equal(qm[f][b, :, :n], gq[f][b, :, :n]), f


def test_compressed_store_feeds_the_attention_oracle():
    # the store decodes (oracle.dequant, pinned elsewhere) to values within half a step of the inputs
    K, V, packed, counts, c_max, fb = random_case(8, torch.float16)
    kb, vb, qm = oracle.chunk_compress(K, V, packed, counts, fb)
    dk = oracle.dequant(kb, qm, packed, counts, K.shape[2], 128, "k")
    mine, _ = decode(kb, qm, packed, counts, K.shape[2], "k")
    assert np.array_equal(dk, mine)


def test_compression_share_balances_the_two_sides():
    D, delta, B, T0, Tc, R = 64e6, 0.25, 16e9, 0.3e-3, 2.0e-3, 200e9
    th = oracle.compression_share(D, delta, B, T0, Tc, R)
    assert 0 < th < 1
    lhs = T0 + (D * (1 - th) + D * th * delta) / B           # transmission side of the condition
    rhs = Tc + D * th / R                                     # computation + decompression side
    assert abs(lhs - rhs) <= 1e-12 * max(lhs, rhs) + 1e-15
    # already hidden without compression
    assert oracle.compression_share(D, delta, B, 0.0, 10e-3, R) == 0.0
    # not hidden even when everything is compressed
    assert oracle.compression_share(D, delta, 1e9, T0, 1e-3, R) == 1.0
    # a slower link asks for a larger share; a faster decompressor too (each unit of theta then costs less)
    assert oracle.compression_share(D, delta, 14e9, T0, Tc, R) > th
    assert oracle.compression_share(D, delta, B, T0, Tc, 2 * R) > th
    # no gain from compressing (delta = 1): the only effect of theta is the decompression time -> stays hidden iff it was
    assert oracle.compression_share(D, 1.0, B, T0, 10e-3, R) == 0.0


def test_compression_tags_follow_the_selection():
    # closed forms: everything kept -> nothing 4-bit; nothing kept -> every valid chunk 4-bit; slots past
    # n_chunks stay 0; with uniform chunks and one head a token budget of (1 - theta) N keeps exactly that share
    c_max, n = 40, 32
    nc = np.array([n, n - 5], dtype=np.int32)
    all_ids = np.tile(np.arange(c_max, dtype=np.int32), (2, 1, 1))
    full = oracle.compression_tags(nc, all_ids, np.array([[n], [n - 5]], dtype=np.int32), c_max)
    assert not full.any()
    none = oracle.compression_tags(nc, all_ids, np.zeros((2, 1), dtype=np.int32), c_max)
    assert none[0, :n].all() and not none[0, n:].any() and none[1, :n - 5].all() and not none[1, n - 5:].any()
    # selection by score with a budget: the top (1 - theta) share stays 8-bit
    rng = np.random.default_rng(2)
    score = rng.standard_normal((1, 1, c_max)).astype(np.float32)
    off = (np.arange(c_max + 1, dtype=np.int32) * 16)[None, :]
    theta = 0.75
    sel, cnt, tok = oracle.topk_select(score, off, np.array([c_max], dtype=np.int32), 0, int((1 - theta) * c_max * 16), c_max)
    tags = oracle.compression_tags(np.array([c_max], dtype=np.int32), sel, cnt, c_max)
    assert tags.sum() == int(theta * c_max)
    assert set(np.flatnonzero(tags[0] == 0)) == set(np.argsort(-score[0, 0], kind="stable")[: c_max - int(theta * c_max)])
    # two heads: a chunk kept by either head stays 8-bit (union)
    sel2 = np.full((1, 2, c_max), -1, dtype=np.int32)
    sel2[0, 0, :3] = [1, 5, 9]
    sel2[0, 1, :2] = [5, 30]
    t2 = oracle.compression_tags(np.array([n], dtype=np.int32), sel2, np.array([[3, 2]], dtype=np.int32), c_max)
    assert set(np.flatnonzero(t2[0] == 0)) == {1, 5, 9, 30} | set(range(n, c_max))
    # entries past sel_count are ignored
    sel2[0, 0, 3] = 7
    assert np.array_equal(oracle.compression_tags(np.array([n], dtype=np.int32), sel2, np.array([[3, 2]], dtype=np.int32), c_max), t2)


# ---------------------------------------------------------------------------
# oracle.chunk_recompress: a store brought to new 4-bit tags chunk by chunk
# ---------------------------------------------------------------------------
def live_intervals(qm, packed, counts):
    """[start, end) of every chunk's rows in a blob, from its record"""
    out = []
    B, Hkv, _ = qm.shape
    for b in range(B):
        for h in range(Hkv):
            for c in range(counts[b]):
                rec = qm[b, h, c]
                rows = int(packed[b, c + 1] - packed[b, c])
                out.append((int(rec["byte_off"]), int(rec["byte_off"]) + rows * (64 if rec["bits"] == 4 else 128), (b, h, c)))
    return out


def recompress_case(seed, dtype=torch.float16, share_old=0.5, share_new=0.5):
    K, V, packed, counts, c_max, fb_old = random_case(seed, dtype, B=3, Hkv=2, N=200, share=share_old)
    rng = np.random.default_rng(seed + 1000)
    fb_new = rng.random(fb_old.shape) < share_new
    kb, vb, qm = oracle.chunk_compress(K, V, packed, counts, fb_old)
    used = kb.size
    cap = K.shape[0] * K.shape[1] * (K.shape[2] * 128 + 16 * c_max) * 2        # room for every chunk to move once
    kbig, vbig = np.full(cap, 0xEE, dtype=np.uint8), np.full(cap, 0xEE, dtype=np.uint8)
    kbig[:used], vbig[:used] = kb, vb
    return K, V, packed, counts, c_max, fb_old, fb_new, kbig, vbig, qm, used


@pytest.mark.parametrize("seed,share_old,share_new", [(1, 0.5, 0.5), (2, 0.0, 1.0), (3, 1.0, 0.0), (4, 0.3, 0.8), (5, 0.8, 0.2)])
def test_recompress_equals_a_full_compression_under_the_new_tags(seed, share_old, share_new):
    K, V, packed, counts, c_max, fb_old, fb_new, kb, vb, qm, used = recompress_case(seed, share_old=share_old,
                                                                                  share_new=share_new)
    kb0, vb0, qm0 = kb.copy(), vb.copy(), qm.copy()
    rc, used_new, changed = oracle.chunk_recompress(K, V, packed, counts, fb_old, fb_new, kb, vb, qm, used)
    assert rc == 0
    # the store now decodes to exactly what a full compression under the new tags decodes to, chunk by chunk:
    # same format, same scale and zero, same codes (byte offsets may differ: moved chunks, holes)
    kf, vf, qf = oracle.chunk_compress(K, V, packed, counts, fb_new)
    N = K.shape[2]
    for blob, full, which in ((kb, kf, "k"), (vb, vf, "v")):
        got_val, got_codes = decode(blob, qm, packed, counts, N, which)
        want_val, want_codes = decode(full, qf, packed, counts, N, which)
        assert np.array_equal(got_codes, want_codes) and np.array_equal(got_val, want_val)
    for b in range(qm.shape[0]):
        n = counts[b]
        for f in ("bits", "scale_k", "zero_k", "scale_v", "zero_v"):
            assert np.array_equal(qm[b, :, :n][f], qf[b, :, :n][f]), f
    # only chunks whose tag changed were touched: the others keep their record, and their bytes are the old bytes
    n_diff = 0
    for b in range(qm.shape[0]):
        for c in range(counts[b]):
            same = bool(fb_old[b, c]) == bool(fb_new[b, c])
            n_diff += 0 if same else qm.shape[1]
            for h in range(qm.shape[1]):
                if same:
                    assert qm[b, h, c] == qm0[b, h, c]
                    o, rows = int(qm0[b, h, c]["byte_off"]), int(packed[b, c + 1] - packed[b, c])
                    nbytes = rows * (64 if fb_old[b, c] else 128)
                    assert np.array_equal(kb[o:o + nbytes], kb0[o:o + nbytes]) and np.array_equal(vb[o:o + nbytes], vb0[o:o + nbytes])
                elif fb_new[b, c]:
                    assert qm[b, h, c]["byte_off"] == qm0[b, h, c]["byte_off"]       # shrinks where it lies
                else:
                    assert qm[b, h, c]["byte_off"] >= used                            # moves to fresh room
    assert changed == n_diff
    # the live chunks do not overlap (brute force over all pairs), lie below the new high-water mark, and the
    # mark grew by exactly the room of the moved chunks; nothing past it was written
    iv = sorted(live_intervals(qm, packed, counts))
    for (s0, e0, _), (s1, e1, _) in zip(iv, iv[1:]):
        assert e0 <= s1
    assert iv[-1][1] <= used_new
    grow = sum(((int(packed[b, c + 1] - packed[b, c]) * 128 + 15) // 16 * 16) * qm.shape[1]
               for b in range(qm.shape[0]) for c in range(counts[b]) if fb_old[b, c] and not fb_new[b, c])
    assert used_new == used + grow
    assert np.all(kb[used_new:] == 0xEE) and np.all(vb[used_new:] == 0xEE)
    # moved chunks follow each other in (b, h, chunk) order from the old mark
    moved = [(int(qm[b, h, c]["byte_off"]), (b, h, c)) for b in range(qm.shape[0]) for h in range(qm.shape[1])
             for c in range(counts[b]) if fb_old[b, c] and not fb_new[b, c]]
    assert [k for _, k in sorted(moved)] == [k for _, k in moved]
    if moved:
        assert moved[0][0] == used


def test_recompress_with_the_same_tags_changes_nothing_and_back_and_forth_returns_the_codes():
    K, V, packed, counts, c_max, fb_old, fb_new, kb, vb, qm, used = recompress_case(9)
    kb0, vb0, qm0 = kb.copy(), vb.copy(), qm.copy()
    rc, used1, changed = oracle.chunk_recompress(K, V, packed, counts, fb_old, fb_old, kb, vb, qm, used)
    assert (rc, used1, changed) == (0, used, 0)
    assert np.array_equal(kb, kb0) and np.array_equal(vb, vb0) and np.array_equal(qm, qm0)
    # there and back: the codes, scales and zeros are those of the first store again
    rc, used2, _ = oracle.chunk_recompress(K, V, packed, counts, fb_old, fb_new, kb, vb, qm, used)
    rc2, used3, _ = oracle.chunk_recompress(K, V, packed, counts, fb_new, fb_old, kb, vb, qm, used2)
    assert rc == 0 and rc2 == 0 and used3 >= used2 >= used
    N = K.shape[2]
    for blob, blob0, which in ((kb, kb0, "k"), (vb, vb0, "v")):
        _, codes = decode(blob, qm, packed, counts, N, which)
        _, codes0 = decode(blob0, qm0, packed, counts, N, which)
        assert np.array_equal(codes, codes0)


def test_recompress_without_room_changes_nothing():
    K, V, packed, counts, c_max, fb_old, fb_new, kb, vb, qm, used = recompress_case(12, share_old=1.0, share_new=0.0)
    tight_k, tight_v = kb[: used + 64].copy(), vb[: used + 64].copy()       # room for 64 more bytes only
    qm0 = qm.copy()
    rc, used1, changed = oracle.chunk_recompress(K, V, packed, counts, fb_old, fb_new, tight_k, tight_v, qm, used)
    assert rc == 1 and used1 == used and changed == 0
    assert np.array_equal(tight_k, kb[: used + 64]) and np.array_equal(tight_v, vb[: used + 64]) and np.array_equal(qm, qm0)
