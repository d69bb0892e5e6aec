"""Pins for oracle.score_pin (always-kept chunks): what the selection does with the pinned scores is fixed by
the order of Sec. 4.2 - the largest score first, ties by index - so the expected kept sets are written out."""
import numpy as np

import oracle


def test_pinned_chunks_are_kept_first_and_only_as_far_as_they_fit():
    c_max, n = 12, 10
    off = (np.arange(c_max + 1, dtype=np.int32) * 8).clip(max=n * 8)[None, :]
    nc = np.array([n], dtype=np.int32)
    score = np.array([[[5, 1, 9, 2, 8, 3, 7, 4, 6, 0, -1, -1]]], dtype=np.float32)
    pinned = oracle.score_pin(score, nc, 2, 1)
    big = np.finfo(np.float32).max
    assert list(np.flatnonzero(pinned[0, 0] == big)) == [0, 1, 9]
    assert np.array_equal(pinned[0, 0, 2:9], score[0, 0, 2:9]) and np.array_equal(pinned[0, 0, n:], score[0, 0, n:])
    # budget of 5 chunks: the three pinned ones, then the two best of the rest (chunks 2 and 4)
    sel, cnt, tok = oracle.topk_select(pinned, off, nc, 0, 5 * 8, c_max)
    assert list(sel[0, 0, :cnt[0, 0]]) == [0, 1, 2, 4, 9]
    # budget of 2 chunks: pinned chunks in index order, the tail no longer fits
    sel, cnt, tok = oracle.topk_select(pinned, off, nc, 0, 2 * 8, c_max)
    assert list(sel[0, 0, :cnt[0, 0]]) == [0, 1]
    # nothing pinned: unchanged; counts beyond the sequence pin everything
    assert np.array_equal(oracle.score_pin(score, nc, 0, 0), score)
    assert (oracle.score_pin(score, nc, 7, 7)[0, 0, :n] == big).all()
    # overlapping head and tail on a short sequence
    short = oracle.score_pin(score, np.array([3], dtype=np.int32), 2, 2)
    assert (short[0, 0, :3] == big).all() and np.array_equal(short[0, 0, 3:], score[0, 0, 3:])


def test_pin_applies_to_every_head_of_a_sequence_only():
    score = np.arange(2 * 3 * 6, dtype=np.float32).reshape(2, 3, 6)
    out = oracle.score_pin(score, np.array([6, 4], dtype=np.int32), 1, 1)
    big = np.finfo(np.float32).max
    assert (out[0, :, 0] == big).all() and (out[0, :, 5] == big).all() and np.array_equal(out[0, :, 1:5], score[0, :, 1:5])
    assert (out[1, :, 0] == big).all() and (out[1, :, 3] == big).all() and np.array_equal(out[1, :, 4:], score[1, :, 4:])
