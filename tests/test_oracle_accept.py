"""Pins for the oracle's lossless greedy acceptance + commit: brute force over every match
pattern, the two extremes, invariants, tie-breaking, forced (prefill) commits.  CPU only."""
import itertools

import numpy as np
import pytest

import synth
from oracle import sfo

SHAPE = synth.ModelShape("pin", 1, 16, 2, 1, 8, 32, 23, "f32")


def make(B, q_max=8, cap=64):
    tw = synth.target_weights(SHAPE, 1)
    return sfo.Oracle(SHAPE.cfg(), tw, None, B, cap, q_max)


def logits_for(ids, V):
    """[B,q,V] logits whose arg-max is ids (with distractors below)."""
    B, q = ids.shape
    lg = np.random.default_rng(0).uniform(-1, 0, (B, q, V))
    for b in range(B):
        for i in range(q):
            lg[b, i, ids[b, i]] = 1.0 + 0.1 * i
    return lg


@pytest.mark.parametrize("k", [1, 2, 3, 4, 6])
def test_every_match_pattern(k):
    V = SHAPE.vocab
    pats = list(itertools.product([0, 1], repeat=k))
    B = len(pats)
    o = make(B)
    o.kv_len[:] = np.arange(B) % 7 + 3
    len0 = o.kv_len.copy()
    rs = np.random.default_rng(k)
    tgt = rs.integers(0, V, (B, k + 1)).astype(np.int32)
    draft = tgt[:, :k].copy()
    for b, pat in enumerate(pats):
        for i, m in enumerate(pat):
            if not m:
                draft[b, i] = (tgt[b, i] + 1 + rs.integers(0, V - 1)) % V   # any other token
    acc, out = o.accept_commit(k, draft, logits_for(tgt, V))
    for b, pat in enumerate(pats):
        n = 0                                                # longest all-ones prefix, by definition
        while n < k and pat[n]:
            n += 1
        assert acc[b] == n + 1
        assert 1 <= acc[b] <= k + 1
        np.testing.assert_array_equal(out[b, :n + 1], tgt[b, :n + 1])
        assert np.all(out[b, n + 1:] == -1)
        assert o.pending[b] == tgt[b, n]
        assert o.kv_len[b] == len0[b] + n + 1
        assert o.n_new[b] == n + 1
    np.testing.assert_array_equal(o.cu_new, np.concatenate([[0], np.cumsum(acc)]))


def test_extremes_and_no_draft():
    V, k = SHAPE.vocab, 4
    o = make(2)
    tgt = np.array([[1, 2, 3, 4, 5], [6, 7, 8, 9, 10]], np.int32)
    draft = np.array([[1, 2, 3, 4], [0, 7, 8, 9]], np.int32)       # all right / first wrong
    acc, out = o.accept_commit(k, draft, logits_for(tgt, V))
    assert list(acc) == [5, 1]
    assert list(out[0]) == [1, 2, 3, 4, 5] and list(out[1]) == [6, -1, -1, -1, -1]
    # a later match after a mismatch must not count
    o = make(1)
    acc, _ = o.accept_commit(k, np.array([[1, 0, 3, 4]], np.int32), logits_for(tgt[:1], V))
    assert acc[0] == 2
    # k = 0 is plain autoregressive decoding: always exactly one token (the "W/o SD" rows, kappa = 1)
    o = make(3)
    acc, out = o.accept_commit(0, np.zeros((3, 0), np.int32), logits_for(tgt[[0, 1, 0], :1], V))
    assert list(acc) == [1, 1, 1] and list(out[:, 0]) == [1, 6, 1]


def test_ties_take_the_lowest_index():
    V, k = SHAPE.vocab, 1
    o = make(1)
    lg = np.zeros((1, 2, V)); lg[0, 0, [4, 9]] = 2.0; lg[0, 1, [7, 3]] = 1.0
    acc, out = o.accept_commit(k, np.array([[4]], np.int32), lg)
    assert acc[0] == 2 and list(out[0]) == [4, 3]
    o = make(1)
    acc, out = o.accept_commit(k, np.array([[9]], np.int32), lg)   # 9 ties with 4 but 4 wins
    assert acc[0] == 1 and list(out[0]) == [4, -1]


def test_forced_commit():
    V, k = SHAPE.vocab, 3
    o = make(3)
    o.pending[:] = 99
    tgt = np.arange(12, dtype=np.int32).reshape(3, 4) % V
    acc, out = o.accept_commit(k, np.zeros((3, 3), np.int32), logits_for(tgt, V), force_len=[4, 0, 2])
    assert list(acc) == [4, 0, 2]
    assert list(o.kv_len) == [4, 0, 2] and list(o.n_new) == [4, 0, 2]
    assert list(o.pending) == [tgt[0, 3], 99, tgt[2, 1]]            # nothing committed: unchanged
    assert list(o.cu_new) == [0, 4, 4, 6]
    assert list(out[1]) == [-1] * 4 and list(out[2]) == [tgt[2, 0], tgt[2, 1], -1, -1]
