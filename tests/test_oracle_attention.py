"""Pins for the oracle's hybrid-mask ragged attention (SpecFormer: unidirectional along the
context, bidirectional along the draft block).  CPU only."""
import math

import numpy as np
import pytest
import torch

import synth
from oracle import sfo
from oracle.sfo import MASK_BIDIR, MASK_CAUSAL


def brute(q, kc, vc, lens, mode):
    """Explicit exp / sum attention with python loops, written from the mask's definition."""
    B, nq, Hq, hd = q.shape
    Hkv = kc.shape[1]
    G = Hq // Hkv
    out = np.zeros_like(q, dtype=np.float64)
    for b in range(B):
        for i in range(nq):
            keys = list(range(int(lens[b])))                      # the committed prefix
            keys += [int(lens[b]) + j for j in range(nq) if mode == MASK_BIDIR or j <= i]
            for h in range(Hq):
                g = h // G
                e = [math.exp(sum(q[b, i, h, t] * kc[b, g, p, t] for t in range(hd)) / math.sqrt(hd))
                     for p in keys]
                z = sum(e)
                for t in range(hd):
                    out[b, i, h, t] = sum(e[n] / z * vc[b, g, p, t] for n, p in enumerate(keys))
    return out


def rand(seed, B, nq, Hq, Hkv, hd, cap):
    q, kc, vc = synth.random_qkv(seed, B, nq, Hq, Hkv, hd, cap, "f32")
    return q.astype(np.float64), kc.astype(np.float64), vc.astype(np.float64)


@pytest.mark.parametrize("mode", [MASK_CAUSAL, MASK_BIDIR])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (6, 2)])
def test_brute_force_tiny(mode, Hq, Hkv):
    B, nq, hd, cap = 2, 3, 8, 12
    q, kc, vc = rand(1, B, nq, Hq, Hkv, hd, cap)
    lens = np.array([5, 0], np.int32)
    got = sfo.attention(q, kc, vc, lens, mode)
    np.testing.assert_allclose(got, brute(q, kc, vc, lens, mode), rtol=1e-12, atol=1e-14)


def test_single_slot_hybrid_is_causal_decode():
    """k = 1: the hybrid mask degenerates to ordinary single-token causal decode attention."""
    B, Hq, Hkv, hd, cap = 3, 4, 2, 16, 40
    q, kc, vc = rand(2, B, 1, Hq, Hkv, hd, cap)
    lens = np.array([7, 0, 39], np.int32)
    a = sfo.attention(q, kc, vc, lens, MASK_BIDIR)
    b = sfo.attention(q, kc, vc, lens, MASK_CAUSAL)
    np.testing.assert_array_equal(a, b)
    # textbook decode: softmax over the len+1 keys [0, len], via the library softmax
    for s in range(B):
        n = int(lens[s]) + 1
        for h in range(Hq):
            g = h // (Hq // Hkv)
            sc = torch.from_numpy(kc[s, g, :n] @ q[s, 0, h] / math.sqrt(hd))
            want = torch.softmax(sc, 0).numpy() @ vc[s, g, :n]
            np.testing.assert_allclose(a[s, 0, h], want, rtol=1e-12, atol=1e-14)


def test_no_prefix_bidir_is_plain_self_attention():
    B, nq, H, hd = 2, 5, 2, 8
    q, kc, vc = rand(3, B, nq, H, H, hd, 8)
    lens = np.zeros(B, np.int32)
    got = sfo.attention(q, kc, vc, lens, MASK_BIDIR)
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)                  # [B,H,nq,hd]
    tk = torch.from_numpy(kc[:, :, :nq]); tv = torch.from_numpy(vc[:, :, :nq])
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
    # and with the causal flag the block is an ordinary causal self-attention
    got_c = sfo.attention(q, kc, vc, lens, MASK_CAUSAL)
    want_c = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    np.testing.assert_allclose(got_c, want_c.permute(0, 2, 1, 3).numpy(), rtol=1e-10, atol=1e-12)


def test_block_causal_rows_equal_successive_decodes():
    """Row i of a causal block == a single-token decode whose prefix is len+i (verify == AR)."""
    B, nq, Hq, Hkv, hd, cap = 2, 4, 4, 2, 8, 24
    q, kc, vc = rand(4, B, nq, Hq, Hkv, hd, cap)
    lens = np.array([9, 3], np.int32)
    blk = sfo.attention(q, kc, vc, lens, MASK_CAUSAL)
    for i in range(nq):
        one = sfo.attention(q[:, i:i + 1], kc, vc, lens + i, MASK_CAUSAL)
        np.testing.assert_array_equal(blk[:, i:i + 1], one)


def test_visibility_by_perturbation():
    B, nq, Hq, Hkv, hd, cap = 2, 3, 2, 1, 8, 16
    q, kc, vc = rand(5, B, nq, Hq, Hkv, hd, cap)
    lens = np.array([6, 2], np.int32)
    for mode in (MASK_CAUSAL, MASK_BIDIR):
        base = sfo.attention(q, kc, vc, lens, mode)
        for b in range(B):
            for p in range(cap):
                k2, v2 = kc.copy(), vc.copy()
                k2[b, 0, p] += 1.0; v2[b, 0, p] -= 2.0
                out = sfo.attention(q, k2, v2, lens, mode)
                other = 1 - b
                np.testing.assert_array_equal(out[other], base[other])     # other sequence's slab
                for i in range(nq):
                    j = p - int(lens[b])
                    vis = p < lens[b] or (0 <= j < nq and (mode == MASK_BIDIR or j <= i))
                    changed = not np.array_equal(out[b, i], base[b, i])
                    assert changed == vis, (mode, b, p, i)


def test_bidir_sees_later_slots_causal_does_not():
    q, kc, vc = rand(6, 1, 4, 2, 2, 8, 16)
    lens = np.array([5], np.int32)
    v2 = vc.copy(); v2[0, :, 5 + 3] += 1.0                         # V of the last slot
    assert not np.array_equal(sfo.attention(q, kc, v2, lens, MASK_BIDIR)[0, 0],
                              sfo.attention(q, kc, vc, lens, MASK_BIDIR)[0, 0])
    np.testing.assert_array_equal(sfo.attention(q, kc, v2, lens, MASK_CAUSAL)[0, 0],
                                  sfo.attention(q, kc, vc, lens, MASK_CAUSAL)[0, 0])


def test_bidir_is_permutation_equivariant_over_slots():
    q, kc, vc = rand(7, 1, 4, 2, 2, 8, 16)
    lens = np.array([6], np.int32)
    perm = np.array([2, 0, 3, 1])
    base = sfo.attention(q, kc, vc, lens, MASK_BIDIR)
    k2, v2 = kc.copy(), vc.copy()
    k2[0][:, 6:10] = kc[0][:, 6 + perm]; v2[0][:, 6:10] = vc[0][:, 6 + perm]
    out = sfo.attention(q[:, perm], k2, v2, lens, MASK_BIDIR)
    np.testing.assert_allclose(out, base[:, perm], rtol=1e-12, atol=1e-14)


def test_ragged_batch_equals_each_sequence_alone():
    B, nq, Hq, Hkv, hd, cap = 4, 3, 4, 2, 8, 40
    q, kc, vc = rand(8, B, nq, Hq, Hkv, hd, cap)
    lens = np.array([0, 37, 5, 18], np.int32)
    for mode in (MASK_CAUSAL, MASK_BIDIR):
        full = sfo.attention(q, kc, vc, lens, mode)
        for b in range(B):
            one = sfo.attention(q[b:b + 1], kc[b:b + 1], vc[b:b + 1], lens[b:b + 1], mode)
            np.testing.assert_array_equal(full[b:b + 1], one)


def test_zero_query_gives_mean_of_visible_values_and_softmax_invariances():
    B, nq, Hq, Hkv, hd, cap = 1, 3, 2, 2, 8, 16
    q, kc, vc = rand(9, B, nq, Hq, Hkv, hd, cap)
    lens = np.array([4], np.int32)
    out = sfo.attention(np.zeros_like(q), kc, vc, lens, MASK_CAUSAL)
    for i in range(nq):
        np.testing.assert_allclose(out[0, i], vc[0, :, :4 + i + 1].mean(1), rtol=1e-13)
    out = sfo.attention(np.zeros_like(q), kc, vc, lens, MASK_BIDIR)
    for i in range(nq):
        np.testing.assert_allclose(out[0, i], vc[0, :, :4 + nq].mean(1), rtol=1e-13)
    base = sfo.attention(q, kc, vc, lens, MASK_BIDIR)
    # outputs are convex combinations of the value rows
    lo, hi = vc[0, :, :7].min(1), vc[0, :, :7].max(1)
    assert np.all(base[0] >= lo[None] - 1e-12) and np.all(base[0] <= hi[None] + 1e-12)
    # huge scores: max-subtraction keeps the softmax finite and picks the arg-max key
    qb = q * 1e4
    big = sfo.attention(qb, kc, vc, lens, MASK_BIDIR)
    assert np.all(np.isfinite(big))
