"""GPU parity of the single operations of the path against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import synth
from oracle import sfo
from paper_2511_20340_amd import binding as sfb

from gpu_common import dev, engine_only, rel_err, to_np

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2     # max relative error w.r.t. max |ref|, bf16 mode
F32_TOL = 1e-4      # fp32 mode


def shape_for(dtype, Hq, Hkv, hd, d=None):
    d = d or Hq * hd
    return synth.ModelShape("t", 1, d, Hq, Hkv, hd, 256, 512, dtype)


def run_attention(dtype, B, nq, Hq, Hkv, hd, cap, lens, mode, seed=1, poison=False):
    q, kc, vc = synth.random_qkv(seed, B, nq, Hq, Hkv, hd, cap, dtype)
    lens = np.asarray(lens, np.int32)
    ref = sfo.attention(q, kc, vc, lens, mode)
    kc_g, vc_g = kc.copy(), vc.copy()
    if poison:                               # dead slots beyond len+nq hold NaN / huge values
        for b in range(B):
            kc_g[b, :, lens[b] + nq:] = np.nan
            vc_g[b, :, lens[b] + nq:] = np.nan
    eng = engine_only(shape_for(dtype, Hq, Hkv, hd), B, cap, nq - 1 if nq > 1 else 1)
    eng.sf_kv_import(kc_g, "dk"); eng.sf_kv_import(vc_g, "dv")
    kvl = torch.from_numpy(lens).cuda()
    out = eng.sf_op_attention(dev(q, dtype), eng.dk, eng.dv, kvl, nq, mode)
    torch.cuda.synchronize()
    return to_np(out), ref


@pytest.mark.parametrize("mode", [sfb.SF_MASK_CAUSAL, sfb.SF_MASK_BIDIR])
@pytest.mark.parametrize("Hq,Hkv,hd,nq", [(8, 2, 128, 5), (10, 2, 128, 5), (8, 2, 64, 5), (8, 2, 128, 7),
                                          (4, 4, 128, 1), (16, 2, 128, 5),
                                          # blocks of many rows (k = 8; prefill blocks): several 32-row tiles
                                          (8, 2, 128, 9), (8, 2, 64, 33), (8, 2, 128, 64), (10, 2, 128, 64)])
def test_attention_bf16_ragged(mode, Hq, Hkv, hd, nq):
    # lengths span: empty prefix, inside one tile, tile boundary, several chunks + ragged tail
    lens = [0, 27, 32, 1500, 511, min(2000, 2048 - nq)]
    got, ref = run_attention("bf16", 6, nq, Hq, Hkv, hd, 2048, lens, mode)
    assert np.all(np.isfinite(got))
    assert rel_err(got, ref) < BF16_TOL


def test_attention_bf16_ignores_dead_slots():
    lens = [0, 27, 700, 1000]
    got, ref = run_attention("bf16", 4, 5, 8, 2, 128, 1024, lens, sfb.SF_MASK_CAUSAL, poison=True)
    assert np.all(np.isfinite(got))
    assert rel_err(got, ref) < BF16_TOL


def test_attention_bf16_single_slot_equals_both_masks():
    lens = [5, 900]
    a, ref = run_attention("bf16", 2, 1, 8, 2, 128, 1024, lens, sfb.SF_MASK_CAUSAL)
    b, _ = run_attention("bf16", 2, 1, 8, 2, 128, 1024, lens, sfb.SF_MASK_BIDIR)
    np.testing.assert_array_equal(a, b)          # k = 1: hybrid mask == causal decode


@pytest.mark.parametrize("mode", [sfb.SF_MASK_CAUSAL, sfb.SF_MASK_BIDIR])
def test_attention_f32(mode):
    lens = [0, 64, 700, 33]
    got, ref = run_attention("f32", 4, 5, 4, 4, 64, 768, lens, mode)
    assert rel_err(got, ref) < F32_TOL
    got, ref = run_attention("f32", 4, 3, 8, 2, 32, 768, lens, mode, seed=2)
    assert rel_err(got, ref) < F32_TOL


@pytest.mark.parametrize("M,N,K", [(320, 512, 4096), (77, 264, 200), (160, 3072, 2048), (640, 384, 1024),
                                   (1, 128, 64), (333, 1000, 520)])
def test_linear_bf16(M, N, K):
    g = synth.rng(5, M * 7 + N)
    x = synth.to_bf16_values(g.standard_normal((M, K), dtype=np.float32))
    w = synth.to_bf16_values(g.standard_normal((N, K), dtype=np.float32) * 0.05)
    bias = synth.to_bf16_values(g.standard_normal(N, dtype=np.float32))
    res = synth.to_bf16_values(g.standard_normal((M, N), dtype=np.float32))
    eng = engine_only(shape_for("bf16", 2, 2, 64), 1, 64, 1)
    ref = sfo.linear(x, w)
    y = eng.sf_op_linear(dev(x, "bf16"), dev(w, "bf16"), out_f32=True)
    assert rel_err(to_np(y), ref) < 1e-5          # fp32 accumulators, unrounded
    y = eng.sf_op_linear(dev(x, "bf16"), dev(w, "bf16"))
    assert rel_err(to_np(y), ref) < BF16_TOL
    ref2 = sfo.linear(x, w, bias) + res
    y = eng.sf_op_linear(dev(x, "bf16"), dev(w, "bf16"), bias=dev(bias, "bf16"), residual=dev(res, "bf16"))
    assert rel_err(to_np(y), ref2) < BF16_TOL
    r, xd, wd = dev(res, "bf16"), dev(x, "bf16"), dev(w, "bf16")     # residual aliasing the output
    eng.sf_op_linear(xd, wd, residual=r, y=r)
    torch.cuda.synchronize()
    assert rel_err(to_np(r), sfo.linear(x, w) + res) < BF16_TOL


@pytest.mark.parametrize("M,N,K", [(333, 520, 1792), (160, 264, 2048), (200, 136, 520)])  # the last: a K tail of 8
def test_linear_bf16_every_tile_and_split_gives_the_same_bits(M, N, K):
    """The K partition, hence the fp32 summation order, depends on K and the split factor only: every
    tile configuration must return identical bits, for the whole batch and for a few of its rows."""
    g = synth.rng(15, M + N)
    x = synth.to_bf16_values(g.standard_normal((M, K), dtype=np.float32))
    w = synth.to_bf16_values(g.standard_normal((N, K), dtype=np.float32) * 0.05)
    ref = sfo.linear(x, w)
    eng = engine_only(shape_for("bf16", 2, 2, 64), 1, 64, 1)
    L = sfb.lib()
    xd, wd = dev(x, "bf16"), dev(w, "bf16")
    packed = eng.sf_pack_weight(wd)
    try:
        for split in (1, 2, 4):
            first = None
            for tile in range(1, L.sf_linear_num_tiles() + 1):
                eng.sf_tune_linear(tile, split)
                y = eng.sf_op_linear(xd, None, out_f32=True, packed=(packed, N))
                few = eng.sf_op_linear(xd[:7].contiguous(), None, out_f32=True, packed=(packed, N))
                torch.cuda.synchronize()
                assert rel_err(to_np(y), ref) < 1e-5, (tile, split)
                if first is None:
                    first = y.clone()
                assert torch.equal(y, first), (tile, split)
                assert torch.equal(few, first[:7]), (tile, split)
    finally:
        eng.sf_tune_linear(0, 0)


def test_linear_bf16_epilogues_of_every_tile_agree():
    """Bias + residual (the output aliasing the residual) and the fused SwiGLU gate go through every tile
    configuration, the tall ones included (their waves hold more than five 32x32 tiles and take the residual
    in groups): all must leave the same bits, and those must match the oracle."""
    M, N, K, F = 650, 392, 512, 224
    g = synth.rng(23, M + N)
    x = synth.to_bf16_values(g.standard_normal((M, K), dtype=np.float32))
    w = synth.to_bf16_values(g.standard_normal((N, K), dtype=np.float32) * 0.05)
    wgu = synth.to_bf16_values(g.standard_normal((2 * F, K), dtype=np.float32) * 0.05)
    bias = synth.to_bf16_values(g.standard_normal(N, dtype=np.float32))
    res = synth.to_bf16_values(g.standard_normal((M, N), dtype=np.float32))
    eng = engine_only(shape_for("bf16", 2, 2, 64), 1, 64, 1)
    xd, wd, bd, wgud = dev(x, "bf16"), dev(w, "bf16"), dev(bias, "bf16"), dev(wgu, "bf16")
    packed = eng.sf_pack_weight(wd)
    ref = sfo.linear(x, w, bias) + res
    gu = sfo.linear(x, wgu)
    ref_glu = gu[:, :F] / (1.0 + np.exp(-gu[:, :F])) * gu[:, F:]
    try:
        first = first_glu = None
        for tile in range(1, sfb.lib().sf_linear_num_tiles() + 1):
            eng.sf_tune_linear(tile, 1)
            r = dev(res, "bf16")
            eng.sf_op_linear(xd, None, bias=bd, residual=r, y=r, packed=(packed, N))
            a = eng.sf_op_linear_swiglu(xd, wgud)
            torch.cuda.synchronize()
            assert rel_err(to_np(r), ref) < BF16_TOL and rel_err(to_np(a), ref_glu) < BF16_TOL, tile
            if first is None:
                first, first_glu = r.clone(), a.clone()
            assert torch.equal(r, first) and torch.equal(a, first_glu), tile
    finally:
        eng.sf_tune_linear(0, 0)


@pytest.mark.parametrize("M,N,K", [(160, 392, 2048), (77, 264, 200), (333, 520, 1792), (5, 128, 4096)])
def test_rmsnorm_linear_fused(M, N, K):
    """The decoder's norm + linear pair as one kernel: against the oracle's RMSNorm followed by its
    linear layer, for every tile configuration and split factor, which must all agree bit for bit and
    must not depend on the rows batched together."""
    g = synth.rng(17, M + N)
    x = synth.to_bf16_values(g.standard_normal((M, K), dtype=np.float32) * 3.0)
    x[0] *= 40.0                                             # rows of very different scale
    x[M - 1] *= 0.01
    x = synth.to_bf16_values(x)
    gain = synth.to_bf16_values(1.0 + 0.5 * g.standard_normal(K, dtype=np.float32))
    w = synth.to_bf16_values(g.standard_normal((N, K), dtype=np.float32) * 0.05)
    ref = sfo.linear(sfo.rmsnorm(x, gain, 1e-6), w)
    eng = engine_only(shape_for("bf16", 2, 2, 64), 1, 64, 1)
    L = sfb.lib()
    xd, gd, wd = dev(x, "bf16"), dev(gain, "bf16"), dev(w, "bf16")
    packed = eng.sf_pack_weight(wd, gain=gd)
    y = eng.sf_op_rmsnorm_linear(xd, gd, None, out_f32=True, packed=(packed, N))
    assert rel_err(to_np(y), ref) < 5e-3                      # weight * gain is rounded to bf16 once
    yb = eng.sf_op_rmsnorm_linear(xd, gd, None, packed=(packed, N))
    assert rel_err(to_np(yb), ref) < BF16_TOL
    try:
        for split in (1, 2, 4):
            first = None
            for tile in range(1, L.sf_linear_num_tiles() + 1):
                eng.sf_tune_linear(tile, split)
                y = eng.sf_op_rmsnorm_linear(xd, gd, None, out_f32=True, packed=(packed, N))
                few = eng.sf_op_rmsnorm_linear(xd[:3].contiguous(), gd, None, out_f32=True, packed=(packed, N))
                torch.cuda.synchronize()
                assert rel_err(to_np(y), ref) < 5e-3, (tile, split)
                if first is None:
                    first = y.clone()
                assert torch.equal(y, first), (tile, split)
                assert torch.equal(few, first[:3]), (tile, split)
    finally:
        eng.sf_tune_linear(0, 0)


@pytest.mark.parametrize("M,N,K", [(20, 768, 256), (77, 264, 200), (130, 1024, 1024)])
def test_linear_f32(M, N, K):
    g = synth.rng(6, M + N)
    x = g.standard_normal((M, K), dtype=np.float32)
    w = g.standard_normal((N, K), dtype=np.float32) * 0.05
    bias = g.standard_normal(N, dtype=np.float32)
    eng = engine_only(shape_for("f32", 2, 2, 64), 1, 64, 1)
    y = eng.sf_op_linear(dev(x, "f32"), dev(w, "f32"), bias=dev(bias, "f32"))
    assert rel_err(to_np(y), sfo.linear(x, w, bias)) < 1e-5


@pytest.mark.parametrize("dtype,tol", [("bf16", BF16_TOL), ("f32", 1e-5)])
def test_rmsnorm_and_group_rmsnorm(dtype, tol):
    g = synth.rng(7, 1)
    d = 520
    x = g.standard_normal((24, d), dtype=np.float32) * 3
    gain = 1 + 0.1 * g.standard_normal((4, d), dtype=np.float32)
    if dtype == "bf16":
        x, gain = synth.to_bf16_values(x), synth.to_bf16_values(gain)
    eng = engine_only(shape_for(dtype, 2, 2, 64), 1, 64, 1)
    y = eng.sf_op_rmsnorm(dev(x, dtype), dev(gain[0], dtype))
    assert rel_err(to_np(y), sfo.rmsnorm(x, gain[0])) < tol
    y = eng.sf_op_rmsnorm(dev(x, dtype), dev(gain, dtype), n_gain=4)      # rows [6][4][d]
    assert rel_err(to_np(y), sfo.group_rmsnorm(x.reshape(6, 4, d), gain).reshape(24, d)) < tol


@pytest.mark.parametrize("dtype,tol,hd", [("bf16", BF16_TOL, 128), ("bf16", BF16_TOL, 64), ("f32", 1e-5, 64)])
def test_rope_kv_append_and_layout_roundtrip(dtype, tol, hd):
    B, nq, Hq, Hkv, cap = 3, 5, 4, 2, 4096 + 64
    lens = np.array([0, 1000, 4096], np.int32)           # large positions: table must stay accurate
    g = synth.rng(8, hd)
    qkv = g.standard_normal((B * nq, (Hq + 2 * Hkv) * hd), dtype=np.float32)
    if dtype == "bf16":
        qkv = synth.to_bf16_values(qkv)
    eng = engine_only(shape_for(dtype, Hq, Hkv, hd), B, cap, nq - 1)
    # layout round trip first: import random plain caches, export them back bit-exactly
    _, kc, vc = synth.random_qkv(3, B, 1, Hq, Hkv, hd, cap, dtype)
    eng.sf_kv_import(kc, "dk"); eng.sf_kv_import(vc, "dv")
    np.testing.assert_array_equal(to_np(eng.sf_kv_export("dk")), kc)
    np.testing.assert_array_equal(to_np(eng.sf_kv_export("dv")), vc)
    q_out = eng.sf_op_rope_kv_append(dev(qkv, dtype), torch.from_numpy(lens).cuda(), nq, eng.dk, eng.dv)
    pos = (lens[:, None] + np.arange(nq)[None]).reshape(-1).astype(np.int32)
    nqc, nkv = Hq * hd, Hkv * hd
    q_ref = sfo.rope(qkv[:, :nqc].reshape(-1, Hq, hd), pos).reshape(-1, nqc)
    k_ref = sfo.rope(qkv[:, nqc:nqc + nkv].reshape(-1, Hkv, hd), pos)
    v_ref = qkv[:, nqc + nkv:].reshape(-1, Hkv, hd)
    assert rel_err(to_np(q_out), q_ref) < tol
    kg, vg = to_np(eng.sf_kv_export("dk")), to_np(eng.sf_kv_export("dv"))
    want_k, want_v = kc.astype(np.float64).copy(), vc.astype(np.float64).copy()
    for b in range(B):
        for i in range(nq):
            want_k[b, :, lens[b] + i] = k_ref[b * nq + i]
            want_v[b, :, lens[b] + i] = v_ref[b * nq + i]
    assert rel_err(kg, want_k) < tol
    np.testing.assert_array_equal(vg, want_v)             # V is copied, not transformed
    untouched = np.ones((B, cap), bool)
    for b in range(B):
        untouched[b, lens[b]:lens[b] + nq] = False
    np.testing.assert_array_equal(kg.transpose(0, 2, 1, 3)[untouched], kc.transpose(0, 2, 1, 3)[untouched])


@pytest.mark.parametrize("dtype,tol,M,F,K", [("bf16", BF16_TOL, 320, 1024, 512), ("bf16", BF16_TOL, 77, 96, 200),
                                             ("bf16", BF16_TOL, 160, 2048, 4096), ("f32", 1e-4, 20, 1024, 256)])
def test_linear_swiglu(dtype, tol, M, F, K):
    g = synth.rng(12, M + F)
    x = g.standard_normal((M, K), dtype=np.float32)
    w = g.standard_normal((2 * F, K), dtype=np.float32) * (2.0 / np.sqrt(K))
    if dtype == "bf16":
        x, w = synth.to_bf16_values(x), synth.to_bf16_values(w)
    eng = engine_only(shape_for(dtype, 2, 2, 64), 1, 64, 1)
    act = eng.sf_op_linear_swiglu(dev(x, dtype), dev(w, dtype))
    ref = sfo.silu_mul(sfo.linear(x, w[:F]), sfo.linear(x, w[F:]))
    assert rel_err(to_np(act), ref) < tol


@pytest.mark.parametrize("dtype,tol", [("bf16", BF16_TOL), ("f32", 1e-5)])
def test_silu_mul(dtype, tol):
    g = synth.rng(9, 1)
    gu = g.standard_normal((37, 2 * 520), dtype=np.float32) * 3
    eng = engine_only(shape_for(dtype, 2, 2, 64), 1, 64, 1)
    act = eng.sf_op_silu_mul(torch.from_numpy(gu).cuda())
    assert rel_err(to_np(act), sfo.silu_mul(gu[:, :520], gu[:, 520:])) < tol


@pytest.mark.parametrize("V", [1000, 1024, 32000, 128256, 7])
def test_argmax_bit_exact(V):
    g = synth.rng(10, V)
    M = 23
    lg = g.standard_normal((M, V), dtype=np.float32)
    lg[0, :] = 0.5                                 # all tied -> index 0
    lg[1, [V - 1, V // 2]] = 9.0                   # tie -> lowest index
    lg[2, 0] = np.nan; lg[2, V - 1] = 50.0         # NaN never wins
    lg[3, :] = -np.inf
    lg[4, :] = np.nan
    eng = engine_only(shape_for("bf16", 2, 2, 64), 1, 64, 1)
    ids = eng.sf_op_argmax(torch.from_numpy(lg).cuda()).cpu().numpy()
    want = np.array([sfo.argmax(lg[r]) for r in range(M)], np.int32)
    np.testing.assert_array_equal(ids, want)


def integer_operands(M, N, K, seed):
    """Small-integer rows and weights: every product and partial sum is exact in fp32, so the GPU's
    accumulators equal the oracle's logits bit for bit and equal values (ties) abound."""
    g = synth.rng(seed, N)
    x = g.integers(-2, 3, (M, K)).astype(np.float32)
    w = g.integers(-3, 4, (N, K)).astype(np.float32)
    return x, w


# fp32 mode serves the small configuration only: its large-vocabulary cases are left out
@pytest.mark.parametrize("dtype,M,V", [("bf16", 5, 32000), ("bf16", 160, 32000), ("bf16", 37, 128256),
                                       ("bf16", 200, 152064), ("bf16", 23, 1000), ("bf16", 3, 136),
                                       ("f32", 5, 32000), ("f32", 23, 1000), ("f32", 3, 136)])
def test_lm_head_fused_argmax_bit_exact(dtype, M, V):
    """The LM head with its arg-max (bf16: per-column-tile partials from the linear kernel's epilogue, logits
    optional) against the oracle's linear + arg-max: planted ties inside a lane group, across the waves of a
    workgroup and across column-tile edges, plus the ties the integer operands produce by themselves."""
    K = 64
    x, w = integer_operands(M, V, K, 21)
    top = np.full(K, 3.0, np.float32)
    for r, (c0, c1) in enumerate([(5, 17), (31, 32), (127, 128), (255, 256), (100, V - 1), (V - 2, V - 1)][:M]):
        x[r] = 2.0                                    # row r: columns c0 and c1 both reach the largest possible logit
        w[c0] = top; w[c1] = top
    if M > 8:
        x[8, 3] = np.nan                              # a row of NaN logits: nothing comparable -> 0
    ref = sfo.linear(x, w)
    want = np.array([sfo.argmax(ref[r]) for r in range(M)], np.int32)
    eng = engine_only(shape_for(dtype, 2, 2, 64), 1, 64, 1)
    xd, wd = dev(x, dtype), dev(w, dtype)
    ids = eng.sf_op_linear_argmax(xd, wd).cpu().numpy()
    np.testing.assert_array_equal(ids, want)
    ids2, lg = eng.sf_op_linear_argmax(xd, wd, want_logits=True)
    np.testing.assert_array_equal(ids2.cpu().numpy(), want)
    finite = ~np.isnan(ref)
    np.testing.assert_array_equal(to_np(lg)[finite], ref[finite])
    if dtype == "bf16" and M == 160:                  # every tile shape leaves the same answer
        packed = eng.sf_pack_weight(wd)
        try:
            for tile in range(1, sfb.lib().sf_linear_num_tiles() + 1):
                eng.sf_tune_linear(tile, 0)
                got = eng.sf_op_linear_argmax(xd, None, packed=(packed, V)).cpu().numpy()
                np.testing.assert_array_equal(got, want, err_msg=f"tile {tile}")
        finally:
            eng.sf_tune_linear(0, 0)


@pytest.mark.parametrize("mode", [sfb.SF_MASK_CAUSAL, sfb.SF_MASK_BIDIR])
@pytest.mark.parametrize("Hq,Hkv,hd,nq,chunk", [(8, 2, 64, 5, 0), (8, 2, 128, 5, 0), (16, 2, 128, 5, 0),
                                                 (8, 2, 64, 5, 16), (8, 2, 128, 7, 16), (4, 4, 128, 1, 0),
                                                 (8, 2, 128, 33, 0), (8, 2, 64, 64, 16)])
def test_rope_attention_fused(mode, Hq, Hkv, hd, nq, chunk):
    """The target layers' kernel (rotate Q and K, append K and V, attend) against the oracle's rope +
    attention and, bit for bit, against the two separate kernels.  Lengths: empty prefix, a block that
    ends on / crosses a tile boundary, one that crosses a split-KV chunk boundary (510 with 16-tile
    chunks), a long ragged one, and a block that fills the cache to its last slot."""
    cap = 2048
    lens = np.array([0, 27, 29, 30, 32, 510, 1500, cap - nq], np.int32)  # all four residues of 4: the V rows go out in groups of four positions
    B = len(lens)
    g = synth.rng(21, Hq * hd + nq)
    qkv = synth.to_bf16_values(g.standard_normal((B * nq, (Hq + 2 * Hkv) * hd), dtype=np.float32))
    _, kc, vc = synth.random_qkv(4, B, 1, Hq, Hkv, hd, cap, "bf16")
    for b in range(B):                       # dead slots hold NaN: nothing past the block may be read
        kc[b, :, lens[b] + nq:] = np.nan
        vc[b, :, lens[b] + nq:] = np.nan
    pos = (lens[:, None] + np.arange(nq)[None]).reshape(-1).astype(np.int32)
    nqc, nkv = Hq * hd, Hkv * hd
    q_ref = synth.to_bf16_values(sfo.rope(qkv[:, :nqc].reshape(-1, Hq, hd), pos).astype(np.float32))
    k_ref = synth.to_bf16_values(sfo.rope(qkv[:, nqc:nqc + nkv].reshape(-1, Hkv, hd), pos).astype(np.float32))
    v_ref = qkv[:, nqc + nkv:].reshape(-1, Hkv, hd)
    kc_ref, vc_ref = np.nan_to_num(kc.astype(np.float64)), np.nan_to_num(vc.astype(np.float64))
    for b in range(B):
        for i in range(nq):
            kc_ref[b, :, lens[b] + i] = k_ref[b * nq + i]
            vc_ref[b, :, lens[b] + i] = v_ref[b * nq + i]
    ref = sfo.attention(q_ref.reshape(B, nq, Hq, hd), kc_ref, vc_ref, lens, mode)

    kvl = torch.from_numpy(lens).cuda()
    if True:
        eng = engine_only(shape_for("bf16", Hq, Hkv, hd), B, cap, max(nq - 1, 1))
        eng.sf_tune_attention(chunk)
        eng.sf_kv_import(kc, "dk"); eng.sf_kv_import(vc, "dv")
        out = eng.sf_op_rope_attention(dev(qkv, "bf16"), kvl, nq, eng.dk, eng.dv, mode)
        torch.cuda.synchronize()
        got, kg, vg = to_np(out), to_np(eng.sf_kv_export("dk")), to_np(eng.sf_kv_export("dv"))
        # the two-kernel route on a second pair of caches
        eng2 = engine_only(shape_for("bf16", Hq, Hkv, hd), B, cap, max(nq - 1, 1))
        eng2.sf_tune_attention(chunk)
        eng2.sf_kv_import(kc, "dk"); eng2.sf_kv_import(vc, "dv")
        q_rot = eng2.sf_op_rope_kv_append(dev(qkv, "bf16"), kvl, nq, eng2.dk, eng2.dv)
        out2 = eng2.sf_op_attention(q_rot.view(B, nq, Hq, hd), eng2.dk, eng2.dv, kvl, nq, mode)
        torch.cuda.synchronize()
        got2, kg2, vg2 = to_np(out2), to_np(eng2.sf_kv_export("dk")), to_np(eng2.sf_kv_export("dv"))
    assert np.all(np.isfinite(got))
    assert rel_err(got, ref) < BF16_TOL
    live = np.zeros((B, cap), bool)
    for b in range(B):
        live[b, :lens[b] + nq] = True
    for a, c in ((kg, kg2), (vg, vg2)):
        np.testing.assert_array_equal(a.transpose(0, 2, 1, 3)[live], c.transpose(0, 2, 1, 3)[live])
    assert rel_err(kg.transpose(0, 2, 1, 3)[live], kc_ref.transpose(0, 2, 1, 3)[live]) < BF16_TOL
    np.testing.assert_array_equal(vg.transpose(0, 2, 1, 3)[live], vc_ref.transpose(0, 2, 1, 3)[live])
    np.testing.assert_array_equal(got, got2)
