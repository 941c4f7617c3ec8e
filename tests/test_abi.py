"""The C-ABI library loads without a GPU, exports every symbol include/specformer.h and
include/specformer_aux.h declare, and its host-side argument checking returns the documented status
codes.  No kernel is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2511_20340_amd import binding as sfb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in ("specformer.h", "specformer_aux.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(sf_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported():
    L = sfb.lib()
    names = declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), n
    assert sorted(sfb.EXPORTS) == names
    assert b"gfx950" in L.sf_version()


def cfg(**kw):
    base = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=1024, vocab=1024,
                rope_theta=10000.0, rms_eps=1e-6, dtype=sfb.SF_F32)
    base.update(kw)
    return sfb.ModelCfg(*[base[n] for n, _ in sfb.ModelCfg._fields_])


def create(t, d, B=4, k=4):
    ctx = C.c_void_p()
    return sfb.lib().sf_create(C.byref(t), C.byref(d), B, k, C.byref(ctx)), ctx


def test_create_validates_arguments():
    L = sfb.lib()
    st, ctx = create(cfg(), cfg(n_layers=1))
    assert st == sfb.SF_OK and ctx.value
    assert L.sf_workspace_bytes(ctx, 4, 4, 128) > 0
    assert L.sf_workspace_bytes(ctx, 5, 4, 128) == 0            # B > max_B
    assert L.sf_workspace_bytes(ctx, 4, 5, 128) == 0            # k > max_k
    assert L.sf_workspace_bytes(ctx, 4, 4, 100) == 0            # cap not a multiple of 32
    assert L.sf_kv_cache_bytes(ctx, 0, 4, 128) == 2 * 4 * 4 * 128 * 64 * 4
    assert L.sf_kv_cache_bytes(ctx, 1, 4, 128) == 4 * 4 * 128 * 64 * 4
    assert L.sf_destroy(ctx) == sfb.SF_OK
    assert create(cfg(), cfg(n_layers=2))[0] == sfb.SF_EINVAL               # draft block is one layer
    assert create(cfg(), cfg(n_layers=1, d_ffn=512))[0] == sfb.SF_EINVAL    # widths must agree
    assert create(cfg(n_q_heads=6), cfg(n_layers=1, n_q_heads=6))[0] == sfb.SF_EINVAL   # Hq % Hkv
    assert create(cfg(), cfg(n_layers=1), B=0)[0] == sfb.SF_EINVAL
    assert create(cfg(), cfg(n_layers=1), k=128)[0] == sfb.SF_EINVAL
    bf = dict(dtype=sfb.SF_BF16, head_dim=96, d_model=384)
    assert create(cfg(**bf), cfg(n_layers=1, **bf))[0] == sfb.SF_EUNSUPPORTED   # bf16 head_dim
    wide = dict(dtype=sfb.SF_BF16, n_q_heads=32, n_kv_heads=2, head_dim=64, d_model=2048)
    assert create(cfg(**wide), cfg(n_layers=1, **wide), k=4)[0] == sfb.SF_OK
    assert create(cfg(**wide), cfg(n_layers=1, **wide), k=64)[0] == sfb.SF_EUNSUPPORTED  # 16*65 rows > 1024


def test_steps_reject_bad_state_before_launching_anything():
    L = sfb.lib()
    st, ctx = create(cfg(), cfg(n_layers=1))
    assert st == sfb.SF_OK
    s = sfb.State()
    s.B, s.cap = 4, 128
    # not bound yet
    assert L.sf_verify_step(ctx, C.byref(s), 4, None, 0, None, None, None) == sfb.SF_ESTATE
    # bind with a missing pointer
    tw = sfb.TargetWeights()
    assert L.sf_bind(ctx, C.byref(tw), None) == sfb.SF_EINVAL
    fake = 0x1000
    arr = (C.c_void_p * 2)(fake, fake)
    for n, _ in sfb.TargetWeights._fields_:
        setattr(tw, n, arr if n not in ("embed", "lm_head", "final_norm") else fake)
    assert L.sf_bind(ctx, C.byref(tw), None) == sfb.SF_OK
    # draft step needs draft weights
    assert L.sf_draft_step(ctx, C.byref(s), 4, 1, 0, None, None, None) == sfb.SF_ESTATE
    # null state buffers
    assert L.sf_verify_step(ctx, C.byref(s), 4, None, 0, None, None, None) == sfb.SF_EINVAL
    for n in ("tk", "tv", "dk", "dv", "kv_len", "pending", "hooks", "n_new", "cu_new"):
        setattr(s, n, fake)
    s.workspace, s.workspace_bytes = 0x10000, 16
    assert L.sf_verify_step(ctx, C.byref(s), 4, fake, 0, None, fake, None) == sfb.SF_ECAPACITY   # workspace
    s.workspace_bytes = L.sf_workspace_bytes(ctx, 4, 4, 128)
    assert L.sf_verify_step(ctx, C.byref(s), 5, fake, 0, None, fake, None) == sfb.SF_EINVAL      # k > max_k
    assert L.sf_verify_step(ctx, C.byref(s), 4, fake, 124, None, fake, None) == sfb.SF_ECAPACITY  # 124+5 > 128
    assert L.sf_verify_step(ctx, C.byref(s), 4, None, 0, None, fake, None) == sfb.SF_EINVAL      # no draft tokens
    assert L.sf_verify_step(ctx, C.byref(s), 4, fake, 0, fake, None, None) == sfb.SF_EINVAL      # no target_ids
    s.workspace = 0x10010
    assert L.sf_verify_step(ctx, C.byref(s), 4, fake, 0, None, fake, None) == sfb.SF_EINVAL      # misaligned
    s.workspace = 0x10000
    assert L.sf_accept_commit(ctx, C.byref(s), 4, fake, None, None, fake, fake, None) == sfb.SF_EINVAL
    # call order: nothing was verified on this context, so there is no block to commit
    assert L.sf_accept_commit(ctx, C.byref(s), 4, fake, fake, None, fake, fake, None) == sfb.SF_ESTATE
    assert L.sf_op_accept(ctx, 4, 4, fake, None, None, fake, fake, fake, fake, fake, fake, None) == sfb.SF_EINVAL
    assert L.sf_tune_linear(ctx, 99, 0) == sfb.SF_EINVAL and L.sf_tune_linear(ctx, 0, 0) == sfb.SF_OK
    assert L.sf_tune_attention(ctx, 3) == sfb.SF_EINVAL and L.sf_tune_attention(None, 0) == sfb.SF_EINVAL
    # the slot attention's own weights come whole or not at all, and the two-stage wiring needs them
    s.workspace = 0x10000
    dw = sfb.DraftWeights()
    for n, _ in sfb.DraftWeights._fields_:
        setattr(dw, n, None if n.startswith("sa_") else fake)
    assert L.sf_bind(ctx, C.byref(tw), C.byref(dw)) == sfb.SF_OK
    two_stage = sfb.SF_MASK_BIDIR | sfb.SF_DRAFT_TWO_STAGE
    assert L.sf_draft_step(ctx, C.byref(s), 4, two_stage, 0, fake, None, None) == sfb.SF_ESTATE
    assert L.sf_draft_step(ctx, C.byref(s), 4, 7, 0, fake, None, None) == sfb.SF_EINVAL     # no such mask
    dw.sa_norm = fake
    assert L.sf_bind(ctx, C.byref(tw), C.byref(dw)) == sfb.SF_EINVAL
    dw.pos_norm = None
    dw.sa_norm = None
    assert L.sf_bind(ctx, C.byref(tw), C.byref(dw)) == sfb.SF_EINVAL
    assert L.sf_last_hip_error(ctx) == 0
    assert b"capacity" in L.sf_strerror(sfb.SF_ECAPACITY)
    L.sf_destroy(ctx)


def test_rope_attention_op_validates_before_launching_anything():
    L = sfb.lib()
    fake = 0x10000
    bf = dict(dtype=sfb.SF_BF16, n_q_heads=8, n_kv_heads=2, head_dim=64, d_model=512)
    st, ctx = create(cfg(**bf), cfg(n_layers=1, **bf))
    assert st == sfb.SF_OK
    need = L.sf_rope_attention_workspace_bytes(ctx, 4, 5, 100)
    assert need >= 4 * 5 * 32 * 8                      # at least the cos/sin table
    assert L.sf_rope_attention_workspace_bytes(ctx, 0, 5, 100) == 0
    call = lambda **kw: L.sf_op_rope_attention(ctx, kw.get("qkv", fake), fake, kw.get("B", 4), kw.get("n_q", 5),
                                               kw.get("cap", 128), kw.get("mask", sfb.SF_MASK_BIDIR),
                                               kw.get("upper", 100), fake, fake, fake, kw.get("ws", fake),
                                               kw.get("ws_bytes", need), None)
    assert call(qkv=None) == sfb.SF_EINVAL
    assert call(cap=100) == sfb.SF_EINVAL              # not a multiple of the 32-key tile
    assert call(mask=9) == sfb.SF_EINVAL
    assert call(upper=124) == sfb.SF_ECAPACITY         # 124 + 5 > 128
    assert call(ws_bytes=need - 1) == sfb.SF_ECAPACITY
    assert call(ws=fake + 16) == sfb.SF_ECAPACITY      # misaligned workspace
    assert call(n_q=257, cap=512, upper=100) == sfb.SF_EUNSUPPORTED   # 4 query heads per kv head x 257 rows > 1024
    L.sf_destroy(ctx)
    st, ctx32 = create(cfg(), cfg(n_layers=1))         # fp32 keeps the two separate kernels
    assert st == sfb.SF_OK
    assert L.sf_op_rope_attention(ctx32, fake, fake, 4, 5, 128, sfb.SF_MASK_BIDIR, 100, fake, fake, fake, fake,
                                  1 << 20, None) == sfb.SF_EUNSUPPORTED
    L.sf_destroy(ctx32)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(sfb, "_lib", None)
    monkeypatch.setattr(sfb, "LIB_PATH", "/nonexistent/libspecformer.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        sfb.lib()
