"""Model-level pins for the oracle: the verify pass against a decoder composed from torch library
routines, block rows == autoregressive decode, the draft block against a torch composition and
its structural special cases, and the lossless invariant (speculative greedy == plain greedy).
CPU only."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle import sfo
from oracle.sfo import DRAFT_TWO_STAGE, MASK_BIDIR, MASK_CAUSAL

SHAPE = synth.ModelShape("pin", 3, 32, 4, 2, 8, 48, 61, "f32")   # odd L: hooks at 0, 1, 2, 3
K_MAX = 4


def weights(std=0.25):
    # larger std than the workloads': makes attention / FFN terms matter in the pins
    return synth.target_weights(SHAPE, 7, std), synth.draft_weights(SHAPE, K_MAX, 7, std)


def T(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float64))


def t_rope(x, pos, theta):
    """x [T,H,hd] -> rotate pairs (i, i+hd/2) as complex numbers by pos * theta^(-2i/hd)."""
    hd = x.shape[-1]
    z = torch.complex(x[..., :hd // 2], x[..., hd // 2:])
    ang = pos.double()[:, None, None] * theta ** (-2.0 * torch.arange(hd // 2).double() / hd)
    z = z * torch.polar(torch.ones_like(ang), ang)
    return torch.cat([z.real, z.imag], -1)


def t_target(tw, toks):
    """Full causal forward of one sequence with torch library ops. Returns logits [T,V] and the
    hidden states after every layer (index 0 = embedding)."""
    m = SHAPE
    h = T(tw["embed"])[torch.as_tensor(toks).long()]
    pos = torch.arange(len(toks))
    hs = [h]
    nq, nkv = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    for l in range(m.n_layers):
        a = F.rms_norm(h, (m.d_model,), T(tw["attn_norm"][l]), m.rms_eps)
        qkv = F.linear(a, T(tw["wqkv"][l]))
        q = t_rope(qkv[:, :nq].view(-1, m.n_q_heads, m.head_dim), pos, m.rope_theta)
        k = t_rope(qkv[:, nq:nq + nkv].view(-1, m.n_kv_heads, m.head_dim), pos, m.rope_theta)
        v = qkv[:, nq + nkv:].view(-1, m.n_kv_heads, m.head_dim)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True, enable_gqa=True)
        h = h + F.linear(o[0].transpose(0, 1).reshape(len(toks), nq), T(tw["wo"][l]))
        a = F.rms_norm(h, (m.d_model,), T(tw["ffn_norm"][l]), m.rms_eps)
        h = h + F.linear(F.silu(F.linear(a, T(tw["w_gate"][l]))) * F.linear(a, T(tw["w_up"][l])),
                         T(tw["w_down"][l]))
        hs.append(h)
    logits = F.linear(F.rms_norm(h, (m.d_model,), T(tw["final_norm"]), m.rms_eps), T(tw["lm_head"]))
    return logits.numpy(), [x.numpy() for x in hs]


def t_draft(dw, lm_head, hooks, k, bidir=True):
    """hooks [T,4,d] of one sequence's whole committed context -> draft logits [k,V]."""
    m = SHAPE
    n, d = hooks.shape[0], m.d_model
    nq, nkv = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    f = torch.stack([F.rms_norm(T(hooks[:, g]), (d,), T(dw["group_norm"][g]), m.rms_eps) for g in range(4)], 1)
    x = F.linear(f.reshape(n, 4 * d), T(dw["w_ds"]))
    s0 = F.linear(F.rms_norm(x[-1], (d,), T(dw["pos_norm"]), m.rms_eps), T(dw["w_pos"])[:k * d],
                  T(dw["b_pos"])[:k * d]).view(k, d)
    seq = torch.cat([x, s0], 0)                                  # context rows then the k slots
    pos = torch.arange(n + k)
    a = F.rms_norm(seq, (d,), T(dw["attn_norm"]), m.rms_eps)
    qkv = F.linear(a, T(dw["wqkv"]))
    q = t_rope(qkv[:, :nq].view(-1, m.n_q_heads, m.head_dim), pos, m.rope_theta)[n:]
    kk = t_rope(qkv[:, nq:nq + nkv].view(-1, m.n_kv_heads, m.head_dim), pos, m.rope_theta)
    v = qkv[:, nq + nkv:].view(-1, m.n_kv_heads, m.head_dim)
    mask = torch.ones(k, n + k, dtype=torch.bool)
    if not bidir:
        mask[:, n:] = torch.tril(torch.ones(k, k, dtype=torch.bool))
    o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kk.transpose(0, 1)[None],
                                       v.transpose(0, 1)[None], attn_mask=mask, enable_gqa=True)
    s1 = s0 + F.linear(o[0].transpose(0, 1).reshape(k, nq), T(dw["wo"]))
    a = F.rms_norm(s1, (d,), T(dw["ffn_norm"]), m.rms_eps)
    s2 = s1 + F.linear(F.silu(F.linear(a, T(dw["w_gate"]))) * F.linear(a, T(dw["w_up"])), T(dw["w_down"]))
    return F.linear(F.rms_norm(s2, (d,), T(dw["out_norm"]), m.rms_eps), T(lm_head)).numpy()


def new_oracle(tw, dw, B, cap=64, q_max=24, rb=False):
    return sfo.Oracle(SHAPE.cfg(), tw, dw, B, cap, q_max, round_bf16=rb)


def test_prefill_and_verify_match_torch_decoder():
    tw, dw = weights()
    lens = [9, 4, 13]
    prompts = synth.prompts(lens, SHAPE.vocab, 3)
    o = new_oracle(tw, dw, 3)
    first = o.prefill(prompts)
    for b, p in enumerate(prompts):
        lg, hs = t_target(tw, p)
        assert first[b] == int(np.argmax(lg[-1]))
        L = SHAPE.n_layers
        for g, layer in enumerate([0, L // 2, L - 1, L]):
            np.testing.assert_allclose(o.hooks[b, :len(p), g], hs[layer], rtol=1e-9, atol=1e-11)
    np.testing.assert_array_equal(o.kv_len, lens)
    # one verify block of k+1 tokens behind the ragged prefixes
    k = 3
    draft = np.random.default_rng(0).integers(0, SHAPE.vocab, (3, k)).astype(np.int32)
    logits = o.verify_step(k, draft)
    for b, p in enumerate(prompts):
        seq = list(p) + [int(first[b])] + list(draft[b])
        lg, hs = t_target(tw, seq)
        np.testing.assert_allclose(logits[b], lg[len(p):], rtol=1e-8, atol=1e-10)
        np.testing.assert_allclose(o.hooks[b, :k + 1, 3], hs[SHAPE.n_layers][len(p):], rtol=1e-8, atol=1e-10)


def test_verify_rows_equal_autoregressive_steps():
    """Logits of block row i == logits of a single-token step after committing the first i block
    tokens: exact, because every row is computed independently in a fixed order."""
    tw, dw = weights()
    prompts = synth.prompts([6, 11], SHAPE.vocab, 4)
    k = 3
    draft = np.random.default_rng(1).integers(0, SHAPE.vocab, (2, k)).astype(np.int32)
    o = new_oracle(tw, dw, 2)
    o.prefill(prompts)
    blk = o.verify_step(k, draft)
    o2 = new_oracle(tw, dw, 2)
    o2.prefill(prompts)
    for i in range(k + 1):
        one = o2.verify_step(0, np.zeros((2, 0), np.int32))
        np.testing.assert_array_equal(one[:, 0], blk[:, i])
        o2.accept_commit(0, np.zeros((2, 0), np.int32), one)
        if i < k:
            o2.pending[:] = draft[:, i]                         # teacher-force the block's next token
    np.testing.assert_array_equal(o2.tk[:, :, :, :17], o.tk[:, :, :, :17])


@pytest.mark.parametrize("bidir", [True, False])
def test_draft_block_matches_torch_composition(bidir):
    tw, dw = weights()
    lens = [7, 12]
    prompts = synth.prompts(lens, SHAPE.vocab, 5)
    o = new_oracle(tw, dw, 2)
    o.prefill(prompts)
    k = K_MAX
    draft, lg = o.draft_step(k, MASK_BIDIR if bidir else MASK_CAUSAL, want_logits=True)
    for b, p in enumerate(prompts):
        _, hs = t_target(tw, p)
        L = SHAPE.n_layers
        hooks = np.stack([hs[0], hs[L // 2], hs[L - 1], hs[L]], 1)
        want = t_draft(dw, tw["lm_head"], hooks, k, bidir)
        np.testing.assert_allclose(lg[b], want, rtol=1e-8, atol=1e-10)
        np.testing.assert_array_equal(draft[b], want.argmax(-1))


def test_draft_incremental_context_equals_one_shot():
    """Feeding the committed rows step by step (the draft layer's own KV cache) gives the same
    draft as recomputing the whole context: the cache is the (L+1)-th layer's cache."""
    tw, dw = weights()
    prompts = synth.prompts([8, 5], SHAPE.vocab, 6)
    k = 3
    o = new_oracle(tw, dw, 2)
    o.prefill(prompts)
    o.draft_step(k)                                   # fills the draft cache for the prompt
    rs = np.random.default_rng(2)
    seqs = [list(p) for p in prompts]
    for _ in range(3):
        d = rs.integers(0, SHAPE.vocab, (2, k)).astype(np.int32)
        lg = o.verify_step(k, d)
        pend = o.pending.copy()
        acc, _ = o.accept_commit(k, d, lg, force_len=rs.integers(1, k + 2, 2))
        for b in range(2):
            seqs[b] += ([int(pend[b])] + list(d[b]))[:acc[b]]
        _, dl = o.draft_step(k, want_logits=True)
        for b in range(2):
            _, hs = t_target(tw, seqs[b])
            L = SHAPE.n_layers
            hooks = np.stack([hs[0], hs[L // 2], hs[L - 1], hs[L]], 1)
            np.testing.assert_allclose(dl[b], t_draft(dw, tw["lm_head"], hooks, k), rtol=1e-7, atol=1e-9)


def t_draft_two_stage(dw, lm_head, hooks, k, bidir=True):
    """The draft block with its two attentions kept apart (first and third equation of the SpecFormer
    section), composed from torch library ops: I_D = X + MSA(RMS(X)) causal over the context, slots
    from the newest row of I_D, then self-attention over the k slots alone with its own weights."""
    m = SHAPE
    n, d = hooks.shape[0], m.d_model
    nq, nkv = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim

    def attn(x, norm, wqkv, wo, causal):
        t = x.shape[0]
        pos = torch.arange(t)
        a = F.rms_norm(x, (d,), T(norm), m.rms_eps)
        qkv = F.linear(a, T(wqkv))
        q = t_rope(qkv[:, :nq].view(-1, m.n_q_heads, m.head_dim), pos, m.rope_theta)
        kk = t_rope(qkv[:, nq:nq + nkv].view(-1, m.n_kv_heads, m.head_dim), pos, m.rope_theta)
        v = qkv[:, nq + nkv:].view(-1, m.n_kv_heads, m.head_dim)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kk.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=causal, enable_gqa=True)
        return x + F.linear(o[0].transpose(0, 1).reshape(t, nq), T(wo))
    f = torch.stack([F.rms_norm(T(hooks[:, g]), (d,), T(dw["group_norm"][g]), m.rms_eps) for g in range(4)], 1)
    x = F.linear(f.reshape(n, 4 * d), T(dw["w_ds"]))
    i_d = attn(x, dw["attn_norm"], dw["wqkv"], dw["wo"], True)
    s0 = F.linear(F.rms_norm(i_d[-1], (d,), T(dw["pos_norm"]), m.rms_eps), T(dw["w_pos"])[:k * d],
                  T(dw["b_pos"])[:k * d]).view(k, d)
    s1 = attn(s0, dw["sa_norm"], dw["sa_wqkv"], dw["sa_wo"], not bidir)
    a = F.rms_norm(s1, (d,), T(dw["ffn_norm"]), m.rms_eps)
    s2 = s1 + F.linear(F.silu(F.linear(a, T(dw["w_gate"]))) * F.linear(a, T(dw["w_up"])), T(dw["w_down"]))
    return F.linear(F.rms_norm(s2, (d,), T(dw["out_norm"]), m.rms_eps), T(lm_head)).numpy()


@pytest.mark.parametrize("bidir", [True, False])
def test_two_stage_draft_matches_torch_composition(bidir):
    tw, dw = weights()
    lens = [7, 12]
    prompts = synth.prompts(lens, SHAPE.vocab, 5)
    o = new_oracle(tw, dw, 2)
    o.prefill(prompts)
    k = K_MAX
    mode = (MASK_BIDIR if bidir else MASK_CAUSAL) | DRAFT_TWO_STAGE
    draft, lg = o.draft_step(k, mode, want_logits=True)
    for b, p in enumerate(prompts):
        _, hs = t_target(tw, p)
        L = SHAPE.n_layers
        hooks = np.stack([hs[0], hs[L // 2], hs[L - 1], hs[L]], 1)
        want = t_draft_two_stage(dw, tw["lm_head"], hooks, k, bidir)
        np.testing.assert_allclose(lg[b], want, rtol=1e-8, atol=1e-10)
        np.testing.assert_array_equal(draft[b], want.argmax(-1))
    # and it is not the single-attention wiring in disguise
    o2 = new_oracle(tw, dw, 2); o2.prefill(prompts)
    _, lg_h = o2.draft_step(k, MASK_BIDIR if bidir else MASK_CAUSAL, want_logits=True)
    assert not np.allclose(lg_h, lg)


def test_two_stage_draft_incremental_context_equals_one_shot():
    """The context attention of the two-stage wiring reads the draft layer's KV cache: feeding the
    committed rows step by step equals recomputing the whole context."""
    tw, dw = weights()
    prompts = synth.prompts([8, 5], SHAPE.vocab, 6)
    k = 3
    o = new_oracle(tw, dw, 2)
    o.prefill(prompts)
    o.draft_step(k, MASK_BIDIR | DRAFT_TWO_STAGE)
    rs = np.random.default_rng(2)
    seqs = [list(p) for p in prompts]
    for _ in range(3):
        d = rs.integers(0, SHAPE.vocab, (2, k)).astype(np.int32)
        lg = o.verify_step(k, d)
        pend = o.pending.copy()
        acc, _ = o.accept_commit(k, d, lg, force_len=rs.integers(1, k + 2, 2))
        for b in range(2):
            seqs[b] += ([int(pend[b])] + list(d[b]))[:acc[b]]
        _, dl = o.draft_step(k, MASK_BIDIR | DRAFT_TWO_STAGE, want_logits=True)
        for b in range(2):
            _, hs = t_target(tw, seqs[b])
            L = SHAPE.n_layers
            hooks = np.stack([hs[0], hs[L // 2], hs[L - 1], hs[L]], 1)
            np.testing.assert_allclose(dl[b], t_draft_two_stage(dw, tw["lm_head"], hooks, k), rtol=1e-7, atol=1e-9)


def test_two_stage_slots_do_not_see_the_context_keys_directly():
    """In the two-stage wiring the context reaches the slots only through the newest row of I_D.
    With W_P zeroed the slot states are b_P alone, and since the slot attention has no cached keys
    the draft then cannot depend on the context at all; the single hybrid attention still reads the
    draft cache and does."""
    tw, dw = weights()
    k = 3
    dw0 = dict(dw)
    dw0["w_pos"] = np.zeros_like(dw["w_pos"])
    outs = []
    for seed in (11, 12):
        prompts = synth.prompts([5, 9], SHAPE.vocab, seed)
        o = new_oracle(tw, dw0, 2); o.prefill(prompts)
        outs.append(o.draft_step(k, MASK_BIDIR | DRAFT_TWO_STAGE, want_logits=True)[1])
    np.testing.assert_array_equal(outs[0], outs[1])          # slots = b_P only: context-free
    np.testing.assert_array_equal(outs[0][0], outs[0][1])    # and the same for every sequence
    outs_h = []
    for seed in (11, 12):
        prompts = synth.prompts([5, 9], SHAPE.vocab, seed)
        o = new_oracle(tw, dw0, 2); o.prefill(prompts)
        outs_h.append(o.draft_step(k, MASK_BIDIR, want_logits=True)[1])
    assert not np.allclose(outs_h[0], outs_h[1])             # one hybrid attention still reads the cache


def test_positional_ffn_slots_use_their_own_rows_of_w_pos():
    """W_P has k * d * d position-specific weights; slot s is produced by rows [s*d,(s+1)*d)."""
    tw, dw = weights()
    d = SHAPE.d_model
    assert dw["w_pos"].shape == (K_MAX * d, d) and dw["w_pos"].size == K_MAX * d * d
    prompts = synth.prompts([6], SHAPE.vocab, 8)
    base = new_oracle(tw, dw, 1); base.prefill(prompts)
    _, lg0 = base.draft_step(K_MAX, MASK_CAUSAL, want_logits=True)
    dw2 = dict(dw); wp = dw["w_pos"].copy(); wp[2 * d:3 * d] *= 1.5; dw2["w_pos"] = wp
    o = new_oracle(tw, dw2, 1); o.prefill(prompts)
    _, lg1 = o.draft_step(K_MAX, MASK_CAUSAL, want_logits=True)
    # causal block: slots before the edited one are untouched, the edited one and later ones move
    np.testing.assert_array_equal(lg1[0, :2], lg0[0, :2])
    assert not np.allclose(lg1[0, 2], lg0[0, 2]) and not np.allclose(lg1[0, 3], lg0[0, 3])


def run_spec(o, prompts, k, steps, draft_fn):
    first = o.prefill(prompts)
    outs = [[int(t)] for t in first]
    accs = []
    for _ in range(steps):
        natural = o.draft_step(k)
        d = draft_fn(natural, outs)
        lg = o.verify_step(k, d)
        acc, out = o.accept_commit(k, d, lg)
        accs.append(acc.copy())
        for b in range(o.B):
            outs[b] += [int(t) for t in out[b, :acc[b]]]
    return outs, np.array(accs)


def run_ar(o, prompts, n_tokens):
    first = o.prefill(prompts)
    outs = [[int(t)] for t in first]
    none = np.zeros((o.B, 0), np.int32)
    while min(len(x) for x in outs) < n_tokens:
        lg = o.verify_step(0, none)
        acc, out = o.accept_commit(0, none, lg)
        assert np.all(acc == 1)
        for b in range(o.B):
            outs[b].append(int(out[b, 0]))
    return outs


@pytest.mark.parametrize("rb", [False, True])
def test_lossless_speculative_equals_plain_greedy(rb):
    """Speculative greedy output is token-identical to plain autoregressive greedy decoding of the
    target for ANY draft: natural, all wrong, all right, partly right."""
    tw, dw = weights()
    k, steps = 3, 5
    prompts = synth.prompts([5, 9, 7], SHAPE.vocab, 9)
    ar = run_ar(new_oracle(tw, dw, 3, cap=96, rb=rb), prompts, 1 + steps * (k + 1))

    def natural(nat, outs):
        return nat

    def all_wrong(nat, outs):
        return np.array([[(ar[b][len(outs[b]) + i] + 1) % SHAPE.vocab for i in range(k)]
                         for b in range(3)], np.int32)

    def all_right(nat, outs):
        return np.array([[ar[b][len(outs[b]) + i] for i in range(k)] for b in range(3)], np.int32)

    def partly(nat, outs):
        d = all_right(nat, outs)
        d[0, 1] = (d[0, 1] + 1) % SHAPE.vocab
        d[2, 2] = (d[2, 2] + 1) % SHAPE.vocab
        return d

    for fn, want_acc in ((natural, None), (all_wrong, 1), (all_right, k + 1), (partly, None)):
        outs, accs = run_spec(new_oracle(tw, dw, 3, cap=96, rb=rb), prompts, k, steps, fn)
        for b in range(3):
            assert outs[b] == ar[b][:len(outs[b])], fn.__name__
        assert accs.min() >= 1 and accs.max() <= k + 1
        if want_acc is not None:
            assert np.all(accs == want_acc)
        if fn is partly:
            assert np.all(accs[:, 0] == 2) and np.all(accs[:, 1] == k + 1) and np.all(accs[:, 2] == 3)


def test_round_bf16_mode_stays_close_to_exact_mode_and_rounds_what_is_stored():
    """The rounding emulation moves the pin model's logits by well under the bf16 tolerance of the
    GPU parity tests, stores bf16 values in hooks and caches, and leaves the residual stream wider:
    HS[L] as hooked is the bf16 rounding of a row that is itself not bf16-representable (the final
    logits depend on the unrounded row)."""
    tw, dw = weights(0.1)
    tw = {n: ([synth.to_bf16_values(a) for a in v] if isinstance(v, list) else synth.to_bf16_values(v))
          for n, v in tw.items()}
    prompts = synth.prompts([9, 6], SHAPE.vocab, 12)
    k = 3
    draft = np.random.default_rng(3).integers(0, SHAPE.vocab, (2, k)).astype(np.int32)
    lg = {}
    for rb in (False, True):
        o = new_oracle(tw, dw, 2, rb=rb)
        o.prefill(prompts)
        lg[rb] = o.verify_step(k, draft)
        if rb:
            hk = o.hooks[:, :k + 1]
            np.testing.assert_array_equal(hk, synth.to_bf16_values(hk.astype(np.float32)))
            n = int(o.kv_len.min())
            np.testing.assert_array_equal(o.tk[:, :, :, :n], synth.to_bf16_values(o.tk[:, :, :, :n].astype(np.float32)))
            # logits from the rounded hook HS[L] differ from the real ones: the stream itself is not rounded
            a = sfo.rmsnorm(hk[:, :, 3], tw["final_norm"], SHAPE.rms_eps)
            from_hook = sfo.linear(synth.to_bf16_values(a.astype(np.float32)).astype(np.float64), tw["lm_head"])
            assert not np.array_equal(from_hook.astype(np.float32), lg[True].astype(np.float32))
    err = np.abs(lg[True] - lg[False]).max() / np.abs(lg[False]).max()
    assert 0 < err < 1e-2, err
