"""GPU parity at the benchmark workloads' real sizes, in the launch configuration bench.py times.

The oracle cannot run a whole 1B / 8B batch, so each test compares a SAMPLE of the outputs that the
oracle computes one by one from the same seeded inputs (whole sequences of the attention, sampled rows
x columns of the linear layers, two of the 32 sequences of a whole 1B step), plus properties that
hold at any size (the speculative stream equals the plain-greedy stream; graph replay equals eager).
"""
import numpy as np
import pytest
import torch

import synth
from oracle import sfo
from paper_2511_20340_amd import binding as sfb
from paper_2511_20340_amd.engine import Engine

from gpu_common import engine_only, rel_err, to_np

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2


def device_normal(shape, seed, dtype=torch.bfloat16):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randn(*shape, generator=g, device="cuda", dtype=torch.float32).to(dtype)


# ---- attention: workload shapes, ragged lengths, a few whole sequences against the oracle -------------
@pytest.mark.parametrize("name,B,Hq,Hkv,hd,lo,hi,nq,mode", [
    ("1b verify", 32, 32, 8, 64, 512, 512, 5, sfb.SF_MASK_CAUSAL),
    ("1b draft slots", 32, 32, 8, 64, 512, 512, 4, sfb.SF_MASK_BIDIR),
    ("8b verify", 64, 32, 8, 128, 256, 2048, 5, sfb.SF_MASK_CAUSAL),
    ("8b sweep", 256, 32, 8, 128, 1024, 1024, 5, sfb.SF_MASK_CAUSAL),
    ("14b verify", 128, 40, 8, 128, 1024, 4096, 5, sfb.SF_MASK_CAUSAL),
])
def test_attention_full_shape_sampled_sequences(name, B, Hq, Hkv, hd, lo, hi, nq, mode):
    lens = synth.prefix_lengths(B, lo, hi, 31)
    cap = synth.kv_capacity(int(lens.max()), 2, nq)
    shape = synth.ModelShape("t", 1, Hq * hd, Hq, Hkv, hd, 256, 512, "bf16")
    eng = engine_only(shape, B, cap, max(nq - 1, 1))
    q = device_normal((B, nq, Hq, hd), 1)
    kc = device_normal((B, Hkv, cap, hd), 2)
    vc = device_normal((B, Hkv, cap, hd), 3)
    eng.sf_kv_import(kc, "dk")
    eng.sf_kv_import(vc, "dv")
    kvl = torch.from_numpy(lens).cuda()
    # the bound bench.py's graph capture uses: the capacity, not the longest sequence
    out = eng.sf_op_attention(q, eng.dk, eng.dv, kvl, nq, mode, len_upper=cap - nq)
    torch.cuda.synchronize()
    order = np.argsort(lens)
    for b in {int(order[0]), int(order[-1]), int(order[B // 2]), 0, B - 1}:
        ref = sfo.attention(to_np(q[b:b + 1]), to_np(kc[b:b + 1]), to_np(vc[b:b + 1]), lens[b:b + 1], mode)
        assert rel_err(to_np(out[b:b + 1]), ref) < BF16_TOL, (name, b, int(lens[b]))


# ---- linear layers: real weight shapes, sampled rows x columns -----------------------------------------
@pytest.mark.parametrize("M,N,K,glu", [
    (160, 3072, 2048, False), (160, 2048, 8192, False), (160, 32000, 2048, False), (160, 16384, 2048, True),
    (32, 2048, 8192, False), (320, 6144, 4096, False), (320, 4096, 14336, False), (320, 28672, 4096, True),
    (1280, 28672, 4096, True), (640, 5120, 13824, False),
    # wide layers that take the tall tiles (320 / 256 / 224 / 192 rows per workgroup)
    (640, 27648, 5120, True), (1024, 28672, 4096, True), (896, 27648, 5120, False), (768, 28672, 4096, False)])
def test_linear_full_shape_sampled_outputs(M, N, K, glu):
    x = device_normal((M, K), 5)
    w = (device_normal((N, K), 6, torch.float32) * 0.02).to(torch.bfloat16)
    eng = engine_only(synth.ModelShape("t", 1, 128, 2, 2, 64, 64, 64, "bf16"), 1, 64, 1)
    g = np.random.default_rng(N + K)
    rows = np.unique(np.concatenate([[0, M - 1], g.integers(0, M, 24)]))
    if glu:
        F = N // 2
        y = eng.sf_op_linear_swiglu(x, w)
        cols = np.unique(np.concatenate([[0, F - 1], g.integers(0, F, 96)]))
        xs, wg, wu = to_np(x[rows]), to_np(w[cols]), to_np(w[F + cols])
        gate, up = sfo.linear(xs, wg), sfo.linear(xs, wu)
        ref = sfo.silu_mul(gate, up)
        got = to_np(y)[np.ix_(rows, cols)]
        assert rel_err(got, ref) < BF16_TOL
    else:
        y = eng.sf_op_linear(x, w, out_f32=True)
        cols = np.unique(np.concatenate([[0, N - 1], g.integers(0, N, 96)]))
        ref = sfo.linear(to_np(x[rows]), to_np(w[cols]))
        got = to_np(y)[np.ix_(rows, cols)]
        assert rel_err(got, ref) < 1e-5          # fp32 accumulators, unrounded output


# ---- acceptance at full vocabulary / batch ---------------------------------------------------------------
@pytest.mark.parametrize("B,k,V", [(64, 4, 128256), (256, 4, 32000)])
def test_accept_commit_full_size_bit_exact(B, k, V):
    g = np.random.default_rng(B + V)
    logits = g.standard_normal((B, k + 1, V), dtype=np.float32)
    top = logits.argmax(-1)
    draft = top[:, :k].astype(np.int32)                       # all accepted ...
    cut = g.integers(0, k + 1, B)                             # ... up to a random first mismatch
    for b in range(B):
        if cut[b] < k:
            draft[b, cut[b]] = (draft[b, cut[b]] + 1) % V
    shape = synth.ModelShape("t", 1, 128, 2, 2, 64, 64, V, "f32")
    tw = synth.target_weights(shape, 1)
    orc = sfo.Oracle(shape.cfg(), tw, None, B, 64, q_max=k + 1)
    lens = g.integers(1, 20, B).astype(np.int32)
    orc.kv_len[:] = lens
    acc_o, out_o = orc.accept_commit(k, draft, logits.astype(np.float64))
    eng = engine_only(shape, B, 64, k)
    eng.bind(tw)
    eng.set_state(kv_len=lens, pending=np.zeros(B, np.int32), n_new=np.ones(B, np.int32))
    ids = eng.sf_op_argmax(torch.from_numpy(logits).cuda().reshape(B * (k + 1), V)).reshape(B, k + 1)
    acc_g, out_g = eng.sf_op_accept(k, torch.from_numpy(draft).cuda(), ids)
    np.testing.assert_array_equal(acc_g.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(acc_o, np.minimum(cut, k) + 1)
    np.testing.assert_array_equal(out_g.cpu().numpy(), out_o)
    np.testing.assert_array_equal(eng.kv_len.cpu().numpy(), orc.kv_len)
    np.testing.assert_array_equal(eng.pending.cpu().numpy(), orc.pending)
    np.testing.assert_array_equal(eng.cu_new.cpu().numpy(), orc.cu_new)


# ---- whole steps at real width: oracle sequences inside a GPU batch ----------------------------------------
def top2_gap(logits):
    s = np.sort(logits, axis=-1)
    return s[..., -1] - s[..., -2]


def safe_positions(got, want):
    """Rows whose arg-max provably agrees: every logit of the row moved by at most e = max_v |got - want|,
    so the oracle's winner stays ahead when its lead over the runner-up exceeds 2 e."""
    return top2_gap(want) > 2.0 * np.abs(got - want).max(-1)


def greedy_chain(orc, k):
    """The oracle's own plain-greedy continuation of every sequence, k tokens after the pending one
    (k single-token verify + accept steps on a state that is restored afterwards)."""
    snap = orc.snapshot()
    none = np.zeros((orc.B, 0), np.int32)
    chain = []
    for _ in range(k):
        lg = orc.verify_step(0, none)
        chain.append(orc.accept_commit(0, none, lg)[1][:, 0].copy())
    orc.restore(snap)
    return np.stack(chain, 1).astype(np.int32)


def seed_oracle_state(orc, lens, vocab, g):
    for name in ("tk", "tv", "dk", "dv", "hooks"):
        a = getattr(orc, name)
        a[...] = synth.to_bf16_values(g.standard_normal(a.shape, dtype=np.float32))
    orc.kv_len[:] = lens
    orc.n_new[:] = 1
    orc.pending[:] = g.integers(0, vocab, orc.B)


def push_state(eng, orc, rows, k):
    """Teacher forcing: batch rows `rows` of the engine take the oracle's caches, hooks, lengths, tokens."""
    for which, src, layers in (("tk", orc.tk, orc.L), ("tv", orc.tv, orc.L), ("dk", orc.dk[None], 1), ("dv", orc.dv[None], 1)):
        for l in range(layers):
            plain = eng.sf_kv_export(which, l)
            plain[rows] = torch.from_numpy(src[l].astype(np.float32)).cuda().to(eng.tdtype)
            eng.sf_kv_import(plain, which, l)
    eng.hooks[rows] = torch.from_numpy(orc.hooks[:, :k + 1].astype(np.float32)).cuda().to(eng.tdtype)
    for name in ("kv_len", "pending", "n_new"):
        getattr(eng, name)[rows] = torch.from_numpy(getattr(orc, name)).cuda()


def check_step_against_oracle(eng, orc, ref, rows, k, draft_o, tally):
    """One draft -> verify -> accept step of the engine, whose batch rows `rows` start from the oracle's
    state: logits / hooks / appended K,V within BF16_TOL of the exact oracle `ref`, ids exact against the
    rounding oracle `orc` at provably safe positions, acceptance exact on identical inputs."""
    B, Bp = eng.B, len(rows)
    m_vocab = eng.V
    # draft
    d_o, dl_o = orc.draft_step(k, want_logits=True)
    _, dl_ref = ref.draft_step(k, want_logits=True)
    dl_g = torch.empty(B, k, m_vocab, dtype=torch.float32, device="cuda")
    d_g = eng.sf_draft_step(k, logits_out=dl_g)
    got = to_np(dl_g[rows])
    e_draft = rel_err(got, dl_ref)
    assert e_draft < BF16_TOL, e_draft
    safe = safe_positions(got, dl_o)
    np.testing.assert_array_equal(d_g[rows].cpu().numpy()[safe], d_o[safe])
    np.testing.assert_array_equal(d_g[rows].cpu().numpy(), got.argmax(-1))          # fused arg-max == arg-max
    tally["safe"] += int(safe.sum()); tally["n"] += safe.size
    # verify: the given drafts (else the rounding oracle's own) for the oracle's sequences, the GPU's own for the rest
    if draft_o is None:
        draft_o = d_o
    draft = d_g.clone()
    draft[rows] = torch.from_numpy(draft_o).cuda()
    lens0 = orc.kv_len.copy()
    lg_o = orc.verify_step(k, draft_o)
    lg_ref = ref.verify_step(k, draft_o)
    lg_g, tid_g = eng.sf_verify_step(k, draft)
    got = to_np(lg_g[rows])
    e_exact, e_emul = rel_err(got, lg_ref), rel_err(got, lg_o)
    assert e_exact < BF16_TOL, (e_exact, e_emul)
    tid = tid_g[rows].cpu().numpy()
    np.testing.assert_array_equal(tid, got.argmax(-1))                              # fused arg-max == arg-max
    safe = safe_positions(got, lg_o)
    np.testing.assert_array_equal(tid[safe], lg_o.argmax(-1)[safe])
    tally["safe"] += int(safe.sum()); tally["n"] += safe.size
    assert rel_err(to_np(eng.hooks[rows]), ref.hooks[:, :k + 1]) < BF16_TOL
    for l in (0, orc.L - 1):
        kg, vg = to_np(eng.sf_kv_export("tk", l)[rows]), to_np(eng.sf_kv_export("tv", l)[rows])
        for i in range(Bp):
            blk = slice(int(lens0[i]), int(lens0[i]) + k + 1)
            assert rel_err(kg[i][:, blk], ref.tk[l][i][:, blk]) < BF16_TOL
            assert rel_err(vg[i][:, blk], ref.tv[l][i][:, blk]) < BF16_TOL
    # accept: exact against the oracle's rule applied to the engine's own logits (no guard band) ...
    kv_before, pend_before = orc.kv_len.copy(), orc.pending.copy()
    acc_own, out_own = orc.accept_commit(k, draft_o, got)          # oracle rule on the GPU's logits
    kv_own, pend_own = orc.kv_len.copy(), orc.pending.copy()
    orc.kv_len[:] = kv_before; orc.pending[:] = pend_before
    acc_o, out_o = orc.accept_commit(k, draft_o, lg_o)             # and on its own logits: the trajectory
    acc_g, out_g = eng.sf_accept_commit(k, draft, tid_g)
    np.testing.assert_array_equal(acc_g[rows].cpu().numpy(), acc_own)
    np.testing.assert_array_equal(out_g[rows].cpu().numpy(), out_own)
    np.testing.assert_array_equal(eng.kv_len[rows].cpu().numpy(), kv_own)
    np.testing.assert_array_equal(eng.pending[rows].cpu().numpy(), pend_own)
    # ... and against the oracle's own result wherever every position the rule looks at -- up to and including
    # the first mismatch -- is provably safe
    ok = np.array([safe[i, :acc_o[i]].all() for i in range(Bp)])
    np.testing.assert_array_equal(acc_g[rows].cpu().numpy()[ok], acc_o[ok])
    np.testing.assert_array_equal(out_g[rows].cpu().numpy()[ok], out_o[ok])
    tally["rows_ok"] += int(ok.sum()); tally["rows"] += ok.size
    tally["acc"].append(acc_o.copy())
    tally["err"].append((round(e_draft, 5), round(e_exact, 5), round(e_emul, 5)))
    return d_g, lg_g, acc_g, out_g, draft


def corrupt_chain(chain, vocab):
    """Sequence b keeps the first b % (k+1) tokens of its true continuation, the rest are wrong."""
    d = chain.copy()
    k = d.shape[1]
    for b in range(d.shape[0]):
        d[b, b % (k + 1):] = (d[b, b % (k + 1):] + 1) % vocab
    return d


def test_1b_full_step_oracle_sequences_and_graph_replay():
    """The benchmarked 1B workload at its real size (16 layers, batch 32, prefix 512, k 4), launch grids
    pinned as in the HIP graph that bench.py replays; four of the 32 sequences are run by the oracle."""
    wl = synth.WORKLOADS[1]
    m, B, k = wl.model, wl.batch, wl.k
    prefix, Bp = int(wl.prefix_hi), 4
    rows = [0, 9, 20, 31]
    cap = synth.kv_capacity(prefix, 4, k)
    tw_d, dw_d = synth.device_weights(m, k, wl.seed)
    tw, dw = synth.host_weights(tw_d, dw_d)
    orc = sfo.Oracle(m.cfg(), tw, dw, Bp, cap, q_max=k + 1, round_bf16=True)
    ref = sfo.Oracle(m.cfg(), tw, dw, Bp, cap, q_max=k + 1, round_bf16=False)
    g = synth.rng(wl.seed, 777)
    seed_oracle_state(orc, prefix, m.vocab, g)
    ref.restore(orc.snapshot())

    eng = Engine(m.cfg(), B, cap, k)
    eng.bind(tw_d, dw_d)
    del tw_d, dw_d
    # the other sequences: random state of their own
    for which in ("tk", "tv", "dk", "dv"):
        buf = getattr(eng, which)
        buf.copy_(device_normal((buf.numel(),), 100 + len(which) + ord(which[0])))
    eng.hooks.copy_(device_normal(tuple(eng.hooks.shape), 9))
    eng.set_state(kv_len=np.full(B, prefix, np.int32), pending=synth.rng(wl.seed, 5).integers(0, m.vocab, B).astype(np.int32),
                  n_new=np.ones(B, np.int32))
    push_state(eng, orc, rows, k)
    eng.pin_len_upper()                               # the launch grids of bench.py's graph capture
    snap = {n: getattr(eng, n).clone() for n in ("kv_len", "pending", "n_new", "cu_new", "hooks")}

    draft_o = corrupt_chain(greedy_chain(orc, k), m.vocab)
    tally = {"safe": 0, "n": 0, "rows_ok": 0, "rows": 0, "acc": [], "err": []}
    d_g, lg_g, acc_g, out_g, draft = check_step_against_oracle(eng, orc, ref, rows, k, draft_o, tally)
    print("1b full step: rel. error (draft vs exact, verify vs exact, verify vs rounding oracle)", tally["err"],
          "; positions provably safe", tally["safe"], "of", tally["n"], "; accept rows fully safe", tally["rows_ok"],
          "of", tally["rows"], "; oracle accept lengths", tally["acc"])
    # Random-init logits have small leads (top-2 gap about sigma / sqrt(2 ln V), exponentially distributed) and 16
    # layers of bf16 operands move a logit by up to ~2 % of the largest: about half of the positions are provably
    # safe.  Whole accept rows that are provably safe are therefore few here (printed); acceptance is exact on
    # identical inputs above, and provably-safe rows are required of the two-layer tests below.
    assert tally["safe"] >= 0.3 * tally["n"]
    assert np.max(tally["acc"]) > 1                   # acceptance beyond the bonus token was exercised

    # the same step as ONE graph replay from the same state gives the same bits
    eager = (d_g.clone(), lg_g.clone(), acc_g.clone(), out_g.clone(), eng.kv_len.clone())
    for n, t in snap.items():
        getattr(eng, n).copy_(t)
    d2 = torch.empty_like(d_g); lg2 = torch.empty_like(lg_g); acc2 = torch.empty_like(acc_g); out2 = torch.empty_like(out_g)
    tid2 = torch.empty(B, k + 1, dtype=torch.int32, device="cuda")
    fixed = draft.clone()

    def step():
        eng.sf_draft_step(k, draft_out=d2)
        eng.sf_verify_step(k, fixed, logits_out=lg2, ids_out=tid2)
        eng.sf_accept_commit(k, fixed, tid2, accept_out=acc2, tokens_out=out2)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        step()
    for n, t in snap.items():
        getattr(eng, n).copy_(t)
    gr.replay()
    torch.cuda.synchronize()
    assert torch.equal(d2, eager[0]) and torch.equal(lg2, eager[1])
    assert torch.equal(acc2, eager[2]) and torch.equal(out2, eager[3]) and torch.equal(eng.kv_len, eager[4])


# ---- the larger workloads at their real widths, reduced depth: whole teacher-forced steps ------------------
@pytest.mark.parametrize("index,k,fixed_prefix", [(2, 4, None), (3, 6, 1024), (4, 4, None)])
def test_real_width_two_layer_steps_teacher_forced(index, k, fixed_prefix):
    """Baseline configurations 3, 4 and 5 at their real d_model / heads / d_ffn / vocabulary with two layers,
    four sequences with prefix lengths from the configuration's range inside a batch of six, four whole
    draft -> verify -> accept steps, every step restarted from the rounding oracle's state."""
    wl = synth.WORKLOADS[index]
    m = wl.model.scaled(n_layers=2)
    B, Bp, steps = 6, 4, 4
    rows = [0, 2, 3, 5]
    g = synth.rng(wl.seed, 778)
    if fixed_prefix is None:
        lens = np.array([wl.prefix_lo, wl.prefix_hi] + list(g.integers(wl.prefix_lo, wl.prefix_hi + 1, Bp - 2)), np.int32)
    else:
        lens = np.full(Bp, fixed_prefix, np.int32)
    cap = synth.kv_capacity(int(lens.max()), steps + 1, k)
    tw_d, dw_d = synth.device_weights(m, k, wl.seed)
    tw, dw = synth.host_weights(tw_d, dw_d)
    orc = sfo.Oracle(m.cfg(), tw, dw, Bp, cap, q_max=k + 1, round_bf16=True)
    ref = sfo.Oracle(m.cfg(), tw, dw, Bp, cap, q_max=k + 1, round_bf16=False)
    seed_oracle_state(orc, lens, m.vocab, g)
    ref.restore(orc.snapshot())
    eng = Engine(m.cfg(), B, cap, k)
    eng.bind(tw_d, dw_d)
    del tw_d, dw_d
    for which in ("tk", "tv", "dk", "dv"):
        buf = getattr(eng, which)
        buf.copy_(device_normal((buf.numel(),), 200 + len(which) + ord(which[0])))
    eng.hooks.copy_(device_normal(tuple(eng.hooks.shape), 10))
    all_lens = g.integers(wl.prefix_lo, wl.prefix_hi + 1, B).astype(np.int32)
    eng.set_state(kv_len=all_lens, pending=g.integers(0, m.vocab, B).astype(np.int32), n_new=np.ones(B, np.int32))
    tally = {"safe": 0, "n": 0, "rows_ok": 0, "rows": 0, "acc": [], "err": []}
    for step in range(steps):
        push_state(eng, orc, rows, k)
        eng.len_upper = int(max(eng.kv_len.max().item(), 0))
        # even steps: the true continuation, partly corrupted; odd steps: the draft block's own tokens
        draft_o = corrupt_chain(greedy_chain(orc, k), m.vocab) if step % 2 == 0 else None
        check_step_against_oracle(eng, orc, ref, rows, k, draft_o, tally)
        ref.restore(orc.snapshot())               # the exact oracle follows the rounding oracle's trajectory
    print(wl.name, "two layers: rel. errors per step (draft vs exact, verify vs exact, verify vs rounding oracle)",
          tally["err"], "; positions provably safe", tally["safe"], "of", tally["n"], "; accept rows fully safe",
          tally["rows_ok"], "of", tally["rows"], "; oracle accept lengths", [list(a) for a in tally["acc"]])
    assert tally["safe"] >= 0.5 * tally["n"] and tally["rows_ok"] >= 1
    assert np.max(tally["acc"]) > 1


# ---- a verify pass over more attention workgroups than the chip holds: sequences ranked by length ---------
def test_batch128_step_bits_do_not_depend_on_the_linear_tiles():
    """The 14B-shaped model at one layer, the benchmark's batch (128 sequences, k = 4: 640 rows, where the
    wide layers run on the tall tiles): drafts, target choices, logits-free hooks and the appended K/V must be
    bit-identical when every linear layer is forced onto the 160-row and the 128-row tiles instead."""
    wl = synth.WORKLOADS[4]
    m = wl.model.scaled(n_layers=1)
    B, k = 128, 4
    g = synth.rng(wl.seed, 991)
    lens = g.integers(40, 97, B).astype(np.int32)
    cap = synth.kv_capacity(int(lens.max()), 2, k)
    eng = Engine(m.cfg(), B, cap, k)
    eng.bind(*synth.device_weights(m, k, wl.seed))
    for which in ("tk", "tv", "dk", "dv"):
        buf = getattr(eng, which)
        buf.copy_(device_normal((buf.numel(),), 300 + ord(which[0]) + ord(which[1])))
    hooks0 = device_normal(tuple(eng.hooks.shape), 11)
    results = []
    try:
        for tile in (0, 9, 4):
            eng.sf_tune_linear(tile, 0)
            eng.hooks.copy_(hooks0)
            eng.set_state(kv_len=lens, pending=g.integers(0, m.vocab, B).astype(np.int32) if not results else pending,
                          n_new=np.ones(B, np.int32))
            if not results:
                pending = eng.pending.cpu().numpy().copy()
            draft = eng.sf_draft_step(k)
            _, ids = eng.sf_verify_step(k, draft, logits=False)
            torch.cuda.synchronize()
            results.append((draft.clone(), ids.clone(), eng.hooks.clone(), eng.tk.clone(), eng.dv.clone()))
    finally:
        eng.sf_tune_linear(0, 0)
    for other in results[1:]:
        for a, b in zip(results[0], other):
            assert torch.equal(a, b)
    assert (results[0][1] >= 0).all() and (results[0][1] < m.vocab).all()


def test_verify_with_length_ranked_attention_three_sequences_against_oracle():
    """272 ragged sequences x 2 kv heads = 544 attention workgroups: above 512 the verify pass starts the
    longest sequences first (a device-side ranking).  The longest, the shortest and a middle sequence,
    sitting at scattered batch indices, must still come out as the oracle computes them one by one."""
    m = synth.ModelShape("ranked", 2, 256, 4, 2, 64, 512, 512, "bf16")
    B, k, cap = 272, 4, 768
    probes = [3, 137, 260]
    Bp = len(probes)
    g = synth.rng(31, 5)
    lens = g.integers(5, 700, B).astype(np.int32)
    lens[probes[0]], lens[probes[1]], lens[probes[2]] = 730, 1, 333
    tw, dw = synth.target_weights(m, 31), synth.draft_weights(m, k, 31)
    orc = sfo.Oracle(m.cfg(), tw, dw, Bp, cap, q_max=k + 1, round_bf16=True)
    ref = sfo.Oracle(m.cfg(), tw, dw, Bp, cap, q_max=k + 1, round_bf16=False)
    for name in ("tk", "tv"):
        a = getattr(orc, name)
        a[...] = synth.to_bf16_values(g.standard_normal(a.shape, dtype=np.float32))
    orc.kv_len[:] = lens[probes]
    orc.n_new[:] = 1
    orc.pending[:] = g.integers(0, m.vocab, Bp)
    ref.restore(orc.snapshot())
    draft_o = g.integers(0, m.vocab, (Bp, k)).astype(np.int32)

    eng = Engine(m.cfg(), B, cap, k)
    eng.bind(tw, dw)
    for which, src in (("tk", orc.tk), ("tv", orc.tv)):
        for l in range(m.n_layers):
            plain = device_normal((B, m.n_kv_heads, cap, m.head_dim), 300 + 7 * l + len(which))
            plain[probes] = torch.from_numpy(src[l].astype(np.float32)).cuda().to(torch.bfloat16)
            eng.sf_kv_import(plain, which, l)
    pend = g.integers(0, m.vocab, B).astype(np.int32)
    pend[probes] = orc.pending
    eng.set_state(kv_len=lens, pending=pend, n_new=np.ones(B, np.int32))
    draft = torch.from_numpy(g.integers(0, m.vocab, (B, k)).astype(np.int32)).cuda()
    draft[probes] = torch.from_numpy(draft_o).cuda()

    lg_o, lg_ref = orc.verify_step(k, draft_o), ref.verify_step(k, draft_o)
    got = to_np(eng.sf_verify_step(k, draft)[0][probes])
    assert rel_err(got, lg_ref) < BF16_TOL
    assert rel_err(got, lg_o) < BF16_TOL
    # the block's K/V rows landed in the probes' own caches, at their own positions
    for l in range(m.n_layers):
        kg = to_np(eng.sf_kv_export("tk", l))[probes]
        vg = to_np(eng.sf_kv_export("tv", l))[probes]
        for i, b in enumerate(probes):
            rows = slice(int(lens[b]), int(lens[b]) + k + 1)
            assert rel_err(kg[i][:, rows], orc.tk[l][i][:, rows]) < BF16_TOL
            assert rel_err(vg[i][:, rows], orc.tv[l][i][:, rows]) < BF16_TOL
            np.testing.assert_array_equal(kg[i][:, :rows.start], orc.tk[l][i][:, :rows.start])


# ---- property at full size: speculative decoding emits exactly the plain-greedy stream -------------------
def test_1b_full_size_lossless_under_graph_replay():
    wl = synth.WORKLOADS[1]
    m, B, k, steps = wl.model, wl.batch, wl.k, 12
    P = 48                                             # a short real prefill keeps the test quick
    lens = np.full(B, P, np.int32)
    prompts = synth.prompts(lens, m.vocab, wl.seed)
    cap = synth.kv_capacity(P, 2 * steps + 4, k)
    eng = Engine(m.cfg(), B, cap, k)
    eng.bind(*synth.device_weights(m, k, wl.seed))
    eng.prefill(prompts)
    torch.cuda.synchronize()
    snap = {n: getattr(eng, n).clone() for n in ("kv_len", "pending", "n_new", "cu_new", "hooks")}
    n_ar = steps * (k + 1) + k + 2
    ar = torch.zeros(B, n_ar, dtype=torch.int64, device="cuda")
    ar[:, 0] = eng.pending
    none = torch.zeros(B, 0, dtype=torch.int32, device="cuda")
    for j in range(1, n_ar):                           # plain greedy continuation (k = 0 steps)
        _, ids = eng.sf_verify_step(0, none, logits=False)
        ar[:, j] = eng.sf_accept_commit(0, none, ids)[1][:, 0]
    for n, t in snap.items():
        getattr(eng, n).copy_(t)
    eng.len_upper = P
    # drafts: the true continuation with every other slot corrupted -> acceptance lengths vary
    gen = torch.Generator(device="cuda"); gen.manual_seed(3)
    inj = (ar + (torch.rand(B, n_ar, generator=gen, device="cuda") > 0.6).long()) % m.vocab
    draft = torch.zeros(B, k, dtype=torch.int32, device="cuda")
    tids = torch.empty(B, k + 1, dtype=torch.int32, device="cuda")
    acc = torch.zeros(B, dtype=torch.int32, device="cuda")
    toks = torch.empty(B, k + 1, dtype=torch.int32, device="cuda")
    slot = torch.arange(k, device="cuda")[None, :]

    def step():
        eng.sf_draft_step(k, draft_out=draft)
        idx = (eng.kv_len.long() - P + 1)[:, None] + slot
        draft.copy_(torch.gather(inj, 1, idx.clamp_(max=n_ar - 1)))
        eng.sf_verify_step(k, draft, ids_out=tids, logits=False)     # the timed path: logits never stored
        eng.sf_accept_commit(k, draft, tids, accept_out=acc, tokens_out=toks)
    eng.pin_len_upper()
    keep = {n: getattr(eng, n).clone() for n in ("kv_len", "pending", "n_new", "cu_new", "hooks")}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr):
        step()
    for n, t in keep.items():
        getattr(eng, n).copy_(t)
    emitted, accepted = 0, []
    for _ in range(steps):
        pos = eng.kv_len.long() - P + 1
        gr.replay()
        torch.cuda.synchronize()
        want = torch.gather(ar, 1, (pos[:, None] + torch.arange(k + 1, device="cuda")[None]).clamp(max=n_ar - 1))
        live = toks >= 0
        assert bool(((toks.long() == want) | ~live).all())
        assert bool((live.sum(1) == acc).all())
        emitted += int(live.sum())
        accepted.append(acc.clone())
    a = torch.stack(accepted)
    assert int(a.max()) > 1 and int(a.min()) >= 1 and emitted == int(a.sum())
