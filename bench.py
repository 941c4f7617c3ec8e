#!/usr/bin/env python3
"""Benchmark of the SpecFormer draft -> verify -> accept step on one MI355X.

A "step" is one pass of the whole hot path (sf_draft_step, sf_verify_step, sf_accept_commit) over
the batch.  Inputs (weights, prompts, caches after a real chunked prefill) are resident in HBM
before the timed region.  Prints ONE JSON line: accepted tokens/s, the roofline of the dominant
kernel class (per-kernel HIP-event timings collected in a second, identical pass), and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK = 8.0e12
MFMA_BF16_PEAK = 2.5e15
FP32_PEAK = 157.3e12
# kappa (mean tokens per target call) of the paper's model-size table at k=4 / k=2, by model class
DEFAULT_CONFIG = 4
PAPER_KAPPA = {"1b-bf16": 1.84, "8b-bf16": 1.75, "14b-bf16": 1.71, "tiny-f32": 1.84}


def solve_alpha(kappa, k):
    """Per-slot acceptance probability alpha with 1 + a + a^2 + ... + a^k == kappa."""
    lo, hi = 0.0, 1.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if sum(mid ** i for i in range(k + 1)) < kappa:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def gemm_shapes(m, B, k, qm, two_stage=False):
    """One dict per linear launch of a step: rows M, output features N, reduction K, and the bytes the launch
    must write (`out_bytes`) and read besides weights and input rows (`res_bytes`).  bf16 mode: the residual
    stream is float (read 4 + written 4 bytes per element) with a bf16 copy for the next matrix product (2
    more); gate/up leave M x F gated activations, never the 2F pre-activations; the LM heads leave one token
    id per row (their logits are reduced inside the kernel)."""
    es = 2 if m.dtype == "bf16" else 4
    stream_out = 4 + (2 if m.dtype == "bf16" else 0)
    d, F, V = m.d_model, m.d_ffn, m.vocab
    nq, nkv = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    M, Mh, Ms = B * (k + 1), B * qm, B * k

    def lin(rows, N, K, out_bytes, res_bytes=0):
        return {"M": rows, "N": N, "K": K, "out_bytes": out_bytes, "res_bytes": res_bytes}

    def layer(rows, last_copy=True):
        return [lin(rows, nq + 2 * nkv, d, rows * (nq + 2 * nkv) * es),
                lin(rows, d, nq, rows * d * stream_out, rows * d * 4),
                lin(rows, 2 * F, d, rows * F * es),
                lin(rows, d, F, rows * d * (stream_out if last_copy else 4), rows * d * 4)]

    def head(rows):
        return lin(rows, V, d, rows * 4 if m.dtype == "bf16" else rows * V * 4)
    out = layer(M) * m.n_layers + [head(M)]
    if k > 0:
        out += [lin(Mh, d, 4 * d, Mh * d * es), lin(Mh, 2 * nkv, d, Mh * 2 * nkv * es),
                lin(B, k * d, d, Ms * d * stream_out)] + layer(Ms, last_copy=False) + [head(Ms)]
        if two_stage:   # query and output projection of the context attention's newest row
            out += [lin(B, nq, d, B * nq * es), lin(B, d, nq, B * d * 4, B * d * es)]
    return out


def gemm_work(shapes, es):
    by = sum(s["K"] * s["N"] * es + s["M"] * s["K"] * es + s["out_bytes"] + s["res_bytes"] for s in shapes)
    fl = sum(2.0 * s["M"] * s["N"] * s["K"] for s in shapes)
    return by, fl


def cpu_baseline(wl, seed, budget_s=25.0):
    """The oracle, as it stands, on a bounded sample: B' = 2 sequences of the same model at the workload's
    mean prefix length, seeded caches, natural drafts; whole steps (draft + verify + accept).  Models whose
    weights would take minutes to draw and tens of GB to hold on the host are sampled in depth too: whole
    steps at L' = 1 and L' = 4 target layers (same widths, same heads), extrapolated linearly to L layers --
    every layer costs the same, the draft block and the two LM heads are in both measurements."""
    import synth
    from oracle import sfo
    m, k = wl.model, wl.k
    Bp = min(2, wl.batch)
    prefix = int((wl.prefix_lo + wl.prefix_hi) // 2)
    cap = synth.kv_capacity(prefix, 4, k)
    per_layer = m.d_model * ((m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim + m.n_q_heads * m.head_dim + 3 * m.d_ffn)
    full_depth = m.n_layers * per_layer < 1.5e9
    depths = [m.n_layers] if full_depth else [1, 4]
    t0 = time.time()
    tw_d, dw_d = synth.device_weights(m.scaled(n_layers=depths[-1]), k, seed)
    tw, dw = synth.host_weights(tw_d, dw_d)
    del tw_d, dw_d
    setup = time.time() - t0

    def run(depth, budget):
        mm = m.scaled(n_layers=depth)
        twd = {n: (v[:depth] if isinstance(v, list) else v) for n, v in tw.items()}
        orc = sfo.Oracle(mm.cfg(), twd, dw, Bp, cap, q_max=k + 1)
        g = synth.rng(seed, 777)
        for name in ("tk", "tv", "dk", "dv"):
            getattr(orc, name)[...] = g.standard_normal(getattr(orc, name).shape, dtype=np.float32)
        orc.hooks[...] = g.standard_normal(orc.hooks.shape, dtype=np.float32)
        orc.kv_len[:] = prefix
        orc.n_new[:] = 1
        orc.pending[:] = g.integers(0, m.vocab, Bp)
        steps, tokens, t_used = 0, 0, 0.0
        while steps < 1 or (t_used < budget and steps < 12 and t_used / steps * (steps + 1) < budget):
            t1 = time.time()
            d = orc.draft_step(k)
            lg = orc.verify_step(k, d)
            acc, _ = orc.accept_commit(k, d, lg)
            t_used += time.time() - t1
            tokens += int(acc.sum())
            steps += 1
        return t_used / steps, tokens / steps, steps, t_used
    runs = [run(depth, budget_s / len(depths)) for depth in depths]
    if full_depth:
        t_step, tok_step = runs[0][0], runs[0][1]
        how = f"{runs[0][2]} whole step(s) at all {m.n_layers} layers"
    else:
        slope = (runs[1][0] - runs[0][0]) / (depths[1] - depths[0])
        t_step = runs[0][0] + slope * (m.n_layers - depths[0])
        tok_step = runs[1][1]
        how = (f"whole steps at L'={depths[0]} ({runs[0][2]} steps, {1e3 * runs[0][0]:.0f} ms each) and L'={depths[1]} "
               f"({runs[1][2]} steps, {1e3 * runs[1][0]:.0f} ms each) of {m.n_layers} target layers at the real widths, "
               f"extrapolated linearly in depth")
    return {"value": tok_step / t_step, "unit": "accepted tokens/s", "cores": sfo.ncores(), "kind": "oracle",
            "sample": f"draft+verify+accept at B'={Bp} of {wl.batch} sequences, prefix {prefix}, k={k}, seeded caches, "
                      f"natural drafts; {how}; fp64 naive C + OpenMP; {sum(r[3] for r in runs):.1f}s timed, "
                      f"{setup:.1f}s weight setup; per-sequence cost is batch-independent",
            "ms_per_step_sample": 1e3 * t_step}


def stream_copy_rate(torch, sfb):
    """What a plain copy kernel reaches on this GPU (read + write bytes per second), as context for the
    roofline fractions, which are quoted against the published 8 TB/s."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    L = sfb.lib()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(7):
        if i == 2:
            e0.record()
        sfb.check(L.sf_calib_copy(dst.data_ptr(), src.data_ptr(), n, None), "sf_calib_copy")
    e1.record()
    torch.cuda.synchronize()
    s = e0.elapsed_time(e1) * 1e-3 / 5
    return {"GB/s": round(2 * n / s / 1e9, 1), "what": "1 GiB device-to-device copy kernel, bytes read + written"}


def profile_traffic(workload, kernel_class):
    """HBM bytes per launch of the dominant kernel class as the hardware counters saw them: read from the
    committed rocprofv3 summary of this workload (FETCH_SIZE / WRITE_SIZE runs scaled by a copy kernel of
    known size), since counters cannot be collected from inside this process.  None if there is none."""
    import re
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                        f"step_kernels__{workload.replace('..', 'to')}.md")
    if not os.path.exists(path):
        return None
    text = open(path).read()
    got = [re.search(rf"^traffic_per_launch {re.escape(kernel_class)} {c}: ([0-9.e+]+) bytes", text, re.M)
           for c in ("FETCH_SIZE", "WRITE_SIZE")]
    return sum(float(g.group(1)) for g in got) if all(got) else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=DEFAULT_CONFIG,
                    help="index into the baseline's configs (default: the 14B-shaped batch-128 workload)")
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--draft-wiring", choices=["hybrid", "two-stage"], default="hybrid",
                    help="hybrid: one draft attention over cached context + slots (default); two-stage: context "
                         "attention and slot attention kept apart, as the SpecFormer section writes them")
    ap.add_argument("--draft-mask", choices=["bidir", "causal"], default="bidir",
                    help="mask inside the slot block (causal = the paper's '+Att Mask' ablation)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--attn-chunk", type=int, default=0,
                    help="tuning aid: force the attention's split-KV chunk (32-key tiles, >= 16; 0 = automatic)")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--calib-copy", type=int, default=0,
                    help="first run this many plain 1 GiB device copies (reference dispatches for scaling "
                         "rocprofv3 byte counters)")
    ap.add_argument("--seeded-state", action="store_true",
                    help="skip prefill and the plain-greedy reference run: seed caches, hooks and pending tokens "
                         "directly (values do not change the work); only the natural-draft pass runs. For profilers.")
    ap.add_argument("--prefill-block", type=int, default=64,
                    help="prompt tokens per sequence and sf_verify_step call during the chunked prefill")
    ap.add_argument("--no-graph", dest="graph", action="store_false",
                    help="launch every kernel eagerly instead of replaying one HIP graph per step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    from paper_2511_20340_amd.engine import Engine
    from paper_2511_20340_amd import binding as sfb

    wl = synth.WORKLOADS[args.config]
    m, B = wl.model, wl.batch
    k = args.k if args.k is not None else wl.k
    steps = args.steps if args.steps is not None else min(wl.steps, 64)
    warm = args.warmup
    es = 2 if m.dtype == "bf16" else 4
    torch.cuda.set_device(0)

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        from paper_2511_20340_amd import binding as _b
        for _ in range(args.calib_copy):
            _b.check(_b.lib().sf_calib_copy(dst.data_ptr(), src.data_ptr(), src.numel(), None), "sf_calib_copy")
        torch.cuda.synchronize()
        del src, dst

    lens = synth.prefix_lengths(B, wl.prefix_lo, wl.prefix_hi, wl.seed)
    prompts = synth.prompts(lens, m.vocab, wl.seed)
    n_pass = 2 if args.no_profile else 3
    total_steps = n_pass * (steps + warm) + 6
    cap = synth.kv_capacity(int(lens.max()), total_steps, k)
    eng = Engine(m.cfg(), B, cap, k)
    if args.attn_chunk:
        eng.sf_tune_attention(args.attn_chunk)
    two_stage = args.draft_wiring == "two-stage"
    draft_mode = (sfb.SF_MASK_BIDIR if args.draft_mask == "bidir" else sfb.SF_MASK_CAUSAL) | \
        (sfb.SF_DRAFT_TWO_STAGE if two_stage else 0)
    tw, dw = synth.device_weights(m, k, wl.seed, two_stage)
    eng.bind(tw, dw)
    del tw, dw

    t0 = time.time()
    if args.seeded_state:
        gs = torch.Generator(device="cuda"); gs.manual_seed(wl.seed + 1)
        for name in ("tk", "tv", "dk", "dv"):
            buf = getattr(eng, name)
            for off in range(0, buf.numel(), 1 << 28):
                chunk = buf[off:off + (1 << 28)]
                chunk.copy_(torch.randn(chunk.numel(), generator=gs, device="cuda", dtype=torch.float32))
        eng.hooks.copy_(torch.randn(eng.hooks.shape, generator=gs, device="cuda", dtype=torch.float32))
        eng.set_state(kv_len=lens, pending=synth.rng(wl.seed, 5).integers(0, m.vocab, B).astype(np.int32),
                      n_new=np.ones(B, np.int32))
    else:
        eng.prefill(prompts, block=max(args.prefill_block, k + 1))
    torch.cuda.synchronize()
    t_prefill = time.time() - t0
    snap = {n: getattr(eng, n).clone() for n in ("kv_len", "pending", "n_new", "cu_new", "hooks")}
    len0 = int(lens.max())

    # plain greedy continuation of the target (k = 0 steps), for the calibrated drafts
    n_ar = total_steps * (k + 1) + k + 2
    ar = torch.zeros(B, n_ar, dtype=torch.int32, device="cuda")
    ar[:, 0] = eng.pending
    none = torch.zeros(B, 0, dtype=torch.int32, device="cuda")
    id1 = torch.empty(B, 1, dtype=torch.int32, device="cuda")
    for j in range(1, n_ar):
        if eng.len_upper + 1 > cap or args.seeded_state:
            break
        eng.sf_verify_step(0, none, ids_out=id1, logits=False)
        _, out = eng.sf_accept_commit(0, none, id1)
        ar[:, j] = out[:, 0]
    torch.cuda.synchronize()
    for n, t in snap.items():
        getattr(eng, n).copy_(t)
    eng.len_upper = len0

    kappa_t = PAPER_KAPPA.get(m.name, 1.75)
    alpha = solve_alpha(min(kappa_t, k + 1.0), k) if k > 0 else 0.0
    gen = torch.Generator(device="cuda"); gen.manual_seed(wl.seed)
    corrupt = (torch.rand(B, n_ar, generator=gen, device="cuda") > alpha).to(torch.int32)
    inj = (ar + corrupt) % m.vocab
    len_t = torch.from_numpy(lens).cuda().to(torch.int64)
    slot = torch.arange(max(k, 1), device="cuda", dtype=torch.int64)[None, :k]

    draft = torch.zeros(B, k, dtype=torch.int32, device="cuda")
    tids = torch.empty(B, k + 1, dtype=torch.int32, device="cuda")     # the target's choices; logits are never stored
    toks = torch.empty(B, k + 1, dtype=torch.int32, device="cuda")

    n_rec = steps + warm + 2
    tok_hist = torch.full((n_rec, B, k + 1), -1, dtype=torch.int32, device="cuda")
    tok_pos = torch.zeros(n_rec, B, dtype=torch.int64, device="cuda")
    hist_i = [0]
    acc_buf = torch.zeros(B, dtype=torch.int32, device="cuda")
    acc_sum = torch.zeros(B, dtype=torch.int64, device="cuda")

    def one_step(calibrated):
        """draft -> (optional draft replacement) -> verify -> accept; everything on the current stream"""
        eng.sf_draft_step(k, mask=draft_mode, draft_out=draft)
        if calibrated and k > 0:
            idx = (eng.kv_len.to(torch.int64) - len_t + 1)[:, None] + slot
            draft.copy_(torch.gather(inj, 1, idx.clamp_(max=n_ar - 1)))
        eng.sf_verify_step(k, draft, ids_out=tids, logits=False)
        eng.sf_accept_commit(k, draft, tids, accept_out=acc_buf, tokens_out=toks)
        acc_sum.add_(acc_buf)

    def run_eager(n, calibrated, len_hist=None, phase_ev=None, record=False):
        for i in range(n):
            if phase_ev is not None:
                phase_ev[i][0].record()
            eng.sf_draft_step(k, mask=draft_mode, draft_out=draft)
            if calibrated and k > 0:
                idx = (eng.kv_len.to(torch.int64) - len_t + 1)[:, None] + slot
                draft.copy_(torch.gather(inj, 1, idx.clamp_(max=n_ar - 1)))
            if phase_ev is not None:
                phase_ev[i][1].record()
            if len_hist is not None:
                len_hist[i].copy_(eng.kv_len)
            eng.sf_verify_step(k, draft, ids_out=tids, logits=False)
            if phase_ev is not None:
                phase_ev[i][2].record()
            if record:   # where in the plain-greedy stream this step's first output token belongs
                tok_pos[hist_i[0]].copy_(eng.kv_len.to(torch.int64) - len_t + 1)
            eng.sf_accept_commit(k, draft, tids, accept_out=acc_buf,
                                 tokens_out=tok_hist[hist_i[0]] if record else toks)
            acc_sum.add_(acc_buf)
            if record:
                hist_i[0] += 1
            if phase_ev is not None:
                phase_ev[i][3].record()

    # One HIP graph per draft mode replays the whole step: the library's launch grids depend only on
    # the host-side length bound, which is pinned to its maximum for the capture.
    graphs = {}
    if args.graph:
        for cal in ((False,) if args.seeded_state else (False, True)):
            keep = {n: getattr(eng, n).clone() for n in ("kv_len", "pending", "n_new", "cu_new", "hooks")}
            eng.pin_len_upper()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                one_step(cal)                      # warm up (lazy kernel attributes) outside the capture
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                one_step(cal)
            torch.cuda.synchronize()
            graphs[cal] = g
            for n, t in keep.items():              # the capture's warm-up advanced the state: rewind
                getattr(eng, n).copy_(t)

    def run(n, calibrated):
        if args.graph:
            for _ in range(n):
                graphs[calibrated].replay()
        else:
            run_eager(n, calibrated)

    step_marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]

    def timed_pass(calibrated):
        run(warm, calibrated)
        torch.cuda.synchronize()
        acc_sum.zero_()
        torch.cuda.synchronize()
        t = time.perf_counter()
        if args.graph:                      # one event between replays: the per-step spread
            for i in range(steps):
                step_marks[i].record()
                graphs[calibrated].replay()
            step_marks[steps].record()
        else:
            run(steps, calibrated)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        spread = None
        if args.graph:
            us = np.array([step_marks[i].elapsed_time(step_marks[i + 1]) for i in range(steps)]) * 1e3
            spread = {q: round(float(np.percentile(us, p)), 1) for q, p in (("p10", 10), ("p50", 50), ("p90", 90))}
        return dt, int(acc_sum.sum().item()), spread

    # Plain autoregressive decoding of the same target (the "W/o SD" row of the paper's tables): an
    # engine of its own with k = 0, so its linear layers are planned for B rows rather than B*(k+1);
    # same packed weights, a copy of the prefilled target cache, timed over as many target calls.
    ar_ms = None
    if not args.seeded_state and k > 0:
        # it works on the same target caches: its rows land behind the prefixes, where the speculative passes
        # that follow overwrite them (dead slots until committed)
        eng0 = Engine(m.cfg(), B, cap, 0, share_caches=eng)
        eng0.bind_shared(eng)
        eng0.set_state(kv_len=lens, pending=snap["pending"].cpu().numpy(), n_new=np.ones(B, np.int32))
        eng0.len_upper = len0
        acc1 = torch.empty(B, dtype=torch.int32, device="cuda")
        out1 = torch.empty(B, 1, dtype=torch.int32, device="cuda")

        def ar_step():
            eng0.sf_verify_step(0, none, ids_out=id1, logits=False)
            eng0.sf_accept_commit(0, none, id1, accept_out=acc1, tokens_out=out1)
        if args.graph:
            eng0.pin_len_upper()
            eng0.len_upper = eng.cap - (k + 1)    # the same attention grid bound as the k-step graph
            ar_step()
            torch.cuda.synchronize()
            g0 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g0):
                ar_step()
            step0 = g0.replay
        else:
            step0 = ar_step
        for _ in range(warm):
            step0()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            step0()
        torch.cuda.synchronize()
        ar_ms = 1e3 * (time.perf_counter() - t) / steps
        if args.graph:
            del g0
        del eng0

    dt_nat, tok_nat, spread_nat = timed_pass(False)
    dt_cal, tok_cal, _ = (dt_nat, tok_nat, None) if args.seeded_state else timed_pass(True)

    result = {
        "metric": "accepted tokens/s at batch B (draft+verify+accept step)",
        "value": tok_nat / dt_nat, "unit": "accepted tokens/s", "n_gpus": 1, "steps": steps, "warmup": warm,
        "ms_per_step": 1e3 * dt_nat / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": m.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "baseline_config_index": args.config, "batch": B, "k": k,
                   "prefix": [int(wl.prefix_lo), int(wl.prefix_hi)], "layers": m.n_layers, "d_model": m.d_model,
                   "q_heads": m.n_q_heads, "kv_heads": m.n_kv_heads, "head_dim": m.head_dim, "d_ffn": m.d_ffn,
                   "vocab": m.vocab, "draft_wiring": args.draft_wiring, "draft_mask": args.draft_mask, "drafts": "natural (the random-init draft block's own tokens)",
                   "state": "seeded caches (no prefill)" if args.seeded_state else
                            f"real chunked prefill through sf_verify_step, blocks of {max(args.prefill_block, k + 1)} "
                            "prompt tokens", "prefill_s": round(t_prefill, 3),
                   "launch": "one HIP graph replay per step" if args.graph else "eager launches"},
        "kappa": tok_nat / (steps * B),
        "step_us": 1e6 * dt_nat / steps,
        "step_us_spread": spread_nat,      # per-replay, HIP events between graph replays (None when eager)
        "calibrated": {"what": "draft tokens replaced after sf_draft_step by the target's greedy continuation, "
                               "each slot corrupted with probability 1-alpha, so kappa matches the paper's model class",
                       "kappa_target": kappa_t, "alpha": alpha, "kappa": tok_cal / (steps * B),
                       "value": tok_cal / dt_cal, "unit": "accepted tokens/s", "ms_per_step": 1e3 * dt_cal / steps},
    }

    if ar_ms is not None:
        # the paper's table format: TPS, speed-up over no-SD, kappa, theta = kappa / speed-up
        ar_tps = B / (ar_ms * 1e-3)
        result["vs_plain_decoding"] = {
            "plain_tokens_per_s": ar_tps, "plain_ms_per_step": ar_ms,
            "natural": {"speedup": result["value"] / ar_tps, "kappa": result["kappa"],
                        "theta": result["kappa"] / (result["value"] / ar_tps)},
            "calibrated": {"speedup": result["calibrated"]["value"] / ar_tps, "kappa": result["calibrated"]["kappa"],
                           "theta": result["calibrated"]["kappa"] / (result["calibrated"]["value"] / ar_tps)}}

    if not args.no_profile:
        # identical pass with every kernel launch bracketed by HIP events on the launch stream
        eng.pin_len_upper(False)
        eng.len_upper = min(cap - (k + 1), int(eng.kv_len.max().item()))
        cal3 = not args.seeded_state
        run_eager(warm, cal3, record=True)
        len_hist = torch.zeros(steps, B, dtype=torch.int32, device="cuda")
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        torch.cuda.synchronize()
        eng.sf_profile_begin()
        run_eager(steps, cal3, len_hist=len_hist, phase_ev=ev, record=True)
        prof = eng.sf_profile_end()
        torch.cuda.synchronize()
        # lossless property at full size: every token the speculative path emitted equals the target's
        # own plain-greedy continuation at that place of the stream
        nrec = hist_i[0]
        pos = tok_pos[:nrec, :, None] + torch.arange(k + 1, device="cuda")[None, None, :]
        want = torch.gather(ar.to(torch.int64)[None].expand(nrec, B, n_ar), 2, pos.clamp(max=n_ar - 1))
        got = tok_hist[:nrec].to(torch.int64)
        emitted = got >= 0
        lossless = {"tokens_compared": int(emitted.sum().item()),
                    "mismatches": int(((got != want) & emitted).sum().item())}

        result["lossless_check"] = "n/a (seeded state has no reference run)" if args.seeded_state else lossless

        phases = {"draft_us": np.mean([e[0].elapsed_time(e[1]) for e in ev]) * 1e3,
                  "verify_us": np.mean([e[1].elapsed_time(e[2]) for e in ev]) * 1e3,
                  "accept_us": np.mean([e[2].elapsed_time(e[3]) for e in ev]) * 1e3}
        result["phase_us_profiled_pass"] = {a: round(float(b), 1) for a, b in phases.items()}
        eager_us = np.array([e[0].elapsed_time(e[3]) for e in ev]) * 1e3
        result["step_us_eager_profiled"] = {q: round(float(np.percentile(eager_us, p)), 1)
                                            for q, p in (("p10", 10), ("p50", 50), ("p90", 90))}
        qm = k + 1
        shapes = gemm_shapes(m, B, k, qm, two_stage)
        g_bytes, g_flops = gemm_work(shapes, es)
        lsum = len_hist.to(torch.float64).sum(1).cpu().numpy()        # sum_b kv_len per step
        kvb = 2 * m.head_dim * es * m.n_kv_heads
        att_v = m.n_layers * (kvb * (lsum + B * (k + 1)) + 2 * B * (k + 1) * m.n_q_heads * m.head_dim * es)
        att_d = (kvb * (lsum + B * k) + 2 * B * k * m.n_q_heads * m.head_dim * es) if k > 0 else 0 * lsum
        if two_stage and k > 0:   # one context row over the cache, then the k slots among themselves
            att_d = (kvb * lsum + 2 * B * m.n_q_heads * m.head_dim * es) + \
                    (kvb * B * k + 2 * B * k * m.n_q_heads * m.head_dim * es)
        att_bytes = float(np.mean(att_v + att_d))
        att_flops = float(np.mean(4.0 * m.n_q_heads * m.head_dim *
                                  (m.n_layers * (k + 1) * (lsum + B * (k + 1)) + k * (lsum + B * k))))
        # fp32 mode scans stored logits; bf16 mode has no such pass (the class is then absent)
        arg_bytes = 4.0 * m.vocab * B * ((k + 1) + k)
        kernels = {}
        for name, (ms, cnt) in prof.items():
            if cnt == 0:
                continue
            ent = {"ms_per_step": ms / steps, "launches_per_step": cnt / steps, "avg_us": 1e3 * ms / cnt}
            t = ms / steps * 1e-3
            if name == "linear":
                hb, mf = g_bytes / t, g_flops / t
                ent.update({"GB/s": hb / 1e9, "TFLOP/s": mf / 1e12, "frac_hbm": hb / HBM_PEAK,
                            "frac_mfma": mf / (MFMA_BF16_PEAK if es == 2 else FP32_PEAK),
                            "bytes_per_step": g_bytes, "flops_per_step": g_flops})
            elif name == "attention":
                ent.update({"GB/s": att_bytes / t / 1e9, "frac_hbm": att_bytes / t / HBM_PEAK,
                            "TFLOP/s": att_flops / t / 1e12, "bytes_per_step": att_bytes})
            elif name == "argmax":
                ent.update({"GB/s": arg_bytes / t / 1e9, "frac_hbm": arg_bytes / t / HBM_PEAK,
                            "bytes_per_step": arg_bytes})
            kernels[name] = ent
        result["kernels"] = kernels
        dom = max(kernels, key=lambda n: kernels[n]["ms_per_step"])
        e = kernels[dom]
        peak_f = MFMA_BF16_PEAK if es == 2 else FP32_PEAK
        if dom == "linear" and e["frac_mfma"] > e["frac_hbm"]:
            roof = {"bound": "mfma" if es == 2 else "alu", "achieved": e["TFLOP/s"], "peak": peak_f / 1e12,
                    "unit": "TFLOP/s", "frac": e["frac_mfma"]}
        else:
            roof = {"bound": "hbm", "achieved": e.get("GB/s", 0.0), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                    "frac": e.get("frac_hbm", 0.0)}
        roof.update({"kernel": dom, "avg_launch_us": e["avg_us"], "launches_per_step": e["launches_per_step"],
                     "algorithmic_per_launch": (e.get("bytes_per_step", 0.0) if roof["unit"] == "GB/s" else
                                                e.get("flops_per_step", 0.0)) / e["launches_per_step"],
                     "traffic": profile_traffic(wl.name, dom),
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this workload, scaled by a copy "
                                       "kernel of known size; read from the summary under profiles/ (hardware counters "
                                       "cannot be collected from inside this process)",
                     "how": "HIP events around every launch of the class on the launch stream, same steps as the timed pass"})
        result["roofline"] = roof

    result["hbm_stream_copy_measured"] = stream_copy_rate(torch, sfb)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, wl.seed)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
