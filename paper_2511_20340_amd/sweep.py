"""Throughput of the target forward against batch size x tokens per sequence, on this GPU.

The paper's first figure and its analysis of batch-wise parallel capability (Eq. 2-3) say: one
forward over bs * (k+1) tokens costs about the same as over bs tokens while bs * (k+1) stays
below the hardware ridge rho = peak FLOP/s / peak bytes/s, so the largest draft worth verifying
is k <= rho / bs.  This sweep measures that on MI355X with the verify pass of the library
(sf_verify_step over seeded caches, no draft block): for every batch size B and block length
q = k+1 it times the pass and prints, per B, the time relative to q = 1 and the largest q whose
pass costs at most `--knee` times the single-token pass.

  python -m paper_2511_20340_amd.sweep --config 1 --batches 1,4,16,64,256 --blocks 1,2,3,5,9

One JSON line per (B, q) on stdout, then a table on stderr.
"""
import argparse
import json
import sys

import numpy as np
import torch

import synth
from .engine import Engine

MFMA_BF16_PEAK, HBM_PEAK = 2.5e15, 8.0e12


def forward_work(m, B, q, prefix):
    """Algorithmic FLOP and HBM bytes of one verify pass (weights once, KV once; the logits are reduced to
    the target's choices inside the LM-head kernel and never stored)."""
    es = 2 if m.dtype == "bf16" else 4
    d, F, V, L = m.d_model, m.d_ffn, m.vocab, m.n_layers
    nq, nkv = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    w_elems = L * ((nq + 2 * nkv) * d + d * nq + 3 * d * F) + V * d
    M = B * q
    flops = 2.0 * M * w_elems + 4.0 * M * m.n_q_heads * m.head_dim * (prefix + q) * L
    kv_bytes = L * B * 2 * nkv * es * (prefix + q)
    return flops, w_elems * es + kv_bytes


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=1, help="index into synth.WORKLOADS: which target model")
    ap.add_argument("--batches", default="1,2,4,8,16,32,64,128,256")
    ap.add_argument("--blocks", default="1,2,3,5,9", help="tokens per sequence per pass, q = k+1")
    ap.add_argument("--prefix", type=int, default=512)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--knee", type=float, default=1.25)
    args = ap.parse_args()
    wl = synth.WORKLOADS[args.config]
    m = wl.model
    Bs = [int(x) for x in args.batches.split(",")]
    qs = sorted(int(x) for x in args.blocks.split(","))
    G = m.n_q_heads // m.n_kv_heads
    qs = [q for q in qs if m.dtype != "bf16" or G * q <= 1024]
    torch.cuda.set_device(0)
    tw, _ = synth.device_weights(m, 1, wl.seed)
    rows, shared = [], None
    for B in Bs:
        cap = synth.kv_capacity(args.prefix, 2, max(qs))
        eng = Engine(m.cfg(), B, cap, max(qs) - 1)
        if shared is None:
            eng.bind(tw, None)
            shared = eng
            del tw
        else:
            eng.bind_shared(shared)
        gs = torch.Generator(device="cuda")
        gs.manual_seed(wl.seed + B)
        for name in ("tk", "tv"):
            buf = getattr(eng, name)
            for off in range(0, buf.numel(), 1 << 28):
                chunk = buf[off:off + (1 << 28)]
                chunk.copy_(torch.randn(chunk.numel(), generator=gs, device="cuda", dtype=torch.float32))
        pend = synth.rng(wl.seed, 5).integers(0, m.vocab, B).astype(np.int32)
        base = None
        for q in qs:
            k = q - 1
            eng.set_state(kv_len=np.full(B, args.prefix, np.int32), pending=pend, n_new=np.ones(B, np.int32))
            eng.pin_len_upper()                     # every pass sees the same prefix: nothing is committed
            eng.len_upper = args.prefix
            draft = torch.randint(0, m.vocab, (B, k), dtype=torch.int32, device="cuda")
            ids = torch.empty(B, q, dtype=torch.int32, device="cuda")
            for _ in range(2):
                eng.sf_verify_step(k, draft, ids_out=ids, logits=False)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                eng.sf_verify_step(k, draft, ids_out=ids, logits=False)
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3 / args.steps
            flops, by = forward_work(m, B, q, args.prefix)
            base = t if q == qs[0] else base
            row = {"model": m.name, "B": B, "q": q, "tokens": B * q, "ms": 1e3 * t, "tokens_per_s": B * q / t,
                   "TFLOP/s": flops / t / 1e12, "frac_mfma": flops / t / MFMA_BF16_PEAK, "GB/s": by / t / 1e9,
                   "frac_hbm": by / t / HBM_PEAK, "time_vs_first_block": t / base}
            rows.append(row)
            print(json.dumps(row), flush=True)
        if eng is not shared:
            del eng
    rho = MFMA_BF16_PEAK / HBM_PEAK
    print(f"\n{m.name}, prefix {args.prefix}: pass time relative to q={qs[0]}  (ridge rho = {rho:.0f} FLOP/B, "
          f"so Eq. 3 predicts a free block up to q ~ rho/B)", file=sys.stderr)
    print("    B | " + " | ".join(f"q={q:<2d}" for q in qs) + f" | largest q within {args.knee}x | rho/B", file=sys.stderr)
    for B in Bs:
        r = [x for x in rows if x["B"] == B]
        knee = max([x["q"] for x in r if x["time_vs_first_block"] <= args.knee], default=qs[0])
        print(f"{B:5d} | " + " | ".join(f"{x['time_vs_first_block']:4.2f}" for x in r) + f" | {knee:>3d} | {rho / B:6.1f}",
              file=sys.stderr)


if __name__ == "__main__":
    main()
