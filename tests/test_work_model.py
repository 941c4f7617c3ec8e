"""Host arithmetic of the measurement code (no GPU): the algorithmic work the roofline fractions are
computed from, checked against figures worked out by hand from the model shapes."""
import importlib.util
import os

import synth
from paper_2511_20340_amd import sweep

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_verify_pass_work_of_the_8b_shape():
    m = synth.WORKLOADS[2].model                    # L=32, d=4096, Hq=32, Hkv=8, hd=128, F=14336, V=128256
    per_layer = (4096 + 2 * 1024) * 4096 + 4096 * 4096 + 3 * 4096 * 14336
    weights = 32 * per_layer + 128256 * 4096        # 7.50 G parameters (no embedding: it is gathered)
    assert abs(weights - 7.50e9) < 0.01e9
    B, q, P = 64, 5, 1152
    flops, by = sweep.forward_work(m, B, q, P)
    attn = 4.0 * B * q * 32 * 128 * (P + q) * 32
    assert flops == 2.0 * B * q * weights + attn
    assert abs(2.0 * B * q * weights - 4.80e12) < 0.01e12          # 4.80 TFLOP of linear layers per pass
    kv = 32 * B * 2 * 1024 * 2 * (P + q)
    assert by == weights * 2 + kv                                  # logits are reduced in the LM-head kernel
    assert abs(weights * 2 - 15.01e9) < 0.01e9                     # 15.01 GB of weights read once


def test_linear_launch_list_of_one_step():
    bench = load_bench()
    m = synth.WORKLOADS[1].model                    # 1B shape: L=16, d=2048, F=8192, V=32000
    B, k = 32, 4
    shapes = bench.gemm_shapes(m, B, k, k + 1)
    # 4 per target layer + LM head; draft: W_D, K/V of the context rows, W_P, 4 of its layer, LM head
    assert len(shapes) == 4 * 16 + 1 + 3 + 4 + 1 == 73
    key = lambda s: (s["M"], s["N"], s["K"], s["out_bytes"], s["res_bytes"])
    assert key(shapes[0]) == (160, 3072, 2048, 160 * 3072 * 2, 0)
    # O projection: adds into the float residual stream (4 B read, 4 B written) and leaves its bf16 copy (2 B)
    assert key(shapes[1]) == (160, 2048, 2048, 160 * 2048 * 6, 160 * 2048 * 4)
    # gate/up: 2F output features are computed, F gated activations in bf16 are stored
    assert key(shapes[2]) == (160, 16384, 2048, 160 * 8192 * 2, 0)
    assert key(shapes[3]) == (160, 2048, 8192, 160 * 2048 * 6, 160 * 2048 * 4)
    # LM heads: one token id per row leaves the kernel
    assert (160, 32000, 2048, 160 * 4, 0) in map(key, shapes) and (128, 32000, 2048, 128 * 4, 0) in map(key, shapes)
    assert len(bench.gemm_shapes(m, B, k, k + 1, two_stage=True)) == 75
    by, fl = bench.gemm_work(shapes, 2)
    assert fl == sum(2.0 * s["M"] * s["N"] * s["K"] for s in shapes)
    # weights dominate the bytes: 2 bytes per parameter of every launch, read once
    w_bytes = sum(s["N"] * s["K"] * 2 for s in shapes)
    assert w_bytes < by < 1.12 * w_bytes
    assert abs(by - 2.656e9) < 0.005e9                             # 2.66 GB per step at the 1B workload (2.40 GB of it weights)
    assert len(bench.gemm_shapes(m, B, 0, 1)) == 4 * 16 + 1       # plain decoding: no draft launches


def test_calibration_solves_for_the_wanted_acceptance():
    bench = load_bench()
    for k in (2, 4, 8):
        for kappa in (1.2, 1.75, 2.4):
            a = bench.solve_alpha(kappa, k)
            assert 0.0 < a < 1.0
            assert abs(sum(a ** i for i in range(k + 1)) - kappa) < 1e-6   # E[accepted] of a geometric chain
