"""Shared helpers of the GPU parity tests: build an oracle and an engine from the same seeded
synthetic inputs.  The HIP library and the oracle never see each other; only this test code does."""
import numpy as np
import torch

import synth
from oracle import sfo
from paper_2511_20340_amd import binding as sfb
from paper_2511_20340_amd.engine import Engine


def have_gpu():
    return torch.cuda.is_available()


def rel_err(got, ref):
    """max |got - ref| / max |ref| over the tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16 if dtype == "bf16" else torch.float32).contiguous()


def make_pair(shape: synth.ModelShape, B, cap, k, seed, std=0.02, round_bf16=False, with_draft=True):
    tw = synth.target_weights(shape, seed, std)
    dw = synth.draft_weights(shape, k, seed, std) if with_draft else None
    orc = sfo.Oracle(shape.cfg(), tw, dw, B, cap, q_max=cap, round_bf16=round_bf16)
    eng = Engine(shape.cfg(), B, cap, k)
    eng.bind(tw, dw)
    return orc, eng, tw, dw


def engine_only(shape, B, cap, k):
    return Engine(shape.cfg(), B, cap, k)
