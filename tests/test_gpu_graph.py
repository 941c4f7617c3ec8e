"""A whole step (draft -> verify -> accept) captured in a HIP graph replays to the same bits as
eager launches, replay after replay, with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

import synth

from gpu_common import make_pair
from test_gpu_e2e import SLICES

pytestmark = pytest.mark.gpu


def test_graph_replay_equals_eager():
    m = SLICES["8b-slice"]
    B, k, seed, cap = 5, 4, 31, 256
    lens = [70, 33, 120, 64, 9]
    prompts = synth.prompts(lens, m.vocab, seed)
    _, eager, _, _ = make_pair(m, B, cap, k, seed, std=0.05)
    _, graph, _, _ = make_pair(m, B, cap, k, seed, std=0.05)
    eager.prefill(prompts)
    graph.prefill(prompts)

    def buffers():
        return (torch.zeros(B, k, dtype=torch.int32, device="cuda"),
                torch.zeros(B, k + 1, m.vocab, dtype=torch.float32, device="cuda"),
                torch.zeros(B, dtype=torch.int32, device="cuda"),
                torch.zeros(B, k + 1, dtype=torch.int32, device="cuda"),
                torch.zeros(B, k + 1, dtype=torch.int32, device="cuda"))

    def step(eng, bufs):
        d, lg, acc, out, ids = bufs
        eng.sf_draft_step(k, draft_out=d)
        eng.sf_verify_step(k, d, logits_out=lg, ids_out=ids)
        eng.sf_accept_commit(k, d, ids, accept_out=acc, tokens_out=out)

    gb, eb = buffers(), buffers()
    graph.pin_len_upper()                      # grids depend only on this host-side bound
    keep = {n: getattr(graph, n).clone() for n in ("kv_len", "pending", "n_new", "cu_new", "hooks")}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(graph, gb)                        # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(graph, gb)
    for n, t in keep.items():
        getattr(graph, n).copy_(t)
    torch.cuda.synchronize()
    for it in range(8):
        step(eager, eb)                        # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b, name in zip(gb, eb, ("draft", "logits", "accept_len", "out_tokens", "target_ids")):
            assert torch.equal(a, b), (it, name)
        for name in ("kv_len", "pending", "n_new", "cu_new", "hooks"):
            assert torch.equal(getattr(graph, name), getattr(eager, name)), (it, name)
    assert int(eager.kv_len.min().item()) >= min(lens) + 8
