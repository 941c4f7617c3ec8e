"""The acceptance rule (arg-max over stored logits + sf_op_accept, the launch behind sf_accept_commit) against
the oracle: bit-exact on identical logits, no guard band."""
import numpy as np
import pytest
import torch

import synth
from oracle import sfo

from gpu_common import engine_only

pytestmark = pytest.mark.gpu


def planted_logits(B, k, V, seed, match_p):
    """Random logits + a draft that matches the row arg-max with probability match_p per slot."""
    g = synth.rng(seed, 1)
    lg = g.standard_normal((B, k + 1, V), dtype=np.float32)
    top = lg.argmax(-1).astype(np.int32)
    draft = top[:, :k].copy()
    wrong = g.random((B, k)) > match_p
    draft[wrong] = (draft[wrong] + 1 + g.integers(0, V - 1, int(wrong.sum()))) % V
    return lg, draft.astype(np.int32)


@pytest.mark.parametrize("B,k,V", [(64, 4, 4096), (256, 6, 1000), (5, 1, 77), (1, 0, 512), (700, 2, 64)])
@pytest.mark.parametrize("forced", [False, True])
def test_accept_commit_bit_exact(B, k, V, forced):
    shape = synth.ModelShape("t", 1, 64, 2, 2, 64, 64, V, "bf16")
    lg, draft = planted_logits(B, k, V, B + k, 0.7)
    lg[0, 0, [3, V - 1]] = 30.0                                   # a tie: lowest index wins
    g = synth.rng(3, 3)
    len0 = g.integers(0, 50, B).astype(np.int32)
    pend0 = g.integers(0, V, B).astype(np.int32)
    force = g.integers(0, k + 2, B).astype(np.int32) if forced else None
    orc = sfo.Oracle(shape.cfg(), synth.target_weights(shape, 1), None, B, 64, k + 1)
    orc.kv_len[:] = len0; orc.pending[:] = pend0
    acc_o, out_o = orc.accept_commit(k, draft, lg, force_len=force)

    eng = engine_only(shape, B, 64, k)
    eng.bind(synth.target_weights(shape, 1))
    eng.set_state(kv_len=len0, pending=pend0, n_new=np.zeros(B, np.int32))
    d = torch.from_numpy(draft).cuda()
    fl = torch.from_numpy(force).cuda() if forced else None
    ids = eng.sf_op_argmax(torch.from_numpy(lg).cuda().reshape(B * (k + 1), V)).reshape(B, k + 1)
    acc, out = eng.sf_op_accept(k, d, ids, force_len=fl)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(acc.cpu().numpy(), acc_o)
    np.testing.assert_array_equal(out.cpu().numpy(), out_o)
    np.testing.assert_array_equal(eng.kv_len.cpu().numpy(), orc.kv_len)
    np.testing.assert_array_equal(eng.pending.cpu().numpy(), orc.pending)
    np.testing.assert_array_equal(eng.n_new.cpu().numpy(), orc.n_new)
    np.testing.assert_array_equal(eng.cu_new.cpu().numpy(), orc.cu_new)
    if not forced:
        assert acc_o.min() >= 1 and acc_o.max() <= k + 1
        assert (acc_o > 1).any() or k == 0                        # acceptance > 1 is exercised
