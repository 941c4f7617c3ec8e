"""The arg-max entry point that allocates nothing (partials in a static device array of the library) against
the entry point it is a variant of, through the C ABI: two calls in a row, the second on a smaller input."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth
from paper_2511_20340_amd import binding as sfb

from gpu_common import engine_only

pytestmark = pytest.mark.gpu


def test_argmax_noalloc_matches_the_workspace_variant_twice_in_a_row():
    eng = engine_only(synth.ModelShape("t", 1, 128, 2, 2, 64, 64, 64, "bf16"), 1, 64, 1)
    g = synth.rng(77, 1)
    for M, V in ((300, 32000), (7, 1000)):                      # the second call: fewer rows, shorter rows
        lg = g.standard_normal((M, V), dtype=np.float32)
        lg[0, :] = 0.25                                         # all tied -> index 0
        lg[1, [V - 1, V // 3]] = 9.0                            # tie -> lowest index
        lg[2, 0] = np.nan; lg[2, V - 2] = 50.0                  # NaN never wins
        lgd = torch.from_numpy(lg).cuda()
        want = eng.sf_op_argmax(lgd)
        ids = torch.full((M,), -7, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        eng.sf_op_argmax_noalloc(lgd, ids)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(ids, want)
        assert ids[0].item() == 0 and ids[1].item() == V // 3 and ids[2].item() == V - 2
    # beyond the static array's size: a clear error, nothing enqueued
    big = torch.zeros(sfb_max_rows() + 1, 8, dtype=torch.float32, device="cuda")
    out = torch.zeros(sfb_max_rows() + 1, dtype=torch.int32, device="cuda")
    st = sfb.lib().sf_op_argmax_noalloc(eng.ctx, C.c_void_p(big.data_ptr()), big.shape[0], 8,
                                        C.c_void_p(out.data_ptr()), None)
    assert st == sfb.SF_ECAPACITY


def sfb_max_rows():
    return 4096
