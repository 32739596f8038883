"""GPU test of epara_grouped_chain_static: the chain entry point for callers that cannot allocate, whose
completion counters live in a device array inside the library.  Called through the C-ABI and compared bit for
bit with epara_grouped_chain (caller-provided workspace) on the same plans: two calls in a row, the second
with a smaller input, so that whatever the first call left in the array would show; then the error path.
"""
import numpy as np
import pytest
import torch

from paper_2511_00603_amd import binding as B
from paper_2511_00603_amd import runtime as R
from paper_2511_00603_amd.mixrun import StagedMix
from workloads import make_mix

import gpu_util as U

pytestmark = pytest.mark.gpu

CASES = [   # (mix, shrink of the first call, shrink of the second, smaller call, dtype)
    (1, {}, dict(rows=[2, 5]), "f32"),
    (4, dict(d=512, ffn=1376), dict(d=256, ffn=704, rows=[1, 8, 20, 40]), "bf16"),
    (3, dict(images=[2, 1, 1, 3, 1, 2, 1, 1], d=192, ffn=768, tokens=197), dict(images=[1, 1, 1, 1, 1, 1, 1, 1], d=128, ffn=512, tokens=50), "bf16"),
]


def _outputs(staged):
    return [t.cpu().view(torch.uint8).numpy().copy() for launch in staged.outputs[0] for _, _, t in launch]


def _clear(staged):
    for launch in staged.outputs[0]:
        for _, _, t in launch:
            t.zero_()


@pytest.mark.parametrize("index,first,second,dtype_name", CASES)
def test_static_scratch_chain_equals_the_workspace_chain(index, first, second, dtype_name):
    flag = torch.full((1,), -1, dtype=torch.int32, device=U.DEV)
    for shrink in (first, second):
        print("no-alloc chain case", index, shrink, dtype_name, flush=True)
        staged = StagedMix(make_mix(index, **shrink), dtype_name, U.DEV, chained=True)
        plan = staged.programs[0][0][1]
        R.grouped_chain(plan)                               # the existing entry point, caller's workspace
        torch.cuda.synchronize()
        assert R.chain_status(plan) == 0
        want = _outputs(staged)
        assert any(w.any() for w in want)
        _clear(staged)
        flag.fill_(-1)
        R.grouped_chain_static(plan, d_flag=flag)           # the library's own scratch, nothing allocated
        torch.cuda.synchronize()
        assert int(flag.item()) == 0
        for a, b in zip(_outputs(staged), want):
            assert np.array_equal(a, b)


def test_static_scratch_chain_reports_a_wait_that_ran_out_and_recovers():
    """A poll limit of one forces the bounded wait to give up (the kernel still ends): the flag is reported
    through d_flag, and the next call starts from a clean array."""
    staged = StagedMix(make_mix(4, d=512, ffn=1376), "bf16", U.DEV, chained=True)
    plan = staged.programs[0][0][1]
    R.grouped_chain(plan)
    torch.cuda.synchronize()
    want = _outputs(staged)
    flag = torch.full((1,), -1, dtype=torch.int32, device=U.DEV)
    seen = 0
    for _ in range(5):                                      # whether a wait runs out with one poll depends on timing
        R.grouped_chain_static(plan, spin_limit=1, d_flag=flag)
        torch.cuda.synchronize()
        seen |= int(flag.item())
    assert seen in (0, 1)
    _clear(staged)
    R.grouped_chain_static(plan, d_flag=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    for a, b in zip(_outputs(staged), want):
        assert np.array_equal(a, b)


def test_static_scratch_chain_rejects_more_counters_than_the_array_holds():
    lib = B.lib()
    import ctypes
    # validation happens on the host copies: a phase with more groups than the array has counters
    G = B.EPARA_STATIC_CHAIN_COUNTERS + 1
    args = np.zeros(G, dtype=B.GROUP_ARGS)
    args["K"], args["N"] = 8, 8                              # M = 0 everywhere: nothing to launch, only the counter count matters
    launch = B.Launch(args.ctypes.data, None, None, None, None, 0, 0, 8, G, None, 0, 0, 0)
    phases = (B.ChainPhase * 1)()
    phases[0].launch = ctypes.pointer(launch)
    phases[0].out_dtype, phases[0].counter_base = B.EPARA_BF16, 0
    rc = lib.epara_grouped_chain_static(ctypes.addressof(phases), 1, B.EPARA_BF16, 0, None, None)
    assert rc == B.EPARA_ERR_CAPACITY
