"""A pass of the library captured into a HIP graph and replayed: the launches only enqueue kernels on the
caller's stream (no allocation, no synchronisation, no memset), so they can be captured; every replay, with
the program's own eager work and synchronisations in between, must reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2511_00603_amd.mixrun import StagedMix
from workloads import make_mix

import gpu_util as U

pytestmark = pytest.mark.gpu


def _raw(staged):
    return [[t.cpu().view(torch.uint8).numpy().copy() if t.dtype != torch.uint8 else t.cpu().numpy().copy() for _, _, t in launch]
            for launch in staged.outputs[0]]


@pytest.mark.parametrize("index,shrink,dtype_name,chained", [
    (1, {}, "f32", False), (2, {}, "bf16", False), (4, dict(d=512, ffn=1376), "bf16", False),
    (4, dict(d=512, ffn=1376), "bf16", True), (2, {}, "bf16", True), (1, {}, "f32", True),
    (4, {}, "bf16", False)])                       # full size: tiles visited in parts of K, counters reset by the kernel
def test_graph_replays_equal_the_eager_pass(index, shrink, dtype_name, chained):
    print("graph case", index, dtype_name, chained, flush=True)
    mix = make_mix(index, **shrink)
    staged = StagedMix(mix, dtype_name, U.DEV, chained=chained)
    staged.run()                                   # eager: also the first call of every kernel (attributes are set here)
    torch.cuda.synchronize()
    want = _raw(staged)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            staged.run()
    torch.cuda.synchronize()
    for factor in (2.0, 0.5, -1.0):
        for launch in staged.outputs[0]:           # eager work between replays: wipe the outputs
            for _, _, t in launch:
                t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = _raw(staged)
        for la, lb in zip(want, got):
            for a, b in zip(la, lb):
                assert np.array_equal(a, b)
        # change the inputs in place: the next replay must follow them, as the eager pass does
        for X in staged.inputs[0]:
            X.mul_(factor)
        staged.run()
        torch.cuda.synchronize()
        want = _raw(staged)
    if chained:
        assert staged.chain_status() == 0


def test_passes_on_two_streams_equal_the_passes_one_after_the_other():
    """Independent passes (their own copies of every buffer) submitted to two streams in turn overlap on the
    GPU; each must still produce what it produces alone."""
    mix = make_mix(4, d=512, ffn=1376)
    staged = StagedMix(mix, "bf16", U.DEV, copies=2)
    raw = lambda c: [[t.cpu().view(torch.uint8).numpy().copy() for _, _, t in launch] for launch in staged.outputs[c]]
    for c in range(2):
        staged.run(copy=c)
    torch.cuda.synchronize()
    want = [raw(0), raw(1)]
    for c in range(2):
        for launch in staged.outputs[c]:
            for _, _, t in launch:
                t.zero_()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    for i in range(6):
        with torch.cuda.stream(streams[i % 2]):
            staged.run(copy=i)
    torch.cuda.synchronize()
    for c in range(2):
        for la, lb in zip(want[c], raw(c)):
            for a, b in zip(la, lb):
                assert np.array_equal(a, b)
