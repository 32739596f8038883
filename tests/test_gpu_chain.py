"""GPU tests of chains of launches run as one kernel (epara_grouped_chain).

A chain computes the same tiles with the same arithmetic as the launches called one after the other, so its
outputs must equal theirs bit for bit wherever the launches do not cut a tile's K into parts (the separate
launches are held to the oracle by test_gpu_parity);
small chains are also compared with the CPU oracle directly.  A wait that cannot be met is forced from the
host with a poll limit of one: the kernel must still end and report it.
"""
import numpy as np
import pytest
import torch

from paper_2511_00603_amd import binding as B
from paper_2511_00603_amd import runtime as R
from paper_2511_00603_amd.mixrun import StagedMix
from workloads import make_mix

import gpu_util as U
import mix_oracle
from parity_util import TOL, assert_close

pytestmark = pytest.mark.gpu

SMALL = [
    (1, {}, "f32"),
    (2, {}, "bf16"),
    (3, dict(images=[2, 1, 1, 3, 1, 2, 1, 1], d=192, ffn=768, tokens=197), "bf16"),
    (4, dict(d=512, ffn=1376), "bf16"),
    (4, dict(d=512, ffn=1376), "fp8"),
    (5, dict(d=640, ffn=1664, total_rows=900, len_lo=60, len_hi=300), "bf16"),
]


def _h_scales(mix, dtype_name):
    return [0.05] * len(mix.services) if dtype_name == "fp8" else None


def _run(mix, dtype_name, chained, n_workgroups=None, host_bits=None, passes=1):
    staged = StagedMix(mix, dtype_name, U.DEV, s_h=_h_scales(mix, dtype_name), n_workgroups=n_workgroups,
                       host_bits=host_bits, chained=chained)
    for _ in range(passes):
        staged.run()
    torch.cuda.synchronize()
    if chained:
        assert staged.n_launches() == 1
        assert staged.chain_status() == 0
    return staged


def _raw(staged):
    """Outputs as stored (bit patterns), per launch and group."""
    return [[t.cpu().view(torch.uint8).numpy().copy() if t.dtype != torch.uint8 else t.cpu().numpy().copy() for _, _, t in launch]
            for launch in staged.outputs[0]]


def _cut(staged):
    """Per launch of separately launched passes: does the launch visit tiles in parts of K?"""
    return [p.n_split_tiles > 0 or p.n_panel_split_tiles > 0 for p in staged.plans()]


def _assert_same(mix, dtype_name, sep_raw, sep_vals, ch, cut, what=""):
    """Chain against launches.  Bit for bit, except from the first launch on that visits tiles in parts of K and
    adds the parts in index order (cut[l]), which a chain does not: the same products in another order of
    addition.  There only the services of at most 16 rows (never split) must still agree bit for bit; the rest,
    and every later launch, is held to the parity tolerance; a stored E4M3 value may land on the neighbouring
    code (an eighth apart)."""
    first = cut.index(True) if True in cut else len(cut)
    for l, (la, lb, va, vb) in enumerate(zip(sep_raw, _raw(ch), sep_vals, ch.results())):
        for x, y, (g, label, p), (_, _, q) in zip(la, lb, va, vb):
            if l < first or (l == first and mix.services[g].M <= 16):
                assert np.array_equal(x, y), what
            else:
                stored_fp8 = dtype_name == "fp8" and label == "H"
                assert_close(q, p, 0.13 if stored_fp8 else TOL[dtype_name], "chain against launches, %s svc %d %s %s" % (mix.name, g, label, what))


@pytest.mark.parametrize("index,shrink,dtype_name", SMALL)
@pytest.mark.parametrize("n_workgroups", [None, 8, 64])
def test_chain_equals_separate_launches_bit_for_bit(index, shrink, dtype_name, n_workgroups):
    print("chain case", index, shrink, dtype_name, n_workgroups, flush=True)
    mix = make_mix(index, **shrink)
    sep = _run(mix, dtype_name, False, n_workgroups)
    ch = _run(mix, dtype_name, True, n_workgroups, host_bits=sep.host_bits, passes=3)      # counters reset by the kernel itself
    _assert_same(mix, dtype_name, _raw(sep), sep.results(), ch, _cut(sep))


@pytest.mark.parametrize("index,shrink,dtype_name", [SMALL[0], SMALL[1], SMALL[3]])
def test_chain_against_the_oracle(index, shrink, dtype_name):
    mix = make_mix(index, **shrink)
    ch = _run(mix, dtype_name, True)
    want = mix_oracle.expected(mix, ch.host_bits, dtype_name)
    for lg, lw in zip(ch.results(), want):
        for (g, label, Y), (g2, label2, Yref) in zip(lg, lw):
            assert (g, label) == (g2, label2)
            assert_close(Y, Yref, TOL[dtype_name], "chained %s svc %d %s" % (mix.name, g, label))


@pytest.mark.parametrize("index,dtype_name", [(4, "bf16"), (4, "fp8"), (5, "bf16"), (3, "bf16")])
def test_full_size_chain_equals_separate_launches(index, dtype_name):
    print("full-size chain", index, dtype_name, flush=True)
    mix = make_mix(index)
    sep = _run(mix, dtype_name, False)
    a, vals, cut = _raw(sep), sep.results(), _cut(sep)
    bits = sep.host_bits
    del sep
    torch.cuda.empty_cache()
    ch = _run(mix, dtype_name, True, host_bits=bits, passes=2)
    _assert_same(mix, dtype_name, a, vals, ch, cut)


@pytest.mark.parametrize("index,shrink,dtype_name", [SMALL[0], SMALL[1], SMALL[2], SMALL[3], SMALL[5], (4, {}, "bf16")])
def test_chain_sees_fresh_activations_when_the_inputs_change_between_passes(index, shrink, dtype_name):
    """The hidden activations live at the same addresses in every pass: a consumer that read a line cached from
    the pass before, or read ahead of the producer's stores, would reproduce the OLD inputs' values.  The
    inputs are rescaled in place between passes and every pass is compared with the separate launches."""
    print("fresh activations", index, shrink, dtype_name, flush=True)
    mix = make_mix(index, **shrink)
    ch = StagedMix(mix, dtype_name, U.DEV, chained=True)
    sep = StagedMix(mix, dtype_name, U.DEV, chained=False, host_bits=ch.host_bits)
    for factor in (1.0, -0.5, 3.0, 0.125, -2.0):
        for st in (ch, sep):
            for X in st.inputs[0]:
                X.mul_(factor)
        ch.run()
        sep.run()
        torch.cuda.synchronize()
        assert ch.chain_status() == 0
        _assert_same(mix, dtype_name, _raw(sep), sep.results(), ch, _cut(sep), "factor %g" % factor)
        # the pass did change the outputs (otherwise this test could not see a stale read)
        if factor != 1.0:
            assert not all(np.array_equal(a, b) for la, lb in zip(prev, _raw(ch)) for a, b in zip(la, lb))
        prev = _raw(ch)


def test_device_copies_of_the_chain_plan_are_the_reference_planners():
    from oracle import planner as P
    staged = StagedMix(make_mix(4), "bf16", U.DEV, chained=True)
    chain = staged.programs[0][0][1]
    ref_phases = []
    for ph in chain.phases:
        gated = bool(np.all(ph.args["act"] == B.EPARA_ACT_SWIGLU))
        groups = [(int(a["M"]), int(a["K"]), int(a["N"]), gated) for a in ph.args]
        classes = [tuple(int(v) for v in c) for c in ph.classes]
        tiles = P.plan_groups([g[:3] for g in groups], classes)[3]
        assert [tuple(int(v) for v in t) for t in ph.d_tiles.cpu().numpy()[: ph.tiles.nbytes].view(B.TILE)] == tiles
        ref_phases.append((groups, classes, ph.n_stream_classes, tiles))
    orders = P.schedule_chain(ref_phases, chain.n_workgroups, 8, 1, 4)
    for ph, want in zip(chain.phases, orders):
        assert ph.d_order.cpu().numpy()[: ph.order.nbytes].view(np.int32).tolist() == want
    down = chain.phases[1]
    waits = down.d_waits.cpu().numpy()[: down.waits.nbytes].view(B.CHAIN_WAIT)
    assert [(int(w["counter"]), int(w["need"])) for w in waits] == P.chain_waits(ref_phases[0][3], 0, [0, 1, 2, 3])


def test_a_wait_that_runs_out_is_reported_and_the_kernel_still_ends():
    """Phase one: a single long tile, so almost every workgroup reaches phase two at once and finds the counter
    unmet; with a poll limit of one those waits give up.  The flag must be set, the kernel must end, and the
    workspace must be usable again: the same chain with the default limit then gives the right result."""
    rng = np.random.default_rng(77)
    K0, N0, N1, M = 16384, 32, 4096, 8
    X = rng.standard_normal((M, K0)).astype(np.float32)
    W0 = (rng.standard_normal((K0, N0)) / np.sqrt(K0)).astype(np.float32)
    W1 = (rng.standard_normal((N0, N1)) / np.sqrt(N0)).astype(np.float32)
    dt = B.EPARA_BF16
    g0 = U.Groups([{"X": X, "W": W0, "b": None, "act": "none"}], "bf16")
    Hd = g0.Y[0]
    W1d = R.pack_weights(R.device_tensor_from_bits(U.to_bits(W1, "bf16"), dt, U.DEV), dt)
    Yd = torch.zeros((M, N1), dtype=torch.bfloat16, device=U.DEV)
    a1 = np.array([R.group_args(Hd, W1d, Yd, M, N0, N1, "none")], dtype=B.GROUP_ARGS)
    chain = R.ChainPlan([g0.args, a1], [dt, dt], [None, np.array([0], dtype=np.int32)], dt, U.DEV)
    R.grouped_chain(chain, spin_limit=1)
    assert R.chain_status(chain) == 1
    assert R.chain_status(chain) == 0                      # reading clears it
    R.grouped_chain(chain)
    assert R.chain_status(chain) == 0
    got = Yd.to(torch.float32).cpu().numpy().astype(np.float64)
    R.grouped_forward(g0.plan, dt)
    plain = R.LaunchPlan(a1, dt, U.DEV)
    Yd.zero_()
    R.grouped_forward(plain, dt)
    torch.cuda.synchronize()
    assert np.array_equal(got, Yd.to(torch.float32).cpu().numpy().astype(np.float64))


def test_chain_rejects_what_it_cannot_run_safely():
    mix = make_mix(4, d=512, ffn=1376)
    ok = StagedMix(mix, "bf16", U.DEV, chained=True).programs[0][0][1]
    stream = R.current_stream_handle()
    def status(phases, ws_bytes=None, in_dtype=B.EPARA_BF16):
        try:
            B.epara_grouped_chain(phases, in_dtype, ok.d_workspace.data_ptr(), ok.workspace_bytes if ws_bytes is None else ws_bytes, stream)
        except B.EparaError as e:
            return e.status
        return B.EPARA_OK
    assert status(ok.c, ws_bytes=16) == B.EPARA_ERR_CAPACITY
    big = StagedMix(mix, "bf16", U.DEV, chained=True, n_workgroups=1024).programs[0][0][1]       # more than the GPU keeps resident
    assert status(big.c) == B.EPARA_ERR_SHAPE
    w = ok.phases[1].waits.copy()
    ok.phases[1].waits["need"][0] += 1                                                          # not the producer's tile count
    assert status(ok.c) == B.EPARA_ERR_SHAPE
    ok.phases[1].waits[:] = w
    ok.c[1].counter_base = 0                                                                    # counter ranges overlap
    assert status(ok.c) == B.EPARA_ERR_SHAPE
    ok.c[1].counter_base = ok.phases[1].counter_base
    assert status(ok.c) == B.EPARA_OK
    torch.cuda.synchronize()
    assert R.chain_status(ok) == 0
