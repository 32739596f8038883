"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle on the same seeded
inputs.  Tolerances (max relative error with the group's rms as floor, tests/parity_util.py):
1e-5 fp32, 2e-2 bf16 inputs / fp32 accumulation, 6e-2 fp8 E4M3.  Integer-valued cases must
match bit for bit.  The full-size mixes are compared on every output element, in the launch
configuration bench.py times.
"""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2511_00603_amd import binding as B
from paper_2511_00603_amd import runtime as R
from paper_2511_00603_amd.mixrun import StagedMix
from workloads import casts, make_mix

import gpu_util as U
import mix_oracle
from parity_util import TOL, assert_close

pytestmark = pytest.mark.gpu


def check_mix(mix, dtype_name, rows=None, h_scales=None, host_bits=None):
    """One pass on the GPU against the oracle.  fp8 SwiGLU mixes without h_scales: the oracle runs first and its
    own hidden activations give the static scales (amax / 448) that both sides then use."""
    want = None
    if dtype_name == "fp8" and h_scales is None and mix.services[0].kind == "swiglu":
        host_bits = host_bits if host_bits is not None else StagedMix.stage_host(mix, "fp8")
        h_scales = []
        want = mix_oracle.expected(mix, host_bits, dtype_name, rows=rows, calibrated=h_scales)
    staged = StagedMix(mix, dtype_name, U.DEV, s_h=h_scales, host_bits=host_bits)
    staged.run()
    torch.cuda.synchronize()
    got = staged.results()
    if want is None:
        want = mix_oracle.expected(mix, staged.host_bits, dtype_name, rows=rows, h_scales=h_scales)
    tol = TOL[dtype_name]
    worst = 0.0
    assert len(got) == len(want)
    for lg, lw in zip(got, want):
        assert len(lg) == len(lw)
        for (g, label, Y), (g2, label2, Yref) in zip(lg, lw):
            assert (g, label) == (g2, label2)
            if rows is not None:
                Y = Y[rows[g]]
            if dtype_name == "fp8" and label == "H":
                # Stored E4M3 codes.  The oracle rounds fp64 sums, the GPU fp32 MFMA sums, so the same value
                # cannot be handed to both roundings: nearly all codes must agree exactly, a value on a
                # rounding boundary may land one code apart, and near zero (where codes are an absolute
                # 2^-9 * s_h apart) the difference is bounded by the accumulation error instead.
                Y = Y * h_scales[g]
                rms = float(np.sqrt(np.mean(Yref * Yref)))
                step = np.maximum(0.13 * np.maximum(np.abs(Yref), h_scales[g] * 2.0 ** -6), 1e-3 * rms)
                bad = np.argwhere(~(np.abs(Y - Yref) <= step))
                assert len(bad) == 0, "H codes too far apart at %d places, e.g. %s" % (
                    len(bad), [(tuple(int(v) for v in ij), float(Y[tuple(ij)]), float(Yref[tuple(ij)])) for ij in bad[:8]])
                assert np.mean(Y != Yref) < 0.02
                continue
            worst = max(worst, assert_close(Y, Yref, tol, "%s svc %d %s" % (mix.name, g, label)))
    return worst


# ---- exactness on integer-valued inputs (layout, indexing, tails) -----------------------------

@pytest.mark.parametrize("dtype_name", ["f32", "bf16", "fp8"])
def test_small_integers_are_bit_exact(dtype_name):
    """Small integers: every product and sum is exact in fp32, so the output must be the oracle's, bit for bit,
    after the cast.  fp8 runs with power-of-two per-tensor scales (1/8 for X, 1/4 for W), under which the
    codes, their products and the scale product 2^-5 are all exact."""
    rng = np.random.default_rng(11)
    shapes = [(5, 64, 40), (1, 32, 16), (64, 96, 33), (70, 160, 300), (300, 128, 260), (257, 256, 513), (16, 48, 10)]
    specs = []
    for M, K, N in shapes:
        X = rng.integers(-4, 5, (M, K)).astype(np.float32)
        W = rng.integers(-3, 4, (K, N)).astype(np.float32)
        b = rng.integers(-8, 9, N).astype(np.float32)
        specs.append({"X": X, "W": W, "b": b, "act": "relu", "s_x": 0.125, "s_w": 0.25})
    G = U.Groups(specs, dtype_name)
    got, want = G.run(), G.expected()
    for (M, K, N), y, yref in zip(shapes, got, want):
        if dtype_name != "f32":
            yref = ref.bf16_decode(ref.bf16_encode(yref))
        assert np.array_equal(y, yref), (dtype_name, M, K, N, np.argwhere(y != yref)[:5])


def test_long_k_tiles_visited_in_parts(dtype_name="bf16"):
    """Batches of 17 to 64 rows with K >= 8192 (bf16; fp8 tiles are not split): the launch visits each tile in two
    parts of K whose sums meet in the workspace.  Integer-valued operands make every order of addition exact, so the result must be
    the oracle's bit for bit: ragged K (a part boundary inside a fragment pair, a last fragment cut short),
    ragged rows and columns, next to groups that are not split; twice, on grids of different sizes (who arrives
    last changes), and three times in a row on one plan (the arrival counters return to zero)."""
    rng = np.random.default_rng(17)
    shapes = [(40, 8208, 200), (64, 11024, 136), (17, 8192, 70), (8, 8192, 40), (33, 12304, 24), (64, 4080, 130), (20, 16384, 16)]
    acts = ["relu", "none", "relu", "none", "none", "relu", "none"]
    specs = []
    for (M, K, N), act in zip(shapes, acts):
        X = rng.integers(-4, 5, (M, K)).astype(np.float32)
        W = rng.integers(-3, 4, (K, N)).astype(np.float32)
        b = rng.integers(-8, 9, N).astype(np.float32)
        specs.append({"X": X, "W": W, "b": b, "act": act, "s_x": 0.125, "s_w": 0.25})
    for W_ in (None, 24):
        G = U.Groups(specs, dtype_name, n_workgroups=W_)
        assert G.plan.n_split_tiles > 0
        parts = {int(e >> 28) + 1 for e in G.plan.order if e >= 0}
        assert parts == {1, 2}
        want = [ref.bf16_decode(ref.bf16_encode(y)) for y in G.expected()]
        for rep in range(3):
            for (M, K, N), y, yref in zip(shapes, G.run(), want):
                assert np.array_equal(y, yref), (dtype_name, W_, rep, M, K, N, np.argwhere(y != yref)[:5])
        if dtype_name == "bf16":
            # new activations at the same addresses: the parts that come back from the workspace must be this
            # launch's (the visit that adds them may run on another compute die than the ones that wrote them)
            for i, sp in enumerate(specs):
                G.keep[3 * i].mul_(-2.0)
                G.bits[i]["X"] = casts.bf16_bits(-2.0 * sp["X"])
            want = [ref.bf16_decode(ref.bf16_encode(y)) for y in G.expected()]
            for (M, K, N), y, yref in zip(shapes, G.run(), want):
                assert np.array_equal(y, yref), ("rescaled", W_, M, K, N, np.argwhere(y != yref)[:5])
    # real values: against the oracle at the usual tolerance
    specs = [U.rand_spec(rng, M, K, N, act, bias=True) for (M, K, N), act in zip(shapes, ["gelu_erf", "silu", "none", "relu", "gelu_tanh", "none", "relu"])]
    G = U.Groups(specs, dtype_name)
    for (M, K, N), y, yref in zip(shapes, G.run(), G.expected()):
        assert_close(y, yref, TOL[dtype_name], "split K %s" % ((M, K, N),))


def test_last_round_panel_tiles_visited_in_parts(dtype_name="bf16"):
    """A bf16 launch of panel tiles alone, all of one K: the tiles of the last, partial round are visited in two to four
    parts of K whose raw sums meet in the workspace.  Integer-valued operands make every order of addition exact, so
    the result must be the oracle's bit for bit: ragged rows and columns, a K that is not a multiple of the parts'
    unit, two grid sizes (two and four parts), three calls in a row on one plan (the counters return to zero), and
    (bf16) new activations at the same addresses."""
    rng = np.random.default_rng(19)
    shapes = [(300, 2064, 500), (600, 2064, 300)]
    specs = []
    for (M, K, N), act in zip(shapes, ["relu", "none"]):
        X = rng.integers(-4, 5, (M, K)).astype(np.float32)
        W = rng.integers(-3, 4, (K, N)).astype(np.float32)
        b = rng.integers(-8, 9, N).astype(np.float32)
        specs.append({"X": X, "W": W, "b": b, "act": act, "s_x": 0.125, "s_w": 0.25})
    seen = set()
    for W_ in (8, 24):
        G = U.Groups(specs, dtype_name, n_workgroups=W_)
        assert G.plan.n_panel_split_tiles == 10 % W_ and G.plan.n_split_tiles == 0
        parts = {int(e >> 28) + 1 for e in G.plan.order if e >= 0}
        seen |= parts
        want = [ref.bf16_decode(ref.bf16_encode(y)) for y in G.expected()]
        for rep in range(3):
            for (M, K, N), y, yref in zip(shapes, G.run(), want):
                assert np.array_equal(y, yref), (dtype_name, W_, rep, M, K, N, np.argwhere(y != yref)[:5])
        if dtype_name == "bf16":
            for i, sp in enumerate(specs):
                G.keep[3 * i].mul_(-2.0)
                G.bits[i]["X"] = casts.bf16_bits(-2.0 * sp["X"])
            want = [ref.bf16_decode(ref.bf16_encode(y)) for y in G.expected()]
            for (M, K, N), y, yref in zip(shapes, G.run(), want):
                assert np.array_equal(y, yref), ("rescaled", W_, M, K, N, np.argwhere(y != yref)[:5])
    assert seen == {1, 2, 4}
    # tiles of one launch in three and in four parts (two parts per workgroup on average)
    shapes = [(900, 4112, 300), (600, 4112, 300)]
    specs = []
    for M, K, N in shapes:
        X = rng.integers(-3, 4, (M, K)).astype(np.float32)
        W = rng.integers(-3, 4, (K, N)).astype(np.float32)
        specs.append({"X": X, "W": W, "b": rng.integers(-8, 9, N).astype(np.float32), "act": "none", "s_x": 0.125, "s_w": 0.25})
    G = U.Groups(specs, dtype_name, n_workgroups=24)
    assert G.plan.n_panel_split_tiles == 14 and {int(e >> 28) + 1 for e in G.plan.order if e >= 0} == {3, 4}
    want = [ref.bf16_decode(ref.bf16_encode(y)) for y in G.expected()]
    for rep in range(2):
        for (M, K, N), y, yref in zip(shapes, G.run(), want):
            assert np.array_equal(y, yref), ("mixed parts", rep, M, K, N, np.argwhere(y != yref)[:5])
    shapes = [(300, 2064, 500), (600, 2064, 300)]
    specs = [U.rand_spec(rng, M, K, N, act, bias=True) for (M, K, N), act in zip(shapes, ["gelu_erf", "silu"])]
    G = U.Groups(specs, dtype_name, n_workgroups=8)
    for (M, K, N), y, yref in zip(shapes, G.run(), G.expected()):
        assert_close(y, yref, TOL[dtype_name], "panel split K %s" % ((M, K, N),))


def test_identity_zero_and_ones_weights_bf16():
    rng = np.random.default_rng(12)
    X = rng.standard_normal((37, 64)).astype(np.float32)
    b = (rng.standard_normal(64) * 0.5).astype(np.float32)
    specs = [{"X": X, "W": np.eye(64, dtype=np.float32), "b": b, "act": "none"},
             {"X": X, "W": np.zeros((64, 48), dtype=np.float32), "b": b[:48], "act": "gelu_erf"},
             {"X": np.round(X * 4) / 4, "W": np.ones((64, 20), dtype=np.float32), "b": None, "act": "none"}]
    G = U.Groups(specs, "bf16")
    y, want = G.run(), G.expected()
    Xb = ref.bf16_decode(G.bits[0]["X"])
    assert np.array_equal(y[0], ref.bf16_decode(ref.bf16_encode(Xb + b.astype(np.float64))))
    assert_close(y[1], want[1], TOL["bf16"], "zero weights")
    assert np.all(y[1] == y[1][0])                                   # act(b) broadcast over rows
    assert_close(y[2], want[2], TOL["bf16"], "ones weights")


@pytest.mark.parametrize("dtype_name", ["f32", "bf16"])
def test_linearity_in_x(dtype_name):
    rng = np.random.default_rng(13)
    M, K, N = 90, 128, 72
    X1, X2 = rng.standard_normal((M, K)).astype(np.float32), rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32)
    a, c = 1.75, -0.375
    f = lambda X: U.Groups([{"X": X, "W": W, "b": None, "act": "none"}], dtype_name).run()[0]
    lhs, rhs = f(a * X1 + c * X2), a * f(X1) + c * f(X2)
    assert_close(lhs, rhs, 3 * TOL[dtype_name], "linearity")


def test_fp32_small_batches_with_awkward_shapes():
    """Batches of at most 16 rows take the fp32 path that cuts K into four quarters: K smaller than the number of
    quarters, K not a multiple of the staging step, ragged column tiles, every activation, next to a group of
    the 64-row class in the same launch."""
    rng = np.random.default_rng(21)
    acts = ["none", "relu", "gelu_erf", "gelu_tanh", "silu"]
    shapes = [(1, 1, 1), (7, 3, 10), (16, 7, 65), (3, 17, 130), (16, 100, 64), (9, 513, 77), (2, 2048, 5), (40, 33, 70), (16, 64, 128)]
    specs = [U.rand_spec(rng, M, K, N, acts[i % len(acts)], bias=i % 3 != 0) for i, (M, K, N) in enumerate(shapes)]
    G = U.Groups(specs, "f32")
    assert sorted(set(int(c) for c in G.plan.tiles["cls"])) == [0, 1]
    for (M, K, N), y, yref in zip(shapes, G.run(), G.expected()):
        assert_close(y, yref, TOL["f32"], "fp32 small %s" % ((M, K, N),))
    # and the same values whatever the grid size (fixed summation order)
    y_a = U.Groups(specs, "f32", n_workgroups=8).run()
    y_b = U.Groups(specs, "f32", n_workgroups=256).run()
    for a, b in zip(y_a, y_b):
        assert np.array_equal(a, b)


# ---- independence and determinism ------------------------------------------------------------------

def test_group_order_row_order_and_grid_size_do_not_change_a_single_bit():
    rng = np.random.default_rng(14)
    shapes = [(3, 256, 96, "gelu_erf"), (300, 128, 260, "relu"), (64, 512, 64, "none"), (17, 64, 10, "silu"), (700, 96, 300, "none")]
    specs = [U.rand_spec(rng, M, K, N, act) for M, K, N, act in shapes]
    base = U.Groups(specs, "bf16")
    y0 = base.run()
    raw0 = [t.view(torch.int16).cpu().numpy() for t in base.raw()]
    perm = [3, 0, 4, 2, 1]
    y1 = U.Groups([specs[i] for i in perm], "bf16").run()
    for j, i in enumerate(perm):
        assert np.array_equal(y1[j], y0[i])
    for W in (8, 64, 128):
        g = U.Groups(specs, "bf16", n_workgroups=W)
        g.run()
        for a, t in zip(raw0, g.raw()):
            assert np.array_equal(a, t.view(torch.int16).cpu().numpy())
    # permuting the rows of X permutes the rows of Y; splitting a batch in two reproduces the same rows
    p = rng.permutation(300)
    s = dict(specs[1]); s["X"] = specs[1]["X"][p]
    top, bottom = dict(specs[1]), dict(specs[1])
    top["X"], bottom["X"] = specs[1]["X"][:100], specs[1]["X"][100:]
    ys = U.Groups([s, top, bottom], "bf16").run()
    assert np.array_equal(ys[0], y0[1][p])
    assert_close(np.vstack([ys[1], ys[2]]), y0[1], 1e-2, "split batch")   # tile classes differ: not bitwise
    # run to run
    again = base.run()
    for a, b in zip(y0, again):
        assert np.array_equal(a, b)


# ---- edge cases -------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype_name", ["f32", "bf16", "fp8"])
def test_ragged_and_degenerate_groups(dtype_name):
    rng = np.random.default_rng(15)
    kmul = 16 if dtype_name == "fp8" else 8
    shapes = [(0, 64, 32, "none"), (1, kmul, 1, "none"), (1, 64, 10, "relu"), (64, 5 * kmul, 33, "gelu_erf"),
              (65, 3 * kmul, 31, "silu"), (255, 7 * kmul, 255, "gelu_tanh"), (256, 128, 256, "none"),
              (257, 64 + kmul, 257, "relu"), (0, 32, 8, "none"), (513, 2 * kmul, 7, "none")]
    specs = [U.rand_spec(rng, M, K, N, act) for M, K, N, act in shapes]
    G = U.Groups(specs, dtype_name)
    got, want = G.run(), G.expected()
    for sh, y, yref in zip(shapes, got, want):
        assert y.shape == yref.shape
        if y.size:
            assert_close(y, yref, TOL[dtype_name], str(sh))


@pytest.mark.parametrize("dtype_name", ["bf16", "fp8"])
def test_every_activation_on_whole_and_ragged_panel_tiles(dtype_name):
    """The matrix-core kernels use the hardware's exp / reciprocal and a rational erf in their epilogue;
    whole 256 x 256 tiles run an unrolled epilogue, ragged ones a loop: both against the fp64 oracle, with
    bias, K of one to five stages incl. an odd stage count and a ragged last stage."""
    rng = np.random.default_rng(16)
    kmul = 16 if dtype_name == "fp8" else 8
    acts = ["none", "relu", "gelu_erf", "gelu_tanh", "silu"]
    shapes = [(512, 24 * kmul, 512, acts[i % 5]) if i < 5 else (300, (4 * i + 1) * kmul, 520, acts[i % 5]) for i in range(10)]
    specs = [U.rand_spec(rng, M, K, N, act) for M, K, N, act in shapes]
    for sp in specs:                                                     # activations need arguments of both signs and sizes
        sp["X"] *= 2.0
    G = U.Groups(specs, dtype_name)
    got, want = G.run(), G.expected()
    for sh, y, yref in zip(shapes, got, want):
        assert_close(y, yref, TOL[dtype_name], str(sh))


def test_output_beyond_four_gibibytes_is_addressed_with_64_bits():
    """One group whose output has more than 2^32 bytes (and its last rows more than 2^31 elements in): rows
    sampled from the start, the 4 GiB boundary and the end against the oracle, panel tiles whole and ragged."""
    rng = np.random.default_rng(17)
    M, K, N = 36100, 16, 60040
    sp = U.rand_spec(rng, M, K, N, "relu")
    xb, wb = casts.bf16_bits(sp["X"]), casts.bf16_bits(sp["W"])
    dX = R.device_tensor_from_bits(xb, B.EPARA_BF16, U.DEV)
    dW = R.pack_weights(R.device_tensor_from_bits(wb, B.EPARA_BF16, U.DEV), B.EPARA_BF16)
    db = torch.from_numpy(sp["b"]).to(U.DEV)
    dY = torch.zeros((M, N), dtype=torch.bfloat16, device=U.DEV)
    assert dY.numel() * 2 > 2 ** 32
    plan = R.LaunchPlan(np.array([R.group_args(dX, dW, dY, M, K, N, "relu", bias=db)], dtype=B.GROUP_ARGS), B.EPARA_BF16, U.DEV)
    R.grouped_forward(plan, B.EPARA_BF16)
    torch.cuda.synchronize()
    edge = 2 ** 32 // (2 * N)                                            # the row that straddles byte 2^32
    rows = sorted({0, 1, 255, 256, edge - 1, edge, edge + 1, 2 ** 31 // N, 2 ** 31 // N + 1, M - 257, M - 2, M - 1}
                  | set(int(r) for r in rng.integers(0, M, 12)))
    got = dY[torch.tensor(rows, device=U.DEV)].float().cpu().numpy()
    want = ref.dense_forward(ref.bf16_decode(xb[rows]), ref.bf16_decode(wb), sp["b"], "relu")
    assert_close(got, want, TOL["bf16"], "rows around the 4 GiB boundary")
    # nothing outside the group's rows x columns was touched: the padding rows of the last tile row stay unwritten
    assert torch.count_nonzero(dY[M - 1]).item() > 0
    del dY
    torch.cuda.empty_cache()


def test_nothing_to_do_is_ok():
    G = U.Groups([], "bf16")
    assert G.run() == []
    rng = np.random.default_rng(16)
    G = U.Groups([U.rand_spec(rng, 0, 64, 32), U.rand_spec(rng, 0, 32, 8)], "bf16")
    assert [y.shape for y in G.run()] == [(0, 32), (0, 8)]


def test_every_activation_fp32():
    rng = np.random.default_rng(17)
    specs = [U.rand_spec(rng, 33, 100, 70, act, x_uniform=True) for act in ("none", "relu", "gelu_erf", "gelu_tanh", "silu")]
    for s in specs:
        s["X"] = s["X"] * 3
    G = U.Groups(specs, "f32")
    for s, y, yref in zip(specs, G.run(), G.expected()):
        assert_close(y, yref, TOL["f32"], s["act"])


def test_pack_weights_layout_round_trip():
    # packed fragment (nb, ks), chunk q*16+r holds W[ks*32 + 8q .. +7][nb*16 + r] (bf16), zero padded; the
    # stages of a column block are padded to a multiple of four
    rng = np.random.default_rng(18)
    K, N = 72, 37
    bits = rng.integers(1, 2 ** 15, (K, N)).astype(np.uint16)
    W = R.device_tensor_from_bits(bits, B.EPARA_BF16, U.DEV)
    P = R.pack_weights(W, B.EPARA_BF16)
    torch.cuda.synchronize()
    p = P.cpu().numpy().view(np.uint16).reshape(3, 4, 4, 16, 8)          # [nb][ks][q][r][e]
    want = np.zeros((3, 4, 4, 16, 8), dtype=np.uint16)
    for nb in range(3):
        for ks in range(3):
            for q in range(4):
                for r in range(16):
                    for e in range(8):
                        k, n = ks * 32 + q * 8 + e, nb * 16 + r
                        if k < K and n < N:
                            want[nb, ks, q, r, e] = bits[k, n]
    assert np.array_equal(p, want)


# ---- what the kernel reads is what the reference planner wrote ----------------------------------------

@pytest.mark.parametrize("index,shrink", [(4, {}), (3, {}), (2, {})])
def test_device_copies_of_the_tile_table_and_visit_order_are_the_reference_planners(index, shrink):
    from oracle import planner as P
    staged = StagedMix(make_mix(index, **shrink), None, U.DEV)
    for plan in staged.plans():
        tiles = plan.d_tiles.cpu().numpy()[: plan.tiles.nbytes].view(B.TILE)
        order = plan.d_order.cpu().numpy()[: plan.order.nbytes].view(np.int32)
        args = plan.d_args.cpu().numpy()[: plan.args.nbytes].view(B.GROUP_ARGS)
        assert np.array_equal(args, plan.args)
        gated = bool(np.all(plan.args["act"] == B.EPARA_ACT_SWIGLU))
        groups = [(int(a["M"]), int(a["K"]), int(a["N"])) + ((True,) if gated else ()) for a in plan.args]
        classes = [tuple(int(v) for v in c) for c in plan.classes]
        row_off, x_off, y_off, want_tiles = P.plan_groups([g[:3] for g in groups], classes)
        assert [tuple(int(v) for v in t) for t in tiles] == want_tiles
        want_order = P.schedule_tiles(groups, classes, plan.n_stream_classes, want_tiles, plan.n_workgroups, 8, 1, 4)
        assert order.tolist() == want_order
        assert plan.row_off.tolist() == row_off and plan.x_off.tolist() == x_off and plan.y_off.tolist() == y_off


def test_end_to_end_error_against_the_unrounded_masters_is_reported():
    """Informative: the parity gate compares against an oracle fed the same rounded inputs; this is the error
    against the fp32 masters, i.e. including the storage formats' own rounding (bf16: about 2^-9 per operand)."""
    mix = make_mix(4, d=512, ffn=1376)
    staged = StagedMix(mix, "bf16", U.DEV)
    staged.run()
    torch.cuda.synchronize()
    from parity_util import rel_err
    worst = 0.0
    for (g, label, Y) in staged.results()[-1]:
        svc = mix.services[g]
        _H, Yref = ref.ffn_swiglu(svc.X.astype(np.float64), svc.Wgate.astype(np.float64), svc.Wup.astype(np.float64), svc.Wdown.astype(np.float64))
        worst = max(worst, rel_err(Y, Yref))
    print("end-to-end max relative error vs fp32 masters (bf16 decode FFN, reduced): %.3e" % worst)
    assert worst < 5e-2


# ---- the five mixes ---------------------------------------------------------------------------------

def test_mix1_mlp_fp32_full():
    check_mix(make_mix(1), "f32")


def test_mix2_small_models_bf16_full():
    check_mix(make_mix(2), "bf16")


def test_mix3_vit_reduced_all_rows():
    check_mix(make_mix(3, images=[2, 1, 1, 3, 1, 2, 1, 1], d=192, ffn=768, tokens=197), "bf16")


def test_mix3_vit_full_size_all_rows():
    check_mix(make_mix(3), "bf16")


def test_mix4_decode_reduced_all_rows():
    check_mix(make_mix(4, d=512, ffn=1376), "bf16")


def test_mix4_decode_fp8_reduced_all_rows():
    # the weight-streaming classes with E4M3 inputs and E4M3 hidden activations (static scale from the oracle)
    check_mix(make_mix(4, d=1024, ffn=2752), "fp8")


def test_mix4_decode_full_size():
    check_mix(make_mix(4), "bf16")


def test_mix4_decode_fp8_full_size():
    check_mix(make_mix(4), "fp8")


@pytest.mark.parametrize("dtype_name", ["bf16", "fp8"])
def test_mix5_prefill_reduced_all_rows(dtype_name):
    check_mix(make_mix(5, d=640, ffn=1664, total_rows=900, len_lo=60, len_hi=300), dtype_name)


@pytest.fixture(scope="module")
def mix5():
    return make_mix(5)


@pytest.mark.parametrize("dtype_name", ["bf16", "fp8"])
def test_mix5_prefill_full_size_all_rows(mix5, dtype_name):
    """Every output element of the 8192-row prefill mix against the fp64 oracle (about a minute of oracle time
    per dtype on the host cores)."""
    check_mix(mix5, dtype_name)
