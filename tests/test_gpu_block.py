"""GPU parity of the pieces between a ViT block's dense layers (residual + layer normalisation, attention), through
the C ABI, against oracle/block.py on the same bf16 inputs.

Tolerances.  Layer normalisation: the arithmetic is fp32 on exact bf16 inputs (errors ~ 1e-6), so what is left is
the rounding of the outputs to bf16: half a unit in the last place = 2^-9 of the value; the test allows 2^-8 of
max(|y|, rms).  Attention: both products are bf16 operands with fp32 sums on the matrix cores, the case for which the
forward path's tolerance of 2e-2 of max(|o|, rms) is stated (P is rounded to bf16 before the second product, the
output again; measured: at most 9e-3 over a ViT-B/16 service)."""
import numpy as np
import pytest
import torch

from oracle import block as OB
from oracle import reference as ref
from paper_2511_00603_amd import runtime as R
from workloads import casts

from parity_util import TOL, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_NORM, TOL_ATTN = 2.0 ** -8, TOL["bf16"]


def dev_bf16(a):
    """fp32 master -> (exact values of its bf16 rounding as fp64, device bf16 tensor)."""
    bits = casts.bf16_bits(np.ascontiguousarray(a, dtype=np.float32))
    return ref.bf16_decode(bits), R.device_tensor_from_bits(bits, 1, DEV)


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def fetch(t):
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


def norm_case(rng, shapes, with_r=True, with_s=True, eps=1e-6):
    groups, want = [], []
    for M, d in shapes:
        x, X = dev_bf16(rng.standard_normal((M, d)) * 2.0 + 0.5)
        r, Rt = dev_bf16(rng.standard_normal((M, d))) if with_r else (None, None)
        gamma = (1.0 + 0.2 * rng.standard_normal(d)).astype(np.float32)
        beta = (0.3 * rng.standard_normal(d)).astype(np.float32)
        S = torch.full((M, d), 7.0, dtype=torch.bfloat16, device=DEV) if with_s else None
        Y = torch.full((M, d), 7.0, dtype=torch.bfloat16, device=DEV)
        groups.append({"X": X, "R": Rt, "gamma": dev_f32(gamma), "beta": dev_f32(beta), "S": S, "Y": Y, "eps": eps})
        want.append(OB.add_layer_norm(x, r, gamma.astype(np.float64), beta.astype(np.float64), float(np.float32(eps))))
    return groups, want


def check_norm(groups, want, what):
    plan = R.NormPlan(groups, DEV)
    R.add_layernorm(plan)
    torch.cuda.synchronize()
    for i, (g, (s, y)) in enumerate(zip(groups, want)):
        if y.size == 0:
            continue
        assert_close(fetch(g["Y"]), y, TOL_NORM, "%s group %d Y" % (what, i))
        if g["S"] is not None:
            assert_close(fetch(g["S"]), s, TOL_NORM, "%s group %d S" % (what, i))


@pytest.mark.parametrize("with_r,with_s", [(True, True), (True, False), (False, True), (False, False)])
def test_add_layernorm_mixed_groups(with_r, with_s):
    """Groups of different widths (one, two and sixteen chunks per lane; widths that leave lanes idle) and row counts
    (none, one, a count that is no multiple of the rows per workgroup) in one launch."""
    rng = np.random.default_rng([31, with_r, with_s])
    shapes = [(197, 768), (0, 64), (1, 8), (5, 520), (33, 1024), (3, 8192), (0, 768), (66, 64)]
    groups, want = norm_case(rng, shapes, with_r, with_s)
    check_norm(groups, want, "mixed")


def test_add_layernorm_vit_sizes_and_exact_sums():
    rng = np.random.default_rng(32)
    groups, want = norm_case(rng, [(197 * 8, 768), (197, 768), (197 * 3, 768)])
    check_norm(groups, want, "vit")
    # small integers: x + r is exact in bf16, so S must hold it bit for bit
    M, d = 37, 768
    xi, ri = rng.integers(-60, 60, (M, d)).astype(np.float32), rng.integers(-60, 60, (M, d)).astype(np.float32)
    _, X = dev_bf16(xi)
    _, Rt = dev_bf16(ri)
    S = torch.zeros((M, d), dtype=torch.bfloat16, device=DEV)
    Y = torch.zeros((M, d), dtype=torch.bfloat16, device=DEV)
    g = {"X": X, "R": Rt, "gamma": dev_f32(np.ones(d)), "beta": dev_f32(np.zeros(d)), "S": S, "Y": Y, "eps": 0.0}
    R.add_layernorm(R.NormPlan([g], DEV))
    torch.cuda.synchronize()
    assert np.array_equal(fetch(S), (xi + ri).astype(np.float64))
    y = fetch(Y)
    assert np.abs(y.mean(axis=1)).max() < 2e-3 and np.abs((y * y).mean(axis=1) - 1.0).max() < 1e-2


def test_add_layernorm_in_place_and_constant_rows():
    """S written over X and Y over R (a wave has read its row before it stores); a constant row gives beta."""
    rng = np.random.default_rng(33)
    M, d = 50, 768
    x, X = dev_bf16(rng.standard_normal((M, d)))
    r, Rt = dev_bf16(rng.standard_normal((M, d)))
    gamma, beta = (1.0 + 0.2 * rng.standard_normal(d)).astype(np.float32), (0.3 * rng.standard_normal(d)).astype(np.float32)
    s, y = OB.add_layer_norm(x, r, gamma.astype(np.float64), beta.astype(np.float64), float(np.float32(1e-6)))
    g = {"X": X, "R": Rt, "gamma": dev_f32(gamma), "beta": dev_f32(beta), "S": X, "Y": Rt, "eps": 1e-6}
    R.add_layernorm(R.NormPlan([g], DEV))
    torch.cuda.synchronize()
    assert_close(fetch(X), s, TOL_NORM, "in place S")
    assert_close(fetch(Rt), y, TOL_NORM, "in place Y")
    c, C = dev_bf16(np.full((4, d), 3.25, dtype=np.float32))
    Y = torch.zeros((4, d), dtype=torch.bfloat16, device=DEV)
    R.add_layernorm(R.NormPlan([{"X": C, "gamma": dev_f32(gamma), "beta": dev_f32(beta), "Y": Y, "eps": 1e-6}], DEV))
    torch.cuda.synchronize()
    assert np.array_equal(fetch(Y), np.broadcast_to(ref.bf16_decode(casts.bf16_bits(beta)), (4, d)))


def attn_case(rng, specs, spread=1.0):
    groups, want = [], []
    for images, tokens, heads in specs:
        d = heads * 64
        qkv, Q = dev_bf16(rng.standard_normal((images * tokens, 3 * d)) * spread)
        O = torch.full((images * tokens, d), 7.0, dtype=torch.bfloat16, device=DEV)
        groups.append({"QKV": Q, "O": O, "tokens": tokens, "heads": heads})
        want.append(OB.attention(qkv, tokens, heads) if images else np.zeros((0, d)))
    return groups, want


def check_attn(groups, want, what):
    R.attention(R.AttnPlan(groups, DEV))
    torch.cuda.synchronize()
    for i, (g, o) in enumerate(zip(groups, want)):
        if o.size:
            assert_close(fetch(g["O"]), o, TOL_ATTN, "%s group %d" % (what, i))


def test_attention_token_counts_around_the_block_edges():
    """One key, a partial block, exactly one and two blocks, an odd and an even number of blocks, the ViT count and
    the largest supported one; several images and heads; an empty service in between."""
    rng = np.random.default_rng(41)
    specs = [(2, 1, 1), (1, 5, 2), (3, 16, 1), (1, 17, 3), (2, 32, 2), (0, 197, 12), (1, 33, 1), (2, 197, 3), (1, 208, 1), (1, 224, 2)]
    groups, want = attn_case(rng, specs)
    check_attn(groups, want, "edges")


def test_attention_many_services():
    """More than 64 groups in a launch (the kernel then finds an item's group by bisection), some of them empty."""
    rng = np.random.default_rng(44)
    specs = [((i % 3), 3 + (i % 5), 1 + (i % 2)) for i in range(70)]
    groups, want = attn_case(rng, specs)
    check_attn(groups, want, "seventy services")


def test_attention_vit_b16_service_and_peaked_scores():
    rng = np.random.default_rng(42)
    groups, want = attn_case(rng, [(4, 197, 12), (1, 197, 12)])
    check_attn(groups, want, "vit-b/16")
    # larger projections: scores of +-30 and more, rows dominated by one or two keys (the maximum is taken out first)
    groups, want = attn_case(rng, [(2, 197, 2), (1, 50, 1)], spread=4.0)
    check_attn(groups, want, "peaked")
    # launches whose longest image needs 8, 4 and 2 key blocks (the kernel is compiled per number of blocks)
    for tokens in (100, 128, 65, 64, 33, 20):
        groups, want = attn_case(rng, [(2, tokens, 2), (1, max(1, tokens // 3), 1)])
        check_attn(groups, want, "%d tokens" % tokens)


def test_attention_closed_forms_on_the_gpu():
    """Equal keys -> every output row is the mean of the values; a value constant per head comes back exactly."""
    rng = np.random.default_rng(43)
    T, H = 197, 3
    d = H * 64
    a = rng.standard_normal((T, 3 * d)).astype(np.float32)
    a[:, d:2 * d] = a[0, d:2 * d]
    vals, Q = dev_bf16(a)
    O = torch.zeros((T, d), dtype=torch.bfloat16, device=DEV)
    R.attention(R.AttnPlan([{"QKV": Q, "O": O, "tokens": T, "heads": H}], DEV))
    torch.cuda.synchronize()
    assert_close(fetch(O), np.broadcast_to(vals[:, 2 * d:].mean(axis=0), (T, d)), TOL_ATTN, "equal keys")
    b = rng.standard_normal((T, 3 * d)).astype(np.float32)
    for h in range(H):
        b[:, 2 * d + 64 * h:2 * d + 64 * (h + 1)] = 2.0 + h
    _, Q = dev_bf16(b)
    R.attention(R.AttnPlan([{"QKV": Q, "O": O, "tokens": T, "heads": H}], DEV))
    torch.cuda.synchronize()
    out = fetch(O)
    for h in range(H):
        assert np.abs(out[:, 64 * h:64 * (h + 1)] - (2.0 + h)).max() <= (2.0 + h) * 2.0 ** -7     # sum of weights / row sum, rounded


# ---- a whole encoder block: the dense layers of the grouped forward with the pieces above between them ----

def _oracle_block(x, w, b, p):
    """Pre-norm encoder block (Dosovitskiy et al. 2021) in fp64 on the bf16 values of inputs and weights, never rounding
    in between."""
    g = lambda a: a.astype(np.float64)
    eps = float(np.float32(p.eps))
    y1 = OB.layer_norm(x, g(p.gamma1), g(p.beta1), eps)
    a = OB.attention(ref.dense_forward(y1, w["qkv"], b["qkv"], "none"), p.tokens, p.heads)
    s2, y2 = OB.add_layer_norm(x, ref.dense_forward(a, w["proj"], b["proj"], "none"), g(p.gamma2), g(p.beta2), eps)
    f = ref.dense_forward(ref.dense_forward(y2, w["up"], b["up"], "gelu_erf"), w["down"], b["down"], "none")
    return s2 + f


@pytest.mark.parametrize("shrink", [dict(d=128, ffn=512, tokens=50, images=[2, 1, 3], n_services=3),
                                    dict(images=[2, 1], n_services=2)])
def test_vit_encoder_block_end_to_end(shrink):
    """x -> LN -> QKV -> attention -> projection -> (+ x) -> LN -> FFN (GELU) -> (+) -> LN: every service of the launch
    with its own weights and image count; four grouped forwards, one attention and three normalisation launches
    (a small block and ViT-B/16 itself)."""
    from paper_2511_00603_amd.vitblock import VitBlock
    from workloads import make_mix, make_vit_block
    mix = make_mix(3, **shrink)
    params = make_vit_block(mix)
    blk = VitBlock(mix, params, DEV)
    blk.run()
    torch.cuda.synchronize()
    worst = 0.0
    for i, (p, hb, t) in enumerate(zip(params, blk.bits, blk.tensors[0])):
        x = ref.bf16_decode(hb["X"])
        w = {n: ref.bf16_decode(v) for n, v in hb["W"].items()}
        b = {n: v.astype(np.float64) for n, v in hb["b"].items()}
        g64 = lambda a: a.astype(np.float64)
        eps = float(np.float32(p.eps))
        got = {n: fetch(t[n]) for n in ("y1", "qkv", "attn", "proj", "s2", "y2", "h", "f", "s3", "y3")}
        # stage by stage, each against the reference on the very (bf16) tensors the stage read on the GPU: this isolates
        # the stage's own error from what the roundings before it did to its input
        assert_close(got["y1"], OB.layer_norm(x, g64(p.gamma1), g64(p.beta1), eps), TOL_NORM, "service %d first normalisation" % i)
        assert_close(got["qkv"], ref.dense_forward(got["y1"], w["qkv"], b["qkv"], "none"), TOL["bf16"], "service %d QKV" % i)
        assert_close(got["attn"], OB.attention(got["qkv"], p.tokens, p.heads), TOL_ATTN, "service %d attention" % i)
        assert_close(got["proj"], ref.dense_forward(got["attn"], w["proj"], b["proj"], "none"), TOL["bf16"], "service %d projection" % i)
        want_s2, want_y2 = OB.add_layer_norm(x, got["proj"], g64(p.gamma2), g64(p.beta2), eps)
        assert_close(got["s2"], want_s2, TOL_NORM, "service %d sum after attention" % i)
        assert_close(got["y2"], want_y2, TOL_NORM, "service %d second normalisation" % i)
        assert_close(got["h"], ref.dense_forward(got["y2"], w["up"], b["up"], "gelu_erf"), TOL["bf16"], "service %d FFN up" % i)
        assert_close(got["f"], ref.dense_forward(got["h"], w["down"], b["down"], "none"), TOL["bf16"], "service %d FFN down" % i)
        want_s3, want_y3 = OB.add_layer_norm(got["s2"], got["f"], g64(p.gamma1), g64(p.beta1), eps)
        assert_close(got["s3"], want_s3, TOL_NORM, "service %d block output" % i)
        assert_close(got["y3"], want_y3, TOL_NORM, "service %d block output, normalised" % i)
        # and the whole block against the reference that never rounds in between: nine tensors are rounded to bf16 on
        # the way (2^-9 each, and a score error e changes an attention weight by a factor exp(e)), so twice the
        # single-stage bound
        worst = max(worst, assert_close(got["s3"], _oracle_block(x, w, b, p), 2 * TOL["bf16"], "service %d whole block" % i))
    print("whole block, worst relative error over the services: %.2e" % worst)


def test_block_pieces_in_a_hip_graph():
    """Both calls only enqueue a kernel on the caller's stream, so they can be captured; every replay, with eager work
    and synchronisations in between, must reproduce the eager result bit for bit and follow its inputs."""
    rng = np.random.default_rng(61)
    T, H = 197, 3
    d = H * 64
    _, X = dev_bf16(rng.standard_normal((2 * T, d)))
    _, Rt = dev_bf16(rng.standard_normal((2 * T, d)))
    _, Q = dev_bf16(rng.standard_normal((2 * T, 3 * d)))
    norm = {"X": X, "R": Rt, "gamma": dev_f32(1.0 + 0.1 * rng.standard_normal(d)), "beta": dev_f32(0.1 * rng.standard_normal(d)),
            "S": torch.zeros((2 * T, d), dtype=torch.bfloat16, device=DEV), "Y": torch.zeros((2 * T, d), dtype=torch.bfloat16, device=DEV), "eps": 1e-6}
    attn = {"QKV": Q, "O": torch.zeros((2 * T, d), dtype=torch.bfloat16, device=DEV), "tokens": T, "heads": H}
    np_, ap = R.NormPlan([norm], DEV), R.AttnPlan([attn], DEV)
    outs = (norm["S"], norm["Y"], attn["O"])

    def run():
        R.add_layernorm(np_)
        R.attention(ap)

    def raw():
        return [t.cpu().view(torch.uint8).numpy().copy() for t in outs]

    run()
    torch.cuda.synchronize()
    want = raw()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()
    for factor in (2.0, 0.5, -1.0):
        for t in outs:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, raw()):
            assert np.array_equal(a, b)
        X.mul_(factor)
        Q.mul_(factor)
        run()
        torch.cuda.synchronize()
        want = raw()
