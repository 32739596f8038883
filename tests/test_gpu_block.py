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


def test_attention_vit_b16_service_and_peaked_scores():
    rng = np.random.default_rng(42)
    groups, want = attn_case(rng, [(4, 197, 12), (1, 197, 12)])
    check_attn(groups, want, "vit-b/16")
    # larger projections: scores of +-30 and more, rows dominated by one or two keys (the maximum is taken out first)
    groups, want = attn_case(rng, [(2, 197, 2), (1, 50, 1)], spread=4.0)
    check_attn(groups, want, "peaked")


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
