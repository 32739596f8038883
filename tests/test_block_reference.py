"""Pins of oracle/block.py (layer normalisation, residual, attention) against what the mathematics fixes:
hand-worked rows, closed forms, invariances, brute force with explicit indices, and library routines."""
import math

import numpy as np
import pytest
import torch

from oracle import block as B


# ---- layer normalisation -----------------------------------------------------------------------------

def test_layer_norm_hand_worked_row():
    # x = 1,2,3,4: mean 2.5, biased variance (2.25 + 0.25 + 0.25 + 2.25) / 4 = 1.25, sqrt = 1.118033988...
    y = B.layer_norm([[1.0, 2.0, 3.0, 4.0]], np.ones(4), np.zeros(4), 0.0)
    want = np.array([-1.5, -0.5, 0.5, 1.5]) / math.sqrt(1.25)
    assert np.allclose(y[0], want, rtol=0, atol=1e-15)
    assert abs(y[0][3] - 1.3416407864998738) < 1e-15            # the unbiased variance (5/3) would give 1.1619
    # eps sits under the root, next to the variance: x = -1, 1 has variance 1, eps = 3 -> +-1 / 2
    assert np.array_equal(B.layer_norm([[-1.0, 1.0]], np.ones(2), np.zeros(2), 3.0), [[-0.5, 0.5]])
    # gamma scales and beta shifts per column, after the normalisation
    y = B.layer_norm([[-1.0, 1.0]], [2.0, 10.0], [0.25, -1.0], 3.0)
    assert np.array_equal(y, [[-0.75, 4.0]])


def test_layer_norm_constant_row_gives_beta_and_rows_are_independent():
    rng = np.random.default_rng(1)
    beta, gamma = rng.standard_normal(16), rng.standard_normal(16)
    x = rng.standard_normal((5, 16))
    x[2] = 7.25
    y = B.layer_norm(x, gamma, beta, 1e-6)
    assert np.array_equal(y[2], beta)
    x2 = x.copy()
    x2[0] += 3.0 * rng.standard_normal(16)
    y2 = B.layer_norm(x2, gamma, beta, 1e-6)
    assert np.array_equal(y[1:], y2[1:]) and not np.allclose(y[0], y2[0])


def test_layer_norm_moments_and_affine_invariance():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((7, 48)) * 3.0 + 1.5
    y = B.layer_norm(x, np.ones(48), np.zeros(48), 0.0)
    assert np.allclose(y.mean(axis=1), 0.0, atol=1e-14) and np.allclose((y * y).mean(axis=1), 1.0, atol=1e-13)
    assert np.allclose(B.layer_norm(2.5 * x - 4.0, np.ones(48), np.zeros(48), 0.0), y, atol=1e-12)
    assert np.allclose(B.layer_norm(-x, np.ones(48), np.zeros(48), 0.0), -y, atol=1e-12)
    # with eps the mean square is var / (var + eps)
    eps = 0.5
    var = x.var(axis=1)
    ye = B.layer_norm(x, np.ones(48), np.zeros(48), eps)
    assert np.allclose((ye * ye).mean(axis=1), var / (var + eps), atol=1e-13)


def test_layer_norm_against_library_routine():
    rng = np.random.default_rng(3)
    x, g, b = rng.standard_normal((9, 40)), rng.standard_normal(40), rng.standard_normal(40)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x), (40,), torch.from_numpy(g), torch.from_numpy(b), 1e-6).numpy()
    assert np.allclose(B.layer_norm(x, g, b, 1e-6), want, rtol=0, atol=1e-13)


def test_add_layer_norm_adds_first():
    rng = np.random.default_rng(4)
    x, r = rng.standard_normal((3, 8)), rng.standard_normal((3, 8))
    g, b = rng.standard_normal(8), rng.standard_normal(8)
    s, y = B.add_layer_norm(x, r, g, b, 1e-6)
    assert np.array_equal(s, x + r) and np.array_equal(y, B.layer_norm(x + r, g, b, 1e-6))
    s0, y0 = B.add_layer_norm(x, None, g, b, 1e-6)
    assert np.array_equal(s0, x) and np.array_equal(y0, B.layer_norm(x, g, b, 1e-6))
    # x = -r: the sum is a constant (zero) row, so y = beta
    s1, y1 = B.add_layer_norm(x, -x, g, b, 1e-6)
    assert np.array_equal(y1, np.broadcast_to(b, (3, 8)))


# ---- attention ---------------------------------------------------------------------------------------

def _brute_attention(qkv, tokens, heads):
    """Explicit indices, scalar loops: O[i*T + t, h*dh + c] = sum_u p_tu V[u, c]."""
    M, d3 = len(qkv), len(qkv[0])
    d = d3 // 3
    dh = d // heads
    out = [[0.0] * d for _ in range(M)]
    for i in range(M // tokens):
        for h in range(heads):
            for t in range(tokens):
                q = [qkv[i * tokens + t][h * dh + c] for c in range(dh)]
                scores = []
                for u in range(tokens):
                    k = [qkv[i * tokens + u][d + h * dh + c] for c in range(dh)]
                    scores.append(sum(a * b for a, b in zip(q, k)) / math.sqrt(dh))
                w = [math.exp(s) for s in scores]
                z = sum(w)
                for c in range(dh):
                    out[i * tokens + t][h * dh + c] = sum(w[u] / z * qkv[i * tokens + u][2 * d + h * dh + c] for u in range(tokens))
    return np.array(out)


@pytest.mark.parametrize("tokens,heads,dh,images", [(3, 2, 2, 2), (5, 3, 4, 1), (1, 1, 8, 3), (7, 2, 3, 2)])
def test_attention_against_brute_force(tokens, heads, dh, images):
    rng = np.random.default_rng([5, tokens, heads])
    qkv = rng.standard_normal((images * tokens, 3 * heads * dh))
    assert np.allclose(B.attention(qkv, tokens, heads), _brute_attention(qkv.tolist(), tokens, heads), rtol=0, atol=1e-13)


def test_attention_closed_forms():
    rng = np.random.default_rng(6)
    T, H, dh = 6, 2, 4
    d = H * dh
    qkv = rng.standard_normal((T, 3 * d))
    # all keys equal: every query weighs the values evenly -> the mean of V
    same = qkv.copy()
    same[:, d:2 * d] = same[0, d:2 * d]
    assert np.allclose(B.attention(same, T, H), np.broadcast_to(same[:, 2 * d:].mean(axis=0), (T, d)), atol=1e-14)
    # one token (a single key): the output is its value row
    one = rng.standard_normal((4, 3 * d))
    assert np.allclose(B.attention(one, 1, H), one[:, 2 * d:], atol=1e-15)
    # a key that dominates: q = k_3 * 200 for every query of head 0 -> head 0 returns V[3]
    dom = qkv.copy()
    dom[:, 0:dh] = 0.0
    dom[:, d:d + dh] = 0.0
    dom[3, d:d + dh] = 1.0
    dom[:, 0] = 200.0
    dom[3, d] = 1.0
    out = B.attention(dom, T, H)
    assert np.allclose(out[:, :dh], np.broadcast_to(dom[3, 2 * d:2 * d + dh], (T, dh)), atol=1e-12)
    # a value that is constant per head comes back whatever the weights: pins which columns belong to which head
    const = qkv.copy()
    for h in range(H):
        const[:, 2 * d + h * dh:2 * d + (h + 1) * dh] = 10.0 + h
    out = B.attention(const, T, H)
    assert np.allclose(out[:, :dh], 10.0, atol=1e-13) and np.allclose(out[:, dh:], 11.0, atol=1e-13)


def test_attention_invariances():
    rng = np.random.default_rng(7)
    T, H, dh, images = 9, 3, 4, 2
    d = H * dh
    qkv = rng.standard_normal((images * T, 3 * d))
    base = B.attention(qkv, T, H)
    # keys and values of an image permuted together: outputs unchanged; queries permuted: outputs permuted
    perm = rng.permutation(T)
    p = qkv.copy()
    p[:T, d:] = qkv[:T, d:][perm]
    assert np.allclose(B.attention(p, T, H), base, atol=1e-13)
    p = qkv.copy()
    p[:T] = qkv[:T][perm]
    assert np.allclose(B.attention(p, T, H)[:T], base[:T][perm], atol=1e-13)
    # the same vector added to every key of an image shifts each query's scores by a constant: no change
    p = qkv.copy()
    p[:T, d:2 * d] += rng.standard_normal(d)
    assert np.allclose(B.attention(p, T, H), base, atol=1e-12)
    # images do not see each other; heads do not see each other
    p = qkv.copy()
    p[T:] = rng.standard_normal((T, 3 * d))
    assert np.array_equal(B.attention(p, T, H)[:T], base[:T])
    p = qkv.copy()
    for third in range(3):
        p[:, third * d + dh:third * d + 2 * dh] = rng.standard_normal((images * T, dh))      # head 1 of Q, K and V
    out = B.attention(p, T, H)
    assert np.array_equal(out[:, :dh], base[:, :dh]) and np.array_equal(out[:, 2 * dh:], base[:, 2 * dh:])


def test_attention_against_library_routine():
    rng = np.random.default_rng(8)
    T, H, dh, images = 11, 4, 8, 3
    d = H * dh
    qkv = rng.standard_normal((images * T, 3 * d))
    t = torch.from_numpy(qkv).reshape(images, T, 3, H, dh).permute(2, 0, 3, 1, 4)           # third, image, head, token, c
    want = torch.nn.functional.scaled_dot_product_attention(t[0], t[1], t[2])                # scale 1 / sqrt(d_h) by default
    want = want.permute(0, 2, 1, 3).reshape(images * T, d).numpy()
    assert np.allclose(B.attention(qkv, T, H), want, rtol=0, atol=1e-12)


def test_attention_rejects_shapes_that_do_not_split():
    with pytest.raises(ValueError):
        B.attention(np.zeros((6, 10)), 3, 2)
    with pytest.raises(ValueError):
        B.attention(np.zeros((7, 12)), 3, 2)
    with pytest.raises(ValueError):
        B.attention(np.zeros((6, 18)), 3, 4)
