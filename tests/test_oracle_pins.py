"""Pins for the CPU oracle: each check ties it to something other than itself --
hand-worked tiny cases, closed forms, invariants of the definition, a library
routine in the special case where one exists, and the number formats' published
definitions (PyTorch's CPU casts as the independent implementation)."""
import math

import numpy as np
import pytest
import torch

from oracle import reference as ref


# ---- matmul core ------------------------------------------------------------

def test_one_by_one_by_one():
    Y = ref.dense_forward([[3.0]], [[-2.0]], [0.5], "none")
    assert Y.shape == (1, 1) and Y[0, 0] == -5.5


def test_hand_worked_2x3x2():
    # X (2x3), W (3x2): worked by hand.
    X = [[1, 2, 3], [-1, 0, 2]]
    W = [[1, -1], [0, 2], [2, 1]]
    b = [10, -20]
    # row0: [1+0+6, -1+4+3] = [7, 6];  row1: [-1+0+4, 1+0+2] = [3, 3]
    assert ref.dense_forward(X, W, None, "none").tolist() == [[7.0, 6.0], [3.0, 3.0]]
    assert ref.dense_forward(X, W, b, "none").tolist() == [[17.0, -14.0], [13.0, -17.0]]
    assert ref.dense_forward(X, W, b, "relu").tolist() == [[17.0, 0.0], [13.0, 0.0]]
    # scale applies to the product only, not to the bias
    assert ref.dense_forward(X, W, b, "none", s=0.5).tolist() == [[13.5, -17.0], [11.5, -18.5]]


def test_non_square_catches_transposed_operands():
    # K != N and M != K: a transposed W or X cannot give the right shape AND values.
    X = np.arange(8.0).reshape(2, 4)
    W = np.arange(12.0).reshape(4, 3) - 5.0
    expect = [[sum(X[i, k] * W[k, j] for k in range(4)) for j in range(3)] for i in range(2)]
    assert ref.dense_forward(X, W).tolist() == expect


def test_identity_zero_and_ones_weights():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((5, 7))
    b = rng.standard_normal(7)
    assert np.array_equal(ref.dense_forward(X, np.eye(7), b, "none"), X + b)
    assert np.array_equal(ref.dense_forward(X, np.eye(7), b, "relu"), np.maximum(X + b, 0))
    Y0 = ref.dense_forward(X, np.zeros((7, 3)), b[:3], "none")
    assert np.array_equal(Y0, np.broadcast_to(b[:3], (5, 3)))
    Y1 = ref.dense_forward(X, np.ones((7, 4)))
    rows = np.array([math.fsum(r) for r in X])
    assert np.allclose(Y1, rows[:, None], rtol=1e-14, atol=1e-14)


def test_linearity_in_x():
    rng = np.random.default_rng(2)
    X1, X2 = rng.standard_normal((6, 33)), rng.standard_normal((6, 33))
    W, b = rng.standard_normal((33, 9)), rng.standard_normal(9)
    a, c = 1.75, -0.375
    f = lambda X: ref.dense_forward(X, W)
    assert np.allclose(f(a * X1 + c * X2), a * f(X1) + c * f(X2), rtol=1e-12, atol=1e-12)
    fb = lambda X: ref.dense_forward(X, W, b) - ref.dense_forward(np.zeros_like(X), W, b)
    assert np.allclose(fb(a * X1 + c * X2), a * fb(X1) + c * fb(X2), rtol=1e-12, atol=1e-12)


def test_rows_and_groups_are_independent():
    rng = np.random.default_rng(3)
    X, W, b = rng.standard_normal((9, 20)), rng.standard_normal((20, 11)), rng.standard_normal(11)
    Y = ref.dense_forward(X, W, b, "gelu_erf")
    perm = rng.permutation(9)
    assert np.array_equal(ref.dense_forward(X[perm], W, b, "gelu_erf"), Y[perm])
    top, bottom = ref.dense_forward(X[:4], W, b, "gelu_erf"), ref.dense_forward(X[4:], W, b, "gelu_erf")
    assert np.array_equal(np.vstack([top, bottom]), Y)
    # column subsets: an output column depends on its own weight column only
    cols = [7, 2, 9]
    assert np.array_equal(ref.dense_forward(X, W[:, cols], b[cols], "gelu_erf"), Y[:, cols])


@pytest.mark.parametrize("shape", [(4, 256, 512), (16, 512, 10), (13, 100, 37), (1, 1, 5), (3, 64, 1)])
def test_against_blas_matmul(shape):
    M, K, N = shape
    rng = np.random.default_rng(4)
    X, W, b = rng.uniform(-1, 1, (M, K)), rng.standard_normal((K, N)) / np.sqrt(K), rng.standard_normal(N) * 0.01
    Y = ref.dense_forward(X, W, b, "none", s=0.7)
    assert np.allclose(Y, 0.7 * (X @ W) + b, rtol=1e-12, atol=1e-13)


def test_empty_group():
    Y = ref.dense_forward(np.zeros((0, 8)), np.ones((8, 3)), np.ones(3), "relu")
    assert Y.shape == (0, 3)


# ---- activations --------------------------------------------------------------

def test_activation_closed_forms():
    a = lambda z, n: float(ref.act([z], n)[0])
    assert a(-1.0, "relu") == 0.0 and a(2.5, "relu") == 2.5 and a(0.0, "relu") == 0.0
    assert a(0.0, "silu") == 0.0
    assert abs(a(1.0, "silu") - 0.7310585786300049) < 1e-15        # 1/(1+e^-1)
    assert abs(a(-1.0, "silu") + 0.2689414213699951) < 1e-15       # -1/(1+e)
    assert a(0.0, "gelu_erf") == 0.0
    assert abs(a(1.0, "gelu_erf") - 0.8413447460685429) < 1e-15    # Phi(1)
    assert abs(a(-1.0, "gelu_erf") + 0.15865525393145707) < 1e-15  # -Phi(-1)
    assert abs(a(2.0, "gelu_erf") - 2 * 0.9772498680518208) < 1e-15
    for n in ("silu", "gelu_erf", "gelu_tanh"):
        assert abs(a(40.0, n) - 40.0) < 1e-12 and abs(a(-40.0, n)) < 1e-12
    assert a(-3.25, "none") == -3.25


def test_activations_against_torch_float64():
    z = torch.linspace(-8, 8, 4001, dtype=torch.float64)
    F = torch.nn.functional
    assert np.allclose(ref.act(z.numpy(), "silu"), F.silu(z).numpy(), rtol=1e-13, atol=1e-15)
    assert np.allclose(ref.act(z.numpy(), "gelu_erf"), F.gelu(z).numpy(), rtol=1e-13, atol=1e-15)
    assert np.allclose(ref.act(z.numpy(), "gelu_tanh"), F.gelu(z, approximate="tanh").numpy(), rtol=1e-13, atol=1e-15)
    assert np.array_equal(ref.act(z.numpy(), "relu"), F.relu(z).numpy())


def test_gelu_variants_differ_but_only_slightly():
    z = np.linspace(-6, 6, 2001)
    d = np.abs(ref.act(z, "gelu_erf") - ref.act(z, "gelu_tanh"))
    assert 1e-5 < d.max() < 1e-3


# ---- SwiGLU FFN ---------------------------------------------------------------

def test_swiglu_hidden_matches_its_definition():
    rng = np.random.default_rng(5)
    X, Wg, Wu = rng.standard_normal((5, 24)), rng.standard_normal((24, 10)), rng.standard_normal((24, 10))
    H = ref.swiglu_hidden(X, Wg, Wu, 0.5, 2.0)
    g, u = torch.from_numpy(0.5 * (X @ Wg)), torch.from_numpy(2.0 * (X @ Wu))
    assert np.allclose(H, (torch.nn.functional.silu(g) * u).numpy(), rtol=1e-12, atol=1e-13)
    # gate and up are not interchangeable
    assert not np.allclose(H, ref.swiglu_hidden(X, Wu, Wg, 0.5, 2.0))


def test_swiglu_hand_worked():
    # one row, d=2, f=2: gate sums [0, 1], up sums [3, -2]; SiLU(0)=0, SiLU(1)=1/(1+e^-1)
    X = [[1.0, 1.0]]
    Wg = [[0.0, 0.5], [0.0, 0.5]]
    Wu = [[1.0, -1.0], [2.0, -1.0]]
    Wd = [[1.0, 0.0, 2.0], [1.0, 1.0, 0.0]]
    H, Y = ref.ffn_swiglu(X, Wg, Wu, Wd)
    h1 = -2.0 / (1.0 + math.exp(-1.0))
    assert H.tolist() == [[0.0, h1]]
    assert Y.tolist() == [[h1, h1, 0.0]]


def test_ffn_swiglu_composes_and_requantises():
    rng = np.random.default_rng(6)
    X = rng.standard_normal((4, 16))
    Wg, Wu, Wd = (rng.standard_normal(s) * 0.3 for s in ((16, 12), (16, 12), (12, 16)))
    H, Y = ref.ffn_swiglu(X, Wg, Wu, Wd)
    assert np.allclose(Y, H @ Wd, rtol=1e-12, atol=1e-13)
    s_h = np.abs(H).max() / 448.0
    Hq, Yq = ref.ffn_swiglu(X, Wg, Wu, Wd, s_down=s_h, h_scale=s_h)
    codes = ref.e4m3_encode(H, s_h)
    assert np.array_equal(Hq, ref.e4m3_decode(codes, s_h))
    assert np.allclose(Yq, Hq @ Wd, rtol=1e-12, atol=1e-13)
    assert np.max(np.abs(Hq - H)) <= s_h * 16.0 + 1e-12        # half a step of the top binade


def test_mlp_chain_is_layer_by_layer():
    rng = np.random.default_rng(7)
    X = rng.uniform(-1, 1, (3, 8))
    layers = [(rng.standard_normal((8, 6)), rng.standard_normal(6), "relu"),
              (rng.standard_normal((6, 6)), rng.standard_normal(6), "relu"),
              (rng.standard_normal((6, 2)), rng.standard_normal(2), "none")]
    outs = ref.mlp_chain(X, layers)
    h = X
    for (W, b, a), o in zip(layers, outs):
        h = h @ W + b
        if a == "relu":
            h = np.maximum(h, 0)
        assert np.allclose(o, h, rtol=1e-12, atol=1e-13)


# ---- number formats -----------------------------------------------------------

def test_e4m3_all_codes():
    codes = np.arange(256, dtype=np.uint8)
    v = ref.e4m3_decode(codes)
    assert np.isnan(v[0x7f]) and np.isnan(v[0xff]) and np.isnan(v).sum() == 2
    pos = v[:0x7f]
    assert np.all(np.diff(pos) > 0) and pos[0] == 0.0                  # monotone per sign
    assert pos[-1] == 448.0 and pos[1] == 2.0 ** -9 and pos[8] == 2.0 ** -6
    assert np.array_equal(v[0x80:0xff], -pos)
    # against PyTorch's table
    t = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ok = ~np.isnan(v)
    assert np.array_equal(v[ok], t[ok]) and np.all(np.isnan(t[~ok]))
    # round trip
    back = ref.e4m3_encode(v[ok])
    expect = codes[ok].copy()
    assert np.array_equal(back, expect)


def test_e4m3_rounding_ties_and_saturation():
    pos = ref.e4m3_decode(np.arange(0x7f, dtype=np.uint8))
    mid = (pos[:-1] + pos[1:]) / 2
    enc = ref.e4m3_encode(mid)
    lo = np.arange(0x7e, dtype=np.uint8)
    expect = np.where(lo % 2 == 0, lo, lo + 1)                        # ties go to the even code
    assert np.array_equal(enc, expect)
    assert np.array_equal(ref.e4m3_encode(np.nextafter(mid, np.inf)), lo + 1)
    assert np.array_equal(ref.e4m3_encode(np.nextafter(mid, -np.inf)), lo)
    assert ref.e4m3_encode([448.0, 449.0, 463.9, 464.0, 1e9, np.inf]).tolist() == [0x7e] * 6
    assert ref.e4m3_encode([-500.0, -np.inf]).tolist() == [0xfe] * 2
    assert ref.e4m3_encode([0.0, -0.0, 2.0 ** -11]).tolist() == [0x00, 0x80, 0x00]
    assert ref.e4m3_encode([10.0], scale=0.5).tolist() == ref.e4m3_encode([20.0]).tolist()


def test_e4m3_encode_against_torch_cast():
    rng = np.random.default_rng(8)
    x = np.concatenate([rng.standard_normal(20000) * 100, rng.standard_normal(20000),
                        rng.standard_normal(20000) * 0.01, np.linspace(-448, 448, 7001)])
    x = x[np.abs(x) <= 448].astype(np.float32).astype(np.float64)
    t = torch.from_numpy(x).to(torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = ref.e4m3_encode(x)
    assert np.array_equal(mine & 0x7f, t & 0x7f)                      # magnitudes (sign of zero aside)
    nz = (mine & 0x7f) != 0
    assert np.array_equal(mine[nz], t[nz])


def test_bf16_codec_against_torch():
    # every bf16 pattern decodes like torch; boundary patterns of fp32 round like torch
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    v = ref.bf16_decode(bits)
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    fin = np.isfinite(t)
    assert np.array_equal(v[fin], t[fin]) and np.array_equal(np.isnan(v), np.isnan(t))
    hi = np.arange(65536, dtype=np.uint32) << 16
    for low in (0x0000, 0x0001, 0x7fff, 0x8000, 0x8001, 0xffff):
        f = (hi | low).astype(np.uint32).view(np.float32)
        keep = np.isfinite(f)
        mine = ref.bf16_encode(f[keep])
        theirs = torch.from_numpy(f[keep].copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(mine, theirs), hex(low)


def test_small_integer_products_are_exact_in_every_storage_type():
    # integers small enough to be exact in bf16 and E4M3 and in their fp32 sums
    rng = np.random.default_rng(9)
    X = rng.integers(-4, 5, (6, 32)).astype(np.float64)
    W = rng.integers(-3, 4, (32, 5)).astype(np.float64)
    Y = ref.dense_forward(X, W)
    assert np.array_equal(Y, (X.astype(np.int64) @ W.astype(np.int64)).astype(np.float64))
    assert np.array_equal(ref.bf16_decode(ref.bf16_encode(X)), X)
    assert np.array_equal(ref.e4m3_decode(ref.e4m3_encode(X)), X)
