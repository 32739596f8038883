"""Reference for the pieces of a vision-transformer encoder block that sit between the dense layers
(test infrastructure only; fp64 throughout).

The ViT services of the paper's setting (co-located models, Sec. 3.1 MT; the ViT-B/16 mix) run, per
block, QKV projection -> attention -> output projection -> FFN.  The projections and the FFN are the
grouped dense forward; what lies between them is written out here by its textbook definition:

  layer normalisation (Ba, Kiros, Hinton 2016), per row x of d values:
      mu = mean(x),  var = mean((x - mu)^2)  (the biased variance),
      y = (x - mu) / sqrt(var + eps) * gamma + beta
  residual connection: s = x + r, normalised afterwards (pre-norm block, Dosovitskiy et al. 2021)
  scaled dot-product attention (Vaswani et al. 2017), per image and head h, with Q, K, V the
  head's d_h columns of the three thirds [Q | K | V] of the projection's output rows:
      S = Q K^T / sqrt(d_h),  P = softmax over the keys of every query row,  O = P V
  and the heads' outputs side by side.

No blocking and no running maxima: the score matrix of a head is formed whole.
"""
import numpy as np


def layer_norm(x, gamma, beta, eps):
    """Rows of x [M, d] normalised to zero mean and unit (biased) variance, then scaled and shifted."""
    x = np.asarray(x, dtype=np.float64)
    mu = x.mean(axis=1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, np.float64) + np.asarray(beta, np.float64)


def add_layer_norm(x, r, gamma, beta, eps):
    """(s, y): s = x + r (r may be None: s = x), y = layer_norm(s)."""
    s = np.asarray(x, dtype=np.float64) if r is None else np.asarray(x, np.float64) + np.asarray(r, np.float64)
    return s, layer_norm(s, gamma, beta, eps)


def softmax_rows(s):
    """exp(s_ij) / sum_j exp(s_ij); the row maximum is taken out first, which changes nothing but the range."""
    e = np.exp(s - s.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def attention(qkv, tokens, heads):
    """qkv [images * tokens, 3 * d] = [Q | K | V] -> O [images * tokens, d]; d = heads * d_h."""
    qkv = np.asarray(qkv, dtype=np.float64)
    M, d3 = qkv.shape
    if d3 % 3 or (d3 // 3) % heads or M % tokens:
        raise ValueError("shape does not split into images, thirds and heads")
    d = d3 // 3
    dh = d // heads
    out = np.zeros((M, d))
    for i in range(M // tokens):
        rows = slice(i * tokens, (i + 1) * tokens)
        for h in range(heads):
            cols = slice(h * dh, (h + 1) * dh)
            Q, K, V = qkv[rows, 0 * d:1 * d][:, cols], qkv[rows, 1 * d:2 * d][:, cols], qkv[rows, 2 * d:3 * d][:, cols]
            P = softmax_rows(Q @ K.T / np.sqrt(dh))
            out[rows, cols] = P @ V
    return out
