"""Seeded synthetic service mixes (inputs only; no layer arithmetic lives here).

The paper drives its testbed with production request traces and trained models
(Sec. 5, evaluation set-up); neither is available, so these mixes stand in for
them: co-located services (MT), each with its own weights and a ragged batch of
requests (BS, MF) -- the situation of Sec. 3.1.  Five mixes:

  1  two fp32 MLPs 256-512-512-10, batches of 4 and 16 rows
  2  sixteen small GELU FFN blocks, d in {256,512,1024}, rows ~ Poisson(8) >= 1
  3  eight ViT-B/16 services: QKV projection and GELU FFN, 197 tokens per image
  4  four decode services, 7B-shaped SwiGLU FFN, batches 1/8/32/64
  5  two prefill services, 13B-shaped SwiGLU FFN, prompt lengths U[512,2048], 8192 rows

Recipe: rng = numpy.random.default_rng([seed, mix]); structure first (widths, row
counts, image counts, prompt lengths), then per service in index order each
layer's W then b, then X; all fp32 masters.  "N(0, 1/fan_in)" is a variance,
"N(0, 0.02)" and "N(0, 0.01)" are standard deviations.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

SEED = 603


@dataclass
class Layer:
    W: np.ndarray                 # fp32 master, logical [K, N]
    b: Optional[np.ndarray]       # fp32 [N] or None
    act: str                      # "none" | "relu" | "gelu_erf" | "silu"


@dataclass
class Service:
    X: np.ndarray                 # fp32 master [M, K]
    request_rows: List[int]       # rows each request contributes (sum = M)
    kind: str                     # "mlp" | "ffn" | "vit" | "swiglu"
    layers: List[Layer] = field(default_factory=list)      # mlp / ffn chain; vit: [qkv, up, down]
    Wgate: Optional[np.ndarray] = None                     # swiglu: [d, f]
    Wup: Optional[np.ndarray] = None
    Wdown: Optional[np.ndarray] = None                     # [f, d]

    @property
    def M(self):
        return int(self.X.shape[0])


@dataclass
class BlockParams:
    """What a ViT service needs besides its QKV and FFN layers to run a whole pre-norm encoder block."""
    proj: Layer                   # attention output projection [d, d]
    gamma1: np.ndarray            # fp32 [d]: scale / shift of the normalisation before attention ...
    beta1: np.ndarray
    gamma2: np.ndarray            # ... and of the one before the FFN
    beta2: np.ndarray
    heads: int
    tokens: int                   # rows per image
    eps: float


@dataclass
class Mix:
    index: int
    name: str
    dtype: str                    # arithmetic type of the mix: "f32" | "bf16" (mix 5 also runs "fp8")
    services: List[Service]

    @property
    def requests(self):
        return sum(len(s.request_rows) for s in self.services)

    @property
    def rows(self):
        return sum(s.M for s in self.services)

    def flops(self):
        """2*M*K*N over every GEMM of one pass (real rows and columns only)."""
        total = 0
        for s in self.services:
            if s.kind == "swiglu":
                d, f = s.Wgate.shape
                total += 2 * s.M * d * f * 3
            else:
                for L in s.layers:
                    total += 2 * s.M * L.W.shape[0] * L.W.shape[1]
        return total

    def weight_elems(self):
        total = 0
        for s in self.services:
            if s.kind == "swiglu":
                total += s.Wgate.size + s.Wup.size + s.Wdown.size
            else:
                total += sum(L.W.size for L in s.layers)
        return total


def _normal(rng, shape, std):
    a = rng.standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    return a


def _dense(rng, K, N, act, bias=True):
    W = _normal(rng, (K, N), 1.0 / np.sqrt(K))
    b = _normal(rng, (N,), 0.01) if bias else None
    return Layer(W, b, act)


def make_mix(index, seed=SEED, **shrink):
    """Build mix `index` (1..5).  Keyword overrides give reduced copies for fast tests:

      mix 1: rows=[..]            mix 2: n_services, widths=[..]
      mix 3: d, ffn, tokens, images=[..]
      mix 4: d, ffn, rows=[..]    mix 5: d, ffn, total_rows, len_lo, len_hi
    """
    rng = np.random.default_rng([seed, index])
    if index == 1:
        rows = shrink.get("rows", [4, 16])
        svcs = []
        for M in rows:
            layers = [_dense(rng, 256, 512, "relu"), _dense(rng, 512, 512, "relu"), _dense(rng, 512, 10, "none")]
            X = rng.uniform(-1.0, 1.0, (M, 256)).astype(np.float32)
            svcs.append(Service(X, [1] * M, "mlp", layers))
        return Mix(1, "mlp_fp32", "f32", svcs)
    if index == 2:
        n = shrink.get("n_services", 16)
        widths = shrink.get("widths", [256, 512, 1024])
        d = [int(v) for v in rng.choice(widths, size=n)]
        rows = [int(v) for v in np.maximum(1, rng.poisson(8, size=n))]
        svcs = []
        for g in range(n):
            layers = [_dense(rng, d[g], 4 * d[g], "gelu_erf"), _dense(rng, 4 * d[g], d[g], "none")]
            X = _normal(rng, (rows[g], d[g]), 1.0)
            svcs.append(Service(X, [1] * rows[g], "ffn", layers))
        return Mix(2, "small_models_bf16", "bf16", svcs)
    if index == 3:
        d, ffn, tokens = shrink.get("d", 768), shrink.get("ffn", 3072), shrink.get("tokens", 197)
        n = shrink.get("n_services", 8)
        images = shrink.get("images")
        drawn = [int(v) for v in rng.choice([1, 2, 4, 8, 16, 32], size=n)]
        images = drawn if images is None else images
        svcs = []
        for g in range(n):
            layers = [_dense(rng, d, 3 * d, "none"), _dense(rng, d, ffn, "gelu_erf"), _dense(rng, ffn, d, "none")]
            X = _normal(rng, (images[g] * tokens, d), 1.0)
            svcs.append(Service(X, [tokens] * images[g], "vit", layers))
        return Mix(3, "vit_b16_bf16", "bf16", svcs)
    if index == 4:
        d, ffn = shrink.get("d", 4096), shrink.get("ffn", 11008)
        rows = shrink.get("rows", [1, 8, 32, 64])
        svcs = []
        for M in rows:
            Wg, Wu, Wd = _normal(rng, (d, ffn), 0.02), _normal(rng, (d, ffn), 0.02), _normal(rng, (ffn, d), 0.02)
            X = _normal(rng, (M, d), 1.0)
            svcs.append(Service(X, [1] * M, "swiglu", Wgate=Wg, Wup=Wu, Wdown=Wd))
        return Mix(4, "llm_decode_bf16", "bf16", svcs)
    if index == 5:
        d, ffn = shrink.get("d", 5120), shrink.get("ffn", 13824)
        total = shrink.get("total_rows", 8192)
        lo, hi = shrink.get("len_lo", 512), shrink.get("len_hi", 2048)
        n = shrink.get("n_services", 2)
        lengths, acc = [], 0
        while acc < total:
            L = int(rng.integers(lo, hi + 1))
            L = min(L, total - acc)
            lengths.append(L)
            acc += L
        per = [[lengths[i] for i in range(len(lengths)) if i % n == s] for s in range(n)]
        svcs = []
        for s in range(n):
            Wg, Wu, Wd = _normal(rng, (d, ffn), 0.02), _normal(rng, (d, ffn), 0.02), _normal(rng, (ffn, d), 0.02)
            X = _normal(rng, (sum(per[s]), d), 1.0)
            svcs.append(Service(X, per[s], "swiglu", Wgate=Wg, Wup=Wu, Wdown=Wd))
        return Mix(5, "llm_prefill", "bf16", svcs)
    raise ValueError("mix index must be 1..5")


def make_vit_block(mix, seed=SEED, eps=1e-6):
    """Per service of a ViT mix (index 3, any size): the rest of an encoder block's parameters, from a generator of
    their own (the mix's draws stay what they are): projection W ~ N(0, 1/d) and b ~ N(0, 0.01) like the other layers,
    scales 1 + N(0, 0.1), shifts N(0, 0.1); heads of 64 columns."""
    rng = np.random.default_rng([seed, mix.index, 1])
    out = []
    for svc in mix.services:
        d = svc.X.shape[1]
        proj = _dense(rng, d, d, "none")
        g1, b1 = (1.0 + _normal(rng, (d,), 0.1)).astype(np.float32), _normal(rng, (d,), 0.1)
        g2, b2 = (1.0 + _normal(rng, (d,), 0.1)).astype(np.float32), _normal(rng, (d,), 0.1)
        out.append(BlockParams(proj, g1, b1, g2, b2, d // 64, svc.request_rows[0], eps))
    return out
