"""Stages the ViT services of a mix for a whole pre-norm encoder block and runs it through libepara:

    y1 = LN1(x) -> QKV -> attention -> projection -> s2 = x + proj, y2 = LN2(s2) -> FFN up (GELU) -> FFN down
    -> s3 = s2 + ffn, y3 = LN1(s3)            (the sum that enters the next block, normalised for it)

Four grouped forwards, one attention launch and three normalisation launches per pass, every service with its own
weights and image count in each of them.  Used by the parity tests and the benchmark."""
import numpy as np
import torch

from workloads import casts

from . import binding as B
from . import runtime as R

STEPS = ("norm1", "qkv", "attention", "proj", "norm2", "ffn_up", "ffn_down", "norm3")


class VitBlock:
    def __init__(self, mix, params, device="cuda:0", copies=1, n_workgroups=None):
        self.mix, self.params, self.device, self.copies = mix, params, torch.device(device), copies
        self.bits = []                 # per service: the exact bf16 inputs handed to the GPU
        for svc, p in zip(mix.services, params):
            qkv, up, down = svc.layers
            self.bits.append({"X": casts.bf16_bits(svc.X),
                              "W": {n: casts.bf16_bits(L.W) for n, L in (("qkv", qkv), ("proj", p.proj), ("up", up), ("down", down))},
                              "b": {n: L.b for n, L in (("qkv", qkv), ("proj", p.proj), ("up", up), ("down", down))}})
        self.tensors, self.programs, self._keep = [], [], []
        for _ in range(copies):
            self._stage(n_workgroups)
        torch.cuda.synchronize(self.device)

    def _stage(self, n_workgroups):
        dev, bf = self.device, B.EPARA_BF16
        f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev)
        per = []
        for svc, p, hb in zip(self.mix.services, self.params, self.bits):
            M, d = svc.X.shape
            ffn = svc.layers[1].W.shape[1]
            buf = lambda N: torch.zeros((M, N), dtype=torch.bfloat16, device=dev)
            t = {"x": R.device_tensor_from_bits(hb["X"], bf, dev), "y1": buf(d), "qkv": buf(3 * d), "attn": buf(d), "proj": buf(d),
                 "s2": buf(d), "y2": buf(d), "h": buf(ffn), "f": buf(d), "s3": buf(d), "y3": buf(d)}
            t["W"] = {n: R.pack_weights(R.device_tensor_from_bits(w, bf, dev), bf) for n, w in hb["W"].items()}
            t["b"] = {n: f32(b) for n, b in hb["b"].items()}
            t["ln"] = {n: f32(getattr(p, n)) for n in ("gamma1", "beta1", "gamma2", "beta2")}
            per.append(t)
        self.tensors.append(per)
        svcs = list(zip(self.mix.services, self.params, per))

        def forward(layer, src, dst, act):
            args = []
            for svc, p, t in svcs:
                K = t[src].shape[1]
                N = t[dst].shape[1]
                args.append(R.group_args(t[src], t["W"][layer], t[dst], svc.M, K, N, act, bias=t["b"][layer]))
            return R.LaunchPlan(np.array(args, dtype=B.GROUP_ARGS), bf, dev, n_workgroups)

        def norm(x, r, which, s, y):
            return R.NormPlan([{"X": t[x], "R": None if r is None else t[r], "gamma": t["ln"]["gamma" + which], "beta": t["ln"]["beta" + which],
                                "S": None if s is None else t[s], "Y": t[y], "eps": p.eps} for svc, p, t in svcs], dev)

        attn = R.AttnPlan([{"QKV": t["qkv"], "O": t["attn"], "tokens": p.tokens, "heads": p.heads} for svc, p, t in svcs], dev)
        self.programs.append([("norm", norm("x", None, "1", None, "y1")), ("forward", forward("qkv", "y1", "qkv", "none")),
                              ("attention", attn), ("forward", forward("proj", "attn", "proj", "none")),
                              ("norm", norm("x", "proj", "2", "s2", "y2")), ("forward", forward("up", "y2", "h", "gelu_erf")),
                              ("forward", forward("down", "h", "f", "none")), ("norm", norm("s2", "f", "1", "s3", "y3"))])

    def run_step(self, i, copy=0, stream=None):
        kind, plan = self.programs[copy % self.copies][i]
        if kind == "forward":
            R.grouped_forward(plan, B.EPARA_BF16, stream)
        elif kind == "norm":
            R.add_layernorm(plan, stream)
        else:
            R.attention(plan, stream)

    def run(self, copy=0, stream=None):
        """Enqueue one pass (the eight launches of the block) on the current stream."""
        for i in range(len(STEPS)):
            self.run_step(i, copy, stream)

    def flops(self):
        """2 M K N of the four dense layers plus 4 T^2 d_h per image and head for the two products of attention."""
        total = 0
        for svc, p in zip(self.mix.services, self.params):
            d = svc.X.shape[1]
            ffn = svc.layers[1].W.shape[1]
            total += 2 * svc.M * (d * 3 * d + d * d + 2 * d * ffn) + 4 * (svc.M // p.tokens) * p.heads * p.tokens * p.tokens * 64
        return total
