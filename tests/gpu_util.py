"""Helpers of the GPU parity tests: stage ad-hoc groups, run them through the C-ABI, fetch outputs."""
import numpy as np
import torch

from oracle import reference as ref
from paper_2511_00603_amd import binding as B
from paper_2511_00603_amd import runtime as R
from workloads import casts

DEV = "cuda:0"


def to_bits(a, dtype_name, scale=1.0):
    if dtype_name == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype_name == "bf16":
        return casts.bf16_bits(a)
    return casts.e4m3_codes(a, scale)


def values(bits, dtype_name, scale=1.0):
    """The exact values the bits stand for, by the oracle's own decoders."""
    if dtype_name == "f32":
        return np.asarray(bits, dtype=np.float64)
    if dtype_name == "bf16":
        return ref.bf16_decode(bits)
    return ref.e4m3_decode(bits, scale)


def fetch(t):
    if t.dtype == torch.uint8:
        return t.view(torch.float8_e4m3fn).to(torch.float32).cpu().numpy().astype(np.float64)
    return t.to(torch.float32).cpu().numpy().astype(np.float64)


class Groups:
    """A list of plain groups {X, W, b, act} (fp32 masters) staged for one grouped_forward launch."""

    def __init__(self, specs, dtype_name, n_workgroups=None, out_dtype_name=None):
        self.dtype_name = dtype_name
        dt = B.DTYPE_BY_NAME[dtype_name]
        self.out_dtype = B.DTYPE_BY_NAME[out_dtype_name] if out_dtype_name else (B.EPARA_F32 if dt == B.EPARA_F32 else B.EPARA_BF16)
        self.bits, self.keep, self.Y, args = [], [], [], []
        for sp in specs:
            X, W, b, act = sp["X"], sp["W"], sp.get("b"), sp.get("act", "none")
            M, K = X.shape
            N = W.shape[1]
            sx = sp.get("s_x", casts.e4m3_scale(X)) if dtype_name == "fp8" else 1.0     # per-tensor scales: amax / 448
            sw = sp.get("s_w", casts.e4m3_scale(W)) if dtype_name == "fp8" else 1.0     # unless the case fixes them
            xb, wb = to_bits(X, dtype_name, sx), to_bits(W, dtype_name, sw)
            self.bits.append({"X": xb, "W": wb, "b": b, "act": act, "s": sx * sw})
            dX = R.device_tensor_from_bits(xb, dt, DEV) if M else None
            dW = R.pack_weights(R.device_tensor_from_bits(wb, dt, DEV), dt)
            db = None if b is None else torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(DEV)
            dY = torch.zeros((M, N), dtype=R.TORCH_DTYPE[self.out_dtype], device=DEV)
            self.keep += [dX, dW, db]
            self.Y.append(dY)
            args.append(R.group_args(dX, dW, dY if M else None, M, K, N, act, bias=db, scale=sx * sw))
        self.args = np.array(args, dtype=B.GROUP_ARGS) if args else np.zeros(0, dtype=B.GROUP_ARGS)
        self.plan = R.LaunchPlan(self.args, dt, DEV, n_workgroups)

    def run(self):
        for y in self.Y:
            y.zero_()
        R.grouped_forward(self.plan, self.out_dtype)
        torch.cuda.synchronize()
        return [fetch(y) for y in self.Y]

    def raw(self):
        return [y.clone() for y in self.Y]

    def expected(self):
        out = []
        for b in self.bits:
            X, W = values(b["X"], self.dtype_name), values(b["W"], self.dtype_name)
            out.append(ref.dense_forward(X, W, b["b"], b["act"], s=b["s"]))
        return out


def rand_spec(rng, M, K, N, act="none", bias=True, x_uniform=False):
    X = (rng.uniform(-1, 1, (M, K)) if x_uniform else rng.standard_normal((M, K))).astype(np.float32)
    W = (rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32) if bias else None
    return {"X": X, "W": W, "b": b, "act": act}
