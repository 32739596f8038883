"""Stages a synthetic service mix (workloads.Mix) on the GPU and runs one pass of it through
libepara.  Used by the parity tests, the smoke check and the benchmark.

A pass is the sequence of grouped launches that serves every service of the mix once:
  mix 1  three launches (layer 1, 2, 3 of both MLPs)
  mix 2  two launches   (all FFN-up groups with GELU, then all FFN-down groups)
  mix 3  two launches   (FFN-up groups of every service, then their QKV and FFN-down groups)
  mix 4, 5  one grouped SwiGLU FFN call (gate/up launch, down launch)
Inputs are rounded once on the host (workloads.casts) and the exact bits are kept in
`host_bits` so that a checker can be given the same values.
"""
import numpy as np
import torch

from workloads import casts

from . import binding as B
from . import runtime as R


def _bits(a, dtype, scale=None):
    if dtype == B.EPARA_F32:
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == B.EPARA_BF16:
        return casts.bf16_bits(a)
    return casts.e4m3_codes(a, scale)


class StagedMix:
    def __init__(self, mix, dtype_name=None, device="cuda:0", copies=1, s_h=None, n_workgroups=None, host_bits=None,
                 chained=False):
        """chained: the launches of a pass run as one kernel (epara_grouped_chain) instead of one after the other.
        copies > 1 stages independent replicas of all weights and activations; pass `copy=i` to run()
        to rotate through them (keeps a timing loop out of the last-level cache).
        s_h: per-service scales of the hidden activations for the fp8 SwiGLU path (list of floats)."""
        self.mix = mix
        self.device = torch.device(device)
        self.dtype = B.DTYPE_BY_NAME[dtype_name or mix.dtype]
        self.fp8 = self.dtype == B.EPARA_FP8_E4M3
        if self.fp8 and mix.services[0].kind != "swiglu":
            raise ValueError("the fp8 path is staged for SwiGLU FFN mixes only (chained layers would need fp8 outputs)")
        self.out_dtype = B.EPARA_F32 if self.dtype == B.EPARA_F32 else B.EPARA_BF16
        self.copies = copies
        self.chained = chained
        self.host_bits = []          # per service: dict of the exact inputs handed to the GPU
        self.programs = []           # per copy: list of ("forward", plan, out_dtype) / ("ffn", up, down, h_dtype)
        self.outputs = []            # per copy: list (per launch) of list (per group) of (service, label, tensor)
        self.inputs = []             # per copy: list (per service) of the device tensor holding X
        self.pack_seconds = 0.0
        self.s_h = s_h
        self._keep = []
        if host_bits is not None:        # already rounded by stage_host(); reused so a checker sees the same bits
            self.host_bits = host_bits
        else:
            self._stage_host()
        for _ in range(copies):
            self._stage_device(n_workgroups)
        torch.cuda.synchronize(self.device)

    # ---- host side: round the fp32 masters once -----------------------------------------
    def _stage_host(self):
        dt = self.dtype
        for svc in self.mix.services:
            hb = {}
            sx = casts.e4m3_scale(svc.X) if self.fp8 else 1.0
            hb["X"], hb["s_x"] = _bits(svc.X, dt, sx), sx
            if svc.kind == "swiglu":
                for name in ("Wgate", "Wup", "Wdown"):
                    W = getattr(svc, name)
                    s = casts.e4m3_scale(W) if self.fp8 else 1.0
                    hb[name], hb["s_" + name.lower()] = _bits(W, dt, s), s
            else:
                hb["layers"] = []
                for L in svc.layers:
                    s = casts.e4m3_scale(L.W) if self.fp8 else 1.0
                    hb["layers"].append({"W": _bits(L.W, dt, s), "s_w": s, "b": L.b, "act": L.act})
            self.host_bits.append(hb)

    @classmethod
    def stage_host(cls, mix, dtype_name=None):
        """Only the host half: the rounded inputs of every service (no GPU needed)."""
        self = cls.__new__(cls)
        self.mix, self.host_bits = mix, []
        self.dtype = B.DTYPE_BY_NAME[dtype_name or mix.dtype]
        self.fp8 = self.dtype == B.EPARA_FP8_E4M3
        self._stage_host()
        return self.host_bits

    # ---- device side ------------------------------------------------------------------------
    def _dev(self, bits):
        t = R.device_tensor_from_bits(bits, self.dtype, self.device)
        self._keep.append(t)
        return t

    def _packed(self, bits):
        W = R.device_tensor_from_bits(bits, self.dtype, self.device)
        torch.cuda.synchronize(self.device)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        P = R.pack_weights(W, self.dtype)
        ev1.record()
        torch.cuda.synchronize(self.device)
        self.pack_seconds += ev0.elapsed_time(ev1) * 1e-3
        self._keep.append(P)
        return P

    def _empty(self, M, N, dtype):
        t = torch.zeros((M, N), dtype=R.TORCH_DTYPE[dtype], device=self.device)
        self._keep.append(t)
        return t

    def _stage_device(self, n_workgroups):
        mix, dt = self.mix, self.dtype
        prog, outs, ins = [], [], []
        if mix.services[0].kind == "swiglu":
            ffn = np.zeros(len(mix.services), dtype=B.FFN_DESC)
            o_h, o_y = [], []
            h_dtype = B.EPARA_FP8_E4M3 if self.fp8 else B.EPARA_BF16
            for g, (svc, hb) in enumerate(zip(mix.services, self.host_bits)):
                d, f = svc.Wgate.shape
                X = self._dev(hb["X"])
                ins.append(X)
                Wg, Wu, Wd = self._packed(hb["Wgate"]), self._packed(hb["Wup"]), self._packed(hb["Wdown"])
                H, Y = self._empty(svc.M, f, h_dtype), self._empty(svc.M, d, B.EPARA_BF16)
                rec = ffn[g]
                rec["X"], rec["Wgate"], rec["Wup"], rec["Wdown"] = X.data_ptr(), Wg.data_ptr(), Wu.data_ptr(), Wd.data_ptr()
                rec["H"], rec["Y"] = H.data_ptr(), Y.data_ptr()
                rec["M"], rec["d_model"], rec["d_ff"] = svc.M, d, f
                rec["s_x"], rec["s_wgate"], rec["s_wup"], rec["s_wdown"] = hb["s_x"], hb["s_wgate"], hb["s_wup"], hb["s_wdown"]
                rec["s_h"] = self.s_h[g] if (self.fp8 and self.s_h is not None) else 1.0
                o_h.append((g, "H", H))
                o_y.append((g, "Y", Y))
            up_args, down_args = B.epara_ffn_swiglu_args(ffn, dt)
            if self.chained:
                chain = R.ChainPlan([up_args, down_args], [h_dtype, B.EPARA_BF16], [None, np.arange(len(ffn), dtype=np.int32)],
                                    dt, self.device, n_workgroups)
                prog.append(("chain", chain))
            else:
                up = R.LaunchPlan(up_args, dt, self.device, n_workgroups)
                down = R.LaunchPlan(down_args, dt, self.device, n_workgroups)
                prog.append(("ffn", up, down, h_dtype))
            outs += [o_h, o_y]
            self.ffn_desc = ffn
        else:
            n_layers = len(mix.services[0].layers)
            X0 = [self._dev(hb["X"]) for hb in self.host_bits]
            ins = list(X0)
            W = [[self._packed(l["W"]) for l in hb["layers"]] for hb in self.host_bits]
            bias = [[None if l["b"] is None else self._dev_f32(l["b"]) for l in hb["layers"]] for hb in self.host_bits]
            n_svc = len(mix.services)
            if mix.services[0].kind == "vit":      # layers: 0 = QKV (from X), 1 = FFN up (from X), 2 = FFN down (from 1)
                # QKV depends on nothing but X, so it shares a launch with FFN down: the few long-K tiles of
                # FFN down alone would leave a quarter of the workgroups idle, the scheduler fills them with QKV tiles
                launches = [[(g, 1, "in") for g in range(n_svc)],
                            [(g, 0, "in") for g in range(n_svc)] + [(g, 2, 1) for g in range(n_svc)]]
            else:                                  # a chain: layer l reads layer l-1
                launches = [[(g, l, "in" if l == 0 else l - 1) for g in range(n_svc)] for l in range(n_layers)]
            produced = {}
            phase_args, producers, where = [], [], {}
            for launch in launches:
                args, o = [], []
                producers.append(np.array([-1 if src == "in" else where[(g, src)] for g, l, src in launch], dtype=np.int32))
                where = {(g, l): i for i, (g, l, src) in enumerate(launch)}
                for g, l, src in launch:
                    svc, hb = mix.services[g], self.host_bits[g]
                    lay = hb["layers"][l]
                    K, N = svc.layers[l].W.shape
                    Xin = X0[g] if src == "in" else produced[(g, src)]
                    Y = self._empty(svc.M, N, self.out_dtype)
                    scale = hb["s_x"] * lay["s_w"] if self.fp8 else 1.0
                    args.append(R.group_args(Xin, W[g][l], Y, svc.M, K, N, lay["act"], bias=bias[g][l], scale=scale))
                    produced[(g, l)] = Y
                    o.append((g, "L%d" % l, Y))
                phase_args.append(np.array(args, dtype=B.GROUP_ARGS))
                if not self.chained:
                    plan = R.LaunchPlan(phase_args[-1], dt, self.device, n_workgroups)
                    prog.append(("forward", plan, self.out_dtype))
                outs.append(o)
            if self.chained:
                producers[0] = None
                chain = R.ChainPlan(phase_args, [self.out_dtype] * len(phase_args), producers, dt, self.device, n_workgroups)
                prog.append(("chain", chain))
        self.programs.append(prog)
        self.outputs.append(outs)
        self.inputs.append(ins)

    def _dev_f32(self, a):
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device)
        self._keep.append(t)
        return t

    # ---- running ------------------------------------------------------------------------------
    def run(self, copy=0, stream=None):
        """Enqueue one pass (all launches of the mix) on the current stream."""
        for step in self.programs[copy % self.copies]:
            if step[0] == "forward":
                R.grouped_forward(step[1], step[2], stream)
            elif step[0] == "chain":
                R.grouped_chain(step[1], stream)
            else:
                R.grouped_ffn_swiglu(step[1], step[2], step[3], B.EPARA_BF16, stream)

    def n_launches(self):
        return sum(2 if s[0] == "ffn" else 1 for s in self.programs[0])

    def plans(self, copy=0):
        """The per-launch plans (for a chain: its phases, which carry the same fields)."""
        out = []
        for step in self.programs[copy]:
            out += [step[1]] if step[0] == "forward" else (list(step[1].phases) if step[0] == "chain" else [step[1], step[2]])
        return out

    def chain_status(self, copy=0):
        """After a chained pass: 0 if every wait ended normally (synchronises)."""
        return max([R.chain_status(step[1]) for step in self.programs[copy % self.copies] if step[0] == "chain"] or [0])

    def results(self, copy=0):
        """After a synchronize: list per launch of (service, label, float64 ndarray of output VALUES)."""
        res = []
        for launch in self.outputs[copy]:
            cur = []
            for g, label, t in launch:
                if t.dtype == torch.uint8:      # E4M3 codes: decode with PyTorch's table, scale applied by the caller
                    v = t.view(torch.float8_e4m3fn).to(torch.float32).cpu().numpy().astype(np.float64)
                else:
                    v = t.to(torch.float32).cpu().numpy().astype(np.float64)
                cur.append((g, label, v))
            res.append(cur)
        return res
