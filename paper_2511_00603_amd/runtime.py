"""Marshalling between PyTorch device memory and libepara.  PyTorch is used for allocation,
host<->device copies and streams only; every step of the forward path runs in the library."""
import ctypes
import time

import numpy as np
import torch

from . import binding as B

TORCH_DTYPE = {B.EPARA_F32: torch.float32, B.EPARA_BF16: torch.bfloat16, B.EPARA_FP8_E4M3: torch.uint8}


def _require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("libepara needs a GPU: no CPU fallback exists")


def _upload(a, device):
    """numpy array (any dtype) -> uint8 device tensor holding the same bytes (never empty)."""
    raw = np.ascontiguousarray(a).view(np.uint8).reshape(-1)
    if raw.size == 0:
        return torch.zeros(16, dtype=torch.uint8, device=device)
    return torch.from_numpy(raw.copy()).to(device)


def current_stream_handle():
    return torch.cuda.current_stream().cuda_stream


def n_compute_units(device=None):
    return torch.cuda.get_device_properties(device if device is not None else torch.cuda.current_device()).multi_processor_count


def device_tensor_from_bits(bits, dtype, device):
    """Host bit patterns (float32 / uint16 bf16 / uint8 e4m3 arrays) -> device tensor of that storage type."""
    if dtype == B.EPARA_F32:
        return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.float32)).to(device)
    if dtype == B.EPARA_BF16:
        return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint16).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint8)).to(device)


def pack_weights(W, dtype):
    """W: device tensor holding the logical [K, N] weights in storage type `dtype` -> packed uint8 tensor."""
    _require_gpu()
    K, N = W.shape
    W = W.contiguous()
    nbytes = B.epara_packed_weight_bytes(K, N, dtype)
    out = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    B.epara_pack_weights(W.data_ptr(), K, N, dtype, out.data_ptr(), nbytes, current_stream_handle())
    return out


def group_args(X, W, Y, M, K, N, act, bias=None, W2=None, scale=1.0, scale2=1.0, out_inv_scale=1.0):
    """One GROUP_ARGS record from device tensors (or None)."""
    a = np.zeros(1, dtype=B.GROUP_ARGS)[0]
    ptr = lambda t: 0 if t is None else int(t.data_ptr())
    a["X"], a["W"], a["W2"], a["bias"], a["Y"] = ptr(X), ptr(W), ptr(W2), ptr(bias), ptr(Y)
    a["M"], a["K"], a["N"] = M, K, N
    a["act"] = B.ACT_BY_NAME[act] if isinstance(act, str) else act
    a["scale"], a["scale2"], a["out_inv_scale"] = scale, scale2, out_inv_scale
    return a


def _group_desc(args):
    groups = np.zeros(len(args), dtype=B.GROUP_DESC)
    for f in ("M", "K", "N", "act"):
        groups[f] = args[f]
    groups["has_bias"] = (args["bias"] != 0).astype(np.int32)
    return groups


class LaunchPlan:
    """Host plan + its device copy for one grouped launch (epara_launch).  The plan itself -- class table, tiles,
    visit order -- is the library's (epara_plan_launch); this class only keeps the arrays and uploads them."""

    def __init__(self, args, in_dtype, device, n_workgroups=None, n_xcd=8, panel_m=1, panel_n=4):
        # panel 1 x 4: panel tiles are visited strip by strip (4 tile columns), row by row, so the 32
        # tiles that run together on one die are 8 whole rows of a strip wherever a strip begins
        _require_gpu()
        t0 = time.perf_counter()
        self.args = np.ascontiguousarray(args, dtype=B.GROUP_ARGS)
        G = len(self.args)
        self.in_dtype = in_dtype
        self.groups = _group_desc(self.args)
        if n_workgroups is None:
            n_workgroups = n_compute_units(device)
            n_workgroups -= n_workgroups % n_xcd
        self.n_workgroups = n_workgroups
        info, self.row_off, self.x_off, self.y_off, self.tiles, self.order, split_base = B.epara_plan_launch(
            self.groups, in_dtype, n_workgroups, n_xcd, panel_m, panel_n)
        self.n_split_tiles, self.workspace_bytes = int(info.n_split_tiles), int(info.workspace_bytes)
        self.n_panel_split_tiles = int(info.n_panel_split_tiles)
        if self.n_split_tiles:                               # where each group's split tiles meet in the workspace
            self.args["reserved"] = split_base
        self.makespan, self.narrow, self.classes, self.n_stream_classes = info.makespan, bool(info.narrow), info.class_table(), info.n_stream_classes
        self.plan_seconds = time.perf_counter() - t0
        t0 = time.perf_counter()
        self.d_args = _upload(self.args, device)
        self.d_tiles = _upload(self.tiles, device)
        self.d_order = _upload(self.order, device)
        self.d_workspace = None
        if self.workspace_bytes:
            self.d_workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=device)
            B.epara_workspace_init(self.d_workspace.data_ptr(), self.workspace_bytes, current_stream_handle())
        torch.cuda.synchronize(device)
        self.upload_seconds = time.perf_counter() - t0
        self.c = B.Launch(self.args.ctypes.data, self.d_args.data_ptr(), self.tiles.ctypes.data, self.d_tiles.data_ptr(),
                          self.d_order.data_ptr(), len(self.tiles), len(self.order), n_workgroups, G,
                          None if self.d_workspace is None else self.d_workspace.data_ptr(), self.workspace_bytes, self.n_split_tiles,
                          self.n_panel_split_tiles)


class _Phase:
    """One phase of a ChainPlan: the fields of a LaunchPlan, scheduled together with the other phases."""


class ChainPlan:
    """Host plan + device copy of a chain of grouped launches that runs as one kernel (epara_grouped_chain); planned
    by the library (epara_plan_chain).

    phase_args[p]: GROUP_ARGS array of phase p; out_dtypes[p]: its output dtype; producers[p]: None, or per
    group of phase p the index of the group of phase p-1 whose output it reads (-1: none)."""

    def __init__(self, phase_args, out_dtypes, producers, in_dtype, device, n_workgroups=None, n_xcd=8, panel_m=1, panel_n=4):
        _require_gpu()
        t0 = time.perf_counter()
        if n_workgroups is None:
            n_workgroups = n_compute_units(device)
            n_workgroups -= n_workgroups % n_xcd
        self.n_workgroups, self.in_dtype, self.out_dtypes = n_workgroups, in_dtype, list(out_dtypes)
        P = len(phase_args)
        args = [np.ascontiguousarray(a, dtype=B.GROUP_ARGS) for a in phase_args]
        groups = [_group_desc(a) for a in args]
        self.makespan, planned = B.epara_plan_chain(groups, [None if p == 0 else producers[p] for p in range(P)], in_dtype,
                                                    n_workgroups, n_xcd, panel_m, panel_n)
        self.phases = []
        for p in range(P):
            ph = _Phase()
            ph.args, ph.groups, ph.in_dtype, ph.n_workgroups = args[p], groups[p], in_dtype, n_workgroups
            info = planned[p]["info"]
            ph.narrow, ph.classes, ph.n_stream_classes = bool(info.narrow), info.class_table(), info.n_stream_classes
            ph.tiles, ph.order, ph.waits, ph.counter_base = planned[p]["tiles"], planned[p]["order"], planned[p]["waits"], planned[p]["counter_base"]
            self.phases.append(ph)
        self.n_counters = sum(len(a) for a in args)
        self.plan_seconds = time.perf_counter() - t0
        t0 = time.perf_counter()
        self.c = (B.ChainPhase * P)()
        self._launches = []
        for p, ph in enumerate(self.phases):
            ph.d_args, ph.d_tiles, ph.d_order = _upload(ph.args, device), _upload(ph.tiles, device), _upload(ph.order, device)
            ph.d_waits = None if ph.waits is None else _upload(ph.waits, device)
            ph.c = B.Launch(ph.args.ctypes.data, ph.d_args.data_ptr(), ph.tiles.ctypes.data, ph.d_tiles.data_ptr(),
                            ph.d_order.data_ptr(), len(ph.tiles), len(ph.order), n_workgroups, len(ph.args), None, 0, 0, 0)
            self._launches.append(ph.c)
            self.c[p].launch = ctypes.pointer(ph.c)
            self.c[p].h_waits = None if ph.waits is None else ph.waits.ctypes.data
            self.c[p].d_waits = None if ph.waits is None else ph.d_waits.data_ptr()
            self.c[p].out_dtype, self.c[p].counter_base = int(self.out_dtypes[p]), ph.counter_base
        self.workspace_bytes = B.epara_chain_workspace_bytes(self.n_counters)
        self.d_workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=device)
        B.epara_chain_workspace_init(self.d_workspace.data_ptr(), self.workspace_bytes, current_stream_handle())
        torch.cuda.synchronize(device)
        self.upload_seconds = time.perf_counter() - t0


def grouped_chain(plan, stream=None, spin_limit=0):
    B.epara_grouped_chain(plan.c, plan.in_dtype, plan.d_workspace.data_ptr(), plan.workspace_bytes,
                          current_stream_handle() if stream is None else stream, spin_limit)


def grouped_chain_static(plan, stream=None, spin_limit=0, d_flag=None):
    """The same chain with the counters in the library's own scratch array (nothing is allocated)."""
    B.epara_grouped_chain_static(plan.c, plan.in_dtype, current_stream_handle() if stream is None else stream, spin_limit,
                                 0 if d_flag is None else d_flag.data_ptr())


def chain_status(plan, stream=None):
    """Synchronises; 0 = every wait of the chains run on this plan's workspace ended normally."""
    return B.epara_chain_status(plan.d_workspace.data_ptr(), current_stream_handle() if stream is None else stream)


def grouped_forward(plan, out_dtype, stream=None):
    B.epara_grouped_forward(plan.c, plan.in_dtype, out_dtype, current_stream_handle() if stream is None else stream)


def grouped_ffn_swiglu(up, down, h_dtype, out_dtype, stream=None):
    B.epara_grouped_ffn_swiglu(up.c, down.c, up.in_dtype, h_dtype, out_dtype,
                               current_stream_handle() if stream is None else stream)


# ---- batch forming (the step before and after the grouped forward) ---------------------------------

class SegmentPlan:
    """Copy plan between the requests' own buffers and the services' batches (epara_request_segments),
    host copy + device copy.  request_tensors[g] = list of [rows_r, width] device tensors of service g,
    batch_tensors[g] = [M_g, width] device tensor."""

    def __init__(self, request_tensors, batch_tensors, to_batch, device):
        _require_gpu()
        rows, off, ptrs, row_bytes, batch_row_bytes, bptr = [], [0], [], [], [], []
        for reqs, batch in zip(request_tensors, batch_tensors):
            for t in reqs:
                rows.append(t.shape[0])
                ptrs.append(t.data_ptr() if t.shape[0] else 0)
            off.append(len(rows))
            row_bytes.append((reqs[0].shape[1] * reqs[0].element_size()) if reqs else 16)
            batch_row_bytes.append((batch.shape[1] * batch.element_size()) if batch is not None and batch.dim() == 2 else row_bytes[-1])
            bptr.append(batch.data_ptr() if batch is not None else 0)
        self.G = len(batch_tensors)
        self.segments, self.n_chunks = B.epara_request_segments(rows, off, row_bytes, batch_row_bytes, ptrs, bptr, to_batch)
        self.d_segments = _upload(self.segments, device)
        self.bytes = int(self.segments["bytes"].sum())


def copy_segments(plan, stream=None):
    B.epara_copy_segments(plan.segments, plan.d_segments.data_ptr(), plan.n_chunks,
                          current_stream_handle() if stream is None else stream)


def quantize_segments_e4m3(plan, src_dtype, d_amax, d_scale, stream=None):
    """plan: SegmentPlan whose destinations are the uint8 code tensors; d_amax, d_scale: float32[G] device tensors."""
    B.epara_quantize_segments_e4m3(plan.segments, plan.d_segments.data_ptr(), plan.n_chunks, plan.G, src_dtype,
                                   d_amax.data_ptr(), d_scale.data_ptr(), current_stream_handle() if stream is None else stream)


def patch_scales(launch_plan, d_sx, d_sw, d_sw2=None, d_sout=None, stream=None):
    """Scale products from device memory into the device copy of a launch's group arguments."""
    ptr = lambda t: 0 if t is None else t.data_ptr()
    B.epara_patch_scales(launch_plan.d_args.data_ptr(), len(launch_plan.args), ptr(d_sx), ptr(d_sw), ptr(d_sw2), ptr(d_sout),
                         current_stream_handle() if stream is None else stream)


class NormPlan:
    """Arguments of one epara_add_layernorm launch, host copy + device copy.  groups: per service a dict with the
    device tensors X [M, d] (bf16), gamma, beta (float32 [d]), Y [M, d], optionally R and S [M, d], and eps."""

    def __init__(self, groups, device):
        _require_gpu()
        ptr = lambda t: 0 if t is None else t.data_ptr()
        self.args = np.zeros(len(groups), dtype=B.NORM_ARGS)
        rows = 0
        for i, g in enumerate(groups):
            M, d = (int(v) for v in g["X"].shape)
            live = M > 0
            self.args[i] = (ptr(g["X"]) if live else 0, ptr(g.get("R")) if live else 0, ptr(g["gamma"]), ptr(g["beta"]),
                            ptr(g.get("S")) if live else 0, ptr(g["Y"]) if live else 0, M, d, float(g.get("eps", 1e-6)), rows)
            rows += M
        self.rows = rows
        self.d_args = _upload(self.args, device)


def add_layernorm(plan, stream=None):
    B.epara_add_layernorm(plan.args, plan.d_args.data_ptr(), current_stream_handle() if stream is None else stream)


class AttnPlan:
    """Arguments of one epara_attention launch.  groups: per service a dict with the device tensors QKV [M, 3 d] and
    O [M, d] (bf16), tokens (rows per image) and heads (d = heads * 64)."""

    def __init__(self, groups, device):
        _require_gpu()
        self.args = np.zeros(len(groups), dtype=B.ATTN_ARGS)
        items = 0
        for i, g in enumerate(groups):
            M = int(g["QKV"].shape[0])
            live = M > 0
            self.args[i] = (g["QKV"].data_ptr() if live else 0, g["O"].data_ptr() if live else 0, M, int(g["tokens"]), int(g["heads"]),
                            B.EPARA_ATTN_HEAD_DIM, items, 0)
            items += (M // int(g["tokens"])) * int(g["heads"])
        self.items = items
        self.d_args = _upload(self.args, device)


def attention(plan, stream=None):
    B.epara_attention(plan.args, plan.d_args.data_ptr(), current_stream_handle() if stream is None else stream)
