"""ctypes binding of libepara: the same entry points as include/epara.h, argument marshalling only.

Structured numpy dtypes mirror the C structs byte for byte; device memory is passed as integer
addresses (e.g. torch.Tensor.data_ptr()).  A non-zero status raises EparaError.
"""
import ctypes
import os

import numpy as np

from . import build as _build

# ---- enums (include/epara.h) -------------------------------------------------------------
EPARA_OK, EPARA_ERR_NULL, EPARA_ERR_SHAPE, EPARA_ERR_DTYPE, EPARA_ERR_CAPACITY, EPARA_ERR_ALIGN, EPARA_ERR_HIP = range(7)
EPARA_F32, EPARA_BF16, EPARA_FP8_E4M3 = 0, 1, 2
EPARA_ACT_NONE, EPARA_ACT_RELU, EPARA_ACT_GELU_ERF, EPARA_ACT_GELU_TANH, EPARA_ACT_SILU, EPARA_ACT_SWIGLU = range(6)
EPARA_CAT_LATENCY, EPARA_CAT_FREQUENCY = 0, 1

ACT_BY_NAME = {"none": EPARA_ACT_NONE, "relu": EPARA_ACT_RELU, "gelu_erf": EPARA_ACT_GELU_ERF,
               "gelu_tanh": EPARA_ACT_GELU_TANH, "silu": EPARA_ACT_SILU, "swiglu": EPARA_ACT_SWIGLU}
DTYPE_BY_NAME = {"f32": EPARA_F32, "bf16": EPARA_BF16, "fp8": EPARA_FP8_E4M3}
DTYPE_BYTES = {EPARA_F32: 4, EPARA_BF16: 2, EPARA_FP8_E4M3: 1}

# ---- struct layouts ----------------------------------------------------------------------
GROUP_DESC = np.dtype([("M", "<i4"), ("K", "<i4"), ("N", "<i4"), ("act", "<i4"), ("has_bias", "<i4"), ("category", "<i4")])
TILE_CLASS = np.dtype([("max_M", "<i4"), ("BM", "<i4"), ("BN", "<i4"), ("split_K", "<i4")])
TILE = np.dtype([("group", "<i4"), ("m0", "<i4"), ("n0", "<i4"), ("rows", "<i4"), ("cols", "<i4"), ("cls", "<i4")])
GROUP_ARGS = np.dtype([("X", "<u8"), ("W", "<u8"), ("W2", "<u8"), ("bias", "<u8"), ("Y", "<u8"),
                       ("M", "<i4"), ("K", "<i4"), ("N", "<i4"), ("act", "<i4"),
                       ("scale", "<f4"), ("scale2", "<f4"), ("out_inv_scale", "<f4"), ("reserved", "<i4")])
FFN_DESC = np.dtype([("X", "<u8"), ("Wgate", "<u8"), ("Wup", "<u8"), ("Wdown", "<u8"), ("H", "<u8"), ("Y", "<u8"),
                     ("M", "<i4"), ("d_model", "<i4"), ("d_ff", "<i4"),
                     ("s_x", "<f4"), ("s_wgate", "<f4"), ("s_wup", "<f4"), ("s_h", "<f4"), ("s_wdown", "<f4")])
SEGMENT = np.dtype([("src", "<u8"), ("dst", "<u8"), ("bytes", "<i8"), ("first_chunk", "<i8"), ("group", "<i4"), ("reserved", "<i4")])
CHAIN_WAIT = np.dtype([("counter", "<i4"), ("need", "<i4")])
NORM_ARGS = np.dtype([("X", "<u8"), ("R", "<u8"), ("gamma", "<u8"), ("beta", "<u8"), ("S", "<u8"), ("Y", "<u8"),
                      ("M", "<i4"), ("d", "<i4"), ("eps", "<f4"), ("first_row", "<i4")])
ATTN_ARGS = np.dtype([("QKV", "<u8"), ("O", "<u8"), ("M", "<i4"), ("tokens", "<i4"), ("heads", "<i4"), ("head_dim", "<i4"),
                      ("first_item", "<i4"), ("reserved", "<i4")])
assert NORM_ARGS.itemsize == 64 and ATTN_ARGS.itemsize == 40
EPARA_NORM_MAX_D, EPARA_ATTN_MAX_TOKENS, EPARA_ATTN_HEAD_DIM = 8192, 224, 64
SIM_REQUEST = np.dtype([("arrival_us", "<i8"), ("slo_us", "<i8"), ("service", "<i4"), ("origin", "<i4"), ("frames", "<i4"), ("fps_milli", "<i4")])
assert SIM_REQUEST.itemsize == 32
EPARA_MAX_CHAIN_PHASES = 4
EPARA_STATIC_CHAIN_COUNTERS = 4092
assert CHAIN_WAIT.itemsize == 8
assert GROUP_DESC.itemsize == 24 and TILE_CLASS.itemsize == 16 and TILE.itemsize == 24 and SEGMENT.itemsize == 40
assert GROUP_ARGS.itemsize == 72 and FFN_DESC.itemsize == 80


class LaunchPlanInfo(ctypes.Structure):
    """struct epara_launch_plan."""
    _fields_ = [("classes", ctypes.c_int32 * 16), ("n_classes", ctypes.c_int32), ("n_stream_classes", ctypes.c_int32),
                ("narrow", ctypes.c_int32), ("gated", ctypes.c_int32), ("n_tiles", ctypes.c_int64), ("n_slots", ctypes.c_int64),
                ("makespan", ctypes.c_int64), ("workspace_bytes", ctypes.c_int64), ("n_split_tiles", ctypes.c_int32),
                ("n_panel_split_tiles", ctypes.c_int32)]

    def class_table(self):
        return np.array(list(self.classes), dtype=np.int32)[: 4 * self.n_classes].view(TILE_CLASS).copy()


class ChainPlanPhase(ctypes.Structure):
    """struct epara_chain_plan_phase."""
    _fields_ = [("groups", ctypes.c_void_p), ("producer", ctypes.c_void_p), ("tiles", ctypes.c_void_p), ("order", ctypes.c_void_p),
                ("waits", ctypes.c_void_p), ("tiles_cap", ctypes.c_int64), ("order_cap", ctypes.c_int64), ("G", ctypes.c_int32),
                ("counter_base", ctypes.c_int32), ("plan", LaunchPlanInfo)]


class Launch(ctypes.Structure):
    """struct epara_launch."""
    _fields_ = [("h_args", ctypes.c_void_p), ("d_args", ctypes.c_void_p),
                ("h_tiles", ctypes.c_void_p), ("d_tiles", ctypes.c_void_p), ("d_order", ctypes.c_void_p),
                ("n_tiles", ctypes.c_int64), ("n_slots", ctypes.c_int64),
                ("n_workgroups", ctypes.c_int32), ("G", ctypes.c_int32),
                ("d_workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_int64), ("n_split_tiles", ctypes.c_int32),
                ("n_panel_split_tiles", ctypes.c_int32)]


assert ctypes.sizeof(Launch) == 88


class SimConfig(ctypes.Structure):
    """struct epara_sim_config."""
    _fields_ = [("compute_us", ctypes.c_void_p), ("hop_us", ctypes.c_int64), ("sync_delay_us", ctypes.c_int64),
                ("n_servers", ctypes.c_int32), ("n_services", ctypes.c_int32), ("max_offload", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class SimResult(ctypes.Structure):
    """struct epara_sim_result."""
    _fields_ = [("satisfied", ctypes.c_double), ("local", ctypes.c_int64), ("offloaded", ctypes.c_int64),
                ("timeout", ctypes.c_int64), ("offload_exceeded", ctypes.c_int64), ("insufficient", ctypes.c_int64)]


assert ctypes.sizeof(SimConfig) == 40 and ctypes.sizeof(SimResult) == 48


class PhaseSchedule(ctypes.Structure):
    """struct epara_phase_schedule."""
    _fields_ = [("groups", ctypes.c_void_p), ("classes", ctypes.c_void_p), ("tiles", ctypes.c_void_p), ("order", ctypes.c_void_p),
                ("n_tiles", ctypes.c_int64), ("order_cap", ctypes.c_int64), ("n_slots", ctypes.c_int64),
                ("G", ctypes.c_int32), ("n_classes", ctypes.c_int32), ("n_stream_classes", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class ChainPhase(ctypes.Structure):
    """struct epara_chain_phase."""
    _fields_ = [("launch", ctypes.POINTER(Launch)), ("h_waits", ctypes.c_void_p), ("d_waits", ctypes.c_void_p),
                ("out_dtype", ctypes.c_int32), ("counter_base", ctypes.c_int32)]


assert ctypes.sizeof(PhaseSchedule) == 72 and ctypes.sizeof(ChainPhase) == 32


PHI_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.POINTER(ctypes.c_int32), ctypes.c_int32, ctypes.c_void_p)   # epara_phi_fn


class EparaError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, epara_status_string(status)))


_lib = None


def library_path():
    return _build.LIB


def lib():
    """The loaded shared library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise RuntimeError("libepara.so is not built (%s); run `python -m paper_2511_00603_amd.build`" % path)
        L = ctypes.CDLL(path)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.epara_status_string.argtypes = [i32]
        L.epara_status_string.restype = ctypes.c_char_p
        L.epara_batch_rows.argtypes = [vp, vp, i32, vp, vp]
        L.epara_dp_group_count.argtypes = [i64, i64]
        L.epara_dp_group_count.restype = i64
        L.epara_inter_request_count.argtypes = [i64, i64]
        L.epara_inter_request_count.restype = i64
        L.epara_operator_set.argtypes = [i32, i32]
        L.epara_operator_set.restype = i32
        L.epara_max_inter_frame_count.argtypes = [i64, i64]
        L.epara_max_inter_frame_count.restype = i64
        L.epara_dp_deal.argtypes = [i64, i64, i64, vp, vp]
        L.epara_dp_deal.restype = i32
        L.epara_handle_request.argtypes = [i64, i64, i32, i32, i32, vp, vp, vp, i32, i32, i64, i64, ctypes.c_double, vp, vp]
        L.epara_handle_request.restype = i32
        L.epara_place_full_models.argtypes = [vp, i32, i32, i32, vp, i32, PHI_FN, vp, vp, i32, vp]
        L.epara_place_full_models.restype = i32
        L.epara_place_services.argtypes = [vp, i32, vp, i32, vp, i32, PHI_FN, vp, vp, i32, vp]
        L.epara_place_services.restype = i32
        L.epara_plan_groups.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp, i64, vp]
        L.epara_schedule_tiles.argtypes = [vp, i32, vp, i32, i32, vp, i64, i32, i32, i32, i32, vp, i64, vp]
        L.epara_kernel_classes.argtypes = [i32, i32, i32, vp, i32, vp, vp]
        L.epara_workspace_bytes.argtypes = [vp, i32, i32, i32]
        L.epara_workspace_bytes.restype = i64
        L.epara_split_workspace_bytes.argtypes = [i32, i32]
        L.epara_split_workspace_bytes.restype = i64
        L.epara_panel_split.argtypes = [vp, i32, vp, i32, i32, i32, vp, vp, vp]
        L.epara_panel_split.restype = i32
        L.epara_simulate.argtypes = [vp, vp, i32, vp, i64, vp, vp]
        L.epara_simulate.restype = i32
        L.epara_schedule_chain.argtypes = [vp, i32, i32, i32, i32, i32]
        L.epara_chain_waits.argtypes = [vp, i64, i32, i32, vp, i32, vp]
        L.epara_chain_workspace_bytes.argtypes = [i32]
        L.epara_chain_workspace_bytes.restype = i64
        L.epara_chain_workspace_init.argtypes = [vp, i64, vp]
        L.epara_grouped_chain.argtypes = [vp, i32, i32, vp, i64, ctypes.c_uint32, vp]
        L.epara_chain_status.argtypes = [vp, vp, vp]
        L.epara_grouped_chain_static.argtypes = [vp, i32, i32, ctypes.c_uint32, vp, vp]
        for name in ("epara_schedule_chain", "epara_chain_waits", "epara_chain_workspace_init", "epara_grouped_chain",
                     "epara_chain_status", "epara_grouped_chain_static"):
            getattr(L, name).restype = i32
        L.epara_plan_launch.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, i64, vp, i64, vp, vp]
        L.epara_split_layout.argtypes = [vp, i32, vp, i32, i32, vp, vp, vp]
        L.epara_split_layout.restype = i32
        L.epara_workspace_init.argtypes = [vp, i64, vp]
        L.epara_workspace_init.restype = i32
        L.epara_workspace_bytes.argtypes = [vp, i32, i32, i32]
        L.epara_workspace_bytes.restype = i64
        L.epara_split_workspace_bytes.argtypes = [i32, i32]
        L.epara_split_workspace_bytes.restype = i64
        L.epara_panel_split.argtypes = [vp, i32, vp, i32, i32, i32, vp, vp, vp]
        L.epara_panel_split.restype = i32
        L.epara_plan_launch.restype = i32
        L.epara_plan_chain.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp]
        L.epara_plan_chain.restype = i32
        L.epara_compute_table.argtypes = [vp, vp, i32, vp, i32, vp]
        L.epara_compute_table.restype = i32
        L.epara_ffn_swiglu_args.argtypes = [vp, i32, i32, vp, vp]
        L.epara_packed_weight_bytes.argtypes = [i32, i32, i32]
        L.epara_packed_weight_bytes.restype = i64
        L.epara_pack_weights.argtypes = [vp, i32, i32, i32, vp, i64, vp]
        L.epara_grouped_forward.argtypes = [vp, i32, i32, vp]
        L.epara_grouped_ffn_swiglu.argtypes = [vp, vp, i32, i32, i32, vp]
        L.epara_request_segments.argtypes = [vp, vp, i32, vp, vp, vp, vp, i32, vp, vp]
        L.epara_copy_segments.argtypes = [vp, vp, i64, i64, vp]
        L.epara_quantize_segments_e4m3.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp]
        L.epara_patch_scales.argtypes = [vp, i32, vp, vp, vp, vp, vp]
        L.epara_add_layernorm.argtypes = [vp, vp, i32, vp]
        L.epara_add_layernorm.restype = i32
        L.epara_attention.argtypes = [vp, vp, i32, vp]
        L.epara_attention.restype = i32
        for name in ("epara_batch_rows", "epara_plan_groups", "epara_schedule_tiles", "epara_kernel_classes",
                     "epara_ffn_swiglu_args", "epara_pack_weights", "epara_grouped_forward", "epara_grouped_ffn_swiglu",
                     "epara_request_segments", "epara_copy_segments", "epara_quantize_segments_e4m3", "epara_patch_scales"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def _ptr(a):
    """Address of a numpy array's buffer (None -> NULL)."""
    return None if a is None else a.ctypes.data


def _check(status, where):
    if status != EPARA_OK:
        raise EparaError(status, where)


def epara_status_string(status):
    return lib().epara_status_string(int(status)).decode()


def epara_batch_rows(request_rows, request_off):
    """-> (M int32[G], first_row int64[R])."""
    request_rows = np.ascontiguousarray(request_rows, dtype=np.int32)
    request_off = np.ascontiguousarray(request_off, dtype=np.int64)
    G = len(request_off) - 1
    M = np.zeros(max(G, 0), dtype=np.int32)
    first = np.zeros(len(request_rows), dtype=np.int64)
    _check(lib().epara_batch_rows(_ptr(request_rows), _ptr(request_off), G, _ptr(M), _ptr(first)), "epara_batch_rows")
    return M, first


def epara_request_segments(request_rows, request_off, request_row_bytes, batch_row_bytes, request_ptr, batch_ptr, to_batch):
    """-> (segments SEGMENT[R], n_chunks).  request_ptr / batch_ptr: integer device addresses."""
    request_rows = np.ascontiguousarray(request_rows, dtype=np.int32)
    request_off = np.ascontiguousarray(request_off, dtype=np.int64)
    request_row_bytes = np.ascontiguousarray(request_row_bytes, dtype=np.int64)
    batch_row_bytes = np.ascontiguousarray(batch_row_bytes, dtype=np.int64)
    request_ptr = np.ascontiguousarray(request_ptr, dtype=np.uint64)
    batch_ptr = np.ascontiguousarray(batch_ptr, dtype=np.uint64)
    G = len(request_off) - 1
    segs = np.zeros(len(request_rows), dtype=SEGMENT)
    n = np.zeros(1, dtype=np.int64)
    _check(lib().epara_request_segments(_ptr(request_rows), _ptr(request_off), G, _ptr(request_row_bytes), _ptr(batch_row_bytes), _ptr(request_ptr),
                                        _ptr(batch_ptr), int(bool(to_batch)), _ptr(segs), _ptr(n)), "epara_request_segments")
    return segs, int(n[0])


def epara_copy_segments(h_segments, d_segments, n_chunks, stream=0):
    h_segments = np.ascontiguousarray(h_segments, dtype=SEGMENT)
    _check(lib().epara_copy_segments(_ptr(h_segments), int(d_segments) or None, len(h_segments), int(n_chunks),
                                     int(stream) or None), "epara_copy_segments")


def epara_quantize_segments_e4m3(h_segments, d_segments, n_chunks, G, src_dtype, d_amax, d_scale, stream=0):
    h_segments = np.ascontiguousarray(h_segments, dtype=SEGMENT)
    _check(lib().epara_quantize_segments_e4m3(_ptr(h_segments), int(d_segments) or None, len(h_segments), int(n_chunks), int(G),
                                              int(src_dtype), int(d_amax) or None, int(d_scale) or None, int(stream) or None),
           "epara_quantize_segments_e4m3")


def epara_patch_scales(d_args, G, d_sx, d_sw, d_sw2=0, d_sout=0, stream=0):
    _check(lib().epara_patch_scales(int(d_args) or None, int(G), int(d_sx) or None, int(d_sw) or None, int(d_sw2) or None,
                                    int(d_sout) or None, int(stream) or None), "epara_patch_scales")


def epara_add_layernorm(h_args, d_args, stream=0):
    """h_args: NORM_ARGS[G] (host copy, validated); d_args: device address of the same bytes."""
    h_args = np.ascontiguousarray(h_args, dtype=NORM_ARGS)
    _check(lib().epara_add_layernorm(_ptr(h_args) if len(h_args) else None, int(d_args) or None, len(h_args), int(stream) or None),
           "epara_add_layernorm")


def epara_attention(h_args, d_args, stream=0):
    """h_args: ATTN_ARGS[G] (host copy, validated); d_args: device address of the same bytes."""
    h_args = np.ascontiguousarray(h_args, dtype=ATTN_ARGS)
    _check(lib().epara_attention(_ptr(h_args) if len(h_args) else None, int(d_args) or None, len(h_args), int(stream) or None),
           "epara_attention")


def epara_dp_group_count(rate_required, rate_of_one_group):
    return int(lib().epara_dp_group_count(int(rate_required), int(rate_of_one_group)))


def epara_inter_request_count(batch_size, max_inter_frame_count):
    return int(lib().epara_inter_request_count(int(batch_size), int(max_inter_frame_count)))


EPARA_OP_BS, EPARA_OP_MT, EPARA_OP_MP, EPARA_OP_MF, EPARA_OP_DP = 1, 2, 4, 8, 16


def epara_operator_set(category, multi_gpu):
    return int(lib().epara_operator_set(int(category), int(bool(multi_gpu))))


def epara_max_inter_frame_count(latency_us, fps_milli):
    return int(lib().epara_max_inter_frame_count(int(latency_us), int(fps_milli)))


def epara_dp_deal(first_frame, n_frames, n_groups):
    """-> (frames_per_group int64[n_groups], group_of_frame int32[n_frames])."""
    per = np.zeros(max(int(n_groups), 0), dtype=np.int64)
    who = np.zeros(max(int(n_frames), 0), dtype=np.int32)
    _check(lib().epara_dp_deal(int(first_frame), int(n_frames), int(n_groups), _ptr(per) if per.size else None,
                               _ptr(who) if who.size else None), "epara_dp_deal")
    return per, who


HANDLE_NAMES = ["timeout", "local", "offload", "offload_exceeded", "insufficient"]


def epara_handle_request(now_us, deadline_us, local_can_serve, offload_count, max_offload, theoretical, actual, queued_us,
                         self_index, sync_delay_us, slo_us, u):
    """-> (decision name, destination or None)."""
    th = np.ascontiguousarray(theoretical, dtype=np.float64)
    ac = np.ascontiguousarray(actual, dtype=np.float64)
    qu = np.ascontiguousarray(queued_us, dtype=np.int64)
    out = np.zeros(2, dtype=np.int32)
    _check(lib().epara_handle_request(int(now_us), int(deadline_us), int(bool(local_can_serve)), int(offload_count), int(max_offload),
                                      _ptr(th), _ptr(ac), _ptr(qu), len(th), int(self_index), int(sync_delay_us), int(slo_us),
                                      float(u), _ptr(out[0:1]), _ptr(out[1:2])), "epara_handle_request")
    return HANDLE_NAMES[int(out[0])], (int(out[1]) if out[1] >= 0 else None)


def _phi_callback(phi):
    """Python callable on a list of placement ids -> C callback."""
    return PHI_FN(lambda p, n, _user: float(phi([p[i] for i in range(n)])))


def epara_place_full_models(candidates, is_set, keep_equal, theta0, phi, cap=4096):
    candidates = np.ascontiguousarray(candidates, dtype=np.int32)
    theta0 = np.ascontiguousarray(theta0, dtype=np.int32)
    out, n, cb = np.zeros(max(cap, 1), dtype=np.int32), np.zeros(1, dtype=np.int32), _phi_callback(phi)
    _check(lib().epara_place_full_models(_ptr(candidates) if candidates.size else None, len(candidates), int(bool(is_set)), int(bool(keep_equal)),
                                         _ptr(theta0) if theta0.size else None, len(theta0), cb, None, _ptr(out), int(cap), _ptr(n)),
           "epara_place_full_models")
    return out[: int(n[0])].tolist()


def epara_place_services(partial, X, X_dot, phi, cap=4096):
    arrs = [np.ascontiguousarray(a, dtype=np.int32) for a in (partial, X, X_dot)]
    out, n, cb = np.zeros(max(cap, 1), dtype=np.int32), np.zeros(1, dtype=np.int32), _phi_callback(phi)
    args = []
    for a in arrs:
        args += [_ptr(a) if a.size else None, len(a)]
    _check(lib().epara_place_services(*args, cb, None, _ptr(out), int(cap), _ptr(n)), "epara_place_services")
    return out[: int(n[0])].tolist()


def epara_plan_groups(groups, classes):
    """groups: GROUP_DESC array, classes: TILE_CLASS array -> (row_off, x_off, y_off, tiles)."""
    groups = np.ascontiguousarray(groups, dtype=GROUP_DESC)
    classes = np.ascontiguousarray(classes, dtype=TILE_CLASS)
    G = len(groups)
    n = np.zeros(1, dtype=np.int64)
    row_off, x_off, y_off = (np.zeros(G + 1, dtype=np.int64) for _ in range(3))
    _check(lib().epara_plan_groups(_ptr(groups), G, _ptr(classes), len(classes), _ptr(row_off), _ptr(x_off),
                                   _ptr(y_off), None, 0, _ptr(n)), "epara_plan_groups")
    tiles = np.zeros(int(n[0]), dtype=TILE)
    _check(lib().epara_plan_groups(_ptr(groups), G, _ptr(classes), len(classes), _ptr(row_off), _ptr(x_off),
                                   _ptr(y_off), _ptr(tiles), len(tiles), _ptr(n)), "epara_plan_groups")
    return row_off, x_off, y_off, tiles


def epara_schedule_tiles(groups, classes, n_stream_classes, tiles, n_workgroups, n_xcd=8, panel_m=8, panel_n=4):
    groups = np.ascontiguousarray(groups, dtype=GROUP_DESC)
    classes = np.ascontiguousarray(classes, dtype=TILE_CLASS)
    tiles = np.ascontiguousarray(tiles, dtype=TILE)
    n = np.zeros(1, dtype=np.int64)
    args = (_ptr(groups), len(groups), _ptr(classes), len(classes), int(n_stream_classes), _ptr(tiles), len(tiles),
            int(n_workgroups), int(n_xcd), int(panel_m), int(panel_n))
    _check(lib().epara_schedule_tiles(*args, None, 0, _ptr(n)), "epara_schedule_tiles")
    order = np.zeros(int(n[0]), dtype=np.int32)
    _check(lib().epara_schedule_tiles(*args, _ptr(order), len(order), _ptr(n)), "epara_schedule_tiles")
    return order


def epara_workspace_bytes(groups, in_dtype):
    groups = np.ascontiguousarray(groups, dtype=GROUP_DESC)
    return int(lib().epara_workspace_bytes(_ptr(groups), len(groups), int(in_dtype)))


def epara_plan_launch(groups, in_dtype, n_workgroups, n_xcd=8, panel_m=1, panel_n=4):
    """-> (info: LaunchPlanInfo, row_off, x_off, y_off, tiles, order, split_base): the library's whole planning decision of a launch."""
    groups = np.ascontiguousarray(groups, dtype=GROUP_DESC)
    G = len(groups)
    gp = _ptr(groups) if G else None
    info = LaunchPlanInfo()
    _check(lib().epara_plan_launch(gp, G, int(in_dtype), n_workgroups, n_xcd, panel_m, panel_n, None, None, None, None, 0, None, 0,
                                   None, ctypes.addressof(info)), "epara_plan_launch")
    row_off, x_off, y_off = (np.zeros(G + 1, dtype=np.int64) for _ in range(3))
    tiles, order = np.zeros(info.n_tiles, dtype=TILE), np.zeros(info.n_slots, dtype=np.int32)
    split_base = np.full(G, -1, dtype=np.int32)
    _check(lib().epara_plan_launch(gp, G, int(in_dtype), n_workgroups, n_xcd, panel_m, panel_n, _ptr(row_off), _ptr(x_off), _ptr(y_off),
                                   _ptr(tiles) if len(tiles) else None, len(tiles), _ptr(order) if len(order) else None, len(order),
                                   _ptr(split_base) if G else None, ctypes.addressof(info)), "epara_plan_launch")
    return info, row_off, x_off, y_off, tiles, order, split_base


def epara_split_layout(groups, classes, n_stream_classes):
    """-> (split_base [G], n_split_tiles, workspace_bytes)."""
    groups = np.ascontiguousarray(groups, dtype=GROUP_DESC)
    classes = np.ascontiguousarray(classes, dtype=TILE_CLASS)
    base = np.full(len(groups), -1, dtype=np.int32)
    n, nbytes = ctypes.c_int32(0), ctypes.c_int64(0)
    _check(lib().epara_split_layout(_ptr(groups) if len(groups) else None, len(groups), _ptr(classes), len(classes), int(n_stream_classes),
                                    _ptr(base) if len(base) else None, ctypes.byref(n), ctypes.byref(nbytes)), "epara_split_layout")
    return base, int(n.value), int(nbytes.value)


def epara_workspace_bytes(groups, in_dtype, n_workgroups=256):
    groups = np.ascontiguousarray(groups, dtype=GROUP_DESC)
    return int(lib().epara_workspace_bytes(_ptr(groups) if len(groups) else None, len(groups), int(in_dtype), int(n_workgroups)))


def epara_split_workspace_bytes(n_split_tiles, n_panel_split_tiles):
    return int(lib().epara_split_workspace_bytes(int(n_split_tiles), int(n_panel_split_tiles)))


def epara_panel_split(groups, classes, n_stream_classes, n_workgroups):
    """-> (m, P, n_more): the last m panel tiles of the tile table are visited in parts of K, the first m - n_more of
    them in P parts, the others in P + 1."""
    groups = np.ascontiguousarray(groups, dtype=GROUP_DESC)
    classes = np.ascontiguousarray(classes, dtype=TILE_CLASS)
    n, parts, more = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().epara_panel_split(_ptr(groups) if len(groups) else None, len(groups), _ptr(classes), len(classes), int(n_stream_classes),
                                   int(n_workgroups), ctypes.byref(n), ctypes.byref(parts), ctypes.byref(more)), "epara_panel_split")
    return int(n.value), int(parts.value), int(more.value)


def epara_workspace_init(d_workspace, nbytes, stream=0):
    _check(lib().epara_workspace_init(int(d_workspace), int(nbytes), int(stream) or None), "epara_workspace_init")


def epara_plan_chain(phase_groups, producers, in_dtype, n_workgroups, n_xcd=8, panel_m=1, panel_n=4):
    """phase_groups[p]: GROUP_DESC array; producers[p]: None or int array (per group: the producing group of phase p-1, -1: none).
    -> (finish, list per phase of dict(info, tiles, order, waits, counter_base))."""
    P = len(phase_groups)
    arr = (ChainPlanPhase * P)()
    keep = []
    for p in range(P):
        g = np.ascontiguousarray(phase_groups[p], dtype=GROUP_DESC)
        pr = None if producers[p] is None else np.ascontiguousarray(producers[p], dtype=np.int32)
        keep.append((g, pr))
        arr[p].groups, arr[p].G = (_ptr(g) if len(g) else None), len(g)
        arr[p].producer = None if pr is None or not len(pr) else _ptr(pr)
    finish = ctypes.c_int64(0)
    _check(lib().epara_plan_chain(ctypes.addressof(arr), P, int(in_dtype), n_workgroups, n_xcd, panel_m, panel_n, ctypes.byref(finish)),
           "epara_plan_chain")
    out = []
    for p in range(P):
        tiles, order = np.zeros(arr[p].plan.n_tiles, dtype=TILE), np.zeros(arr[p].plan.n_slots, dtype=np.int32)
        waits = None if keep[p][1] is None else np.zeros(len(keep[p][0]), dtype=CHAIN_WAIT)
        out.append({"tiles": tiles, "order": order, "waits": waits})
        arr[p].tiles, arr[p].tiles_cap = (_ptr(tiles) if len(tiles) else None), len(tiles)
        arr[p].order, arr[p].order_cap = (_ptr(order) if len(order) else None), len(order)
        arr[p].waits = None if waits is None or not len(waits) else _ptr(waits)
    _check(lib().epara_plan_chain(ctypes.addressof(arr), P, int(in_dtype), n_workgroups, n_xcd, panel_m, panel_n, ctypes.byref(finish)),
           "epara_plan_chain")
    for p in range(P):
        info = LaunchPlanInfo()
        ctypes.memmove(ctypes.addressof(info), ctypes.addressof(arr[p].plan), ctypes.sizeof(info))
        out[p]["info"], out[p]["counter_base"] = info, int(arr[p].counter_base)
    return int(finish.value), out


def epara_compute_table(ms_per_pass, requests_per_pass, server_speed):
    """c_ln [n_services, n_servers] in microseconds per request from measured passes (see the header)."""
    ms = np.ascontiguousarray(ms_per_pass, dtype=np.float64)
    rq = np.ascontiguousarray(requests_per_pass, dtype=np.int32)
    sp = np.ascontiguousarray(server_speed, dtype=np.float64)
    out = np.zeros((len(ms), len(sp)), dtype=np.int64)
    _check(lib().epara_compute_table(_ptr(ms) if len(ms) else None, _ptr(rq) if len(rq) else None, len(ms),
                                     _ptr(sp) if len(sp) else None, len(sp), _ptr(out) if out.size else None), "epara_compute_table")
    return out


def compute_table_from_bench_line(line, mix_keys, server_speed):
    """The same from one JSON line of bench.py: service l is the mix named mix_keys[l] (a key of line["mixes"])."""
    mixes = line["mixes"]
    return epara_compute_table([mixes[k]["ms_per_step"] for k in mix_keys], [mixes[k]["requests"] for k in mix_keys], server_speed)


def epara_simulate(n_servers, n_services, compute_us, hop_us, sync_delay_us, max_offload, placements, requests, draws):
    """compute_us: [n_services, n_servers]; requests: SIM_REQUEST array; draws: [n_requests, max_offload] in [0, 1).
    -> dict(satisfied, local, offloaded, timeout, offload_exceeded, insufficient)."""
    compute_us = np.ascontiguousarray(compute_us, dtype=np.int64).reshape(n_services, n_servers)
    placements = np.ascontiguousarray(placements, dtype=np.int32)
    requests = np.ascontiguousarray(requests, dtype=SIM_REQUEST)
    draws = np.ascontiguousarray(draws, dtype=np.float64).reshape(-1)
    cfg = SimConfig(_ptr(compute_us), int(hop_us), int(sync_delay_us), int(n_servers), int(n_services), int(max_offload), 0)
    res = SimResult()
    _check(lib().epara_simulate(ctypes.addressof(cfg), _ptr(placements) if len(placements) else None, len(placements),
                                _ptr(requests) if len(requests) else None, len(requests),
                                _ptr(draws) if len(draws) else None, ctypes.addressof(res)), "epara_simulate")
    return {k: getattr(res, k) for k, _ in SimResult._fields_}


def epara_schedule_chain(phases, n_workgroups, n_xcd=8, panel_m=8, panel_n=4):
    """phases: list of (groups, classes, n_stream_classes, tiles) -> list of order arrays (one per phase)."""
    keep, arr = [], (PhaseSchedule * max(len(phases), 1))()
    for i, (groups, classes, n_stream, tiles) in enumerate(phases):
        groups = np.ascontiguousarray(groups, dtype=GROUP_DESC)
        classes = np.ascontiguousarray(classes, dtype=TILE_CLASS)
        tiles = np.ascontiguousarray(tiles, dtype=TILE)
        keep.append((groups, classes, tiles))
        arr[i].groups, arr[i].classes, arr[i].tiles, arr[i].order = _ptr(groups), _ptr(classes), _ptr(tiles), None
        arr[i].n_tiles, arr[i].order_cap, arr[i].n_slots = len(tiles), 0, 0
        arr[i].G, arr[i].n_classes, arr[i].n_stream_classes = len(groups), len(classes), int(n_stream)
    args = (len(phases), int(n_workgroups), int(n_xcd), int(panel_m), int(panel_n))
    _check(lib().epara_schedule_chain(ctypes.addressof(arr), *args), "epara_schedule_chain")
    orders = [np.zeros(int(arr[i].n_slots), dtype=np.int32) for i in range(len(phases))]
    for i, o in enumerate(orders):
        arr[i].order, arr[i].order_cap = _ptr(o) if len(o) else None, len(o)
    _check(lib().epara_schedule_chain(ctypes.addressof(arr), *args), "epara_schedule_chain")
    return orders


def epara_chain_waits(producer_tiles, G_producer, counter_base, producer):
    """-> CHAIN_WAIT[len(producer)]."""
    producer_tiles = np.ascontiguousarray(producer_tiles, dtype=TILE)
    producer = np.ascontiguousarray(producer, dtype=np.int32)
    waits = np.zeros(len(producer), dtype=CHAIN_WAIT)
    _check(lib().epara_chain_waits(_ptr(producer_tiles), len(producer_tiles), int(G_producer), int(counter_base),
                                   _ptr(producer), len(producer), _ptr(waits)), "epara_chain_waits")
    return waits


def epara_chain_workspace_bytes(n_counters):
    return int(lib().epara_chain_workspace_bytes(int(n_counters)))


def epara_chain_workspace_init(d_workspace, nbytes, stream):
    _check(lib().epara_chain_workspace_init(int(d_workspace), int(nbytes), stream), "epara_chain_workspace_init")


def epara_grouped_chain(phases, in_dtype, d_workspace, workspace_bytes, stream, spin_limit=0):
    """phases: a ctypes array of ChainPhase (kept alive by the caller)."""
    _check(lib().epara_grouped_chain(ctypes.addressof(phases), len(phases), int(in_dtype), int(d_workspace),
                                     int(workspace_bytes), int(spin_limit), stream), "epara_grouped_chain")


def epara_grouped_chain_static(phases, in_dtype, stream, spin_limit=0, d_flag=0):
    """The chain on the library's own scratch array (no workspace argument).  d_flag: device address of an int32 or 0."""
    _check(lib().epara_grouped_chain_static(ctypes.addressof(phases), len(phases), int(in_dtype), int(spin_limit),
                                            int(d_flag) or None, stream), "epara_grouped_chain_static")


def epara_chain_status(d_workspace, stream):
    flag = np.zeros(1, dtype=np.int32)
    _check(lib().epara_chain_status(int(d_workspace), stream, _ptr(flag)), "epara_chain_status")
    return int(flag[0])


def epara_kernel_classes(in_dtype, gated, narrow=False):
    """-> (classes, n_stream_classes)."""
    n = np.zeros(2, dtype=np.int32)
    classes = np.zeros(8, dtype=TILE_CLASS)
    _check(lib().epara_kernel_classes(int(in_dtype), int(bool(gated)), int(bool(narrow)), _ptr(classes), len(classes),
                                      _ptr(n[0:1]), _ptr(n[1:2])),
           "epara_kernel_classes")
    return classes[: int(n[0])].copy(), int(n[1])


def epara_ffn_swiglu_args(ffn, in_dtype):
    ffn = np.ascontiguousarray(ffn, dtype=FFN_DESC)
    up = np.zeros(len(ffn), dtype=GROUP_ARGS)
    down = np.zeros(len(ffn), dtype=GROUP_ARGS)
    _check(lib().epara_ffn_swiglu_args(_ptr(ffn), len(ffn), int(in_dtype), _ptr(up), _ptr(down)), "epara_ffn_swiglu_args")
    return up, down


def epara_packed_weight_bytes(K, N, dtype):
    return int(lib().epara_packed_weight_bytes(int(K), int(N), int(dtype)))


def epara_pack_weights(d_W, K, N, dtype, d_packed, packed_bytes, stream=0):
    _check(lib().epara_pack_weights(int(d_W), int(K), int(N), int(dtype), int(d_packed), int(packed_bytes),
                                    int(stream) or None), "epara_pack_weights")


def epara_grouped_forward(launch, in_dtype, out_dtype, stream=0):
    _check(lib().epara_grouped_forward(ctypes.addressof(launch), int(in_dtype), int(out_dtype), int(stream) or None),
           "epara_grouped_forward")


def epara_grouped_ffn_swiglu(up, down, in_dtype, h_dtype, out_dtype, stream=0):
    _check(lib().epara_grouped_ffn_swiglu(ctypes.addressof(up), ctypes.addressof(down), int(in_dtype), int(h_dtype),
                                          int(out_dtype), int(stream) or None), "epara_grouped_ffn_swiglu")
