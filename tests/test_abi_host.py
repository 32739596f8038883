"""CPU-side checks of libepara: every symbol the header declares is exported, the C++ planner and
scheduler reproduce the reference planner integer for integer, and bad arguments come back as
status codes (the launch functions validate on the host before touching the device)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import planner as P
from paper_2511_00603_amd import binding as B
from workloads import make_mix

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "epara.h")


def test_library_exports_every_declared_symbol():
    text = open(HEADER).read()
    names = sorted(set(re.findall(r"^(?:int32_t|int64_t|const char\*)\s+(epara_[a-z0-9_]+)\s*\(", text, re.M)))
    assert len(names) >= 12, names
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_struct_sizes_match_header_layout():
    assert B.GROUP_ARGS.itemsize == 72 and B.TILE.itemsize == 24 and B.FFN_DESC.itemsize == 80
    assert ctypes.sizeof(B.Launch) == 88


def _desc(groups, act=0):
    g = np.zeros(len(groups), dtype=B.GROUP_DESC)
    for i, (M, K, N) in enumerate(groups):
        g[i]["M"], g[i]["K"], g[i]["N"], g[i]["act"] = M, K, N, act
    return g


def _classes(cl):
    c = np.zeros(len(cl), dtype=B.TILE_CLASS)
    for i, row in enumerate(cl):
        c[i]["max_M"], c[i]["BM"], c[i]["BN"] = row[:3]
        c[i]["split_K"] = row[3] if len(row) > 3 else 0
    return c


def mix_group_shapes():
    """(M, K, N) lists of every launch of the five mixes, from the seeded structure draws."""
    out = []
    m1 = [4, 16]
    out += [[(m, 256, 512) for m in m1], [(m, 512, 512) for m in m1], [(m, 512, 10) for m in m1]]
    d = [512, 512, 1024, 256, 1024, 256, 256, 512, 1024, 1024, 256, 1024, 256, 256, 1024, 256]
    rows = [6, 4, 9, 11, 5, 7, 7, 8, 8, 4, 14, 7, 4, 4, 6, 8]
    out += [[(r, k, 4 * k) for r, k in zip(rows, d)], [(r, 4 * k, k) for r, k in zip(rows, d)]]
    M3 = [197 * i for i in [32, 16, 1, 8, 4, 4, 2, 8]]
    out += [[(m, 768, 3072) for m in M3], [(m, 768, 2304) for m in M3] + [(m, 3072, 768) for m in M3]]
    out += [[(m, 4096, 11008) for m in (1, 8, 32, 64)], [(m, 11008, 4096) for m in (1, 8, 32, 64)]]
    out += [[(4692, 5120, 13824), (3500, 5120, 13824)], [(4692, 13824, 5120), (3500, 13824, 5120)]]
    return out


ADVERSARIAL = [
    [(1, 8, 10)], [(64, 8, 32), (65, 8, 33)], [(255, 16, 255), (256, 16, 256), (257, 16, 257)],
    [(0, 8, 8), (3, 8, 8), (0, 8, 8)], [(0, 8, 8)], [],
    [(63, 40, 31), (513, 24, 1)], [(1000, 64, 1000), (7, 2048, 77), (300, 128, 300), (64, 512, 64)],
]
# (class table, number of leading weight-streaming classes)
CLASS_TABLES = [([(64, 64, 32), (P.INT32_MAX, 256, 256)], 1), ([(64, 64, 32), (P.INT32_MAX, 256, 128)], 0),
                ([(P.INT32_MAX, 64, 64)], 0), ([(16, 16, 64), (64, 64, 64), (512, 128, 128), (P.INT32_MAX, 256, 256)], 2),
                ([(16, 16, 32), (32, 32, 64), (64, 64, 128), (P.INT32_MAX, 256, 256)], 3),
                ([(16, 16, 16), (32, 32, 32), (64, 64, 64), (P.INT32_MAX, 256, 128)], 4),
                ([(16, 16, 32, 0), (32, 32, 64, 512), (64, 64, 128, 128), (P.INT32_MAX, 256, 256, 0)], 3),
                ([(P.INT32_MAX, 64, 64, 8)], 0), ([(64, 64, 32, 0), (P.INT32_MAX, 256, 256, 1024)], 1)]


@pytest.mark.parametrize("groups", mix_group_shapes() + ADVERSARIAL)
@pytest.mark.parametrize("table", CLASS_TABLES)
def test_planner_and_scheduler_match_reference_bit_for_bit(groups, table):
    classes, n_stream = table
    row_off, x_off, y_off, tiles = P.plan_groups(groups, classes)
    r2, x2, y2, t2 = B.epara_plan_groups(_desc(groups), _classes(classes))
    assert r2.tolist() == row_off and x2.tolist() == x_off and y2.tolist() == y_off
    assert [tuple(int(v) for v in t) for t in t2] == tiles
    for W, X, pm, pn in ((256, 8, 8, 4), (8, 8, 2, 2), (48, 4, 3, 5), (1, 1, 1, 1)):
        for gated in (False, True):
            order = P.schedule_tiles([g + (gated,) for g in groups], classes, n_stream, tiles, W, X, pm, pn)
            o2 = B.epara_schedule_tiles(_desc(groups, 5 if gated else 0), _classes(classes), n_stream, t2, W, X, pm, pn)
            assert o2.tolist() == order


def test_mix_structures_are_the_seeded_draws():
    m2, m3 = make_mix(2), make_mix(3, d=16, ffn=32)          # structure draws do not depend on the widths
    assert [s.M for s in m2.services] == [6, 4, 9, 11, 5, 7, 7, 8, 8, 4, 14, 7, 4, 4, 6, 8]
    assert [s.X.shape[1] for s in m2.services] == [512, 512, 1024, 256, 1024, 256, 256, 512, 1024, 1024, 256, 1024, 256, 256, 1024, 256]
    assert [len(s.request_rows) for s in m3.services] == [32, 16, 1, 8, 4, 4, 2, 8]
    m5 = make_mix(5, d=16, ffn=32)
    assert [s.M for s in m5.services] == [4692, 3500] and m5.requests == 9
    assert m5.services[0].request_rows == [881, 593, 1894, 882, 442]


def status_of(fn, *a):
    try:
        fn(*a)
    except B.EparaError as e:
        return e.status
    return B.EPARA_OK


def test_planner_error_codes():
    cl = _classes(CLASS_TABLES[0][0])
    assert status_of(B.epara_plan_groups, _desc([(1, 0, 4)]), cl) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_plan_groups, _desc([(-1, 4, 4)]), cl) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_plan_groups, _desc([(1, 4, 0)]), cl) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_plan_groups, _desc([(1, 4, 4)]), _classes([(64, 64, 32), (64, 256, 256)])) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_plan_groups, _desc([(1, 4, 4)]), _classes([(64, 0, 32)])) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_plan_groups, _desc([(100, 4, 4)]), _classes([(64, 64, 32)])) == B.EPARA_ERR_SHAPE
    L = B.lib()
    n = np.zeros(1, dtype=np.int64)
    g = _desc([(300, 8, 300)])
    assert L.epara_plan_groups(g.ctypes.data, 1, cl.ctypes.data, 2, None, None, None, None, 0, None) == B.EPARA_ERR_NULL
    assert L.epara_plan_groups(None, 1, cl.ctypes.data, 2, None, None, None, None, 0, n.ctypes.data) == B.EPARA_ERR_NULL
    assert L.epara_plan_groups(g.ctypes.data, 1, None, 2, None, None, None, None, 0, n.ctypes.data) == B.EPARA_ERR_NULL
    assert L.epara_plan_groups(g.ctypes.data, -1, cl.ctypes.data, 2, None, None, None, None, 0, n.ctypes.data) == B.EPARA_ERR_SHAPE
    tiles = np.zeros(2, dtype=B.TILE)
    assert L.epara_plan_groups(g.ctypes.data, 1, cl.ctypes.data, 2, None, None, None, tiles.ctypes.data, 2, n.ctypes.data) == B.EPARA_ERR_CAPACITY
    assert n[0] == 4                                                     # needed size still reported
    assert L.epara_plan_groups(None, 0, cl.ctypes.data, 2, None, None, None, None, 0, n.ctypes.data) == B.EPARA_OK and n[0] == 0
    # scheduler: grid must be a positive multiple of the die count
    _, _, _, t = B.epara_plan_groups(g, cl)
    assert status_of(B.epara_schedule_tiles, g, cl, 1, t, 12, 8) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_schedule_tiles, g, cl, 1, t, 0, 8) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_schedule_tiles, g, cl, 3, t, 8, 8) == B.EPARA_ERR_SHAPE     # more streaming classes than classes
    assert status_of(B.epara_schedule_tiles, g, cl, -1, t, 8, 8) == B.EPARA_ERR_SHAPE
    bad = t.copy(); bad[1]["group"] = 5
    assert status_of(B.epara_schedule_tiles, g, cl, 1, bad, 8, 8) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_schedule_tiles, g, cl, 1, t[:3], 8, 8) == B.EPARA_ERR_SHAPE   # not a whole table


def test_batch_accounting_and_paper_numbers():
    M, first = B.epara_batch_rows([197, 197, 197, 5, 0, 7], [0, 3, 3, 6])
    assert M.tolist() == [591, 0, 12] and first.tolist() == [0, 197, 394, 0, 5, 5]
    assert status_of(B.epara_batch_rows, [1, -2], [0, 2]) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_batch_rows, [1, 2], [0, 2, 1]) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_batch_rows, [2 ** 30, 2 ** 30, 2 ** 30], [0, 3]) == B.EPARA_ERR_SHAPE
    golden = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_numbers.txt")
    for line in open(golden):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, args, expect, _ = [f.strip() for f in line.split(";", 3)]
        a = [int(v) for v in args.split()]
        if name == "dp_group_count":
            assert B.epara_dp_group_count(*a) == int(expect)
        elif name == "inter_request_count":
            assert B.epara_inter_request_count(*a) == int(expect)
    assert B.epara_dp_group_count(1, 0) == -1 and B.epara_inter_request_count(4, 0) == -1


def test_kernel_classes_and_packed_sizes():
    c, ns = B.epara_kernel_classes(B.EPARA_BF16, 0)
    assert [tuple(int(v) for v in x) for x in c] == [(16, 16, 32, 0), (32, 32, 64, 8192), (64, 64, 128, 8192), (P.INT32_MAX, 256, 256, 1024)] and ns == 3
    c, ns = B.epara_kernel_classes(B.EPARA_FP8_E4M3, 1)
    assert [tuple(int(v) for v in x) for x in c] == [(16, 16, 16, 0), (32, 32, 32, 0), (64, 64, 64, 0), (P.INT32_MAX, 256, 128, 0)] and ns == 3   # fp8 tiles are not split
    c, ns = B.epara_kernel_classes(B.EPARA_F32, 0)
    assert [tuple(int(v) for v in x) for x in c] == [(16, 16, 64, 0), (P.INT32_MAX, 64, 64, 0)] and ns == 0
    c, ns = B.epara_kernel_classes(B.EPARA_BF16, 0, narrow=True)
    assert [tuple(int(v) for v in x) for x in c] == [(16, 16, 32, 0), (32, 32, 64, 8192), (64, 64, 64, 8192), (P.INT32_MAX, 256, 256, 1024)] and ns == 3
    assert status_of(B.epara_kernel_classes, B.EPARA_F32, 1) == B.EPARA_ERR_DTYPE
    assert status_of(B.epara_kernel_classes, 7, 0) == B.EPARA_ERR_DTYPE
    assert B.epara_workspace_bytes(_desc([(5, 8, 8)]), B.EPARA_BF16) == 0 and B.epara_workspace_bytes(_desc([]), 9) == -1
    assert B.epara_workspace_bytes(_desc([(5, 8, 8)]), B.EPARA_BF16, 0) == -1 and B.epara_split_workspace_bytes(-1, 0) == -1
    assert B.epara_split_workspace_bytes(3, 2) == 256 + 3 * 4 * 32768 + 2 * 4 * 262144 and B.epara_split_workspace_bytes(0, 0) == 0
    assert B.epara_packed_weight_bytes(4096, 11008, B.EPARA_BF16) == 4096 * 11008 * 2
    assert B.epara_packed_weight_bytes(40, 10, B.EPARA_BF16) == 1 * 4 * 1024          # 2 stages of K, padded to 4
    assert B.epara_packed_weight_bytes(40, 10, B.EPARA_FP8_E4M3) == 4 * 1024
    assert B.epara_packed_weight_bytes(160, 17, B.EPARA_BF16) == 2 * 8 * 1024        # 5 stages -> 8, 2 column blocks
    assert B.epara_packed_weight_bytes(3, 5, B.EPARA_F32) == 60
    assert B.epara_packed_weight_bytes(0, 5, B.EPARA_BF16) == -1 and B.epara_packed_weight_bytes(3, 5, 9) == -1


def test_ffn_args_fill():
    ffn = np.zeros(1, dtype=B.FFN_DESC)
    r = ffn[0]
    r["X"], r["Wgate"], r["Wup"], r["Wdown"], r["H"], r["Y"] = 0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000
    r["M"], r["d_model"], r["d_ff"] = 7, 64, 256
    r["s_x"], r["s_wgate"], r["s_wup"], r["s_h"], r["s_wdown"] = 0.5, 0.25, 2.0, 4.0, 0.125
    up, down = B.epara_ffn_swiglu_args(ffn, B.EPARA_FP8_E4M3)
    assert (up[0]["X"], up[0]["W"], up[0]["W2"], up[0]["Y"]) == (0x1000, 0x2000, 0x3000, 0x5000)
    assert (up[0]["M"], up[0]["K"], up[0]["N"], up[0]["act"]) == (7, 64, 256, B.EPARA_ACT_SWIGLU)
    assert (up[0]["scale"], up[0]["scale2"], up[0]["out_inv_scale"]) == (0.125, 1.0, 0.25)
    assert (down[0]["X"], down[0]["W"], down[0]["Y"]) == (0x5000, 0x4000, 0x6000)
    assert (down[0]["K"], down[0]["N"], down[0]["act"], down[0]["scale"]) == (256, 64, B.EPARA_ACT_NONE, 0.5)
    up, down = B.epara_ffn_swiglu_args(ffn, B.EPARA_BF16)
    assert up[0]["scale"] == 1.0 and down[0]["scale"] == 1.0 and up[0]["out_inv_scale"] == 1.0
    assert status_of(B.epara_ffn_swiglu_args, ffn, B.EPARA_F32) == B.EPARA_ERR_DTYPE
    ffn[0]["s_h"] = 0.0
    assert status_of(B.epara_ffn_swiglu_args, ffn, B.EPARA_FP8_E4M3) == B.EPARA_ERR_SHAPE


def _host_launch(args, tiles, order_len, W=8):
    """A Launch whose device pointers are fake but non-NULL: only the host-side validation is exercised,
    and every case below must be rejected before anything is enqueued."""
    L = B.Launch(args.ctypes.data, 0x1000, tiles.ctypes.data if len(tiles) else None, 0x2000, 0x3000,
                 len(tiles), order_len, W, len(args), None, 0, 0, 0)
    return L


def test_launch_validation_rejects_bad_arguments_without_a_gpu():
    from paper_2511_00603_amd.runtime import group_args
    lib = B.lib()

    class T:   # stand-in for a device tensor
        def __init__(self, p): self.p = p
        def data_ptr(self): return self.p
    mk = lambda **kw: np.array([group_args(T(0x10000), T(0x20000), T(0x30000), kw.pop("M", 100), kw.pop("K", 64), kw.pop("N", 300),
                                           kw.pop("act", "none"), **kw)], dtype=B.GROUP_ARGS)
    cl, _ = B.epara_kernel_classes(B.EPARA_BF16, 0)

    def plan(a):
        g = np.zeros(1, dtype=B.GROUP_DESC)
        for f in ("M", "K", "N"): g[f] = a[f]
        return B.epara_plan_groups(g, cl)[3]

    fwd = lambda L, i=B.EPARA_BF16, o=B.EPARA_BF16: lib.epara_grouped_forward(ctypes.addressof(L), i, o, None)
    a = mk(); t = plan(a)
    assert lib.epara_grouped_forward(None, B.EPARA_BF16, B.EPARA_BF16, None) == B.EPARA_ERR_NULL
    assert fwd(_host_launch(a, t, 8), B.EPARA_BF16, B.EPARA_F32) == B.EPARA_ERR_DTYPE
    assert fwd(_host_launch(a, t, 8), 5, B.EPARA_BF16) == B.EPARA_ERR_DTYPE
    assert fwd(_host_launch(a, t, 8), B.EPARA_F32, B.EPARA_BF16) == B.EPARA_ERR_DTYPE
    assert fwd(_host_launch(a, t, 7)) == B.EPARA_ERR_SHAPE                     # slots not a multiple of the grid
    assert fwd(_host_launch(a, t, 0)) == B.EPARA_ERR_SHAPE                     # fewer slots than tiles
    L = _host_launch(a, t, 8); L.d_order = None
    assert fwd(L) == B.EPARA_ERR_NULL
    L = _host_launch(a, t, 8); L.n_workgroups = 0
    assert fwd(L) == B.EPARA_ERR_SHAPE
    b = mk(); b[0]["X"] = 0
    assert fwd(_host_launch(b, t, 8)) == B.EPARA_ERR_NULL
    b = mk(); b[0]["W"] = 0x20008
    assert fwd(_host_launch(b, t, 8)) == B.EPARA_ERR_ALIGN
    b = mk(K=36); assert fwd(_host_launch(b, plan(b), 8)) == B.EPARA_ERR_ALIGN   # 72-byte rows
    b = mk(K=(1 << 22) + 8); assert fwd(_host_launch(b, plan(b), 8)) == B.EPARA_ERR_SHAPE   # a row longer than 8 MiB
    b = mk(); b[0]["act"] = 9
    assert fwd(_host_launch(b, t, 8)) == B.EPARA_ERR_DTYPE
    b = mk(act="swiglu")                                                         # no second weight matrix
    assert fwd(_host_launch(b, t, 8)) in (B.EPARA_ERR_NULL, B.EPARA_ERR_SHAPE)
    b = mk(); b[0]["K"] = 0
    assert fwd(_host_launch(b, t, 8)) == B.EPARA_ERR_SHAPE
    bad = t.copy(); bad[0]["rows"] = 7
    assert fwd(_host_launch(a, bad, 8)) == B.EPARA_ERR_SHAPE
    bad = t.copy(); bad[1]["n0"] = 250
    assert fwd(_host_launch(a, bad, 8)) == B.EPARA_ERR_SHAPE
    bad = t.copy(); bad[0]["cls"] = 2                                            # 100 rows do not fit a streaming class
    assert fwd(_host_launch(a, bad, 8)) == B.EPARA_ERR_SHAPE
    bad = t.copy(); bad[0]["group"] = 3
    assert fwd(_host_launch(a, bad, 8)) == B.EPARA_ERR_SHAPE
    # nothing to do is fine and touches nothing: no tiles, G = 0
    empty = np.zeros(0, dtype=B.GROUP_ARGS)
    assert fwd(B.Launch(None, None, None, None, None, 0, 0, 8, 0, None, 0, 0, 0)) == B.EPARA_OK
    z = mk(M=0)
    assert fwd(B.Launch(z.ctypes.data, None, None, None, None, 0, 0, 8, 1, None, 0, 0, 0)) == B.EPARA_OK
    # ffn wrapper: dtype rules and phase consistency
    ffn = lambda u, d, i, h, o: lib.epara_grouped_ffn_swiglu(ctypes.addressof(u), ctypes.addressof(d), i, h, o, None)
    e = B.Launch(None, None, None, None, None, 0, 0, 8, 0, None, 0, 0, 0)
    assert ffn(e, e, B.EPARA_BF16, B.EPARA_BF16, B.EPARA_BF16) == B.EPARA_OK
    assert ffn(e, e, B.EPARA_BF16, B.EPARA_FP8_E4M3, B.EPARA_BF16) == B.EPARA_ERR_DTYPE
    assert ffn(e, e, B.EPARA_F32, B.EPARA_F32, B.EPARA_F32) == B.EPARA_ERR_DTYPE
    assert lib.epara_grouped_ffn_swiglu(None, None, 1, 1, 1, None) == B.EPARA_ERR_NULL
    # pack: argument checks come before any enqueue
    assert lib.epara_pack_weights(None, 8, 8, B.EPARA_BF16, 0x1000, 1024, None) == B.EPARA_ERR_NULL
    assert lib.epara_pack_weights(0x1000, 8, 8, B.EPARA_BF16, 0x2000, 16, None) == B.EPARA_ERR_CAPACITY
    assert lib.epara_pack_weights(0x1000, 0, 8, B.EPARA_BF16, 0x2000, 1024, None) == B.EPARA_ERR_SHAPE
    assert lib.epara_pack_weights(0x1000, 8, 8, 7, 0x2000, 1024, None) == B.EPARA_ERR_DTYPE
    assert lib.epara_pack_weights(0x1000, 8, 8, B.EPARA_BF16, 0x2004, 4096, None) == B.EPARA_ERR_ALIGN
    assert B.epara_status_string(B.EPARA_ERR_ALIGN).startswith("pointer")


# ---- chains of launches ------------------------------------------------------------------------

def _chains():
    """(phases, gated flags): consecutive launches of the mixes that form chains, plus adversarial ones."""
    shapes = mix_group_shapes()
    wide = ([(16, 16, 32), (32, 32, 64), (64, 64, 128), (P.INT32_MAX, 256, 256)], 3)
    gatedt = ([(16, 16, 16), (32, 32, 32), (64, 64, 64), (P.INT32_MAX, 256, 128)], 3)
    narrow = ([(16, 16, 32), (32, 32, 64), (64, 64, 64), (P.INT32_MAX, 256, 256)], 3)
    f32 = ([(P.INT32_MAX, 64, 64)], 0)
    return [
        ([(shapes[0], f32, False), (shapes[1], f32, False), (shapes[2], f32, False)]),
        ([(shapes[3], wide, False), (shapes[4], wide, False)]),
        ([(shapes[5], wide, False), (shapes[6], wide, False)]),
        ([(shapes[7], gatedt, True), (shapes[8], narrow, False)]),
        ([(shapes[7], gatedt, True), (shapes[8], wide, False)]),
        ([(shapes[9], gatedt, True), (shapes[10], wide, False)]),
        ([([(0, 8, 8)], wide, False), ([], wide, False)]),
        ([([(63, 40, 31), (513, 24, 1)], wide, False), ([(63, 31, 77), (513, 1, 300)], narrow, False),
          ([(63, 77, 5), (7, 300, 64)], wide, False), ([(63, 5, 40)], wide, False)]),
    ]


@pytest.mark.parametrize("chain", _chains())
def test_chain_scheduler_matches_reference_and_covers_every_tile_once(chain):
    ref_phases, lib_phases = [], []
    for groups, (classes, n_stream), gated in chain:
        _, _, _, tiles = P.plan_groups(groups, classes)
        ref_phases.append(([g + (gated,) for g in groups], classes, n_stream, tiles))
        t2 = np.array(tiles, dtype=B.TILE) if tiles else np.zeros(0, dtype=B.TILE)
        lib_phases.append((_desc(groups, 5 if gated else 0), _classes(classes), n_stream, t2))
    for W, X, pm, pn in ((256, 8, 1, 4), (8, 8, 2, 2), (48, 4, 3, 5), (1, 1, 1, 1)):
        ref = P.schedule_chain(ref_phases, W, X, pm, pn)
        got = B.epara_schedule_chain(lib_phases, W, X, pm, pn)
        assert [o.tolist() for o in got] == ref
        # what any valid schedule must satisfy, whatever the rule: every tile of every phase exactly once,
        # lists without holes, and (streaming-only chains) the greedy bound max <= mean + largest tile
        total = np.zeros(W, dtype=np.int64)
        biggest, stream_only = 0, True
        for (groups, classes, n_stream, tiles), order in zip(ref_phases, ref):
            o = np.array(order, dtype=np.int64).reshape(-1, W) if order else np.zeros((0, W), dtype=np.int64)
            assert sorted(o[o >= 0].tolist()) == list(range(len(tiles)))
            for b in range(W):
                col = o[:, b]
                assert np.all(col[: int((col >= 0).sum())] >= 0)
                for t in col[col >= 0]:
                    tile = tiles[t]
                    if tile[5] < n_stream:
                        g = groups[tile[0]]
                        c = g[1] * (6 * tile[4] * (2 if g[3] else 1) + (2 * classes[tile[5]][1] if classes[tile[5]][1] >= 32 else 0))
                    else:
                        c, stream_only = 2040 * groups[tile[0]][1], False
                    total[b] += c
                    biggest = max(biggest, c)
        if stream_only and total.sum() > 0:
            assert total.max() <= total.sum() / W + biggest


def test_single_phase_chain_is_the_plain_schedule():
    groups = [(1000, 64, 1000), (7, 2048, 77), (300, 128, 300), (64, 512, 64)]
    classes, n_stream = CLASS_TABLES[4]
    _, _, _, tiles = B.epara_plan_groups(_desc(groups), _classes(classes))
    a = B.epara_schedule_tiles(_desc(groups), _classes(classes), n_stream, tiles, 48, 4, 3, 5)
    b = B.epara_schedule_chain([(_desc(groups), _classes(classes), n_stream, tiles)], 48, 4, 3, 5)[0]
    assert a.tolist() == b.tolist()


def test_chain_balances_a_coarse_phase_against_a_fine_one():
    """Decode-like FFN shapes (K short enough that no tile is split) with the wide table in the down phase: alone,
    its 32 widest tiles are all their owners get and twice the mean; scheduled together with the up phase the
    loads even out."""
    up, down = [(m, 4000, 4096) for m in (1, 8, 32, 64)], [(m, 4000, 4096) for m in (1, 8, 32, 64)]
    gt, nt = [(16, 16, 16), (32, 32, 32), (64, 64, 64), (P.INT32_MAX, 256, 128)], [(16, 16, 32), (32, 32, 64), (64, 64, 128), (P.INT32_MAX, 256, 256)]
    tu, td = P.plan_groups(up, gt)[3], P.plan_groups(down, nt)[3]
    phases = [([g + (True,) for g in up], gt, 3, tu), ([g + (False,) for g in down], nt, 3, td)]

    def loads(phase_list, orders):
        total = np.zeros(256, dtype=np.int64)
        for (groups, classes, _, tiles), order in zip(phase_list, orders):
            for slot, t in enumerate(order):
                if t >= 0:
                    g = groups[tiles[t][0]]
                    total[slot % 256] += g[1] * (6 * tiles[t][4] * (2 if g[3] else 1) + (2 * classes[tiles[t][5]][1] if classes[tiles[t][5]][1] >= 32 else 0))
        return total
    # separate launches: a launch boundary is a barrier, the maxima of the phases add up
    alone = [loads([ph], [P.schedule_tiles(*ph, 256, 8, 1, 4)]) for ph in phases]
    joint = loads(phases, P.schedule_chain(phases, 256, 8, 1, 4))
    assert sum(a.sum() for a in alone) == joint.sum()
    assert sum(a.max() for a in alone) / joint.mean() > 1.3
    assert joint.max() / joint.mean() < 1.05


def test_chain_waits_match_reference_and_reject_bad_indices():
    groups = [(63, 40, 31), (0, 8, 8), (513, 24, 1), (7, 8, 300)]
    classes, _ = CLASS_TABLES[4]
    _, _, _, tiles = B.epara_plan_groups(_desc(groups), _classes(classes))
    producer = [2, -1, 0, 3, 1, 0]
    w = B.epara_chain_waits(tiles, len(groups), 10, producer)
    ref = P.chain_waits([tuple(int(v) for v in t) for t in tiles], 10, producer)
    assert [(int(a["counter"]), int(a["need"])) for a in w] == ref
    # counted independently: tiles per group from the grid rule
    per = {g: -(-M // (16 if M <= 16 else 32 if M <= 32 else 64 if M <= 64 else 256)) * -(-N // {16: 32, 32: 64, 64: 128, 256: 256}[16 if M <= 16 else 32 if M <= 32 else 64 if M <= 64 else 256])
           for g, (M, K, N) in enumerate(groups) if M}
    assert ref[0] == (12, per[2]) and ref[1] == (-1, 0) and ref[4] == (11, 0) and ref[3] == (13, per[3])
    assert status_of(B.epara_chain_waits, tiles, len(groups), 0, [4]) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_chain_waits, tiles, len(groups), 0, [-2]) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_chain_waits, tiles, len(groups), -1, [0]) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_chain_waits, tiles, 2, 0, [0]) == B.EPARA_ERR_SHAPE       # a tile of group 2 or 3 is outside


def test_chain_entry_point_validates_before_touching_the_device():
    L = B.lib()
    assert B.epara_chain_workspace_bytes(0) == 256 and B.epara_chain_workspace_bytes(100) == 512
    assert B.epara_chain_workspace_bytes(-1) == -1
    ws = ctypes.c_void_p(4096)
    assert L.epara_grouped_chain(None, 1, B.EPARA_BF16, ws, 256, 0, None) == B.EPARA_ERR_NULL
    phases = (B.ChainPhase * 1)()
    assert L.epara_grouped_chain(ctypes.addressof(phases), 0, B.EPARA_BF16, ws, 256, 0, None) == B.EPARA_ERR_SHAPE
    assert L.epara_grouped_chain(ctypes.addressof(phases), 5, B.EPARA_BF16, ws, 256, 0, None) == B.EPARA_ERR_SHAPE
    assert L.epara_grouped_chain(ctypes.addressof(phases), 1, B.EPARA_BF16, ws, 256, 0, None) == B.EPARA_ERR_NULL   # no launch
    assert L.epara_grouped_chain(ctypes.addressof(phases), 1, B.EPARA_BF16, ctypes.c_void_p(4100), 256, 0, None) == B.EPARA_ERR_ALIGN
    empty = B.Launch(None, None, None, None, None, 0, 0, 0, 0, None, 0, 0, 0)
    phases[0].launch = ctypes.pointer(empty)
    phases[0].out_dtype = B.EPARA_BF16
    assert L.epara_grouped_chain(ctypes.addressof(phases), 1, B.EPARA_BF16, ws, 16, 0, None) == B.EPARA_ERR_CAPACITY
    assert L.epara_grouped_chain(ctypes.addressof(phases), 1, B.EPARA_BF16, ws, 256, 0, None) == B.EPARA_OK          # nothing to run
    assert L.epara_chain_workspace_init(None, 256, None) == B.EPARA_ERR_NULL
    assert L.epara_chain_status(None, None, None) == B.EPARA_ERR_NULL


def test_chain_rejects_produced_tensors_that_do_not_own_their_cache_lines():
    """A consumer invalidates nothing after its wait, so a tensor that is waited for must start on a 128-byte
    line and nothing else of the chain may overlap the rest of its last line.  Host-side validation only:
    every case is rejected before anything is enqueued (K = N = 72 bf16, M = 3 is 432 bytes, as when groups
    are packed back to back with the planner's y_off)."""
    L = B.lib()

    def chain(y_a, y_b, x_b_of):
        a0 = np.zeros(2, dtype=B.GROUP_ARGS)                  # phase 0: two groups that write Y_A, Y_B
        a1 = np.zeros(2, dtype=B.GROUP_ARGS)                  # phase 1: each reads one of them
        for g, y in enumerate((y_a, y_b)):
            a0[g]["X"], a0[g]["W"], a0[g]["Y"] = 0x100000 + 0x1000 * g, 0x200000 + 0x10000 * g, y
            a0[g]["M"], a0[g]["K"], a0[g]["N"], a0[g]["scale"] = 3, 72, 72, 1.0
            a1[g]["X"], a1[g]["W"], a1[g]["Y"] = x_b_of[g], 0x300000 + 0x10000 * g, 0x400000 + 0x1000 * g
            a1[g]["M"], a1[g]["K"], a1[g]["N"], a1[g]["scale"] = 3, 72, 72, 1.0
        classes, _ = B.epara_kernel_classes(B.EPARA_BF16, False)
        keep, phases = [], (B.ChainPhase * 2)()
        for p, a in enumerate((a0, a1)):
            d = np.zeros(2, dtype=B.GROUP_DESC)
            for f in ("M", "K", "N"):
                d[f] = a[f]
            _, _, _, tiles = B.epara_plan_groups(d, classes)
            launch = _host_launch(a, tiles, 8 * len(tiles), 8)
            keep += [a, tiles, launch]
            phases[p].launch = ctypes.pointer(launch)
            phases[p].out_dtype, phases[p].counter_base = B.EPARA_BF16, 2 * p
        waits = B.epara_chain_waits(keep[1], 2, 0, [0, 1])
        keep.append(waits)
        phases[1].h_waits, phases[1].d_waits = waits.ctypes.data, 0x5000
        return L.epara_grouped_chain(ctypes.addressof(phases), 2, B.EPARA_BF16, ctypes.c_void_p(0x6000), 16, 0, None), keep

    # Y_B begins in the last line of Y_A (432 bytes after it): rejected; so is a produced tensor that starts off a line
    assert chain(0x500000, 0x500000 + 432, [0x500000, 0x500000 + 432])[0] == B.EPARA_ERR_ALIGN
    assert chain(0x500000 + 64, 0x510000, [0x500000 + 64, 0x510000])[0] == B.EPARA_ERR_ALIGN
    # tensors on lines of their own pass this check and reach the next one (the workspace given here is too
    # small on purpose, so that nothing is ever enqueued with these made-up addresses)
    assert chain(0x500000, 0x510000, [0x500000, 0x510000])[0] == B.EPARA_ERR_CAPACITY


def _launches_by_mix():
    s = mix_group_shapes()          # launches in mix order: 3 of mix 1, 2 of mix 2, 2 of mix 3, 2 of mix 4, 2 of mix 5
    return {1: [(s[0], False), (s[1], False), (s[2], False)], 2: [(s[3], False), (s[4], False)], 3: [(s[5], False), (s[6], False)],
            4: [(s[7], True), (s[8], False)], 5: [(s[9], True), (s[10], False)]}


LAUNCHES = _launches_by_mix()


def _ref_cost(group, tile, classes, n_stream, gated, parts=1):
    if tile[5] >= n_stream:
        return 2040 * group[1] if parts == 1 else 2040 * group[1] // parts + 1020000
    bm = classes[tile[5]][1]
    whole = group[1] * (6 * tile[4] * (2 if gated else 1) + (2 * bm if bm >= 32 else 0))
    return whole if parts == 1 else whole // parts + 24 * bm * tile[4] * (2 if gated else 1)


def _visits(order, tiles, groups, classes, n_stream, W=256, gated=False):
    """Checks that a visit order holds every tile the right number of times, each part once."""
    n_panel, panel_parts, panel_more = P.panel_split([g + (gated,) for g in groups], classes, n_stream, W)
    seen = {}
    for e in order:
        if e >= 0:
            t, part, parts = P.order_decode(int(e))
            seen.setdefault(t, []).append((part, parts))
    assert sorted(seen) == list(range(len(tiles)))
    for t, v in seen.items():
        tile = tiles[t]
        want = P.split_parts(groups[tile[0]][1], classes[tile[5]]) if tile[5] < n_stream else (
            1 if t < len(tiles) - n_panel else panel_parts + (1 if t >= len(tiles) - panel_more else 0))
        assert sorted(v) == [(j, want) for j in range(want)]


@pytest.mark.parametrize("index,dtype", [(4, B.EPARA_BF16), (5, B.EPARA_BF16), (3, B.EPARA_BF16), (2, B.EPARA_BF16), (1, B.EPARA_F32), (4, B.EPARA_FP8_E4M3)])
def test_plan_launch_is_a_valid_plan_and_makes_the_choice_the_header_states(index, dtype):
    """epara_plan_launch on the launches of the benchmark mixes (shapes only).  What any plan must satisfy: the
    tiles partition every group, the order holds every tile once, lists have no holes.  The choice between the
    wide and the narrow table and the integers of the chosen plan are also compared with the reference planner
    run on both tables under the cost model of the header (a transcription check: the same rule typed twice)."""
    W = 256
    for groups, gated in LAUNCHES[index]:
        info, row_off, x_off, y_off, tiles, order, split_base = B.epara_plan_launch(_desc(groups, 5 if gated else 0), dtype, W, 8, 1, 4)
        classes = [tuple(int(v) for v in c) for c in info.class_table()]
        # validity
        cover = {g: np.zeros((M, N), dtype=np.int32) for g, (M, K, N) in enumerate(groups) if M}
        for t in tiles:
            cover[int(t["group"])][t["m0"]: t["m0"] + t["rows"], t["n0"]: t["n0"] + t["cols"]] += 1
        assert all(np.all(c == 1) for c in cover.values())
        o = order.reshape(-1, W)
        _visits(order.tolist(), [tuple(int(v) for v in t) for t in tiles], groups, classes, info.n_stream_classes, W, gated)
        ref_base, ref_n, _ = P.split_layout(groups, classes, info.n_stream_classes)
        ref_panel, ref_parts, ref_more = P.panel_split([g + (gated,) for g in groups], classes, info.n_stream_classes, W)
        assert (split_base.tolist(), info.n_split_tiles, info.n_panel_split_tiles) == (ref_base, ref_n, ref_panel)
        assert info.workspace_bytes == P.split_workspace_bytes(ref_n, ref_panel) == B.epara_split_workspace_bytes(ref_n, ref_panel)
        assert B.epara_panel_split(_desc(groups, 5 if gated else 0), _classes(classes), info.n_stream_classes, W) == (ref_panel, ref_parts, ref_more)
        if index == 5 and not gated and dtype == B.EPARA_BF16:
            # 660 tiles on 256 workgroups: the last 148 in 512 parts, two per workgroup: 80 tiles in three, 68 in four
            assert (ref_panel, ref_parts, ref_more) == (148, 3, 68)
        for b in range(W):
            col = o[:, b]
            assert np.all(col[: int((col >= 0).sum())] >= 0)
        assert row_off[-1] == sum(g[0] for g in groups)
        # the choice
        best = None
        big = dtype != B.EPARA_F32 and max(g[0] for g in groups) > 32
        for narrow in ((0, 1) if big else (0,)):
            cls, n_stream = B.epara_kernel_classes(dtype, gated, bool(narrow))
            cls = [tuple(int(v) for v in c) for c in cls]
            _, _, _, rt = P.plan_groups(groups, cls)
            ro = P.schedule_tiles([g + (gated,) for g in groups], cls, n_stream, rt, W, 8, 1, 4)
            dec = [P.order_decode(e) if e >= 0 else None for e in ro]
            loads = [sum(_ref_cost(groups[rt[d[0]][0]], rt[d[0]], cls, n_stream, gated, d[2]) for d in dec[b::W] if d) for b in range(W)]
            if best is None or max(loads) < best[0]:
                best = (max(loads), narrow, cls, rt, ro)
        assert (info.makespan, info.narrow, classes) == best[:3]
        assert [tuple(int(v) for v in t) for t in tiles] == best[3] and order.tolist() == best[4]


def test_plan_chain_picks_tables_jointly_and_writes_waits():
    """epara_plan_chain on the decode FFN (gate/up then down): both phases may take either table; whatever it
    picks, the plan is valid, the waits are those of epara_chain_waits, and no other combination finishes
    earlier under the replay the header describes (run here by the reference scheduler)."""
    W = 256
    up, down = [(m, 4096, 11008) for m in (1, 8, 32, 64)], [(m, 11008, 4096) for m in (1, 8, 32, 64)]
    finish, phases = B.epara_plan_chain([_desc(up, 5), _desc(down, 0)], [None, [0, 1, 2, 3]], B.EPARA_BF16, W, 8, 1, 4)
    assert [ph["counter_base"] for ph in phases] == [0, 4]
    want = B.epara_chain_waits(phases[0]["tiles"], 4, 0, [0, 1, 2, 3])
    assert phases[1]["waits"].tolist() == want.tolist() and phases[0]["waits"] is None
    for ph, groups in zip(phases, (up, down)):
        o = ph["order"].reshape(-1, W)
        assert sorted(o[o >= 0].tolist()) == list(range(len(ph["tiles"])))

    def replay(picks):
        ref_phases = []
        for groups, gated, narrow in ((up, True, picks[0]), (down, False, picks[1])):
            cls, n_stream = B.epara_kernel_classes(B.EPARA_BF16, gated, bool(narrow))
            cls = [tuple(int(v) for v in c) for c in cls]
            ref_phases.append(([g + (gated,) for g in groups], cls, n_stream, P.plan_groups(groups, cls)[3]))
        orders = P.schedule_chain(ref_phases, W, 8, 1, 4)
        clock, ready_prev = [0] * W, None
        for p, ((groups, cls, n_stream, tiles), order) in enumerate(zip(ref_phases, orders)):
            ready = [0] * len(groups)
            for slot, t in enumerate(order):
                if t < 0:
                    continue
                b, g = slot % W, tiles[t][0]
                start = max(clock[b], ready_prev[g]) if p else clock[b]
                clock[b] = start + _ref_cost(groups[g], tiles[t], cls, n_stream, groups[g][3])
                ready[g] = max(ready[g], clock[b])
            ready_prev = ready
        return max(clock)

    all_finishes = {picks: replay(picks) for picks in ((0, 0), (0, 1), (1, 0), (1, 1))}
    assert finish == min(all_finishes.values())
    assert all_finishes[(int(phases[0]["info"].narrow), int(phases[1]["info"].narrow))] == finish


def test_fast_gelu_constants_hold_their_stated_error():
    """The 16- and 8-bit epilogues take the erf form of GELU as z / (1 + 2^(z p(min(z^2, 64)))) with three fitted
    coefficients; the kernel source states |error| < 2.6e-5.  Read the coefficients from the source, evaluate the
    same expression in fp32 and compare with the oracle's GELU over [-20, 20]."""
    import os
    import re
    from oracle import reference as ref
    src = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2511_00603_amd", "csrc", "epara_device.h")).read()
    m = re.search(r"const float u = z \* \((-?[0-9.e-]+)f \+ z2 \* \((-?[0-9.e-]+)f \+ z2 \* (-?[0-9.e-]+)f\)\);", src)
    assert m, "the expression of the fast GELU has changed: update this test with it"
    k0, k1, k2 = (np.float32(v) for v in m.groups())
    z = np.linspace(-20, 20, 200001).astype(np.float32)
    z2 = np.minimum(z * z, np.float32(64))
    u = (z * (k0 + z2 * (k1 + z2 * k2))).astype(np.float32)
    with np.errstate(over="ignore"):
        got = (z / (np.float32(1) + np.exp2(u))).astype(np.float32)
    want = ref.dense_forward(z.astype(np.float64).reshape(-1, 1), np.ones((1, 1)), None, "gelu_erf")[:, 0]
    assert np.all(np.isfinite(got)) and float(np.max(np.abs(got - want))) < 2.6e-5


def test_split_launch_validation_without_a_gpu():
    """A launch whose tiles are visited in parts must bring the layout the library computes and a workspace that holds it;
    every case is rejected on the host, before anything is enqueued."""
    from paper_2511_00603_amd.runtime import group_args
    lib = B.lib()

    class T:
        def __init__(self, p): self.p = p
        def data_ptr(self): return self.p
    groups = [(64, 11008, 4096), (8, 11008, 4096), (32, 8192, 256)]
    g = _desc(groups)
    info, _, _, _, tiles, order, base = B.epara_plan_launch(g, B.EPARA_BF16, 256)
    assert info.n_split_tiles > 0 and info.workspace_bytes == 256 * -(-info.n_split_tiles * 4 // 256) + info.n_split_tiles * 4 * 32768
    assert base.tolist()[1] == -1 and base.tolist()[0] == 0 and base.tolist()[2] > 0
    assert B.epara_workspace_bytes(g, B.EPARA_BF16) >= info.workspace_bytes and B.epara_workspace_bytes(g, B.EPARA_FP8_E4M3) == 0
    args = np.array([group_args(T(0x100000), T(0x200000), T(0x300000), M, K, N, "none") for M, K, N in groups], dtype=B.GROUP_ARGS)
    args["reserved"] = base

    def launch(ws=0x7000000, ws_bytes=None, n_split=None, a=args):
        return B.Launch(a.ctypes.data, 0x1000, tiles.ctypes.data, 0x2000, 0x3000, len(tiles), len(order), 256, len(a),
                        ws, info.workspace_bytes if ws_bytes is None else ws_bytes, info.n_split_tiles if n_split is None else n_split, 0)
    fwd = lambda L, i=B.EPARA_BF16: lib.epara_grouped_forward(ctypes.addressof(L), i, B.EPARA_BF16, None)
    assert fwd(launch(ws=None)) == B.EPARA_ERR_NULL
    assert fwd(launch(ws=0x7000010)) == B.EPARA_ERR_ALIGN
    assert fwd(launch(ws_bytes=info.workspace_bytes - 1)) == B.EPARA_ERR_CAPACITY
    assert fwd(launch(n_split=info.n_split_tiles - 1)) == B.EPARA_ERR_SHAPE
    assert fwd(launch(n_split=-1)) == B.EPARA_ERR_SHAPE
    bad = args.copy(); bad["reserved"][2] = 0
    assert fwd(launch(a=bad)) == B.EPARA_ERR_SHAPE                                   # a group's slots are not where the layout puts them
    assert fwd(launch(), B.EPARA_FP8_E4M3) in (B.EPARA_ERR_SHAPE, B.EPARA_ERR_ALIGN)   # fp8 launches have no split tiles
    # a chain takes no launch with split tiles
    ph = (B.ChainPhase * 1)()
    L = launch()
    ph[0].launch, ph[0].out_dtype = ctypes.pointer(L), B.EPARA_BF16
    assert lib.epara_grouped_chain(ph, 1, B.EPARA_BF16, ctypes.c_void_p(0x9000000), 1 << 20, 0, None) == B.EPARA_ERR_SHAPE
    # the workspace's own entry point
    assert lib.epara_workspace_init(None, 256, None) == B.EPARA_ERR_NULL
    assert lib.epara_workspace_init(ctypes.c_void_p(0x7000004), 256, None) == B.EPARA_ERR_ALIGN


def test_panel_split_decision_and_its_error_paths():
    """epara_panel_split against the reference on the launches of the mixes and on shapes around the rule's edges
    (a full last round, a K below the class's split_K, gated groups, two different K, a streaming group next to
    the panel groups), for several grid sizes; then the argument checks."""
    cls, ns = B.epara_kernel_classes(B.EPARA_BF16, 0)
    table = [tuple(int(v) for v in c) for c in cls]
    cases = [g for g, gated in sum(LAUNCHES.values(), []) if not gated] + [
        [(256 * 16, 2048, 256 * 16)], [(256 * 16, 1023, 256 * 17)], [(256 * 16, 1024, 256 * 17)], [(300, 4096, 300), (300, 2048, 300)],
        [(300, 4096, 300), (8, 4096, 300)], [(0, 4096, 300)], [], [(100000, 8192, 256)]]
    for groups in cases:
        for W in (256, 8, 24, 1):
            assert B.epara_panel_split(_desc(groups), cls, ns, W) == P.panel_split(groups, table, ns, W), (groups, W)
    gcls, gns = B.epara_kernel_classes(B.EPARA_BF16, 1)
    assert B.epara_panel_split(_desc([(4692, 13824, 5120)], 5), gcls, gns, 256) == (0, 1, 0)       # gated groups are not split
    fcls, fns = B.epara_kernel_classes(B.EPARA_FP8_E4M3, 0)
    assert B.epara_panel_split(_desc([(4692, 13824, 5120), (3500, 13824, 5120)]), fcls, fns, 256) == (0, 1, 0)   # nor fp8 ones
    assert B.epara_panel_split(_desc([(4692, 13824, 5120), (3500, 13824, 5120)]), cls, ns, 256) == (148, 3, 68)
    g = _desc([(300, 4096, 300)])
    assert status_of(B.epara_panel_split, g, cls, ns, 0) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_panel_split, g, cls, 9, 8) == B.EPARA_ERR_SHAPE
    assert status_of(B.epara_panel_split, _desc([(300, 0, 300)]), cls, ns, 8) == B.EPARA_ERR_SHAPE
    n, parts, more = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    assert B.lib().epara_panel_split(g.ctypes.data, 1, cls.ctypes.data, len(cls), ns, 8, None, ctypes.byref(parts), ctypes.byref(more)) == B.EPARA_ERR_NULL
    assert B.lib().epara_panel_split(g.ctypes.data, 1, cls.ctypes.data, len(cls), ns, 8, ctypes.byref(n), ctypes.byref(parts), None) == B.EPARA_ERR_NULL
    assert B.lib().epara_panel_split(None, 1, cls.ctypes.data, len(cls), ns, 8, ctypes.byref(n), ctypes.byref(parts), ctypes.byref(more)) == B.EPARA_ERR_NULL


def test_block_pieces_argument_checks():
    """epara_add_layernorm and epara_attention validate the host copy of their arguments before anything is enqueued
    (every case here returns before a launch: an error, or no rows at all)."""
    L = B.lib()
    D = 0x7000000                                    # a pretend device address: never dereferenced on these paths

    def norm(**kw):
        a = np.zeros(1, dtype=B.NORM_ARGS)
        a[0] = (D, D + 0x10000, D + 0x20000, D + 0x30000, D + 0x40000, D + 0x50000, 4, 768, 1e-6, 0)
        for k, v in kw.items():
            a[0][k] = v
        return L.epara_add_layernorm(a.ctypes.data, ctypes.c_void_p(D + 0x60000), 1, None)

    assert struct_bytes(B.NORM_ARGS) == 64 and struct_bytes(B.ATTN_ARGS) == 40
    assert L.epara_add_layernorm(None, None, 0, None) == B.EPARA_OK
    assert L.epara_add_layernorm(None, None, -1, None) == B.EPARA_ERR_SHAPE
    assert L.epara_add_layernorm(None, ctypes.c_void_p(D), 1, None) == B.EPARA_ERR_NULL
    a = np.zeros(1, dtype=B.NORM_ARGS)
    assert L.epara_add_layernorm(a.ctypes.data, None, 1, None) == B.EPARA_ERR_NULL
    assert norm(M=0) == B.EPARA_OK                                      # no rows: nothing to enqueue
    assert norm(M=0, X=0, Y=0, gamma=0, beta=0) == B.EPARA_OK           # and nothing to point to
    for bad in (dict(M=-1), dict(d=0), dict(d=4), dict(d=12), dict(d=B.EPARA_NORM_MAX_D + 8), dict(eps=-1.0), dict(eps=np.inf),
                dict(eps=np.nan), dict(first_row=1)):
        assert norm(**bad) == B.EPARA_ERR_SHAPE, bad
    for missing in ("X", "gamma", "beta", "Y"):
        assert norm(**{missing: 0}) == B.EPARA_ERR_NULL, missing
    for field in ("X", "R", "S", "Y", "gamma", "beta"):
        assert norm(**{field: D + 8}) == B.EPARA_ERR_ALIGN, field
    # first_row is the running sum over the groups
    two = np.zeros(2, dtype=B.NORM_ARGS)
    two[0] = (D, 0, D + 0x20000, D + 0x30000, 0, D + 0x50000, 0, 768, 1e-6, 0)
    two[1] = (D, 0, D + 0x20000, D + 0x30000, 0, D + 0x50000, 0, 64, 0.0, 0)
    assert L.epara_add_layernorm(two.ctypes.data, ctypes.c_void_p(D), 2, None) == B.EPARA_OK
    two[1]["first_row"] = 5
    assert L.epara_add_layernorm(two.ctypes.data, ctypes.c_void_p(D), 2, None) == B.EPARA_ERR_SHAPE

    def attn(**kw):
        a = np.zeros(1, dtype=B.ATTN_ARGS)
        a[0] = (D, D + 0x100000, 2 * 197, 197, 12, 64, 0, 0)
        for k, v in kw.items():
            a[0][k] = v
        return L.epara_attention(a.ctypes.data, ctypes.c_void_p(D + 0x200000), 1, None)

    assert L.epara_attention(None, None, 0, None) == B.EPARA_OK
    assert L.epara_attention(None, None, -1, None) == B.EPARA_ERR_SHAPE
    assert L.epara_attention(None, ctypes.c_void_p(D), 1, None) == B.EPARA_ERR_NULL
    assert attn(M=0) == B.EPARA_OK and attn(M=0, QKV=0, O=0) == B.EPARA_OK
    for bad in (dict(M=-197), dict(M=198), dict(tokens=0), dict(tokens=B.EPARA_ATTN_MAX_TOKENS + 1, M=B.EPARA_ATTN_MAX_TOKENS + 1),
                dict(heads=0), dict(head_dim=32), dict(head_dim=128), dict(first_item=1), dict(O=D)):
        assert attn(**bad) == B.EPARA_ERR_SHAPE, bad
    assert attn(QKV=0) == B.EPARA_ERR_NULL and attn(O=0) == B.EPARA_ERR_NULL
    assert attn(QKV=D + 8) == B.EPARA_ERR_ALIGN and attn(O=D + 0x100008) == B.EPARA_ERR_ALIGN
    two = np.zeros(2, dtype=B.ATTN_ARGS)
    two[0] = (D, D + 0x100000, 0, 197, 12, 64, 0, 0)
    two[1] = (D, D + 0x100000, 0, 50, 3, 64, 0, 0)
    assert L.epara_attention(two.ctypes.data, ctypes.c_void_p(D), 2, None) == B.EPARA_OK
    two[1]["first_item"] = 24
    assert L.epara_attention(two.ctypes.data, ctypes.c_void_p(D), 2, None) == B.EPARA_ERR_SHAPE


def struct_bytes(dtype):
    return dtype.itemsize
