"""Batch forming (the step before and after the grouped forward): pins of the numpy reference
(oracle/rows.py, oracle/planner.request_segments) and the host half of the library against it."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import planner as P
from oracle import reference as ref
from oracle import rows as RW
from paper_2511_00603_amd import binding as B


# ---- the reference against things it does not define itself ---------------------------------------

def test_gather_is_concatenation_and_scatter_inverts_it():
    rng = np.random.default_rng(31)
    reqs = [[rng.standard_normal((r, 24)).astype(np.float32) for r in (3, 0, 5, 1)],
            [rng.standard_normal((r, 8)).astype(np.float32) for r in (7,)],
            []]
    X = RW.gather(reqs)
    assert X[2] is None and X[0].shape == (9, 24) and X[1].shape == (7, 8)
    assert np.array_equal(X[0][3:8], reqs[0][2]) and np.array_equal(X[0][8:], reqs[0][3])
    back = RW.scatter(X[0], [3, 0, 5, 1])
    for a, b in zip(back, reqs[0]):
        assert np.array_equal(a, b)
    # the first rows are the ones the batch accounting gives
    _M, first = P.batch_rows([[3, 0, 5, 1], [7], []])
    assert first[0] == [0, 3, 3, 8]
    with pytest.raises(ValueError):
        RW.scatter(X[0], [3, 5])


def test_scale_closed_forms():
    assert RW.amax_scale(np.zeros((4, 4), np.float32)) == (0.0, 1.0)
    assert RW.amax_scale(np.zeros((0, 4), np.float32)) == (0.0, 1.0)
    a, s = RW.amax_scale(np.array([[-896.0, 3.0]], np.float32))
    assert a == 896.0 and s == 2.0
    x = np.array([896.0, -896.0, 2.0, 0.0, 1.0, -3.5, 2.0 ** -8], np.float32)     # / 2: 448, -448, 1, 0, .5, -1.75, 2^-9
    assert RW.quantize_e4m3(x, s).tolist() == [0x7e, 0xfe, 0x38, 0x00, 0x30, 0xbe, 0x01]
    # the largest magnitude always lands on the largest code, whatever the scale rounding does
    rng = np.random.default_rng(32)
    for _ in range(50):
        v = (rng.standard_normal(64) * 10.0 ** rng.integers(-6, 6)).astype(np.float32)
        a, s = RW.amax_scale(v)
        q = RW.quantize_e4m3(v, s)
        assert (q[np.argmax(np.abs(v))] & 0x7f) == 0x7e and np.all((q & 0x7f) <= 0x7e)


def test_codes_agree_with_an_independent_cast_of_the_fp32_product():
    # PyTorch's CPU conversion to float8_e4m3fn rounds the same fp32 numbers to nearest even
    rng = np.random.default_rng(33)
    for shape, spread in (((37, 48), 1.0), ((5, 1024), 30.0), ((1, 16), 1e-3)):
        x = (rng.standard_normal(shape) * spread).astype(np.float32)
        x.flat[::7] *= 2.0 ** rng.integers(-12, 3)                   # reach the subnormal codes too
        a, s = RW.amax_scale(x)
        q = (x * (np.float32(1.0) / s)).astype(np.float32)
        want = torch.from_numpy(q).clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(RW.quantize_e4m3(x, s), want)
        # and decoding gives back x to within half a code step (relative 2^-4, absolute 2^-10 of the scale)
        back = ref.e4m3_decode(RW.quantize_e4m3(x, s), float(s))
        assert np.all(np.abs(back - x) <= np.maximum(np.abs(x.astype(np.float64)) * 2.0 ** -4, float(s) * 2.0 ** -10) * 1.0001)


def test_scale_products_are_fp32_products():
    s, s2, inv = RW.scale_products([0.1, 3.0], [0.7, 1e-3], [2.0, 5.0], [0.25, 3.0])
    assert s.dtype == np.float32 and s[0] == np.float32(0.1) * np.float32(0.7) and s2[1] == np.float32(15.0)
    assert inv[0] == 4.0 and inv[1] == np.float32(1.0) / np.float32(3.0)


# ---- the library's host half against the reference -------------------------------------------------

def random_tables(rng):
    G = int(rng.integers(1, 6))
    rows = [[int(r) for r in rng.integers(0, 900, size=rng.integers(0, 7))] for _ in range(G)]
    row_bytes = [int(64 * rng.integers(1, 200)) for _ in range(G)]
    batch_bytes = [rb // int(rng.choice([1, 2, 4])) for rb in row_bytes]
    ptrs = [[int(0x10000000 + 0x1000000 * (7 * g + i)) for i in range(len(rows[g]))] for g in range(G)]
    batch = [int(0x7f0000000000 + 0x40000000 * g) for g in range(G)]
    return rows, row_bytes, batch_bytes, ptrs, batch


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("to_batch", [True, False])
def test_request_segments_match_the_reference_integer_for_integer(seed, to_batch):
    rows, row_bytes, batch_bytes, ptrs, batch = random_tables(np.random.default_rng(100 + seed))
    want, want_chunks = P.request_segments(rows, row_bytes, batch_bytes, ptrs, batch, to_batch)
    flat = [r for reqs in rows for r in reqs]
    off = np.cumsum([0] + [len(r) for r in rows])
    got, chunks = B.epara_request_segments(flat, off, row_bytes, batch_bytes, [p for ps in ptrs for p in ps], batch, to_batch)
    assert chunks == want_chunks and len(got) == len(want)
    for g, w in zip(got, want):
        assert (int(g["src"]), int(g["dst"]), int(g["bytes"]), int(g["first_chunk"]), int(g["group"])) == w
    # every chunk of every non-empty segment is found by "last segment whose first_chunk <= c"
    fc = [w[3] for w in want]
    for c in range(0, want_chunks, max(1, want_chunks // 40)):
        i = max(j for j in range(len(fc)) if fc[j] <= c)
        assert want[i][2] > (c - fc[i]) * 16384 >= 0


def test_request_segments_errors():
    L = B.lib()
    n = np.zeros(1, dtype=np.int64)
    segs = np.zeros(4, dtype=B.SEGMENT)
    def call(rows, off, rb, rp, bp, G):
        a = [np.asarray(rows, dtype=np.int32), np.asarray(off, dtype=np.int64), np.asarray(rb, dtype=np.int64),
             np.asarray(rp, dtype=np.uint64), np.asarray(bp, dtype=np.uint64)]        # kept alive across the call
        return L.epara_request_segments(B._ptr(a[0]), B._ptr(a[1]), G, B._ptr(a[2]), B._ptr(a[2]), B._ptr(a[3]), B._ptr(a[4]), 1, B._ptr(segs), B._ptr(n))
    assert call([1, 2], [0, 2], [32], [16, 32], [64], 1) == B.EPARA_OK and n[0] == 2
    assert call([1, -2], [0, 2], [32], [16, 32], [64], 1) == B.EPARA_ERR_SHAPE
    assert call([1, 2], [2, 0], [32], [16, 32], [64], 1) == B.EPARA_ERR_SHAPE
    assert call([1, 2], [0, 2], [0], [16, 32], [64], 1) == B.EPARA_ERR_SHAPE
    assert call([1, 2], [0, 2], [24], [16, 32], [64], 1) == B.EPARA_ERR_ALIGN
    assert call([1, 2], [0, 2], [32], [16, 32], [64], -1) == B.EPARA_ERR_SHAPE
    assert L.epara_request_segments(None, None, 0, None, None, None, None, 1, None, B._ptr(n)) == B.EPARA_OK and n[0] == 0
    assert L.epara_request_segments(None, None, 0, None, None, None, None, 1, None, None) == B.EPARA_ERR_NULL


def test_segment_launches_validate_before_they_enqueue():
    # every call below must be refused on the host: nothing reaches a GPU
    L = B.lib()
    segs, chunks = B.epara_request_segments([3, 2], [0, 2], [4096 * 2], [4096 * 2], [0x1000, 0x200000], [0x40000000], True)
    assert chunks == 3
    fake_dev = ctypes.c_void_p(0x1000)
    copy = lambda s, d, n, c: L.epara_copy_segments(B._ptr(s), d, n, c, None)
    assert copy(segs, fake_dev, 2, 4) == B.EPARA_ERR_SHAPE                   # chunk total
    assert copy(segs, None, 2, 3) == B.EPARA_ERR_NULL
    bad = segs.copy(); bad["first_chunk"][1] = 0
    assert copy(bad, fake_dev, 2, 3) == B.EPARA_ERR_SHAPE
    bad = segs.copy(); bad["src"][0] += 8
    assert copy(bad, fake_dev, 2, 3) == B.EPARA_ERR_ALIGN
    bad = segs.copy(); bad["bytes"][1] = -16
    assert copy(bad, fake_dev, 2, 3) == B.EPARA_ERR_SHAPE
    bad = segs.copy(); bad["dst"][1] = 0
    assert copy(bad, fake_dev, 2, 3) == B.EPARA_ERR_NULL
    assert copy(segs[:0], None, 0, 0) == B.EPARA_OK                          # nothing to do
    quant = lambda s, G, dt, a, sc: L.epara_quantize_segments_e4m3(B._ptr(s), fake_dev, len(s), 3, G, dt, a, sc, None)
    assert quant(segs, 1, B.EPARA_FP8_E4M3, fake_dev, fake_dev) == B.EPARA_ERR_DTYPE
    assert quant(segs, 1, B.EPARA_BF16, None, fake_dev) == B.EPARA_ERR_NULL
    bad = segs.copy(); bad["group"][1] = 1
    assert quant(bad, 1, B.EPARA_BF16, fake_dev, fake_dev) == B.EPARA_ERR_SHAPE
    assert L.epara_patch_scales(None, 2, fake_dev, fake_dev, None, None, None) == B.EPARA_ERR_NULL
    assert L.epara_patch_scales(fake_dev, -1, fake_dev, fake_dev, None, None, None) == B.EPARA_ERR_SHAPE
    assert L.epara_patch_scales(None, 0, None, None, None, None, None) == B.EPARA_OK
