"""Reference for batch forming around the grouped forward (test infrastructure only).

The allocator's BS / MF operators (Sec. 3.1 of the paper) make one ragged batch per service out of
the rows its requests bring, and every request gets its own result rows back.  Nothing here is
arithmetic except the dynamic per-tensor fp8 scale: the rows of all requests of a service are one
tensor, amax = max |x|, scale = amax / 448 (1 for an all-zero or empty tensor; 448 is the largest
finite E4M3 value), code = sat(RNE(x * (1 / scale))) -- the form in which the forward path itself
quantises its hidden activations (a stored reciprocal scale).  Reciprocal and product are taken in
fp32, the precision the GPU kernel decides the integer code in, so the codes can be compared bit
for bit; the fp32 product is an exact double, which the oracle's own E4M3 encoder then rounds.
"""
import numpy as np

from . import reference as ref


def gather(requests_per_service):
    """requests_per_service[g] = list of [rows_r, K_g] arrays -> list of [M_g, K_g] batches."""
    out = []
    for reqs in requests_per_service:
        rows = [np.asarray(r) for r in reqs]
        if not rows:
            out.append(None)
            continue
        out.append(np.concatenate(rows, axis=0))
    return out


def scatter(batch, request_rows):
    """The rows of one service's result, handed back request by request."""
    out, at = [], 0
    for n in request_rows:
        out.append(batch[at:at + n])
        at += n
    if at != len(batch):
        raise ValueError("row counts do not add up to the batch")
    return out


def amax_scale(x):
    """(amax, scale) of one tensor, both fp32."""
    x = np.asarray(x, dtype=np.float32)
    amax = np.float32(np.max(np.abs(x))) if x.size else np.float32(0.0)
    scale = np.float32(amax / np.float32(448.0)) if amax > 0 else np.float32(1.0)
    return amax, scale


def quantize_e4m3(x, scale):
    """E4M3 codes of x * (1 / scale), reciprocal and product rounded to fp32."""
    inv = np.float32(1.0) / np.float32(scale)
    q = (np.asarray(x, dtype=np.float32) * inv).astype(np.float32)
    return ref.e4m3_encode(q.astype(np.float64), 1.0)


def scale_products(sx, sw, sw2=None, sout=None):
    """What the group arguments receive: s = sx*sw, s2 = sx*sw2, 1/sout, all in fp32."""
    sx, sw = np.asarray(sx, np.float32), np.asarray(sw, np.float32)
    s = (sx * sw).astype(np.float32)
    s2 = None if sw2 is None else (sx * np.asarray(sw2, np.float32)).astype(np.float32)
    inv = None if sout is None else (np.float32(1.0) / np.asarray(sout, np.float32)).astype(np.float32)
    return s, s2, inv
