"""Expected outputs of a staged mix, computed by the CPU oracle from the exact input bits.

Intermediate activations stay in fp64 (the GPU rounds them to the storage type; that error is
part of what the tolerance covers), except on the fp8 SwiGLU path where the hidden activations
are requantised with the same static scale the GPU is given.
"""
import numpy as np

from oracle import reference as ref


def decode(bits, dtype_name, scale=1.0):
    if dtype_name == "f32":
        return np.asarray(bits, dtype=np.float64)
    if dtype_name == "bf16":
        return ref.bf16_decode(bits)
    return ref.e4m3_decode(bits, scale)


def expected(mix, host_bits, dtype_name, rows=None, h_scales=None, calibrated=None):
    """-> list per launch of list of (service, label, Yref) in the launch/group order of StagedMix.

    rows: optional list (per service) of row index arrays; only those rows are evaluated.
    h_scales: per-service s_h for the fp8 SwiGLU path; or pass an empty list as `calibrated`: s_h of every
    service is then taken from the oracle's hidden activations (amax / 448) and appended to that list.
    """
    fp8 = dtype_name == "fp8"
    launches = []
    kind = mix.services[0].kind
    n = len(mix.services)
    sel = lambda g: slice(None) if rows is None else rows[g]
    if kind == "swiglu":
        hs, ys = [], []
        for g, hb in enumerate(host_bits):
            X = decode(hb["X"][sel(g)], dtype_name)             # codes as values; scales applied below
            Wg, Wu, Wd = (decode(hb[k], dtype_name) for k in ("Wgate", "Wup", "Wdown"))
            if fp8:
                sx, sg, su, sd = hb["s_x"], hb["s_wgate"], hb["s_wup"], hb["s_wdown"]
                H = ref.swiglu_hidden(X, Wg, Wu, sx * sg, sx * su)
                if calibrated is not None:                      # static scale from the oracle's own hidden activations
                    calibrated.append(float(np.abs(H).max()) / 448.0)
                sh = calibrated[g] if calibrated is not None else h_scales[g]
                H, Y = ref.ffn_swiglu_down(H, Wd, s_down=sh * sd, h_scale=sh)
            else:
                H, Y = ref.ffn_swiglu(X, Wg, Wu, Wd)
            hs.append((g, "H", H))
            ys.append((g, "Y", Y))
        return [hs, ys]
    outs = {}
    for g, hb in enumerate(host_bits):
        X = decode(hb["X"][sel(g)], dtype_name)
        L = hb["layers"]
        W = [decode(l["W"], dtype_name) for l in L]
        if kind == "vit":
            outs[(g, 0)] = ref.dense_forward(X, W[0], L[0]["b"], L[0]["act"])
            outs[(g, 1)] = ref.dense_forward(X, W[1], L[1]["b"], L[1]["act"])
            outs[(g, 2)] = ref.dense_forward(outs[(g, 1)], W[2], L[2]["b"], L[2]["act"])
        else:
            cur = X
            for l in range(len(L)):
                cur = ref.dense_forward(cur, W[l], L[l]["b"], L[l]["act"])
                outs[(g, l)] = cur
    if kind == "vit":
        order = [[(g, 1) for g in range(n)], [(g, 0) for g in range(n)] + [(g, 2) for g in range(n)]]
    else:
        order = [[(g, l) for g in range(n)] for l in range(len(host_bits[0]["layers"]))]
    for launch in order:
        launches.append([(g, "L%d" % l, outs[(g, l)]) for g, l in launch])
    return launches
