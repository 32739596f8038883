"""GPU parity of batch forming: gather / scatter and dynamic E4M3 quantisation through the C ABI,
bit for bit against oracle/rows.py, and the fp8 SwiGLU FFN run with scales that only exist in
device memory against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from oracle import rows as RW
from paper_2511_00603_amd import binding as B
from paper_2511_00603_amd import runtime as R
from workloads import casts

from parity_util import TOL, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_requests(rng, layout, torch_dtype):
    """layout: per service (width, [rows per request]) -> (numpy arrays per request, device tensors per request)."""
    host, dev = [], []
    for width, rows in layout:
        h, d = [], []
        for r in rows:
            if torch_dtype == torch.uint8:
                a = rng.integers(0, 256, size=(r, width), dtype=np.uint8)
                t = torch.from_numpy(a).to(DEV)
            elif torch_dtype == torch.bfloat16:
                bits = casts.bf16_bits((rng.standard_normal((r, width)) * 3.0).astype(np.float32))
                a = bits
                t = torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
            else:
                a = (rng.standard_normal((r, width)) * 3.0).astype(np.float32)
                t = torch.from_numpy(a).to(DEV)
            h.append(a)
            d.append(t)
        host.append(h)
        dev.append(d)
    return host, dev


def raw(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


LAYOUTS = [
    [(64, [3, 0, 5, 1]), (1024, [17]), (16, [0, 0]), (4112, [300, 2, 129])],       # chunk tails, empty requests, an empty service
    [(5120, [881, 593, 442]), (5120, [860, 96])],                                # prompt-sized requests
]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("torch_dtype", [torch.uint8, torch.bfloat16, torch.float32])
def test_gather_and_scatter_move_every_byte_where_the_reference_puts_it(layout, torch_dtype):
    esz = torch.tensor([], dtype=torch_dtype).element_size()
    layout = [(w * (16 // esz) if (w * esz) % 16 else w, rows) for w, rows in layout]
    rng = np.random.default_rng(41)
    host, dev = make_requests(rng, layout, torch_dtype)
    want = RW.gather(host)
    batches = [torch.full((sum(rows), w), 0, dtype=torch_dtype, device=DEV) for w, rows in layout]
    plan = R.SegmentPlan(dev, batches, True, DEV)
    R.copy_segments(plan)
    torch.cuda.synchronize()
    for g, (w, rows) in enumerate(layout):
        if sum(rows):
            assert np.array_equal(raw(batches[g]), want[g]), g
    # and back: result rows to fresh request buffers
    outs = [[torch.zeros_like(t) for t in d] for d in dev]
    back = R.SegmentPlan(outs, batches, False, DEV)
    R.copy_segments(back)
    torch.cuda.synchronize()
    for g, (w, rows) in enumerate(layout):
        for got, piece in zip(outs[g], RW.scatter(want[g], rows) if sum(rows) else []):
            assert np.array_equal(raw(got), piece)


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("src", ["f32", "bf16"])
def test_dynamic_quantisation_gives_the_reference_scales_and_codes(layout, src):
    torch_dtype = torch.float32 if src == "f32" else torch.bfloat16
    rng = np.random.default_rng(42)
    host, dev = make_requests(rng, layout, torch_dtype)
    if src == "f32":
        host[0][0][0, 0] = 0.0
        dev[0][0][0, 0] = 0.0
    G = len(layout)
    codes = [torch.full((sum(rows), w), 0xAA, dtype=torch.uint8, device=DEV) for w, rows in layout]
    plan = R.SegmentPlan(dev, codes, True, DEV)
    amax = torch.full((G,), -1.0, dtype=torch.float32, device=DEV)
    scale = torch.full((G,), -1.0, dtype=torch.float32, device=DEV)
    for _ in range(2):                                                   # a second call must not see the first one's maxima
        R.quantize_segments_e4m3(plan, B.DTYPE_BY_NAME[src], amax, scale)
    torch.cuda.synchronize()
    for g, (w, rows) in enumerate(layout):
        vals = [h if src == "f32" else ref.bf16_decode(h).astype(np.float32) for h in host[g]]
        x = np.concatenate(vals, axis=0) if vals else np.zeros((0, w), np.float32)
        a, s = RW.amax_scale(x)
        assert amax[g].item() == a and scale[g].item() == s, (g, amax[g].item(), a)
        if x.size:
            assert np.array_equal(codes[g].cpu().numpy(), RW.quantize_e4m3(x, s)), g


def test_scales_from_device_memory_reach_the_group_arguments():
    G = 5
    rng = np.random.default_rng(43)
    args = np.zeros(G, dtype=B.GROUP_ARGS)
    args["scale"], args["scale2"], args["out_inv_scale"] = 7.0, 8.0, 9.0
    args["M"] = np.arange(G)
    d_args = torch.from_numpy(args.view(np.uint8).copy()).to(DEV)
    sx, sw, sw2, so = (rng.random(G).astype(np.float32) + 0.01 for _ in range(4))
    t = [torch.from_numpy(a).to(DEV) for a in (sx, sw, sw2, so)]
    B.epara_patch_scales(d_args.data_ptr(), G, t[0].data_ptr(), t[1].data_ptr(), 0, 0, R.current_stream_handle())
    torch.cuda.synchronize()
    got = d_args.cpu().numpy().view(B.GROUP_ARGS)
    s, s2, inv = RW.scale_products(sx, sw, sw2, so)
    assert np.array_equal(got["scale"], s) and np.all(got["scale2"] == 8.0) and np.all(got["out_inv_scale"] == 9.0)
    B.epara_patch_scales(d_args.data_ptr(), G, t[0].data_ptr(), t[1].data_ptr(), t[2].data_ptr(), t[3].data_ptr(), R.current_stream_handle())
    torch.cuda.synchronize()
    got = d_args.cpu().numpy().view(B.GROUP_ARGS)
    assert np.array_equal(got["scale"], s) and np.array_equal(got["scale2"], s2) and np.array_equal(got["out_inv_scale"], inv)
    assert np.array_equal(got["M"], np.arange(G))                       # nothing else was touched


def test_fp8_swiglu_ffn_with_dynamic_scales_end_to_end():
    """Requests -> gather + quantise X -> gate/up launch (H in bf16) -> quantise H -> down launch, every
    activation scale computed on the GPU; the oracle repeats the same steps in fp64 / numpy."""
    rng = np.random.default_rng(44)
    services = [(256, 2048, [40, 0, 30]), (384, 1536, [300, 57])]      # d_model, d_ff, rows per request (the fp8 bound assumes long sums)
    fp8 = B.EPARA_FP8_E4M3
    req_host, req_dev, Wbits, Wdev, sw = [], [], [], [], {"g": [], "u": [], "d": []}
    for d, f, rows in services:
        h, t = make_requests(rng, [(d, rows)], torch.bfloat16)
        req_host.append(h[0]); req_dev.append(t[0])
        Ws = {"g": rng.standard_normal((d, f)).astype(np.float32) * 0.05, "u": rng.standard_normal((d, f)).astype(np.float32) * 0.05,
              "d": rng.standard_normal((f, d)).astype(np.float32) * 0.05}
        bits, dev = {}, {}
        for k, W in Ws.items():
            s = casts.e4m3_scale(W)
            sw[k].append(s)
            bits[k] = casts.e4m3_codes(W, s)
            dev[k] = R.pack_weights(R.device_tensor_from_bits(bits[k], fp8, DEV), fp8)
        Wbits.append(bits); Wdev.append(dev)
    G = len(services)
    M = [sum(rows) for _, _, rows in services]
    X8 = [torch.zeros((M[g], services[g][0]), dtype=torch.uint8, device=DEV) for g in range(G)]
    H16 = [torch.zeros((M[g], services[g][1]), dtype=torch.bfloat16, device=DEV) for g in range(G)]
    H8 = [torch.zeros((M[g], services[g][1]), dtype=torch.uint8, device=DEV) for g in range(G)]
    Y = [torch.zeros((M[g], services[g][0]), dtype=torch.bfloat16, device=DEV) for g in range(G)]
    f32dev = lambda a: torch.tensor(a, dtype=torch.float32, device=DEV)
    d_sw = {k: f32dev(v) for k, v in sw.items()}
    amax_x, s_x, amax_h, s_h = (torch.zeros(G, dtype=torch.float32, device=DEV) for _ in range(4))
    up = R.LaunchPlan(np.array([R.group_args(X8[g], Wdev[g]["g"], H16[g], M[g], services[g][0], services[g][1], "swiglu", W2=Wdev[g]["u"])
                                for g in range(G)], dtype=B.GROUP_ARGS), fp8, DEV)
    down = R.LaunchPlan(np.array([R.group_args(H8[g], Wdev[g]["d"], Y[g], M[g], services[g][1], services[g][0], "none")
                                  for g in range(G)], dtype=B.GROUP_ARGS), fp8, DEV)
    gather = R.SegmentPlan(req_dev, X8, True, DEV)
    requant = R.SegmentPlan([[h] for h in H16], H8, True, DEV)
    R.quantize_segments_e4m3(gather, B.EPARA_BF16, amax_x, s_x)
    R.patch_scales(up, s_x, d_sw["g"], d_sw["u"])
    R.grouped_forward(up, B.EPARA_BF16)
    R.quantize_segments_e4m3(requant, B.EPARA_BF16, amax_h, s_h)
    R.patch_scales(down, s_h, d_sw["d"])
    R.grouped_forward(down, B.EPARA_BF16)
    torch.cuda.synchronize()
    for g, (d, f, rows) in enumerate(services):
        x = np.concatenate([ref.bf16_decode(h).astype(np.float32) for h in req_host[g]], axis=0)
        ax, sx = RW.amax_scale(x)
        assert s_x[g].item() == sx
        Xq = ref.e4m3_decode(RW.quantize_e4m3(x, sx), float(sx))
        Wq = {k: ref.e4m3_decode(Wbits[g][k], sw[k][g]) for k in "gud"}
        Href = ref.swiglu_hidden(Xq, Wq["g"], Wq["u"])
        h16 = ref.bf16_decode(ref.bf16_encode(Href)).astype(np.float32)
        ah, sh = RW.amax_scale(h16)
        assert abs(s_h[g].item() - sh) <= 2.0 ** -7 * sh              # one bf16 step of the largest hidden value
        Hq = ref.e4m3_decode(RW.quantize_e4m3(h16, sh), float(sh))
        Yref = ref.dense_forward(Hq, Wq["d"])
        assert_close(Y[g].float().cpu().numpy(), Yref, TOL["fp8"], "service %d" % g)
