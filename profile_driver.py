"""Small driver for rocprofv3 runs: a few passes of one synthetic mix, then the plain copy kernel
of known size whose HBM traffic calibrates the byte counters.

    rocprofv3 --kernel-trace --stats --output-format csv -d OUT -o run -- python3 profile_driver.py 5 bf16 6
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -o fetch -- python3 profile_driver.py 5 bf16 3
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -o fetch -- python3 profile_driver.py 3 block 6
"""
import sys

import torch

import os

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import bench_probes as P
from paper_2511_00603_amd import binding as B
from paper_2511_00603_amd.mixrun import StagedMix
from workloads import make_mix

COPY_BYTES = 1 << 30


def batch_forming(mix, steps):
    """Gather, gather + dynamic E4M3 quantisation and scatter of the mix's requests (bf16 rows), `steps` times."""
    import numpy as np
    from workloads import casts
    from paper_2511_00603_amd import runtime as R
    dev = "cuda:0"
    reqs, batches, codes = [], [], []
    for svc in mix.services:
        bits = casts.bf16_bits(svc.X)
        at, mine = 0, []
        for n in svc.request_rows:
            mine.append(torch.from_numpy(bits[at:at + n].view(np.int16).copy()).to(dev).view(torch.bfloat16))
            at += n
        reqs.append(mine)
        batches.append(torch.zeros(svc.X.shape, dtype=torch.bfloat16, device=dev))
        codes.append(torch.zeros(svc.X.shape, dtype=torch.uint8, device=dev))
    G = len(reqs)
    gather, quant, scatter = R.SegmentPlan(reqs, batches, True, dev), R.SegmentPlan(reqs, codes, True, dev), R.SegmentPlan(reqs, batches, False, dev)
    amax, scale = torch.zeros(G, dtype=torch.float32, device=dev), torch.zeros(G, dtype=torch.float32, device=dev)
    for _ in range(steps):
        R.copy_segments(gather)
        R.quantize_segments_e4m3(quant, B.EPARA_BF16, amax, scale)
        R.copy_segments(scatter)
    torch.cuda.synchronize()
    print("profile_driver: batch forming of mix %d, %d passes, %d source bytes per pass" % (mix.index, steps, gather.bytes))


def block_pieces(mix, steps):
    """Attention and residual + layer normalisation over the ViT mix's services (tensors of the mix's shapes with
    N(0, 1) values), `steps` times each, then the copy probe."""
    from paper_2511_00603_amd import runtime as R
    dev = "cuda:0"
    d = mix.services[0].X.shape[1]
    tokens, heads = mix.services[0].request_rows[0], d // 64
    bf = lambda M, N: torch.randn((M, N), device=dev).to(torch.bfloat16)
    attn = R.AttnPlan([{"QKV": bf(s.M, 3 * d), "O": bf(s.M, d), "tokens": tokens, "heads": heads} for s in mix.services], dev)
    norm = R.NormPlan([{"X": bf(s.M, d), "R": bf(s.M, d), "gamma": torch.ones(d, device=dev), "beta": torch.zeros(d, device=dev),
                        "S": bf(s.M, d), "Y": bf(s.M, d), "eps": 1e-6} for s in mix.services], dev)
    for _ in range(steps):
        R.attention(attn)
        R.add_layernorm(norm)
    torch.cuda.synchronize()
    copy_probe()
    print("profile_driver: attention and add + layer norm over mix %d, %d launches each, %d rows" % (mix.index, steps, mix.rows))


def copy_probe():
    src = torch.ones(COPY_BYTES, dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros(COPY_BYTES, dtype=torch.uint8, device="cuda:0")
    for _ in range(2):
        P.probe_copy(src.data_ptr(), dst.data_ptr(), COPY_BYTES, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()


def main():
    idx = int(sys.argv[1])
    dtype = sys.argv[2] if len(sys.argv) > 2 else None
    steps = int(sys.argv[3]) if len(sys.argv) > 3 else 4
    mix = make_mix(idx)
    if dtype == "rows":          # batch forming of the mix's requests instead of its forward pass
        return batch_forming(mix, steps)
    if dtype == "block":         # the pieces between a ViT block's dense layers
        return block_pieces(mix, steps)
    s_h = None
    if dtype == "fp8":
        cal = StagedMix(mix, "bf16", "cuda:0")
        cal.run()
        torch.cuda.synchronize()
        s_h = [float(t.abs().max().float().item()) / 448.0 for (_, _, t) in cal.outputs[0][0]]
        del cal
    staged = StagedMix(mix, dtype, "cuda:0")
    for _ in range(steps):
        staged.run()
    torch.cuda.synchronize()
    copy_probe()
    print("profile_driver: mix %d %s, %d passes, copy probe %d bytes" % (idx, dtype or mix.dtype, steps, COPY_BYTES))


if __name__ == "__main__":
    main()
