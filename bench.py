#!/usr/bin/env python3
"""Benchmark of the grouped forward on one MI355X.

A step is one pass of a synthetic service mix through libepara (all its launches), inputs already
resident in HBM.  The headline workload is the prefill mix (two 13B-shaped SwiGLU FFN services,
8192 rows, bf16): `value` is its TFLOP/s.  The same JSON line carries, under "mixes", TFLOP/s,
requests/s and the roofline fraction of every other mix (decode mix against HBM bandwidth; each mix
also timed as one chained kernel), the
roofline object of the headline mix's dominant kernel, and the CPU oracle timed on a bounded
sample of the same workload.

    python bench.py [--steps K] [--warmup W] [--mixes 5,4] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "fp8": 5000.0}
LLC_BYTES = 256 << 20
PREWARM_S = 0.03        # untimed passes before the warm-up steps of a mix (seconds)


def launch_stats(staged, mix, dtype_name):
    """Algorithmic flops and bytes of every launch of one pass: weights once, inputs once, outputs once."""
    from paper_2511_00603_amd import binding as B
    esz = {"f32": 4, "bf16": 2, "fp8": 1}[dtype_name]
    stats = []
    for plan in staged.plans():
        flops = nbytes = 0
        for a in plan.args:
            M, K, N = int(a["M"]), int(a["K"]), int(a["N"])
            gated = int(a["act"]) == B.EPARA_ACT_SWIGLU
            nw = 2 if gated else 1
            flops += 2 * M * K * N * nw
            out_esz = 4 if dtype_name == "f32" else (1 if (gated and dtype_name == "fp8") else 2)
            nbytes += K * N * nw * esz + M * K * esz + M * N * out_esz + (N * 4 if int(a["bias"]) else 0)
        stats.append({"flops": flops, "bytes": nbytes, "tiles": int(len(plan.tiles)), "groups": int(len(plan.args)),
                      # tiles visited in parts of K (weight-streaming tiles / panel tiles of the last round) and their workspace
                      "split_tiles": int(getattr(plan, "n_split_tiles", 0)), "panel_split_tiles": int(getattr(plan, "n_panel_split_tiles", 0)),
                      "workspace_bytes": int(getattr(plan, "workspace_bytes", 0))})
    return stats


def time_mix(mix, dtype_name, steps, warmup, s_h=None):
    import torch
    from paper_2511_00603_amd import runtime as R
    from paper_2511_00603_amd.mixrun import StagedMix

    esz = {"f32": 4, "bf16": 2, "fp8": 1}[dtype_name]
    footprint = mix.weight_elems() * esz
    # cold-cache rule: rotate through copies whose total is at least twice the last-level cache, and never
    # fewer than two unless a single pass already streams six times the cache
    copies = 1 if footprint >= 6 * LLC_BYTES else max(2, min(8, -(-2 * LLC_BYTES // max(footprint, 1))))
    t0 = time.perf_counter()
    staged = StagedMix(mix, dtype_name, "cuda:0", copies=copies, s_h=s_h)
    stage_s = time.perf_counter() - t0
    stats = launch_stats(staged, mix, dtype_name)
    plan_us = sum(p.plan_seconds for p in staged.plans()) * 1e6
    upload_us = sum(p.upload_seconds for p in staged.plans()) * 1e6

    # (a) whole passes, the library's own entry points, events at both ends only.  A pass of the small mixes takes a
    # quarter of a millisecond: W of them do not bring the clocks up from idle, so every mix first runs, untimed, until
    # PREWARM_S have passed; then the W warm-up passes, then the K timed ones.
    t_pre, n_pre = time.perf_counter(), 0
    while time.perf_counter() - t_pre < PREWARM_S:
        for _ in range(4):
            staged.run(copy=n_pre)
            n_pre += 1
        torch.cuda.synchronize()
    for i in range(warmup):
        staged.run(copy=i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        staged.run(copy=i)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / steps

    # (a2) the same passes with an event after each one: median and minimum of a pass (an event pair also spans
    # the few microseconds between two kernels, so these sit slightly above the mean of (a) for short passes)
    pev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    pev[0].record()
    for i in range(steps):
        staged.run(copy=i)
        pev[i + 1].record()
    torch.cuda.synchronize()
    pass_ms = sorted(pev[i].elapsed_time(pev[i + 1]) for i in range(steps))

    # (a') the warm figure, labelled as such: every pass on the same copy, so whatever fits stays in the
    # last-level cache (only differs from (a) for mixes that rotate through copies)
    warm_ms = ms_per_step
    if copies > 1:
        staged.run(copy=0)
        e0.record()
        for i in range(steps):
            staged.run(copy=0)
        e1.record()
        torch.cuda.synchronize()
        warm_ms = e0.elapsed_time(e1) / steps
        for i in range(copies):                    # back to the cold rotation before the per-launch timing
            staged.run(copy=i)
        torch.cuda.synchronize()

    # (b) the same launches one by one with an event between them: per-kernel durations, right after (a) so
    # that the chip is in the same state (passes warmup + steps .. warmup + 2 steps - 1 of these kernels in a
    # kernel trace of this command)
    plans = [staged.plans(c) for c in range(copies)]
    outs = []
    for step in staged.programs[0]:
        outs += [step[2]] if step[0] == "forward" else [step[3], 1]     # out dtype per launch (1 = bf16)
    n_l = len(plans[0])
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(n_l + 1)] for _ in range(steps)]
    for i in range(steps):
        evs[i][0].record()
        for l in range(n_l):
            R.grouped_forward(plans[i % copies][l], outs[l])
            evs[i][l + 1].record()
    torch.cuda.synchronize()
    samples = [sorted(evs[i][l].elapsed_time(evs[i][l + 1]) for i in range(steps)) for l in range(n_l)]
    per_launch_ms = [sum(v) / steps for v in samples]
    # where these passes sit among the grouped_kernel dispatches of a kernel trace of this command
    trace_first_pass = n_pre + warmup + 2 * steps + (1 + steps + copies if copies > 1 else 0)
    # each launch repeated back to back (on its rotating copies) with events at both ends only: without the
    # idle microseconds that an event pair around a single short kernel also spans
    repeated_ms = []
    for l in range(n_l):
        e0.record()
        for i in range(steps):
            R.grouped_forward(plans[i % copies][l], outs[l])
        e1.record()
        torch.cuda.synchronize()
        repeated_ms.append(e0.elapsed_time(e1) / steps)

    # (b2) the same passes captured once into a HIP graph and replayed (no host work per launch)
    side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for c in range(copies):
                staged.run(copy=c)
    torch.cuda.synchronize()
    reps = max(1, steps // copies)
    graph.replay()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    graph_ms = e0.elapsed_time(e1) / (reps * copies)
    del graph

    # (b3) consecutive passes on two streams in turn: passes are independent (each works on its own copy of
    # every buffer), so the start of one fills the compute units that the end of the other leaves idle
    even = copies if copies % 2 == 0 else copies + 1
    pair = staged if even == copies else StagedMix(mix, dtype_name, "cuda:0", copies=even, s_h=s_h, host_bits=staged.host_bits)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    def alternate(n):
        for st in streams:
            st.wait_stream(torch.cuda.current_stream())
        for i in range(n):
            with torch.cuda.stream(streams[i % 2]):
                pair.run(copy=i)                  # an even number of copies: a stream always meets the same buffers
        for st in streams:
            torch.cuda.current_stream().wait_stream(st)
    alternate(2 * warmup)
    torch.cuda.synchronize()
    n2 = 4 * steps
    t0 = time.perf_counter()
    alternate(n2)
    torch.cuda.synchronize()
    two_stream_ms = (time.perf_counter() - t0) * 1e3 / n2
    if pair is not staged:
        del pair
        torch.cuda.empty_cache()

    flops = mix.flops()
    res = {"name": mix.name, "dtype": dtype_name, "ms_per_step": ms_per_step,
           "ms_per_step_median": pass_ms[steps // 2], "ms_per_step_min": pass_ms[0],
           "tflops": flops / (ms_per_step * 1e-3) / 1e12, "requests_per_s": mix.requests / (ms_per_step * 1e-3),
           "requests": mix.requests, "rows": mix.rows, "flops": flops, "launches": n_l, "weight_copies": copies,
           "prewarm_passes": n_pre, "plan_us": plan_us, "plan_upload_us": upload_us, "pack_weights_s": staged.pack_seconds / copies,
           "stage_s": stage_s, "warm_cache_ms_per_step": warm_ms, "graph_replay_ms_per_step": graph_ms,
           "two_streams": {"ms_per_step": two_stream_ms, "tflops": flops / (two_stream_ms * 1e-3) / 1e12,
                           "requests_per_s": mix.requests / (two_stream_ms * 1e-3), "steps": n2,
                           "clock": "host wall clock around the submissions, synchronised at both ends"},
           "kernels": []}
    for l in range(n_l):
        t = per_launch_ms[l] * 1e-3
        st = stats[l]
        gbs, tf = st["bytes"] / t / 1e9, st["flops"] / t / 1e12
        peak_tf = MFMA_PEAK_TFLOPS.get(dtype_name)
        t_mfma = st["flops"] / (peak_tf * 1e12) if peak_tf else 0.0
        t_hbm = st["bytes"] / (HBM_PEAK_GBS * 1e9)
        bound = "mfma" if t_mfma > t_hbm else "hbm"
        k = {"launch": l, "ms": per_launch_ms[l], "ms_median": samples[l][steps // 2], "ms_min": samples[l][0],
             "ms_repeated": repeated_ms[l],
             "tiles": st["tiles"], "groups": st["groups"], "split_tiles": st["split_tiles"], "panel_split_tiles": st["panel_split_tiles"],
             "workspace_bytes": st["workspace_bytes"],
             "flops": st["flops"], "bytes": st["bytes"], "bound": bound}
        if bound == "mfma":
            k.update(achieved=tf, peak=peak_tf, unit="TFLOP/s", frac=tf / peak_tf)
        else:
            k.update(achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS)
        res["kernels"].append(k)
    # the whole pass against the same ceilings: time the roofline allows for all launches / time taken
    t_roof = sum(max(st["flops"] / (MFMA_PEAK_TFLOPS[dtype_name] * 1e12) if dtype_name in MFMA_PEAK_TFLOPS else 0.0,
                     st["bytes"] / (HBM_PEAK_GBS * 1e9)) for st in stats)
    res["kernel_trace"] = {"first_pass": trace_first_pass, "passes": steps, "launches_per_pass": n_l,
                           "what": "passes first_pass .. first_pass + passes - 1 of this mix's grouped_kernel dispatches are the ones timed launch by launch"}
    res["pass_roofline"] = {"frac": t_roof / (ms_per_step * 1e-3), "roofline_ms": t_roof * 1e3,
                            "algorithmic_bytes": sum(st["bytes"] for st in stats), "algorithmic_flops": sum(st["flops"] for st in stats),
                            "GBs": sum(st["bytes"] for st in stats) / (ms_per_step * 1e-3) / 1e9,
                            "what": "sum over the launches of max(flops / MFMA peak, bytes / HBM peak), divided by ms_per_step"}
    # (c) the same pass as ONE kernel (epara_grouped_chain): reported beside the launches above, not instead.
    # The chain is an entry point for one-submission use with long tiles; it is not meant for passes of short
    # streaming tiles (every dependency costs a poll and a drained pipeline), so it is not timed there.
    if mix.index in (2, 4):
        del staged
        torch.cuda.empty_cache()
        return finish_result(res, mix, dtype_name)
    del staged
    torch.cuda.empty_cache()
    chained = StagedMix(mix, dtype_name, "cuda:0", copies=copies, s_h=s_h, chained=True)
    for i in range(warmup):
        chained.run(copy=i)
    torch.cuda.synchronize()
    e0.record()
    for i in range(steps):
        chained.run(copy=i)
    e1.record()
    torch.cuda.synchronize()
    res["chained"] = {"ms_per_step": e0.elapsed_time(e1) / steps, "launches": chained.n_launches(),
                      "wait_error_flag": max(chained.chain_status(c) for c in range(copies))}
    del chained
    torch.cuda.empty_cache()
    return finish_result(res, mix, dtype_name)


def finish_result(res, mix, dtype_name):
    """The roofline object of the mix: its dominant launch; HBM traffic from the counter runs kept under profiles/."""
    from profile_summary import lookup_traffic
    dom = max(res["kernels"], key=lambda k: k["ms"])
    res["roofline"] = {"bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"], "unit": dom["unit"],
                       "frac": dom["frac"], "traffic": lookup_traffic("%s_%s" % (mix.name, dtype_name), dom["launch"]),
                       "traffic_source": "profiles/traffic.txt (rocprofv3 --pmc runs of profile_driver.py; null when the kernels changed since)",
                       "algorithmic_bytes": dom["bytes"], "algorithmic_flops": dom["flops"],
                       "kernel": "grouped_kernel launch %d" % dom["launch"], "avg_ms": dom["ms"],
                       "whole_pass_frac": res["pass_roofline"]["frac"]}
    return res


def measure_peaks():
    """What this GPU sustains on the benchmark's probes (bench_probes.hip): streaming read bandwidth, and the bf16 MFMA rate
    on all-zero operands and on N(0,1) operands (the matrix clock is power limited and data dependent)."""
    import numpy as np
    import torch
    import bench_probes as P
    from workloads import casts
    dev = "cuda:0"
    stream = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(16, dtype=torch.uint8, device=dev)
    out = {}
    nbytes = 2 << 30
    buf = torch.ones(nbytes, dtype=torch.uint8, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    P.probe_read(buf.data_ptr(), nbytes, sink.data_ptr(), 256, stream)
    e0.record()
    for _ in range(5):
        P.probe_read(buf.data_ptr(), nbytes, sink.data_ptr(), 256, stream)
    e1.record()
    torch.cuda.synchronize()
    out["hbm_read_GBs"] = 5 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del buf
    rng = np.random.default_rng(7)
    for name, vals in (("zeros", np.zeros(16384, dtype=np.float32)), ("normal", rng.standard_normal(16384).astype(np.float32))):
        ops = torch.from_numpy(casts.bf16_bits(vals).view(np.int16)).to(dev)
        iters = 20000
        P.probe_mfma(ops.data_ptr(), 2000, sink.data_ptr(), 256, stream)
        e0.record()
        P.probe_mfma(ops.data_ptr(), iters, sink.data_ptr(), 256, stream)
        e1.record()
        torch.cuda.synchronize()
        out["mfma_bf16_TFLOPs_%s_operands" % name] = 256 * 4 * iters * 16 * 2 * 32 * 32 * 16 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    torch.cuda.empty_cache()
    return out


def time_batch_forming(mix, steps, warmup):
    """The step before and after the path on the prefill mix's own requests: every prompt's rows (bf16, in a
    buffer of its own) gathered into its service's batch, gathered with dynamic per-tensor E4M3 quantisation,
    and the result rows scattered back.  HBM-bound: bytes = what each variant has to move."""
    import numpy as np
    import torch
    from paper_2511_00603_amd import binding as B
    from paper_2511_00603_amd import runtime as R
    from workloads import casts
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
    src = gather.bytes
    cases = {"gather_bf16": (lambda: R.copy_segments(gather), 2 * src),
             "gather_quantize_e4m3": (lambda: R.quantize_segments_e4m3(quant, B.EPARA_BF16, amax, scale), 2 * src + src // 2),
             "scatter_bf16": (lambda: R.copy_segments(scatter), 2 * src)}
    out = {"rows": int(mix.rows), "requests": int(mix.requests), "source_bytes": int(src)}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for name, (fn, nbytes) in cases.items():
        for _ in range(warmup):
            fn()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / steps * 1e3
        out[name] = {"us": us, "bytes": int(nbytes), "GBs": nbytes / us / 1e3, "frac_hbm": nbytes / us / 1e3 / HBM_PEAK_GBS}
    # the numpy reference on the host, same requests
    from oracle import reference as ref
    from oracle import rows as RW
    t0 = time.perf_counter()
    for svc in mix.services:
        x = ref.bf16_decode(casts.bf16_bits(svc.X)).astype(np.float32)
        _a, sc = RW.amax_scale(x)
        RW.quantize_e4m3(x, sc)
    dt = time.perf_counter() - t0
    out["cpu_reference"] = {"GBs": (2 * src + src // 2) / dt / 1e9, "kind": "oracle", "sample": "all rows, amax + quantise in numpy, %.1f s" % dt}
    return out


def time_vit_block_pieces(mix, steps, warmup):
    """What lies between the dense layers of a ViT encoder block, on the ViT mix's own tensors: attention over the QKV
    projection's output of every service (one launch), and the residual + layer normalisation that follows a block
    (FFN output + block input; one launch).  Both are bound by HBM traffic at these sizes: bytes = inputs once +
    outputs once.  Six copies of the tensors are rotated so that no pass finds its data in the last-level cache."""
    import torch
    from paper_2511_00603_amd import runtime as R
    from paper_2511_00603_amd.mixrun import StagedMix
    dev = "cuda:0"
    st = StagedMix(mix, "bf16", dev)
    st.run()
    torch.cuda.synchronize()
    by_label = {}
    for launch in st.outputs[0]:
        for g, label, t in launch:
            by_label[(g, label)] = t
    tokens = mix.services[0].request_rows[0]
    d = mix.services[0].X.shape[1]
    heads = d // 64
    copies = 6
    attn, norm = [], []
    for _ in range(copies):
        ga, gn = [], []
        for g, svc in enumerate(mix.services):
            qkv = by_label[(g, "L0")].clone()
            ga.append({"QKV": qkv, "O": torch.empty((svc.M, d), dtype=torch.bfloat16, device=dev), "tokens": tokens, "heads": heads})
            gn.append({"X": by_label[(g, "L2")].clone(), "R": st.inputs[0][g].clone(),
                       "gamma": torch.ones(d, dtype=torch.float32, device=dev), "beta": torch.zeros(d, dtype=torch.float32, device=dev),
                       "S": torch.empty((svc.M, d), dtype=torch.bfloat16, device=dev),
                       "Y": torch.empty((svc.M, d), dtype=torch.bfloat16, device=dev), "eps": 1e-6})
        attn.append(R.AttnPlan(ga, dev))
        norm.append(R.NormPlan(gn, dev))
    M = int(mix.rows)
    images = M // tokens
    cases = {"attention": (attn, R.attention, M * 4 * d * 2, 4 * images * heads * tokens * tokens * 64),
             "add_layernorm": (norm, R.add_layernorm, M * 4 * d * 2, 0)}
    out = {"rows": M, "images": images, "tokens": tokens, "heads": heads, "d": d, "copies": copies}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for name, (plans, fn, nbytes, flops) in cases.items():
        for i in range(max(warmup, copies)):
            fn(plans[i % copies])
        e0.record()
        for i in range(steps):
            fn(plans[i % copies])
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / steps * 1e3
        out[name] = {"us": us, "bytes": int(nbytes), "GBs": nbytes / us / 1e3, "frac_hbm": nbytes / us / 1e3 / HBM_PEAK_GBS}
        if flops:
            out[name]["TFLOPs"] = flops / us / 1e6
    # the fp64 reference on the host for the same two steps, on a bounded sample (the images of the smallest services)
    import numpy as np
    from oracle import block as OB
    small = sorted(range(len(mix.services)), key=lambda g: mix.services[g].M)[:3]
    t0 = time.perf_counter()
    n_img = 0
    for g in small:
        OB.attention(by_label[(g, "L0")].float().cpu().numpy().astype(np.float64), tokens, heads)
        n_img += mix.services[g].M // tokens
    t_attn = time.perf_counter() - t0
    t0 = time.perf_counter()
    n_rows = 0
    for g in small:
        OB.add_layer_norm(by_label[(g, "L2")].float().cpu().numpy().astype(np.float64), st.inputs[0][g].float().cpu().numpy().astype(np.float64),
                          np.ones(d), np.zeros(d), 1e-6)
        n_rows += mix.services[g].M
    t_norm = time.perf_counter() - t0
    out["cpu_reference"] = {"kind": "oracle", "attention_images_per_s": n_img / t_attn, "add_layernorm_rows_per_s": n_rows / t_norm,
                            "sample": "%d images / %d rows of the three smallest services, numpy fp64, %.2f s + %.2f s" % (n_img, n_rows, t_attn, t_norm)}
    del st, attn, norm
    torch.cuda.empty_cache()
    # a whole encoder block of every service: the eight launches back to back, then each launch on its own
    from paper_2511_00603_amd.vitblock import STEPS, VitBlock
    from workloads import make_vit_block
    blk = VitBlock(mix, make_vit_block(mix), dev, copies=2)
    for i in range(warmup):
        blk.run(i)
    e0.record()
    for i in range(steps):
        blk.run(i)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    per = {}
    for k, name in enumerate(STEPS):
        blk.run_step(k, 0)
        e0.record()
        for i in range(steps):
            blk.run_step(k, i)
        e1.record()
        torch.cuda.synchronize()
        per[name] = e0.elapsed_time(e1) / steps * 1e3
    out["block"] = {"what": "LN -> QKV -> attention -> projection -> add + LN -> FFN up (GELU) -> FFN down -> add + LN, all services per launch",
                    "ms_per_step": ms, "launches": len(STEPS), "us_per_launch": per, "flops": blk.flops(),
                    "tflops": blk.flops() / (ms * 1e-3) / 1e12, "requests_per_s": images / (ms * 1e-3)}
    del blk
    torch.cuda.empty_cache()
    return out


def cpu_baseline(mix, budget_s=15.0):
    """The oracle as it stands on the host cores, on a few rows of service 0 of the prefill mix (fp64)."""
    from oracle import reference as ref
    from workloads import casts
    svc = mix.services[0]
    dec = lambda a: ref.bf16_decode(casts.bf16_bits(a))
    Wg, Wu, Wd = dec(svc.Wgate), dec(svc.Wup), dec(svc.Wdown)
    d, f = svc.Wgate.shape
    per_row = 2 * d * f * 3
    threads = ref.threads()
    X = dec(svc.X[:threads])                       # probe: one row per thread
    t0 = time.perf_counter()
    ref.ffn_swiglu(X, Wg, Wu, Wd)
    t_probe = time.perf_counter() - t0
    rows = threads * int(max(1, min(svc.M // threads, budget_s / max(t_probe, 1e-6))))
    X = dec(svc.X[:rows])
    t0 = time.perf_counter()
    ref.ffn_swiglu(X, Wg, Wu, Wd)
    dt = time.perf_counter() - t0
    return {"value": per_row * rows / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": "%d rows of service 0 of the prefill mix (SwiGLU FFN d=%d f=%d), fp64 triple loop, %.1f s" % (rows, d, f, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--mixes", default="5,5fp8,4,4fp8,3,2,1", help="comma list; the first is the headline (default prefill bf16)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measured-ceiling probes")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: every service of a mix is resident on it and nothing is sharded; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from workloads import make_mix
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (libepara has no CPU path)", file=sys.stderr)
        sys.exit(2)

    peaks = None if a.no_peaks else measure_peaks()
    results, cache, cpu, forming, pieces = [], {}, None, None, None
    for tag in a.mixes.split(","):
        idx = int(tag[0])
        dtype_name = "fp8" if tag.endswith("fp8") else None
        if idx not in cache:
            cache.clear()
            cache[idx] = make_mix(idx)
        mix = cache[idx]
        dtype_name = dtype_name or mix.dtype
        s_h = None
        if dtype_name == "fp8":        # static hidden-activation scales from a calibration pass in bf16
            from paper_2511_00603_amd.mixrun import StagedMix
            cal = StagedMix(mix, "bf16", "cuda:0")
            cal.run()
            torch.cuda.synchronize()
            s_h = [float(t.abs().max().float().item()) / 448.0 for (_, _, t) in cal.outputs[0][0]]
            del cal
            torch.cuda.empty_cache()
        results.append(time_mix(mix, dtype_name, a.steps, a.warmup, s_h))
        if idx == 5 and cpu is None and not a.no_cpu_baseline:
            cpu = cpu_baseline(mix)
        if idx == 5 and forming is None:
            forming = time_batch_forming(mix, a.steps, a.warmup)
        if idx == 3 and dtype_name == "bf16" and pieces is None:
            pieces = time_vit_block_pieces(mix, a.steps, a.warmup)
            print("# between the dense layers of a ViT block: attention %.1f us (%.0f GB/s, %.1f TFLOP/s), residual + layer norm %.1f us (%.0f GB/s); a whole encoder block of all services: %.3f ms (%.1f TFLOP/s, %.0f images/s; %s)" % (
                pieces["attention"]["us"], pieces["attention"]["GBs"], pieces["attention"]["TFLOPs"], pieces["add_layernorm"]["us"],
                pieces["add_layernorm"]["GBs"], pieces["block"]["ms_per_step"], pieces["block"]["tflops"], pieces["block"]["requests_per_s"],
                ", ".join("%s %.0f" % kv for kv in pieces["block"]["us_per_launch"].items())), file=sys.stderr, flush=True)
        r = results[-1]
        print("# %s %s: %.3f ms/step (median %.3f, min %.3f), %.1f TFLOP/s, %.0f req/s, roofline %s %.1f%% (whole pass %.1f%%); graph replay %.3f ms; passes on two streams %.3f ms%s" % (
            mix.name, dtype_name, r["ms_per_step"], r["ms_per_step_median"], r["ms_per_step_min"], r["tflops"], r["requests_per_s"],
            r["roofline"]["bound"], 100 * r["roofline"]["frac"], 100 * r["pass_roofline"]["frac"], r["graph_replay_ms_per_step"], r["two_streams"]["ms_per_step"],
            "; as one chained kernel %.3f ms" % r["chained"]["ms_per_step"] if "chained" in r else ""),
            file=sys.stderr, flush=True)

    head = results[0]
    line = {"metric": "grouped forward TFLOP/s + % MFMA/HBM roofline; requests/s per mix, 1 MI355X",
            "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
            "ms_per_step": head["ms_per_step"], "ms_per_step_median": head["ms_per_step_median"], "ms_per_step_min": head["ms_per_step_min"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": head["dtype"], "data": "synthetic",
            "config": {"workload": "%s (%s): %d rows, %d requests per pass, %d launches" % (
                head["name"], head["dtype"], head["rows"], head["requests"], head["launches"])},
            "requests_per_s": head["requests_per_s"], "measured_peaks": peaks,
            "roofline": head["roofline"], "cpu_baseline": cpu, "pass_roofline": head["pass_roofline"], "batch_forming": forming, "vit_block_pieces": pieces,
            "mixes": {("%s_%s" % (r["name"], r["dtype"])): r for r in results}}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
