#!/usr/bin/env python3
"""Benchmark of the FP8 <-> MXFP4 conversion hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic DeepSeek-V3-shaped
activations [65536, 7168]:  FP8 -> MXFP4 quantization, MXFP4 -> FP8 de-quantization, and
row-blocked -> column-blocked MXFP4 conversion.  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line: whole-step algorithmic GB/s as `value`, the roofline of the
dominant kernel (HIP-event durations taken inside the timed region), per-kernel figures,
and the CPU oracle timed on the host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published
# algorithmic bytes per element (paper sec. 3.2: FP8 = 1 + 4/128, MXFP4 = 1/2 + 1/32)
BYTES_PER_ELEM = {"quant": 1.03125 + 0.53125, "dequant": 0.53125 + 1.03125, "row_to_col": 0.53125 + 0.53125}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--rows", type=int, default=65536, help="M of the workload (tokens)")
    p.add_argument("--hidden", type=int, default=7168, help="K of the workload")
    p.add_argument("--seed", type=int, default=0)
    p.add_argument("--cpu-sample-rows", type=int, default=65536)
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--event-stride", type=int, default=8,
                   help="bracket the three kernels with HIP events in every N-th timed step (1 = every step). "
                        "An event between two kernels keeps the second from starting while the first drains: "
                        "with events in every step the step takes 309 us instead of 296 at [65536,7168]")
    p.add_argument("--copy-calibration", action="store_true",
                   help="run only plain device copies of a known size (512 MiB read + 512 MiB written per "
                        "launch): the reference against which rocprofv3's FETCH_SIZE / WRITE_SIZE are scaled")
    p.add_argument("--variants", action="store_true",
                   help="also time the gathered, record-layout and grouped entry points (extra JSON field)")
    p.add_argument("--variant", default=None,
                   help="with --variants: time only the entry point of this name (e.g. row_to_fp8_col), "
                        "so that a profiler run sees that kernel at one launch shape")
    return p.parse_args()


def cpu_baseline(x8, s, rows):
    """The oracle as it stands, over `rows` rows of the same workload, one thread per host core."""
    import numpy as np
    from oracle import parallel as par  # thread pool over row ranges around the oracle
    workers = par.WORKERS
    xs, ss = x8[:rows].cpu().numpy(), s[:rows].cpu().numpy()
    t0 = time.perf_counter()
    q, sf = par.quant(xs, ss, workers)
    t1 = time.perf_counter()
    par.dequant(q, sf, workers)
    t2 = time.perf_counter()
    par.row_to_col(q, sf, workers)
    t3 = time.perf_counter()
    n = xs.size
    total_bytes = n * sum(BYTES_PER_ELEM.values())
    # the same oracle on one thread, on the first 2048 rows
    r1 = min(2048, rows)
    u0 = time.perf_counter()
    q1, sf1 = par.quant(xs[:r1], ss[:r1], 1)
    par.dequant(q1, sf1, 1)
    par.row_to_col(q1, sf1, 1)
    u1 = time.perf_counter()
    return {
        "value": total_bytes / (t3 - t0) * 1e-9, "unit": "GB/s", "cores": workers, "kind": "oracle",
        "sample": f"first {rows} rows x {xs.shape[1]} of the workload, quant+dequant+row_to_col, "
                  f"row ranges over {workers} threads",
        "elements_per_s": {"quant": n / (t1 - t0), "dequant": n / (t2 - t1), "row_to_col": n / (t3 - t2)},
        "seconds": t3 - t0,
        "single_thread_GB/s": r1 * xs.shape[1] * sum(BYTES_PER_ELEM.values()) / (u1 - u0) * 1e-9,
    }


def measured_traffic(kernel, M, K):
    """HBM bytes per launch of `kernel` as rocprofv3 counted them (profiles/hbm_traffic.json), or None
    when no counter run covers this workload."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.json")
    try:
        t = json.load(open(path))
    except (OSError, ValueError):
        return None
    if t.get("workload") != f"target_{M}x{K}" or kernel not in t.get("kernels", {}):
        return None
    k = t["kernels"][kernel]
    return k["read"] + k["written"]


def main():
    a = parse()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU; there is no multi-GPU path "
                         "(the conversions shard by rows with no exchange). Use --gpus 1.\n")
        sys.exit(2)

    import torch
    import paper_2603_02731_amd as mx
    from paper_2603_02731_amd import synth

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    mx.lib()  # fail loudly here if the HIP library is missing

    if a.copy_calibration:
        n = 512 << 20
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(a.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "launches": a.steps, "bytes_read_per_launch": n,
                          "bytes_written_per_launch": n}))
        return

    M, K = a.rows, a.hidden
    x8, s = synth.student_t_fp8(M, K, seed=a.seed, device=dev)
    q = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
    sf = torch.empty((M, K // 32), dtype=torch.uint8, device=dev)
    xb = torch.empty((M, K), dtype=torch.uint8, device=dev)
    sb = torch.empty((M, K // 128), dtype=torch.float32, device=dev)
    qc = torch.empty((K, M // 2), dtype=torch.uint8, device=dev)
    sc = torch.empty((K, M // 32), dtype=torch.uint8, device=dev)

    def step(ev=None):
        if ev:
            ev[0].record()
        mx.mxfp4_quant_from_fp8(x8, s, q=q, sf=sf)
        if ev:
            ev[1].record()
        mx.mxfp4_dequant_to_fp8(q, sf, x=xb, x_scale=sb)
        if ev:
            ev[2].record()
        mx.mxfp4_row_to_col(q, sf, q_col=qc, sf_col=sc)
        if ev:
            ev[3].record()

    for _ in range(a.warmup):
        step()
    stride = max(1, min(a.event_stride, a.steps // 8))  # at least eight bracketed steps, all of them in a short run
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] if i % stride == 0 else None
              for i in range(a.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / a.steps
    events = [e for e in events if e is not None]

    n = M * K
    names = ["quant", "dequant", "row_to_col"]
    kernels = {}
    for j, name in enumerate(names):
        us = sum(e[j].elapsed_time(e[j + 1]) for e in events) * 1e3 / len(events)
        b = n * BYTES_PER_ELEM[name]
        kernels[name] = {"us": us, "GB/s": b / us * 1e-3, "frac_of_hbm_peak": b / us * 1e-3 / HBM_PEAK_GBPS,
                         "elements_per_s": n / us * 1e6, "algorithmic_bytes": b}
    total_bytes = n * sum(BYTES_PER_ELEM.values())
    value = total_bytes / (ms_per_step * 1e-3) * 1e-9

    # what a plain device-to-device copy reaches on this GPU, measured now (470 MB read + 470 MB written)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        xb.copy_(x8)
    c0.record()
    for _ in range(20):
        xb.copy_(x8)
    c1.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * n * 20 / (c0.elapsed_time(c1) * 1e-3) * 1e-9
    for name in names:
        kernels[name]["frac_of_measured_copy"] = kernels[name]["GB/s"] / copy_gbps
        kernels[name]["traffic"] = measured_traffic(name, M, K)  # HBM bytes per launch by rocprofv3 counters
    dom = max(names, key=lambda k: kernels[k]["us"])
    traffic = measured_traffic(dom, M, K)

    out = {
        "metric": "HBM GB/s (% of peak) for FP8<->MXFP4 quant/dequant and MXFP4 row->col",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"target_{M}x{K}: Student-t(df=3) activations with 1% outlier channels x100, "
                               f"FP8 E4M3 + FP32 1x128 scales; step = quant + dequant + row_to_col",
                   "rows": M, "hidden": K, "seed": a.seed},
        "frac_of_hbm_peak": value / HBM_PEAK_GBPS,
        "measured_copy_GB/s": copy_gbps,
        "elements_per_s": 3 * n / (ms_per_step * 1e-3),
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": kernels[dom]["GB/s"], "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": kernels[dom]["frac_of_hbm_peak"], "traffic": traffic},
        "kernels": kernels,
        "per_kernel_events": {"every_nth_step": stride, "steps_with_events": len(events)},
    }

    if a.variants:
        out["variants"] = time_variants(torch, mx, synth, x8, s, q, sf, a)

    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(x8, s, min(a.cpu_sample_rows, M))
    print(json.dumps(out))


def time_variants(torch, mx, synth, x8, s, q, sf, a, iters=10):
    """BF16-source quant, gathered quant (top-8 dispatch emulation), per-token records, FP8 column output,
    grouped forms."""
    dev = x8.device
    M, K = x8.shape
    res = {}

    def want(name):
        return a.variant is None or a.variant == name

    def timed(fn):
        for _ in range(2):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    def entry(us, nbytes, **extra):
        return {**extra, "us": us, "GB/s": nbytes / us * 1e-3, "frac_of_hbm_peak": nbytes / us * 1e-3 / HBM_PEAK_GBPS}

    if want("quant_from_bf16"):
        # the paper's BF16-source row quantizer on the same activations (2 B read + 0.53125 B written per element)
        xbf = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
        for r0 in range(0, M, 8192):
            xbf[r0:r0 + 8192] = (x8[r0:r0 + 8192].view(torch.float8_e4m3fn).float()
                                 * s[r0:r0 + 8192].repeat_interleave(128, dim=1)).to(torch.bfloat16)
        qb = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
        sb = torch.empty((M, K // 32), dtype=torch.uint8, device=dev)
        res["quant_from_bf16"] = entry(timed(lambda: mx.mxfp4_quant_from_bf16(xbf, q=qb, sf=sb)),
                                       M * K * (2.0 + 0.53125))
        del xbf, qb, sb

    if want("quant_gather_top8") or want("quant_gather_top8_records") or want("quant_scatter_top8"):
        top_k = 8
        idx = synth.routing_indices(seed=a.seed, num_tokens=M, top_k=top_k, device=dev)
        Mo = idx.shape[0]
        compulsory = M * K * 1.03125 + Mo * 4 + Mo * K * 0.53125
        if want("quant_gather_top8"):
            qg = torch.empty((Mo, K // 2), dtype=torch.uint8, device=dev)
            sg = torch.empty((Mo, K // 32), dtype=torch.uint8, device=dev)
            us = timed(lambda: mx.mxfp4_quant_from_fp8(x8, s, gather_idx=idx, q=qg, sf=sg))
            logical = Mo * K * BYTES_PER_ELEM["quant"]
            res["quant_gather_top8"] = {"us": us, "logical_GB/s": logical / us * 1e-3,
                                        "compulsory_GB/s": compulsory / us * 1e-3,
                                        "frac_of_hbm_peak_compulsory": compulsory / us * 1e-3 / HBM_PEAK_GBPS}
            del qg, sg
        if want("quant_scatter_top8"):
            # the same payload with every token quantized once and written to its 8 destinations
            dst = torch.argsort(idx.long(), stable=True).to(torch.int32).view(M, top_k).contiguous()
            qg = torch.empty((Mo, K // 2), dtype=torch.uint8, device=dev)
            sg = torch.empty((Mo, K // 32), dtype=torch.uint8, device=dev)
            us = timed(lambda: mx.mxfp4_quant_from_fp8_scatter(x8, s, dst, Mo, q=qg, sf=sg))
            res["quant_scatter_top8"] = {"us": us, "compulsory_GB/s": compulsory / us * 1e-3,
                                         "frac_of_hbm_peak_compulsory": compulsory / us * 1e-3 / HBM_PEAK_GBPS}
            del qg, sg, dst
        if want("quant_gather_top8_records"):
            rec = K // 2 + K // 32
            buf = torch.empty(Mo * rec, dtype=torch.uint8, device=dev)
            us = timed(lambda: mx.mxfp4_quant_from_fp8(x8, s, gather_idx=idx, q=buf, sf=buf[K // 2:],
                                                       ld_q=rec, ld_sf=rec))
            res["quant_gather_top8_records"] = {"us": us, "compulsory_GB/s": compulsory / us * 1e-3}
            del buf

    off, _ = synth.expert_offsets(seed=a.seed, num_experts=32, total_tokens=M - 32 * 128, pad_to=128)
    Mt = int(off[-1])
    offd = off.to(dev)
    f8 = 0.53125 + 1.03125  # row-blocked MXFP4 read, FP8 + FP32 per 128 written
    if any(want(n) for n in ("row_to_fp8_col", "row_to_fp8_col_requant", "row_to_fp8_col_grouped_32_experts",
                             "row_to_fp8_col_ragged_32_experts")):
        # the paper's literal weight-gradient kernel: row-blocked MXFP4 -> column-wise FP8
        xc = torch.empty((K, M), dtype=torch.uint8, device=dev)
        xcs = torch.empty((K, M // 128), dtype=torch.float32, device=dev)
        if want("row_to_fp8_col"):
            res["row_to_fp8_col"] = entry(timed(lambda: mx.mxfp4_row_to_fp8_col(q, sf, x_col=xc, x_col_scale=xcs)),
                                          M * K * f8)
        if want("row_to_fp8_col_requant"):
            # the other reading: scale from the group maximum (two passes over the nibbles in registers)
            res["row_to_fp8_col_requant"] = entry(
                timed(lambda: mx.mxfp4_row_to_fp8_col(q, sf, x_col=xc, x_col_scale=xcs, requant=True)), M * K * f8)
        if want("row_to_fp8_col_grouped_32_experts") and Mt <= M:
            us = timed(lambda: mx.mxfp4_row_to_fp8_col_grouped(q[:Mt], sf[:Mt], offd, x_col=xc.view(-1)[:Mt * K],
                                                               x_col_scale=xcs.view(-1)[:Mt * K // 128]))
            res["row_to_fp8_col_grouped_32_experts"] = entry(us, Mt * K * f8, rows=Mt)
        if want("row_to_fp8_col_ragged_32_experts"):
            # the same expert counts without padding: arbitrary T_e, unaligned rows, partial last groups
            offr, _ = synth.expert_offsets(seed=a.seed, num_experts=32, total_tokens=M - 32 * 128, pad_to=1)
            Mr = int(offr[-1])
            offrd = offr.to(dev)
            us = timed(lambda: mx.mxfp4_row_to_fp8_col_grouped(q[:Mr], sf[:Mr], offrd, x_col=xc.view(-1)[:Mr * K],
                                                               x_col_scale=xcs.view(-1)))
            res["row_to_fp8_col_ragged_32_experts"] = entry(us, Mr * K * f8, rows=Mr)
        del xc, xcs
    if want("row_to_col_grouped_32_experts") and Mt <= M:
        qc = torch.empty(Mt * K // 2, dtype=torch.uint8, device=dev)
        scc = torch.empty(Mt * K // 32, dtype=torch.uint8, device=dev)
        us = timed(lambda: mx.mxfp4_row_to_col_grouped(q[:Mt], sf[:Mt], offd, q_col=qc, sf_col=scc))
        res["row_to_col_grouped_32_experts"] = entry(us, Mt * K * BYTES_PER_ELEM["row_to_col"], rows=Mt)
    if want("row_to_col_ragged_32_experts"):
        # the same expert counts without padding: arbitrary T_e, partial last blocks, k-rows at any byte
        offr, _ = synth.expert_offsets(seed=a.seed, num_experts=32, total_tokens=M - 32 * 128, pad_to=1)
        Mr = int(offr[-1])
        offrd = offr.to(dev)
        qcr = torch.empty(Mr * K // 2 + 32 * K, dtype=torch.uint8, device=dev)
        scr = torch.empty(Mr * K // 32 + 32 * K, dtype=torch.uint8, device=dev)
        us = timed(lambda: mx.mxfp4_row_to_col_grouped(q[:Mr], sf[:Mr], offrd, q_col=qcr, sf_col=scr))
        res["row_to_col_ragged_32_experts"] = entry(us, Mr * K * BYTES_PER_ELEM["row_to_col"], rows=Mr)
    return res


if __name__ == "__main__":
    main()
