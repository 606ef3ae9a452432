#!/usr/bin/env python3
"""Benchmark of the FP8 <-> MXFP4 conversion hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic DeepSeek-V3-shaped
activations [65536, 7168]:  FP8 -> MXFP4 quantization, MXFP4 -> FP8 de-quantization, and
row-blocked -> column-blocked MXFP4 conversion.  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line.

What is timed, and how the caches are kept out of it.  The GPU has a 256 MB memory-side cache; a
kernel that reads what its predecessor has just written, or rewrites its own last output, is served
partly from that cache, not from HBM.  Every figure reported against the HBM peak is therefore
taken over ROTATED buffer sets: a kernel never touches bytes that were read or written during the
last 768 MB of traffic ("cold").  The same kernels on a single buffer set, in the order a training
step would run them, are reported beside it ("in_step"), labelled as such.
  value / ms_per_step  whole step over rotated sets (quant writes set i, dequant reads set i+1 and
                       row_to_col set i+2, all written one or two steps earlier)
  kernels.*.cold       each kernel launched back to back over the rotated sets, HIP events on the
                       launch stream around the whole run, duration = elapsed / launches
  kernels.*.in_step    one buffer set, HIP events around each kernel in every N-th step
  roofline             the kernel with the LOWEST cold fraction of the 8 TB/s HBM peak
  copy                 the library's own 16-byte-per-lane copy over the same rotated sets
  movers               the bytes of each kernel moved in its read : write mix and access pattern, no arithmetic
  configs              the smaller named workloads ([4096,7168], [16384,2048], 32 ragged experts,
                       the top-8 dispatch payload), cold and on a single set
  cpu_baseline         the CPU oracle on the host cores, on a bounded sample of the workload
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published
MALL_BYTES = 256 << 20  # memory-side cache
# algorithmic bytes per element (paper sec. 3.2: FP8 = 1 + 4/128, MXFP4 = 1/2 + 1/32)
FP8_B, MX_B = 1.03125, 0.53125
BYTES_PER_ELEM = {"quant": FP8_B + MX_B, "dequant": MX_B + FP8_B, "row_to_col": MX_B + MX_B}
PHASES = ("step", "in_step", "cold", "copy", "configs", "variants", "cpu")


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--rows", type=int, default=65536, help="M of the workload (tokens)")
    p.add_argument("--hidden", type=int, default=7168, help="K of the workload")
    p.add_argument("--seed", type=int, default=0)
    p.add_argument("--sets", type=int, default=3, help="rotated buffer sets of the workload (at least 3)")
    p.add_argument("--cold-launches", type=int, default=60, help="launches per kernel of the cold measurement")
    p.add_argument("--cpu-sample-rows", type=int, default=65536)
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--event-stride", type=int, default=8,
                   help="in_step: bracket the three kernels with HIP events in every N-th step (1 = every step). "
                        "An event between two kernels keeps the second from starting while the first drains")
    p.add_argument("--phases", default=",".join(PHASES),
                   help="comma-separated subset of " + ",".join(PHASES) + " (a profiler run that should see one "
                        "kind of launch only names one phase, e.g. --phases cold)")
    p.add_argument("--config", type=int, default=None, choices=(2, 3, 4, 5),
                   help="with the configs phase: only this named workload")
    p.add_argument("--variant", default=None,
                   help="with the variants phase: only the entry point of this name (e.g. row_to_fp8_col)")
    p.add_argument("--copy-calibration", action="store_true",
                   help="run only plain device copies of a known size (512 MiB read + 512 MiB written per "
                        "launch): the reference against which rocprofv3's FETCH_SIZE / WRITE_SIZE are scaled")
    return p.parse_args()


def csrc_sha256():
    """Hash of the kernel sources: a recorded counter run only describes the kernels it was taken on."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2603_02731_amd", "csrc")
    for f in sorted(os.listdir(d)):
        if f.endswith((".hip", ".hpp")):
            h.update(f.encode())
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()


def measured_traffic(kernel, M, K):
    """HBM bytes per launch of `kernel` as rocprofv3 counted them (profiles/hbm_traffic.json), or None when no
    counter run covers this workload or the kernels have changed since it was taken."""
    try:
        t = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))
    except (OSError, ValueError):
        return None
    if t.get("workload") != f"target_{M}x{K}" or kernel not in t.get("kernels", {}):
        return None
    if t.get("csrc_sha256") != csrc_sha256():
        return None
    k = t["kernels"][kernel]
    return k["read"] + k["written"]


def cpu_baseline(x8, s, rows):
    """The oracle as it stands, over `rows` rows of the same workload, one thread per host core."""
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


def sets_for(bytes_per_launch, at_least=3):
    """Buffer sets to rotate so that a launch never meets bytes of the last 3 x 256 MB of traffic."""
    return max(at_least, -(-3 * MALL_BYTES // int(bytes_per_launch)))


class Bench:
    def __init__(self, torch, mx, synth, args):
        self.torch, self.mx, self.synth, self.a = torch, mx, synth, args
        self.dev = "cuda:0"

    def timed(self, calls, launches, warm=None):
        """Launch `calls` round-robin (one callable per buffer set) and return the average microseconds per
        launch, from HIP events on the launch stream around the whole run."""
        torch, n = self.torch, len(calls)
        for i in range(n if warm is None else warm):
            calls[i % n]()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(launches):
            calls[i % n]()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / launches

    def timed_graph(self, calls, launches):
        """The same round-robin, with one pass over the buffer sets captured in a HIP graph and replayed: the
        figure for kernels of a few microseconds, which Python cannot launch as fast as they run."""
        torch, n = self.torch, len(calls)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for c in calls:
                c()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for c in calls:
                    c()
            reps = max(2, -(-launches // n))
            graph.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                graph.replay()
            e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * n)

    def entry(self, us, nbytes, **extra):
        return {**extra, "us": us, "GB/s": nbytes / us * 1e-3, "frac_of_hbm_peak": nbytes / us * 1e-3 / HBM_PEAK_GBPS}

    def cold_and_single(self, calls, nbytes, launches, **extra):
        """A workload timed over its rotated sets (cold: HBM) and on the first set alone (its working set stays
        in the memory-side cache when it fits)."""
        cold = self.entry(self.timed(calls, launches), nbytes)
        single = self.entry(self.timed(calls[:1], launches, warm=3), nbytes)
        out = {**extra, "algorithmic_bytes": nbytes, "sets": len(calls), "cold": cold, "single_set": single}
        if cold["us"] < 40.0:  # launch-bound from Python: the same rotation replayed from a HIP graph
            out["cold_graph_replay"] = self.entry(self.timed_graph(calls, launches), nbytes)
        return out

    def empty(self, *shape, dtype=None):
        return self.torch.empty(shape, dtype=dtype or self.torch.uint8, device=self.dev)


def main():
    a = parse()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU; there is no multi-GPU path "
                         "(the conversions shard by rows with no exchange). Use --gpus 1.\n")
        sys.exit(2)
    phases = [p for p in a.phases.split(",") if p]
    for p in phases:
        if p not in PHASES:
            sys.stderr.write(f"bench.py: unknown phase {p!r}; known: {', '.join(PHASES)}\n")
            sys.exit(2)
    if a.no_cpu_baseline and "cpu" in phases:
        phases.remove("cpu")

    import torch
    import paper_2603_02731_amd as mx
    from paper_2603_02731_amd import synth

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    mx.lib()  # fail loudly here if the HIP library is missing
    B = Bench(torch, mx, synth, a)

    if a.copy_calibration:
        n = 512 << 20
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(a.steps):
            mx.mxfp4_stream_copy(src, dst, policy=1)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "launches": a.steps, "bytes_read_per_launch": n,
                          "bytes_written_per_launch": n}))
        return

    M, K = a.rows, a.hidden
    R = max(3, a.sets)
    n = M * K
    names = ["quant", "dequant", "row_to_col"]
    alg = {k: n * BYTES_PER_ELEM[k] for k in names}
    total_bytes = sum(alg.values())

    # ---- the workload: R buffer sets holding the same synthetic activations at different addresses
    x8_0, s_0 = synth.student_t_fp8(M, K, seed=a.seed, device=dev)
    S = []
    for r in range(R):
        S.append({"x8": x8_0 if r == 0 else x8_0.clone(), "s": s_0 if r == 0 else s_0.clone(),
                  "q": B.empty(M, K // 2), "sf": B.empty(M, K // 32), "xb": B.empty(M, K),
                  "sb": B.empty(M, K // 128, dtype=torch.float32), "qc": B.empty(K, M // 2), "sc": B.empty(K, M // 32)})

    def quant(t):
        mx.mxfp4_quant_from_fp8(t["x8"], t["s"], q=t["q"], sf=t["sf"])

    def dequant(t):
        mx.mxfp4_dequant_to_fp8(t["q"], t["sf"], x=t["xb"], x_scale=t["sb"])

    def row_to_col(t):
        mx.mxfp4_row_to_col(t["q"], t["sf"], q_col=t["qc"], sf_col=t["sc"])

    fns = {"quant": quant, "dequant": dequant, "row_to_col": row_to_col}
    for t in S:  # every set holds valid MXFP4 before anything reads it
        quant(t), dequant(t), row_to_col(t)
    torch.cuda.synchronize()

    out = {
        "metric": "HBM GB/s (% of peak) for FP8<->MXFP4 quant/dequant and MXFP4 row->col",
        "value": None, "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"target_{M}x{K}: Student-t(df=3) activations with 1% outlier channels x100, "
                               f"FP8 E4M3 + FP32 1x128 scales; step = quant + dequant + row_to_col over {R} "
                               f"rotated buffer sets (every input comes from HBM, not from the memory-side cache)",
                   "rows": M, "hidden": K, "seed": a.seed, "buffer_sets": R},
        "phases": phases,
    }

    # ---- the whole step over rotated sets: `value`
    if "step" in phases:
        def step(i):
            quant(S[i % R])
            dequant(S[(i + 1) % R])
            row_to_col(S[(i + 2) % R])

        for i in range(a.warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(a.steps):
            step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms = (t1 - t0) * 1e3 / a.steps
        out["ms_per_step"] = ms
        out["value"] = total_bytes / (ms * 1e-3) * 1e-9
        out["frac_of_hbm_peak"] = out["value"] / HBM_PEAK_GBPS
        out["elements_per_s"] = 3 * n / (ms * 1e-3)

    kernels = {k: {"algorithmic_bytes": alg[k], "traffic": measured_traffic(k, M, K)} for k in names}

    # ---- one buffer set, the kernels in training order, events around each kernel in every N-th step
    if "in_step" in phases:
        t = S[0]
        stride = max(1, min(a.event_stride, a.steps // 8))  # at least eight bracketed steps
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] if i % stride == 0 else None
                  for i in range(a.steps)]
        for _ in range(a.warmup):
            quant(t), dequant(t), row_to_col(t)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for ev in events:
            for j, k in enumerate(names):
                if ev:
                    ev[j].record()
                fns[k](t)
            if ev:
                ev[3].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        events = [e for e in events if e is not None]
        for j, k in enumerate(names):
            us = sum(e[j].elapsed_time(e[j + 1]) for e in events) * 1e3 / len(events)
            kernels[k]["in_step"] = B.entry(us, alg[k])
        ms1 = (t1 - t0) * 1e3 / a.steps
        out["in_step"] = {"ms_per_step": ms1, "GB/s": total_bytes / (ms1 * 1e-3) * 1e-9,
                          "note": "one buffer set: dequant and row_to_col read what quant has just written "
                                  "(249.6 MB, inside the 256 MB memory-side cache)",
                          "events_every_nth_step": stride, "steps_with_events": len(events)}

    # ---- each kernel on its own over the rotated sets: the figures held against the HBM peak
    if "cold" in phases:
        for k in names:
            us = B.timed([lambda t=t, k=k: fns[k](t) for t in S], a.cold_launches)
            kernels[k]["cold"] = B.entry(us, alg[k], elements_per_s=n / us * 1e6, launches=a.cold_launches)
        worst = min(names, key=lambda k: kernels[k]["cold"]["frac_of_hbm_peak"])
        c = kernels[worst]["cold"]
        out["roofline"] = {"bound": "hbm", "kernel": worst, "achieved": c["GB/s"], "peak": HBM_PEAK_GBPS,
                           "unit": "GB/s", "frac": c["frac_of_hbm_peak"], "traffic": kernels[worst]["traffic"],
                           "how": f"lowest of the three kernels; algorithmic bytes / average duration of "
                                  f"{a.cold_launches} back-to-back launches over {R} rotated buffer sets "
                                  f"(HIP events on the launch stream)"}
    out["kernels"] = kernels

    # ---- the measured roof: the library's 16-byte-per-lane copy over the same rotated sets (470 MB each way)
    if "copy" in phases:
        pol = {}
        for p, label in ((0, "plain"), (1, "nt_load"), (2, "nt_store"), (3, "nt_both")):
            us = B.timed([lambda t=t, p=p: mx.mxfp4_stream_copy(t["x8"].view(-1), t["xb"].view(-1), policy=p)
                          for t in S], 30)
            pol[label] = 2 * n / us * 1e-3
        best = max(pol.values())
        out["copy"] = {"GB/s": best, "frac_of_hbm_peak": best / HBM_PEAK_GBPS, "by_policy_GB/s": pol,
                       "what": "mxfp4_stream_copy, 16-byte loads and stores, rotated sets"}
        # the same bytes as each kernel moves (without its scales), in its read : write mix and access pattern,
        # by kernels that do no arithmetic: what this GPU gives the pattern itself
        movers = {
            "quant": ("mxfp4_stream_mix 2:1 (16 B read, 8 B written per lane)", 1.5 * n,
                      lambda t: mx.mxfp4_stream_mix(t["x8"].view(-1), t["q"].view(-1), 1)),
            "dequant": ("mxfp4_stream_mix 1:2 (8 B read, 16 B written per lane)", 1.5 * n,
                        lambda t: mx.mxfp4_stream_mix(t["q"].view(-1), t["xb"].view(-1), 2)),
            "row_to_col": ("mxfp4_tile_copy (256 x 128-byte tiles read, 256 pieces of 128 B written each)", 1.0 * n,
                           lambda t: mx.mxfp4_tile_copy(t["q"], t["xb"].view(-1))),
            "read_only": ("mxfp4_stream_mix read only", 1.0 * n,
                          lambda t: mx.mxfp4_stream_mix(t["x8"].view(-1), t["sb"].view(torch.uint8).view(-1), 3)),
        }
        out["movers"] = {}
        for k, (what, nbytes, fn) in movers.items():
            us = B.timed([lambda t=t, fn=fn: fn(t) for t in S], 30)
            out["movers"][k] = {"what": what, "us": us, "bytes": nbytes, "GB/s": nbytes / us * 1e-3,
                                "frac_of_hbm_peak": nbytes / us * 1e-3 / HBM_PEAK_GBPS}
        for k in names:
            if "cold" in kernels[k]:
                kernels[k]["cold"]["frac_of_measured_copy"] = kernels[k]["cold"]["GB/s"] / best
                kernels[k]["cold"]["frac_of_its_mover"] = kernels[k]["cold"]["GB/s"] / out["movers"][k]["GB/s"]
        if "roofline" in out:  # the same kernel against a kernel that only moves its bytes in its access pattern
            w = out["roofline"]["kernel"]
            out["roofline"]["mover"] = {"what": out["movers"][w]["what"], "GB/s": out["movers"][w]["GB/s"],
                                        "frac_of_hbm_peak": out["movers"][w]["frac_of_hbm_peak"],
                                        "kernel_rate_over_mover_rate": kernels[w]["cold"]["frac_of_its_mover"]}
        for t in S:  # the movers wrote over the MXFP4 and FP8 outputs: every set holds valid data again
            quant(t), dequant(t), row_to_col(t)
        torch.cuda.synchronize()

    if "configs" in phases:
        out["configs"] = time_configs(B, S[0])
    if "variants" in phases:
        out["variants"] = time_variants(B, S)
    if "cpu" in phases:
        out["cpu_baseline"] = cpu_baseline(x8_0, s_0, min(a.cpu_sample_rows, M))
    print(json.dumps(out))


def time_configs(B, target):
    """The named workloads besides the target shape, each cold (rotated sets) and on a single set."""
    torch, mx, synth, a = B.torch, B.mx, B.synth, B.a
    dev = B.dev
    res = {}

    def want(c):
        return a.config is None or a.config == c

    def clones(t, r):
        return [t] + [t.clone() for _ in range(r - 1)]

    if want(2):
        # activation quantize / de-quantize at the hidden size: [4096, 7168], 45.9 MB per launch
        M, K = 4096, 7168
        nb = M * K * BYTES_PER_ELEM["quant"]
        r = sets_for(nb)
        x8, s = synth.student_t_fp8(M, K, seed=a.seed, device=dev)
        xs, ss = clones(x8, r), clones(s, r)
        qs = [B.empty(M, K // 2) for _ in range(r)]
        sfs = [B.empty(M, K // 32) for _ in range(r)]
        xo = [B.empty(M, K) for _ in range(r)]
        so = [B.empty(M, K // 128, dtype=torch.float32) for _ in range(r)]
        res["config2_quant_4096x7168"] = B.cold_and_single(
            [lambda i=i: mx.mxfp4_quant_from_fp8(xs[i], ss[i], q=qs[i], sf=sfs[i]) for i in range(r)], nb, 200)
        res["config2_dequant_4096x7168"] = B.cold_and_single(
            [lambda i=i: mx.mxfp4_dequant_to_fp8(qs[i], sfs[i], x=xo[i], x_scale=so[i]) for i in range(r)], nb, 200)
        del xs, ss, qs, sfs, xo, so

    if want(3):
        # expert-FFN activations silu(a)*b as row-blocked MXFP4 [16384, 2048] -> column-blocked, 35.7 MB per launch
        M, K = 16384, 2048
        nb = M * K * BYTES_PER_ELEM["row_to_col"]
        r = sets_for(nb)
        x8, s = synth.swiglu_fp8(M, K, seed=a.seed, device=dev)
        q, sf = mx.mxfp4_quant_from_fp8(x8, s)
        qs, sfs = clones(q, r), clones(sf, r)
        qc = [B.empty(K, M // 2) for _ in range(r)]
        sc = [B.empty(K, M // 32) for _ in range(r)]
        res["config3_row_to_col_16384x2048"] = B.cold_and_single(
            [lambda i=i: mx.mxfp4_row_to_col(qs[i], sfs[i], q_col=qc[i], sf_col=sc[i]) for i in range(r)], nb, 200)
        xc = [B.empty(K, M) for _ in range(r)]
        xcs = [B.empty(K, M // 128, dtype=torch.float32) for _ in range(r)]
        nb8 = M * K * (MX_B + FP8_B)
        res["config3_row_to_fp8_col_16384x2048"] = B.cold_and_single(
            [lambda i=i: mx.mxfp4_row_to_fp8_col(qs[i], sfs[i], x_col=xc[i], x_col_scale=xcs[i]) for i in range(r)],
            nb8, 200)
        del qs, sfs, qc, sc, xc, xcs

    if want(4):
        # 32 local experts, Zipf(1.2) token counts summing to 65536: FP8 [T_e, 7168] for the grouped quantizer,
        # MXFP4 [T_e, 2048] for the grouped transposing kernels; padded to 128 rows as the config says, and
        # the same counts without padding
        for pad, tag in ((128, "padded128"), (1, "unpadded")):
            off, counts = synth.expert_offsets(seed=a.seed, num_experts=32, total_tokens=65536, pad_to=pad)
            Mt = int(off[-1])
            offd = off.to(dev)
            if pad == 128:
                K = 7168
                nb = Mt * K * BYTES_PER_ELEM["quant"]
                r = sets_for(nb)
                x8, s = synth.student_t_fp8(Mt, K, seed=a.seed + 4, device=dev)
                synth.zero_padding_rows(x8, s, off, counts)
                xs, ss = clones(x8, r), clones(s, r)
                qs = [B.empty(Mt, K // 2) for _ in range(r)]
                sfs = [B.empty(Mt, K // 32) for _ in range(r)]
                res[f"config4_quant_grouped_{tag}_K7168"] = B.cold_and_single(
                    [lambda i=i: mx.mxfp4_quant_from_fp8_grouped(xs[i], ss[i], offd, q=qs[i], sf=sfs[i])
                     for i in range(r)], nb, 40, rows=Mt)
                del xs, ss, qs, sfs, x8, s
            K = 2048
            x8, s = synth.swiglu_fp8(Mt, K, seed=a.seed + 4, device=dev)
            if pad == 128:
                synth.zero_padding_rows(x8, s, off, counts)
            q, sf = mx.mxfp4_quant_from_fp8(x8, s)
            nb = Mt * K * BYTES_PER_ELEM["row_to_col"]
            r = sets_for(nb)
            qs, sfs = clones(q, r), clones(sf, r)
            qc = [B.empty(K * (Mt // 2 + 32)) for _ in range(r)]
            sc = [B.empty(K * (Mt // 32 + 32)) for _ in range(r)]
            res[f"config4_row_to_col_grouped_{tag}_K2048"] = B.cold_and_single(
                [lambda i=i: mx.mxfp4_row_to_col_grouped(qs[i], sfs[i], offd, q_col=qc[i], sf_col=sc[i])
                 for i in range(r)], nb, 100, rows=Mt)
            del qc, sc
            nb8 = Mt * K * (MX_B + FP8_B)
            r8 = min(r, sets_for(nb8))
            xc = [B.empty(K * Mt) for _ in range(r8)]
            xcs = [B.empty(K * (Mt // 128 + 32), dtype=torch.float32) for _ in range(r8)]
            res[f"config4_row_to_fp8_col_grouped_{tag}_K2048"] = B.cold_and_single(
                [lambda i=i: mx.mxfp4_row_to_fp8_col_grouped(qs[i], sfs[i], offd, x_col=xc[i], x_col_scale=xcs[i])
                 for i in range(r8)], nb8, 100, rows=Mt)
            del qs, sfs, xc, xcs

    if want(5):
        # dispatch payload: 65536 tokens x top-8 into 3808-byte records (nibbles then scale bytes), each token
        # read and quantized once and written to its 8 destinations; then the 524288 records de-quantized.
        # Compulsory bytes: the source once, the indices, the payload; every launch moves gigabytes, so two sets
        # are a cold rotation.
        x8, s = target["x8"], target["s"]
        M, K = x8.shape
        top_k = 8
        idx = synth.routing_indices(seed=a.seed, num_tokens=M, top_k=top_k, device=dev)
        Mo = idx.shape[0]
        dst = torch.argsort(idx.long(), stable=True).to(torch.int32).view(M, top_k).contiguous()
        rec = K // 2 + K // 32
        bufs = [B.empty(Mo * rec) for _ in range(2)]
        nbq = M * K * FP8_B + Mo * 4 + Mo * rec
        res["config5_quant_scatter_top8_records"] = B.cold_and_single(
            [lambda b=b: mx.mxfp4_quant_from_fp8_scatter(x8, s, dst, Mo, q=b, sf=b[K // 2:], ld_q=rec, ld_sf=rec)
             for b in bufs], nbq, 10, rows_out=Mo, bytes_are="compulsory: source once + indices + payload")
        xo = [B.empty(Mo, K) for _ in range(2)]
        so = [B.empty(Mo, K // 128, dtype=torch.float32) for _ in range(2)]
        nbd = Mo * K * BYTES_PER_ELEM["dequant"]
        res["config5_dequant_records"] = B.cold_and_single(
            [lambda i=i: mx.mxfp4_dequant_to_fp8(bufs[i], bufs[i][K // 2:], M=Mo, K=K, ld_q=rec, ld_sf=rec,
                                                 x=xo[i], x_scale=so[i]) for i in range(2)], nbd, 10, rows=Mo)
        del xo, so
        # the gather form of the same payload (every token read and quantized once per destination)
        res["config5_quant_gather_top8_records"] = B.cold_and_single(
            [lambda b=b: mx.mxfp4_quant_from_fp8(x8, s, gather_idx=idx, q=b, sf=b[K // 2:], ld_q=rec, ld_sf=rec)
             for b in bufs], nbq, 5, rows_out=Mo, bytes_are="compulsory: source once + indices + payload")
        # the write traffic of the scatter without the quantizer: 65536 ready records, each written to the same 8
        # destinations (a mover: it reads half the bytes of the quantizer and does no arithmetic)
        recs = torch.randint(0, 256, (M, rec), dtype=torch.uint8, device=dev)
        res["config5_record_fanout_mover"] = B.cold_and_single(
            [lambda b=b: mx.mxfp4_record_fanout(recs, dst, b) for b in bufs], M * rec + Mo * 4 + Mo * rec, 10,
            rows_out=Mo, bytes_are="the mover's own: records once + indices + payload")
        res["config5_quant_scatter_top8_records"]["cold"]["time_of_its_mover_over_its_time"] = (
            res["config5_record_fanout_mover"]["cold"]["us"] / res["config5_quant_scatter_top8_records"]["cold"]["us"])
        del bufs, recs
    return res


def time_variants(B, S):
    """The other entry points at the target shape, over the rotated sets (cold)."""
    torch, mx, synth, a = B.torch, B.mx, B.synth, B.a
    dev = B.dev
    M, K = S[0]["x8"].shape
    R = len(S)
    res = {}

    def want(name):
        return a.variant is None or a.variant == name

    f8 = MX_B + FP8_B  # row-blocked MXFP4 read, FP8 + FP32 per 128 written
    if want("quant_from_bf16"):
        # the paper's BF16-source row quantizer on the same activations (2 B read + 0.53125 B written per element)
        xbf = []
        for t in S[:2]:
            v = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
            for r0 in range(0, M, 8192):
                v[r0:r0 + 8192] = (t["x8"][r0:r0 + 8192].view(torch.float8_e4m3fn).float()
                                   * t["s"][r0:r0 + 8192].repeat_interleave(128, dim=1)).to(torch.bfloat16)
            xbf.append(v)
        res["quant_from_bf16"] = B.entry(B.timed(
            [lambda i=i: mx.mxfp4_quant_from_bf16(xbf[i], q=S[i]["qc"].view(M, K // 2), sf=S[i]["sc"].view(M, K // 32))
             for i in range(2)], 20), M * K * (2.0 + MX_B))
        del xbf
    for name, requant in (("row_to_fp8_col", False), ("row_to_fp8_col_requant", True)):
        if want(name):
            # the paper's literal weight-gradient kernel: row-blocked MXFP4 -> column-wise FP8 (both readings)
            xcs = [B.empty(K, M // 128, dtype=torch.float32) for _ in range(R)]
            res[name] = B.entry(B.timed(
                [lambda i=i: mx.mxfp4_row_to_fp8_col(S[i]["q"], S[i]["sf"], x_col=S[i]["xb"].view(K, M),
                                                     x_col_scale=xcs[i], requant=requant) for i in range(R)], 30),
                M * K * f8)
    # grouped forms on the target's MXFP4 rows: 32 Zipf-sized experts, padded to 128 rows and un-padded
    for pad, tag in ((128, "grouped_32_experts"), (1, "ragged_32_experts")):
        off, _ = synth.expert_offsets(seed=a.seed, num_experts=32, total_tokens=M - 32 * 128, pad_to=pad)
        Mt = int(off[-1])
        if Mt > M:
            continue
        offd = off.to(dev)
        if want("row_to_col_" + tag):
            scr = [B.empty(K * (Mt // 32 + 32)) for _ in range(R)]
            res["row_to_col_" + tag] = B.entry(B.timed(
                [lambda i=i: mx.mxfp4_row_to_col_grouped(S[i]["q"][:Mt], S[i]["sf"][:Mt], offd,
                                                         q_col=S[i]["xb"].view(-1), sf_col=scr[i])
                 for i in range(R)], 30), Mt * K * BYTES_PER_ELEM["row_to_col"], rows=Mt)
        for name, requant in (("row_to_fp8_col_" + tag, False), ("row_to_fp8_col_requant_" + tag, True)):
            if want(name):
                xcs = [B.empty(K * (Mt // 128 + 32), dtype=torch.float32) for _ in range(R)]
                res[name] = B.entry(B.timed(
                    [lambda i=i: mx.mxfp4_row_to_fp8_col_grouped(S[i]["q"][:Mt], S[i]["sf"][:Mt], offd,
                                                                 x_col=S[i]["xb"].view(-1), x_col_scale=xcs[i],
                                                                 requant=requant) for i in range(R)], 30),
                    Mt * K * f8, rows=Mt)
    return res


if __name__ == "__main__":
    main()
