#!/usr/bin/env python3
"""Benchmark of the FBSR hot path on one MI355X.

Headline metric: fp32 -> fp8 few-bit stochastic rounding throughput (elements/s) and achieved
HBM GB/s against the 8 TB/s peak, at N = 2, 4, 8 random bits, on 2^28 full-range elements
(the benchmark's third workload, the size the 70 %-of-peak target is quoted on).

One "step" = one pass over the batch for every (format, N, variant) of the headline sweep:
{E4M3, E5M2} x {2, 4, 8} x {SRFF, SRF, SRC} = 18 fbsr_round launches of 2^28 elements each, all
through the C ABI.  Inputs are resident in HBM before the timed region starts.  The other paths
(bf16 rounding, fused SGD update, bias statistics, and the RNE launch that serves as a
streaming ceiling) are timed separately and reported under "paths".

Prints ONE JSON line.
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
# Vector-ALU ceiling for the paths that HBM does not bound: the part's published fp32 vector peak of 157.3 TFLOP/s is
# 78.6 x 10^12 fused multiply-adds a second, i.e. one-lane operations a second at the widest issue the vector ALUs have
# (256 compute units x 128 lanes x 2.4 GHz).  No instruction mix can pass it; the integer / conversion / fp64 instructions
# these kernels are made of run at about half that rate, so read the fraction as an upper-bound-normalised figure.
ALU_PEAK_LANE_OPS = 157.3e12 / 2
# Counter-derived figures (VALU instructions per element per path, HBM traffic of the headline launch) come from
# profiles/kernel_counters.json, which `python -m paper_2504_20634_amd.profile_summary` writes from rocprofv3 --pmc runs
# of this file together with a hash of the kernel sources.  When the sources have changed since, the figures are
# stale and are left out.
COUNTERS_JSON = os.path.join(ROOT, "profiles", "kernel_counters.json")
# The kernel each secondary path launches, as rocprofv3 names it (template arguments: round_tiles<fmt, variant, W>,
# round16_tiles<src, fmt, variant, W>, format8_tiles<src, ties, W, 16-bit codes>, block_tiles<fmt, variant, W>,
# format8_lut_tiles<src, W>, sgd_tiles<variant, W>, stats_spans<fmt, variant, W>, stats8_spans<W>, qat_tiles<codec, W>; fmt 0 bf16, 1 E4M3, 2 E5M2, 3 binary8p4;
# variant 0 RNE, 1 SRFF, 2 SRF, 3 SRC; W the slot width).  The profile summary joins counters to paths through these.
PATH_KERNELS = {
    "stream_4to1_no_arithmetic_ceiling": "fbsr::stream41_tiles", "stream_7to5_no_arithmetic_ceiling": "fbsr::stream75_tiles",
    "round_e4m3_rne_ceiling": "fbsr::round_tiles<1, 0, 8>",
    "round_bf16_N4_srf": "fbsr::round_tiles<0, 2, 4>", "round_bf16_N8_srf": "fbsr::round_tiles<0, 2, 8>",
    "round_bf16_N16_srf": "fbsr::round_tiles<0, 2, 16>",
    "round_from_bf16_e4m3_N3_src": "fbsr::round16_tiles<0, 1, 3, 4>", "round_from_bf16_e5m2_N3_srf": "fbsr::round16_tiles<0, 2, 2, 4>",
    "round_from_bf16_e4m3_N8_srff": "fbsr::round16_tiles<0, 1, 1, 8>", "round_from_bf16_e4m3_N20_srff": "fbsr::round16_tiles<0, 1, 1, 32>",
    "round_binary8p4_N3_src": "fbsr::round_tiles<3, 3, 4>", "round_binary8p4_N8_srff": "fbsr::round_tiles<3, 1, 8>",
    "round_e4m3_N20_classical_sr": "fbsr::round_tiles<1, 1, 32>", "round_e4m3_N24_src": "fbsr::round_tiles<1, 3, 32>",
    "round_from_bf16_binary8p4_N3_src": "fbsr::round16_tiles<0, 3, 3, 4>",
    "round_format8_binary8p4_from_fp32_N3_src": "fbsr::format8_tiles<2, true, 4, false>",
    "round_format8_binary8p4_from_fp32_N8_srf": "fbsr::format8_tiles<2, false, 8, false>",
    "round_format8_binary8p4_from_fp32_N3_src_ties_odd": "fbsr::format8_tiles<2, true, 4, false>",
    "round_format8_binary8p4_from_fp32_N20_srff": "fbsr::format8_tiles<2, false, 32, false>",
    "round_format8_binary8p4_from_bf16_N3_src": "fbsr::format8_lut_tiles<0, 4>",
    "round_format8_binary8p4_from_bf16_N3_srff": "fbsr::format8_lut_tiles<0, 4>",
    "round_format16_binary16_from_fp32_N3_src": "fbsr::format8_tiles<2, true, 4, true>",
    "round_format16_binary16_from_fp32_N8_srf": "fbsr::format8_tiles<2, false, 8, true>",
    "round_block_scaled_e4m3_N3_src": "fbsr::block_tiles<1, 3, 4>", "round_block_scaled_e5m2_N8_srf": "fbsr::block_tiles<2, 2, 8>",
    "round_block_scaled_e4m3_N20_srff": "fbsr::block_tiles<1, 1, 32>",
    "qat_adamw_e4m3_N3_src": "fbsr::qat_tiles<fbsr::FixedCodec<1, 3>, 4>", "qat_adamw_e4m3_N3_srff": "fbsr::qat_tiles<fbsr::FixedCodec<1, 1>, 4>",
    "qat_adamw_binary8p4_N3_src": "fbsr::qat_tiles<fbsr::FixedCodec<3, 3>, 4>", "qat_adamw_binary8p4_N3_srff": "fbsr::qat_tiles<fbsr::FixedCodec<3, 1>, 4>",
    "qat_adamw_format8_binary8p4_N3_src": "fbsr::qat_tiles<fbsr::Codec8<true, true>, 4>",
    "qat_adamw_format8_binary8p4_N3_srff": "fbsr::qat_tiles<fbsr::Codec8<false, true>, 4>",
    "sgd_update_bf16_N2_srf": "fbsr::sgd_tiles<2, 2>", "sgd_update_bf16_N4_srf": "fbsr::sgd_tiles<2, 4>", "sgd_update_bf16_N8_srf": "fbsr::sgd_tiles<2, 8>",
    "bias_stats_e4m3_N3_srf": "fbsr::stats_spans<1, 2, 4>", "bias_stats_e4m3_N8_srf": "fbsr::stats_spans<1, 2, 8>",
    "bias_stats_bf16_N2_srf": "fbsr::stats_spans<0, 2, 2>", "bias_stats_bf16_N8_srf": "fbsr::stats_spans<0, 2, 8>",
    "bias_stats_format8_binary8p4_N3_srf": "fbsr::stats8_spans<4>", "bias_stats_format8_binary8p4_N3_src": "fbsr::stats8_spans<4>",
}
N_ELEMS = 1 << 28
SGD_ELEMS = 1 << 27
HEADLINE_NBITS = (2, 4, 8)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--elems-log2", type=int, default=28, help="log2 of the batch size (default 28)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-paths", action="store_true", help="skip the secondary paths (profiling runs)")
    ap.add_argument("--no-workloads", action="store_true", help="skip the five-workload report")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run two plain device copies of the 1 GiB input (a kernel of known traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def kernel_sources_hash():
    """sha256 over the kernel sources and headers, in a fixed order (what the counter figures belong to)."""
    import hashlib
    h = hashlib.sha256()
    for folder in (os.path.join(ROOT, "paper_2504_20634_amd", "csrc"), os.path.join(ROOT, "include")):
        for name in sorted(os.listdir(folder)):
            if name.endswith((".hip", ".h")):
                h.update(name.encode())
                with open(os.path.join(folder, name), "rb") as fh:
                    h.update(fh.read())
    return h.hexdigest()


def load_counters():
    """(figures, note): the counter-derived figures if they belong to the sources at hand, else ({}, why not)."""
    try:
        with open(COUNTERS_JSON) as fh:
            c = json.load(fh)
    except (OSError, ValueError):
        return {}, "no profiles/kernel_counters.json"
    if c.get("sources_sha256") != kernel_sources_hash():
        return {}, "profiles/kernel_counters.json belongs to other kernel sources (stale): counter-derived figures left out"
    return c, "profiles/kernel_counters.json"


# Every secondary path is timed over this many launches, after launches of the same call have kept the GPU busy for
# WARM_MS: when load sets in after a pause the part's clocks dip for some tens of milliseconds and recover, which a short
# burst of a dozen launches of an arithmetic-heavy kernel reads as anything from 70 % to 100 % of its steady rate.
TIMED_LAUNCHES = 12
WARM_MS = 40.0


def keep_busy(torch, fn, ms=WARM_MS, batch=8):
    """Launches fn() in batches until they have kept the GPU busy for `ms` milliseconds."""
    t0 = time.perf_counter()
    while True:
        for _ in range(batch):
            fn()
        torch.cuda.synchronize()
        if (time.perf_counter() - t0) * 1e3 >= ms:
            return


def timed_launches(torch, fn, reps=TIMED_LAUNCHES):
    """Average duration (ms) of fn()'s GPU work over `reps` launches in the steady state, from events recorded on
    the stream the kernels are launched on (torch's current stream)."""
    keep_busy(torch, fn)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in evs) / reps


def timed_sweep(torch, launches, reps=3):
    """Average duration (ms) of one pass over `launches` (a list of callables), from events around whole passes."""
    def one_pass():
        for fn in launches:
            fn()
    keep_busy(torch, one_pass, batch=1)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        for fn in launches:
            fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def five_workloads(torch, np, fbsr, workloads, x_e5m2):
    """Throughput on the five synthetic workloads at their own sizes (elements/s and algorithmic GB/s per launch,
    averaged over each workload's sweep).  x_e5m2: 2^28 full-range inputs already on the device."""
    rep = {}

    def entry(elements, launches, ms, bytes_per_elem, note):
        per = ms / launches
        return {"elements": elements, "launches": launches, "ms_per_launch": round(per, 4), "gelem_s": round(elements / per / 1e6, 1),
                "gb_s": round(bytes_per_elem * elements / per / 1e6, 1), "bytes_per_elem": bytes_per_elem, "note": note}

    # 1: Fig. 1 sweep, 1024 X values x 5000 samples -> bf16, N = 2, rounded values and per-X statistics in one pass
    x1 = torch.from_numpy(workloads.fig1_grid()[0]).cuda()
    n1 = x1.numel()
    out1 = torch.empty(n1, dtype=torch.uint16, device="cuda")
    st1 = torch.zeros((1024, 4), dtype=torch.float64, device="cuda")
    ws1 = torch.empty(fbsr.bias_stats_workspace_bytes(n1, 1024) // 8 + 1, dtype=torch.float64, device="cuda")
    ls = [lambda v=v: fbsr.fbsr_bias_stats(x1, fbsr.FMT_BF16, v, 2, 0, 0, 5000, 0, 1024, stats=st1, out=out1, workspace=ws1)
          for v in (fbsr.SRFF, fbsr.SRF, fbsr.SRC)]
    rep["1_fig1_sweep_bf16_N2"] = entry(n1, len(ls), timed_sweep(torch, ls, 10), 6.0,
                                        "fbsr_bias_stats with codes written; 20 MB input, resident in the last-level cache")
    del x1, out1
    # 2: 2^24 scaled normals -> E4M3, N in {1,2,3,4,6,8} x 3 variants
    x2 = torch.from_numpy(workloads.scaled_normal(1 << 24, seed=1)).cuda()
    out2 = torch.empty(1 << 24, dtype=torch.uint8, device="cuda")
    ls = [lambda nb=nb, v=v: fbsr.fbsr_round(x2, fbsr.FMT_E4M3, v, nb, seed=1, out=out2)
          for nb in (1, 2, 3, 4, 6, 8) for v in (fbsr.SRFF, fbsr.SRF, fbsr.SRC)]
    rep["2_e4m3_scaled_normal_2p24"] = entry(1 << 24, len(ls), timed_sweep(torch, ls, 5), 5.0,
                                             "64 MiB input, resident in the 256 MB last-level cache: not an HBM figure")
    del x2, out2
    # 3: 2^28 full-range -> E5M2 and bf16, N in {4,8,16} x 3 variants
    n3 = x_e5m2.numel()
    xb = torch.from_numpy(workloads.full_range(n3, "bf16", seed=2)).cuda()
    o8 = [torch.empty(n3, dtype=torch.uint8, device="cuda") for _ in range(2)]
    o16 = [torch.empty(n3, dtype=torch.uint16, device="cuda") for _ in range(2)]
    ls = [lambda nb=nb, v=v, k=k: fbsr.fbsr_round(x_e5m2, fbsr.FMT_E5M2, v, nb, seed=2, out=o8[k % 2])
          for k, (nb, v) in enumerate((nb, v) for nb in (4, 8, 16) for v in (fbsr.SRFF, fbsr.SRF, fbsr.SRC))]
    rep["3_e5m2_full_range_2p28"] = entry(n3, len(ls), timed_sweep(torch, ls, 3), 5.0, "N in {4,8,16} x {srff,srf,src}")
    ls = [lambda nb=nb, v=v, k=k: fbsr.fbsr_round(xb, fbsr.FMT_BF16, v, nb, seed=2, out=o16[k % 2])
          for k, (nb, v) in enumerate((nb, v) for nb in (4, 8, 16) for v in (fbsr.SRFF, fbsr.SRF, fbsr.SRC))]
    rep["3_bf16_full_range_2p28"] = entry(n3, len(ls), timed_sweep(torch, ls, 3), 6.0, "N in {4,8,16} x {srff,srf,src}")
    del xb, o8, o16
    # 4: fused SGD update, 2^27 bf16 weights, fresh gradients, N in {2,4,8} x 3 variants and RNE
    n4 = 1 << 27
    w4 = [torch.from_numpy(workloads.sgd_weights(n4, seed=3 + k).view(np.int16)).cuda() for k in range(3)]
    g4 = [torch.from_numpy(workloads.sgd_grads(n4, k, seed=3)).cuda() for k in range(3)]
    cases = [(fbsr.RNE, 0)] + [(v, nb) for nb in (2, 4, 8) for v in (fbsr.SRFF, fbsr.SRF, fbsr.SRC)]
    ls = [lambda v=v, nb=nb, k=k: fbsr.fbsr_sgd_update(w4[k % 3], g4[k % 3], 1e-3, v, nb, seed=4, step=k) for k, (v, nb) in enumerate(cases)]
    rep["4_sgd_update_bf16_2p27"] = entry(n4, len(ls), timed_sweep(torch, ls, 5), 8.0, "RNE and N in {2,4,8} x {srff,srf,src}")
    del w4, g4
    # 5: 2^30 inputs in 4096 log-spaced bins of 2^18 over [2^-10, 2^10), statistics only, E4M3 and bf16 x 3 variants x N = 1..12
    nb5, grp = 4096, 1 << 18
    edges = torch.exp2(-10.0 + 20.0 * torch.arange(nb5 + 1, dtype=torch.float64, device="cuda") / nb5).float().double()
    x5 = torch.empty(nb5 * grp, dtype=torch.float32, device="cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    for b0 in range(0, nb5, 256):
        u = torch.rand((256, grp), dtype=torch.float64, device="cuda", generator=gen)
        lo, hi = edges[b0:b0 + 256, None], edges[b0 + 1:b0 + 257, None]
        x5[b0 * grp:(b0 + 256) * grp] = torch.minimum(lo + u * (hi - lo), torch.nextafter(hi.float(), lo.float()).double()).float().reshape(-1)
        del u
    st5 = torch.zeros((nb5, 4), dtype=torch.float64, device="cuda")
    ws5 = torch.empty(fbsr.bias_stats_workspace_bytes(nb5 * grp, nb5) // 8 + 1, dtype=torch.float64, device="cuda")
    for f, name in ((fbsr.FMT_E4M3, "e4m3"), (fbsr.FMT_BF16, "bf16")):
        ls = [lambda v=v, nb=nb: fbsr.fbsr_bias_stats(x5, f, v, nb, 5, 0, grp, 0, nb5, stats=st5, workspace=ws5)
              for v in (fbsr.SRFF, fbsr.SRF, fbsr.SRC) for nb in range(1, 13)]
        rep["5_bias_stats_%s_2p30" % name] = entry(nb5 * grp, len(ls), timed_sweep(torch, ls, 1), 4.0,
                                                   "statistics only (out = NULL), 3 variants x N = 1..12; inputs drawn on the device")
    return rep


def cpu_baseline(x_host, fmts, variants, threads):
    """The oracle as it stands, timed on the host cores over a bounded sample of the same
    workload: the first 2^25 elements, every (format, N, variant) of the headline sweep."""
    from oracle import fbsr_oracle as oracle
    sample = 1 << 25
    done = 0
    t0 = time.perf_counter()
    for fmt in fmts:
        xs = x_host[fmt][:sample]
        for nbits in HEADLINE_NBITS:
            for variant in variants:
                oracle.round_(xs, fmt, variant, nbits, seed=2, offset=0, nthreads=threads)
                done += xs.size
    dt = time.perf_counter() - t0
    # the same sweep on one thread, over the first 2^22 elements
    one = 1 << 22
    done1 = 0
    t1 = time.perf_counter()
    for fmt in fmts:
        for nbits in HEADLINE_NBITS:
            for variant in variants:
                oracle.round_(x_host[fmt][:one], fmt, variant, nbits, seed=2, offset=0, nthreads=1)
                done1 += one
    dt1 = time.perf_counter() - t1
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            model = next((ln.split(":", 1)[1].strip() for ln in fh if ln.startswith("model name")), "unknown")
    except OSError:
        pass
    return {"value": done / dt, "unit": "elements/s", "cores": threads, "host_cpus": os.cpu_count(), "kind": "oracle",
            "sample": "first 2^25 elements of the same inputs x 18 (format, N, variant) launches, "
                      "oracle_round_threads with %d threads, %.1f s wall" % (threads, dt),
            "single_thread_value": done1 / dt1, "single_thread_sample": "first 2^22 elements x the same 18 launches, %.1f s" % dt1,
            "cpu_model": model}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards without communication, but no "
              "multi-GPU run is part of it); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2504_20634_amd as fbsr
    from paper_2504_20634_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    fbsr.binding.lib()
    n = 1 << args.elems_log2
    fmts = (fbsr.FMT_E4M3, fbsr.FMT_E5M2)
    variants = (fbsr.SRFF, fbsr.SRF, fbsr.SRC)
    target = {fbsr.FMT_E4M3: "e4m3", fbsr.FMT_E5M2: "e5m2", fbsr.FMT_BF16: "bf16"}

    x_host = {f: workloads.full_range(n, target[f], seed=2) for f in fmts}
    x_dev = {f: torch.from_numpy(x_host[f]).cuda() for f in fmts}
    # Consecutive launches rotate through several input and output buffers (3 GiB of inputs per
    # format, 1 GiB of outputs) so the 256 MB last-level cache cannot serve any of the traffic.
    x_rot = {f: [x_dev[f]] + [torch.from_numpy(workloads.full_range(n, target[f], seed=20 + k)).cuda() for k in (1, 2)]
             for f in fmts}
    out_rot = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(4)]
    out8 = out_rot[0]
    sweep = [(f, nb, v) for f in fmts for nb in HEADLINE_NBITS for v in variants]
    turn = [0]

    def launch(f, nb, v):
        turn[0] += 1
        fbsr.fbsr_round(x_rot[f][turn[0] % 3], f, v, nb, seed=2, offset=0, out=out_rot[turn[0] % 4])

    if args.copy_probe:
        probe = torch.empty_like(x_dev[fbsr.FMT_E4M3])
        for _ in range(2):
            probe.copy_(x_dev[fbsr.FMT_E4M3])
        torch.cuda.synchronize()
        del probe

    def step():
        for f, nb, v in sweep:
            launch(f, nb, v)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The timed region: exactly args.steps steps between two synchronizations, an event on the launch stream at every
    # step boundary.  The average launch duration of the roofline object is the events' span of the region over its
    # launches (so it includes the gaps between launches); the wall clock gives the value.
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for k in range(args.steps):
        step()
        marks[k + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    value = len(sweep) * n * args.steps / wall
    step_ms = [marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps)]
    avg_ms = sum(step_ms) / (args.steps * len(sweep))
    achieved = 5.0 * n / (avg_ms * 1e-3) / 1e9

    # A second pass, outside the timed region, with an event pair around every launch: the break-down by format, N and
    # variant (the pairs cost each launch a few microseconds, which is why they are not in the timed region).
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in sweep]
           for _ in range(args.steps)]
    for k in range(args.steps):
        for i, (f, nb, v) in enumerate(sweep):
            evs[k][i][0].record()
            launch(f, nb, v)
            evs[k][i][1].record()
    torch.cuda.synchronize()
    per = {}
    for i, (f, nb, v) in enumerate(sweep):
        ms = sum(evs[k][i][0].elapsed_time(evs[k][i][1]) for k in range(args.steps)) / args.steps
        per["%s_N%d_%s" % (target[f], nb, fbsr.binding.VARIANT_NAMES[v])] = {
            "ms": round(ms, 4), "gelem_s": round(n / ms / 1e6, 2), "gb_s": round(5.0 * n / ms / 1e6, 1),
            "kernel": "fbsr::round_tiles<%d, %d, %d>" % (f, v, 1 << (nb - 1).bit_length()), "elements": n}
    by_n = {"N%d" % nb: round(sum(5.0 * n / p["ms"] / 1e6 for k, p in per.items() if "_N%d_" % nb in k) /
                              sum(1 for k in per if "_N%d_" % nb in k), 1) for nb in HEADLINE_NBITS}

    paths = {}
    if not args.no_paths:
        # practical ceiling of the launch shape: the same tiles with no arithmetic (plain 4:1 read:write stream)
        def probe():
            turn[0] += 1
            fbsr.binding.fbsr_probe_stream41(x_rot[fbsr.FMT_E4M3][turn[0] % 3], out_rot[turn[0] % 4])
        ms = timed_launches(torch, probe)
        paths["stream_4to1_no_arithmetic_ceiling"] = {"ms": round(ms, 4), "gb_s": round(5.0 * n / ms / 1e6, 1)}
        # the RNE launch draws no random bits (same 4:1 read:write byte mix)
        ms = timed_launches(torch, lambda: fbsr.fbsr_round(x_dev[fbsr.FMT_E4M3], fbsr.FMT_E4M3, fbsr.RNE, 0, 2, 0, out=out8))
        paths["round_e4m3_rne_ceiling"] = {"ms": round(ms, 4), "gb_s": round(5.0 * n / ms / 1e6, 1)}
        out16 = torch.empty(n, dtype=torch.uint16, device="cuda")
        for nb in (4, 8, 16):
            ms = timed_launches(torch, lambda: fbsr.fbsr_round(x_dev[fbsr.FMT_E5M2], fbsr.FMT_BF16, fbsr.SRF, nb, 2, 0, out=out16))
            paths["round_bf16_N%d_srf" % nb] = {"ms": round(ms, 4), "gb_s": round(6.0 * n / ms / 1e6, 1)}
        del out16
        # narrow-source rounding (bf16 -> fp8, 3 B/element), N = 3 as in the paper's experiments
        x16 = [torch.from_numpy(workloads.sgd_weights(n, seed=30 + k).view(np.int16)).cuda() for k in range(3)]
        rot16 = [0]

        def from16(f, v, nb):
            rot16[0] += 1
            fbsr.fbsr_round_from16(x16[rot16[0] % 3], fbsr.SRC_BF16, f, v, nb, seed=2, offset=0, out=out_rot[rot16[0] % 4])
        for f, v, nb in ((fbsr.FMT_E4M3, fbsr.SRC, 3), (fbsr.FMT_E5M2, fbsr.SRF, 3), (fbsr.FMT_E4M3, fbsr.SRFF, 8)):
            ms = timed_launches(torch, lambda: from16(f, v, nb))
            paths["round_from_bf16_%s_N%d_%s" % (target[f], nb, fbsr.binding.VARIANT_NAMES[v])] = {
                "ms": round(ms, 4), "gb_s": round(3.0 * n / ms / 1e6, 1), "gelem_s": round(n / ms / 1e6, 1)}
        ms = timed_launches(torch, lambda: from16(fbsr.FMT_E4M3, fbsr.SRFF, 20))       # more than 16 random bits: 32-bit slots
        paths["round_from_bf16_e4m3_N20_srff"] = {"ms": round(ms, 4), "gb_s": round(3.0 * n / ms / 1e6, 1), "gelem_s": round(n / ms / 1e6, 1)}
        # the format Sec. IV trains in (P3109 binary8p4) as a target id: hardware converts on 2 x
        def p4round(v, nb):
            turn[0] += 1
            fbsr.fbsr_round(x_rot[fbsr.FMT_E4M3][turn[0] % 3], fbsr.FMT_BINARY8P4, v, nb, seed=2, offset=0, out=out_rot[turn[0] % 4])
        for v, nb in ((fbsr.SRC, 3), (fbsr.SRFF, 8)):
            ms = timed_launches(torch, lambda: p4round(v, nb))
            paths["round_binary8p4_N%d_%s" % (nb, fbsr.binding.VARIANT_NAMES[v])] = {"ms": round(ms, 4), "gb_s": round(5.0 * n / ms / 1e6, 1)}

        # classical SR from fp32 (N = D = 20 for E4M3): more than 16 bits per element, 32-bit slots and the wide rounding
        def many_bits():
            turn[0] += 1
            fbsr.fbsr_round(x_rot[fbsr.FMT_E4M3][turn[0] % 3], fbsr.FMT_E4M3, fbsr.SRFF, 20, seed=2, offset=0, out=out_rot[turn[0] % 4])
        ms = timed_launches(torch, many_bits)
        paths["round_e4m3_N20_classical_sr"] = {"ms": round(ms, 4), "gb_s": round(5.0 * n / ms / 1e6, 1),
                                                                   "gelem_s": round(n / ms / 1e6, 1)}

        # 24 bits with the corrected variant: past what the hardware converts apply to every input, so waves that hold
        # values below the normal range (most waves of this full-range input) take the integer rounding
        def most_bits():
            turn[0] += 1
            fbsr.fbsr_round(x_rot[fbsr.FMT_E4M3][turn[0] % 3], fbsr.FMT_E4M3, fbsr.SRC, 24, seed=2, offset=0, out=out_rot[turn[0] % 4])
        ms = timed_launches(torch, most_bits)
        paths["round_e4m3_N24_src"] = {"ms": round(ms, 4), "gb_s": round(5.0 * n / ms / 1e6, 1), "gelem_s": round(n / ms / 1e6, 1)}

        def p4from16(v, nb):
            rot16[0] += 1
            fbsr.fbsr_round_from16(x16[rot16[0] % 3], fbsr.SRC_BF16, fbsr.FMT_BINARY8P4, v, nb, seed=2, offset=0, out=out_rot[rot16[0] % 4])
        ms = timed_launches(torch, lambda: p4from16(fbsr.SRC, 3))
        paths["round_from_bf16_binary8p4_N3_src"] = {"ms": round(ms, 4), "gb_s": round(3.0 * n / ms / 1e6, 1), "gelem_s": round(n / ms / 1e6, 1)}
        # generic-format path (descriptor given at run time): the same format, from fp32 and from bf16 (N = 3)
        p4 = fbsr.format8_named("p3109_binary8p4")
        rotg = [0]

        def generic(src, v, nb):
            rotg[0] += 1
            xin = x_rot[fbsr.FMT_E4M3][rotg[0] % 3] if src == fbsr.FROM_FP32 else x16[rotg[0] % 3]
            fbsr.fbsr_round_format8(xin, src, p4, v, nb, seed=2, offset=0, out=out_rot[rotg[0] % 4])
        for src, v, nb, tag in ((fbsr.FROM_FP32, fbsr.SRC, 3, "src"), (fbsr.FROM_FP32, fbsr.SRF, 8, "srf"),
                                (fbsr.FROM_FP32, fbsr.SRC_TIES_ODD, 3, "src_ties_odd"), (fbsr.FROM_FP32, fbsr.SRFF, 20, "srff"),
                                (fbsr.FROM_BF16, fbsr.SRC, 3, "src"), (fbsr.FROM_BF16, fbsr.SRFF, 3, "srff")):
            ms = timed_launches(torch, lambda: generic(src, v, nb))
            bpe = 5.0 if src == fbsr.FROM_FP32 else 3.0
            paths["round_format8_binary8p4_from_%s_N%d_%s" % ("fp32" if src == fbsr.FROM_FP32 else "bf16", nb, tag)] = {
                "ms": round(ms, 4), "gb_s": round(bpe * n / ms / 1e6, 1), "gelem_s": round(n / ms / 1e6, 1)}
        del x16
        # IEEE binary16 as a generic 16-bit target (4 B read, 2 B written per element)
        b16 = fbsr.format8_named("ieee_binary16")
        o16 = [torch.empty(n, dtype=torch.uint16, device="cuda") for _ in range(2)]

        def wide16(v, nb):
            rotg[0] += 1
            fbsr.fbsr_round_format16(x_rot[fbsr.FMT_E4M3][rotg[0] % 3], fbsr.FROM_FP32, b16, v, nb, seed=2, offset=0, out=o16[rotg[0] % 2])
        for v, nb, tag in ((fbsr.SRC, 3, "src"), (fbsr.SRF, 8, "srf")):
            ms = timed_launches(torch, lambda: wide16(v, nb))
            paths["round_format16_binary16_from_fp32_N%d_%s" % (nb, tag)] = {"ms": round(ms, 4), "gb_s": round(6.0 * n / ms / 1e6, 1),
                                                                              "gelem_s": round(n / ms / 1e6, 1)}
        del o16
        # block-scaled fp8 target (one scale byte per 32 elements: 4 B read + 1 + 1/32 B written per element)
        sc = torch.empty(n // 32, dtype=torch.uint8, device="cuda")
        rotb = [0]

        def blockscaled(f, v, nb):
            rotb[0] += 1
            fbsr.fbsr_round_block_scaled(x_rot[f][rotb[0] % 3], f, v, nb, seed=2, offset=0, out=out_rot[rotb[0] % 4], scales=sc)
        for f, v, nb in ((fbsr.FMT_E4M3, fbsr.SRC, 3), (fbsr.FMT_E5M2, fbsr.SRF, 8), (fbsr.FMT_E4M3, fbsr.SRFF, 20)):
            ms = timed_launches(torch, lambda: blockscaled(f, v, nb))
            paths["round_block_scaled_%s_N%d_%s" % (target[f], nb, fbsr.binding.VARIANT_NAMES[v])] = {
                "ms": round(ms, 4), "gb_s": round((5.0 + 1.0 / 32) * n / ms / 1e6, 1)}
        del sc
        # fused QAT step of Alg. 1 (7 B read + 5 B written per element), N = 3, 2^27 weights, rotated buffers
        nq = min(SGD_ELEMS, n)
        qs = [(torch.from_numpy((workloads.sgd_weights(nq, seed=40 + k) & 0x7777).view(np.uint8)[:nq].copy()).cuda(),
               torch.from_numpy(workloads.sgd_weights(nq, seed=50 + k).view(np.int16)).cuda(),
               torch.zeros(nq, dtype=torch.int16, device="cuda"), torch.zeros(nq, dtype=torch.int16, device="cuda"))
              for k in range(3)]
        tq = [0]

        # the step's loads and stores with the arithmetic taken out: the ceiling of its 7 : 5 read : write stream
        def stream75_twice():                        # two launches on two buffer sets; each set gets an even count in all,
            for k in range(2):                       # so the buffers end as they began
                w8_, g_, m_, v_ = qs[k]
                fbsr.binding.fbsr_probe_stream75(w8_, g_, m_, v_)
        ms = timed_launches(torch, stream75_twice) / 2
        paths["stream_7to5_no_arithmetic_ceiling"] = {"ms": round(ms, 4), "gb_s": round(12.0 * nq / ms / 1e6, 1),
                                                      "gelem_s": round(nq / ms / 1e6, 1)}

        def qat(v):
            tq[0] += 1
            w8_, g_, m_, v_ = qs[tq[0] % 3]
            t = 1 + tq[0] // 3
            fbsr.fbsr_qat_adamw_step(w8_, g_, m_, v_, fbsr.FMT_E4M3, (1e-3, 0.9, 0.999, 1e-8, 0.01, 1 - 0.9 ** t, 1 - 0.999 ** t),
                                     v, 3, seed=6, step=t)
        for v in (fbsr.SRC, fbsr.SRFF):
            ms = timed_launches(torch, lambda: qat(v))
            paths["qat_adamw_e4m3_N3_%s" % fbsr.binding.VARIANT_NAMES[v]] = {
                "ms": round(ms, 4), "gb_s": round(12.0 * nq / ms / 1e6, 1), "gelem_s": round(nq / ms / 1e6, 1)}
        # the same step with the weights in P3109 binary8p4 (the format Sec. IV trains in): as a target id ...
        # (fresh weights: a byte 0x80, E4M3's -0 left behind by the runs above, is binary8p4's NaN)
        for k in range(3):
            qs[k][0].copy_(torch.from_numpy((workloads.sgd_weights(nq, seed=60 + k) & 0x7777).view(np.uint8)[:nq].copy()))

        def qatp4(v):
            tq[0] += 1
            w8_, g_, m_, v_ = qs[tq[0] % 3]
            t = 1 + tq[0] // 3
            fbsr.fbsr_qat_adamw_step(w8_, g_, m_, v_, fbsr.FMT_BINARY8P4, (1e-3, 0.9, 0.999, 1e-8, 0.01, 1 - 0.9 ** t, 1 - 0.999 ** t),
                                     v, 3, seed=6, step=t)
        for v in (fbsr.SRC, fbsr.SRFF):
            ms = timed_launches(torch, lambda: qatp4(v))
            paths["qat_adamw_binary8p4_N3_%s" % fbsr.binding.VARIANT_NAMES[v]] = {
                "ms": round(ms, 4), "gb_s": round(12.0 * nq / ms / 1e6, 1), "gelem_s": round(nq / ms / 1e6, 1)}
        # ... and through the generic entry point (descriptor at run time, weights decoded through a table)
        for k in range(3):
            qs[k][0].copy_(torch.from_numpy((workloads.sgd_weights(nq, seed=60 + k) & 0x7777).view(np.uint8)[:nq].copy()))
        p4q = fbsr.format8_named("p3109_binary8p4")

        def qat8(v):
            tq[0] += 1
            w8_, g_, m_, v_ = qs[tq[0] % 3]
            t = 1 + tq[0] // 3
            fbsr.fbsr_qat_adamw_step_format8(w8_, g_, m_, v_, p4q, (1e-3, 0.9, 0.999, 1e-8, 0.01, 1 - 0.9 ** t, 1 - 0.999 ** t),
                                             v, 3, seed=6, step=t)
        for v in (fbsr.SRC, fbsr.SRFF):
            ms = timed_launches(torch, lambda: qat8(v))
            paths["qat_adamw_format8_binary8p4_N3_%s" % fbsr.binding.VARIANT_NAMES[v]] = {
                "ms": round(ms, 4), "gb_s": round(12.0 * nq / ms / 1e6, 1), "gelem_s": round(nq / ms / 1e6, 1)}
        del qs
        ns = min(SGD_ELEMS, n)
        # rotate through 3 weight and 3 gradient buffers (2.25 GiB) so the last-level cache cannot help
        ws_ = [torch.from_numpy(workloads.sgd_weights(ns, seed=3 + k).view(np.int16)).cuda() for k in range(3)]
        gs_ = [torch.from_numpy(workloads.sgd_grads(ns, k, seed=3)).cuda() for k in range(3)]
        step_no = [0]

        def sgd(nb):
            k = step_no[0] % 3
            fbsr.fbsr_sgd_update(ws_[k], gs_[k], 1e-3, fbsr.SRF, nb, seed=4, step=step_no[0])
            step_no[0] += 1
        for nb in (2, 4, 8):
            ms = timed_launches(torch, lambda: sgd(nb))
            paths["sgd_update_bf16_N%d_srf" % nb] = {"ms": round(ms, 4), "gb_s": round(8.0 * ns / ms / 1e6, 1)}
        del ws_, gs_
        # bias statistics on the fifth workload's recipe at 2^28 elements: 1024 log-spaced bins of 2^18
        # over [2^-10, 2^10), statistics only (out = NULL); rotated over two input buffers
        group = 1 << 18
        nbins = n // group
        xs_ = [torch.from_numpy(workloads.log_bins(nbins, group, seed=5 + k)[0]).cuda() for k in range(2)]
        ws = torch.empty(fbsr.bias_stats_workspace_bytes(n, nbins) // 8 + 1, dtype=torch.float64, device="cuda")
        stats = torch.zeros((nbins, 4), dtype=torch.float64, device="cuda")
        rot = [0]

        def stat(f, nb):
            rot[0] += 1
            fbsr.fbsr_bias_stats(xs_[rot[0] % 2], f, fbsr.SRF, nb, 5, 0, group, 0, nbins, stats=stats, workspace=ws)
        for f, nb in ((fbsr.FMT_E4M3, 3), (fbsr.FMT_E4M3, 8), (fbsr.FMT_BF16, 2), (fbsr.FMT_BF16, 8)):
            ms = timed_launches(torch, lambda: stat(f, nb))
            paths["bias_stats_%s_N%d_srf" % (target[f], nb)] = {"ms": round(ms, 4), "gb_s": round(4.0 * n / ms / 1e6, 1)}

        # the same statistics with the target given by its descriptor (P3109 binary8p4, the format Sec. IV trains in)
        def stat8(v, nb):
            rot[0] += 1
            fbsr.fbsr_bias_stats_format8(xs_[rot[0] % 2], p4, v, nb, 5, 0, group, 0, nbins, stats=stats, workspace=ws)
        for v, nb, tag in ((fbsr.SRF, 3, "srf"), (fbsr.SRC, 3, "src")):
            ms = timed_launches(torch, lambda: stat8(v, nb))
            paths["bias_stats_format8_binary8p4_N%d_%s" % (nb, tag)] = {"ms": round(ms, 4), "gb_s": round(4.0 * n / ms / 1e6, 1)}
        del xs_

    # every path names its kernel and its elements per launch; where the committed counter figures belong to the kernel
    # sources at hand, a path also carries its vector-ALU figures: instructions per element x elements per second against
    # the ALU ceiling, and the share of the kernel's time with vector-ALU work in flight (rocprofv3's VALUBusy)
    counters, counters_note = load_counters()
    for name, entry in paths.items():
        elems = min(SGD_ELEMS, n) if name.startswith(("qat", "sgd", "stream_7to5")) else n
        entry["kernel"] = PATH_KERNELS.get(name)
        entry["elements"] = elems
        entry["launches"] = TIMED_LAUNCHES * (2 if name.startswith("stream_7to5") else 1)   # of the kernel, in the timed region
        per_elem = counters.get("valu_per_elem", {}).get(name)
        if per_elem is not None:
            rate = per_elem * elems / (entry["ms"] * 1e-3)
            entry["alu_roofline"] = {"bound": "alu", "achieved": round(rate / 1e12, 2), "peak": round(ALU_PEAK_LANE_OPS / 1e12, 2),
                                     "unit": "T lane-ops/s", "frac": round(rate / ALU_PEAK_LANE_OPS, 3), "valu_per_elem": per_elem,
                                     "valu_busy_pct": counters.get("valu_busy_pct", {}).get(name)}
    workloads_report = None
    if not args.no_paths and not args.no_workloads and args.elems_log2 == 28:
        del x_rot, out_rot
        workloads_report = five_workloads(torch, np, fbsr, workloads, x_dev[fbsr.FMT_E5M2])

    result = {
        "metric": "FBSR fp32->fp8 elements/s (achieved HBM GB/s and fraction of peak under roofline), N=2,4,8",
        "value": value,
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": "full-range fp32 (random sign, exponent uniform over the target's range incl. "
                               "subnormals and overflow, random mantissa), 2^%d elements, seed 2; "
                               "step = {e4m3,e5m2} x N{2,4,8} x {srff,srf,src} = 18 launches" % args.elems_log2,
                   "elements": n, "launches_per_step": len(sweep)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": counters.get("headline_traffic_bytes_2p28") if args.elems_log2 == 28 else None,
                     "traffic_source": counters_note,
                     "kernel": "round_tiles<fmt,variant,W> (average over the 18 launches of a step)",
                     "bytes_per_launch": 5 * n, "avg_launch_ms": avg_ms, "gb_s_by_nbits": by_n,
                     "step_ms_min_max": [round(min(step_ms), 4), round(max(step_ms), 4)]},
        "per_launch": per,
        "paths": paths,
    }
    if workloads_report is not None:
        result["workloads"] = workloads_report
    if not args.no_cpu_baseline:
        threads = min(16, os.cpu_count() or 1)
        result["cpu_baseline"] = cpu_baseline(x_host, fmts, variants, threads)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
