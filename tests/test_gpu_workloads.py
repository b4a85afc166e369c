"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.
Where the oracle cannot cover the whole array in seconds it checks sampled windows: legal
because every element's bits depend only on its global index."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from gpu_util import assert_stats_close, dev, first_mismatch, host

pytestmark = pytest.mark.gpu
BF16, E4M3, E5M2 = 0, 1, 2
RNE, SRFF, SRF, SRC = 0, 1, 2, 3
THREADS = 16


def _windows(n, count, width, seed):
    rng = np.random.default_rng(seed)
    starts = [0, n - width] + [int(s) for s in rng.integers(0, n - width, count)]
    # some windows deliberately start off a tile boundary
    return sorted(set(starts))


def test_workload2_e4m3_scaled_normal_full(fbsr, oracle):
    """2^24 scaled-normal values -> E4M3, N in {1,2,3,4,6,8}, all variants, seed 1: every byte."""
    from paper_2504_20634_amd import workloads
    n = 1 << 24
    x = workloads.scaled_normal(n, seed=1)
    xd = dev(x)
    frac_sub = np.mean(np.abs(x) < 2.0 ** -6)
    assert 0.05 < frac_sub < 0.5      # a good share lands in E4M3's subnormal range (|z| 2^6 stays below 448)
    for nbits in (1, 2, 3, 4, 6, 8):
        for variant in (SRFF, SRF, SRC):
            print("case nbits=%d variant=%d" % (nbits, variant), flush=True)
            got = host(fbsr.fbsr_round(xd, E4M3, variant, nbits, seed=1))
            want = oracle.round_(x, E4M3, variant, nbits, seed=1, nthreads=THREADS)
            assert first_mismatch(got, want) is None, (nbits, variant, first_mismatch(got, want))


@pytest.mark.parametrize("fmt,target", [(E5M2, "e5m2"), (BF16, "bf16"), (E4M3, "e4m3")])
def test_workload3_full_range_2_28(fbsr, oracle, fmt, target):
    """2^28 full-range values, N in {4,8,16} (and 2 for the headline), all variants, seed 2:
    one combination compared over the whole array, the rest on 40 sampled windows of 2^16."""
    from paper_2504_20634_amd import workloads
    n = 1 << 28
    x = workloads.full_range(n, target, seed=2, specials_every=(100003 if fmt == BF16 else 0))
    xd = dev(x)
    print("case fmt=%d full array SRF N=8" % fmt, flush=True)
    got = host(fbsr.fbsr_round(xd, fmt, SRF, 8, seed=2))
    want = oracle.round_(x, fmt, SRF, 8, seed=2, nthreads=THREADS)
    assert first_mismatch(got, want) is None, first_mismatch(got, want)
    del got, want
    width = 1 << 16
    wins = _windows(n, 40, width, seed=fmt)
    for nbits in (2, 4, 8, 16):
        for variant in (SRFF, SRF, SRC):
            print("case fmt=%d nbits=%d variant=%d windows" % (fmt, nbits, variant), flush=True)
            out = fbsr.fbsr_round(xd, fmt, variant, nbits, seed=2)
            for s in wins:
                got = host(out[s:s + width])
                want = oracle.round_(x[s:s + width], fmt, variant, nbits, seed=2, offset=s)
                assert first_mismatch(got, want) is None, (nbits, variant, s, first_mismatch(got, want))
            del out


def test_workload4_sgd_2_27_two_steps(fbsr, oracle):
    """2^27 bf16 weights, fp32 gradients of std 1e-3, lr 1e-3: two full-size steps, every weight."""
    from paper_2504_20634_amd import workloads
    n = 1 << 27
    w = workloads.sgd_weights(n, seed=3)
    wd = dev(w)
    for t in range(2):
        g = workloads.sgd_grads(n, t, seed=3)
        fbsr.fbsr_sgd_update(wd, dev(g), 1e-3, SRF, 4, seed=4, step=t)
        with ThreadPoolExecutor(THREADS) as pool:
            cuts = np.linspace(0, n, THREADS + 1).astype(np.int64)
            parts = list(pool.map(lambda ab: oracle.sgd_update(w[ab[0]:ab[1]], g[ab[0]:ab[1]], 1e-3, SRF, 4, 4, t, int(ab[0])),
                                  zip(cuts[:-1], cuts[1:])))
        w = np.concatenate(parts)
        print("case step=%d" % t, flush=True)
        assert first_mismatch(host(wd), w) is None, t


def test_workload5_log_bins_2_30(fbsr, oracle):
    """2^30 inputs in 4096 log-spaced bins of 2^18 over [2^-10, 2^10): statistics only (out = NULL), the whole
    sweep of the workload: {E4M3, bf16} x {SRFF, SRF, SRC} x N = 1..12 = 72 passes.  In every pass the oracle
    checks 66 bins in full (every 64th bin, which takes in 13 bins of E4M3's subnormal range below 2^-6 and 3 of
    its saturated range above 448, plus the two bins that straddle 2^-6 and 448); the remaining bins are checked
    through properties: count = 2^18, |mean error| < 1 ulp in range, SRFF's bias near -2^-(N+1) and SRF / SRC
    near 0 away from E4M3's saturation."""
    from paper_2504_20634_amd import workloads
    nbins, group = 4096, 1 << 18
    straddle = [int(np.floor((np.log2(v) + 10.0) / 20.0 * nbins)) for v in (2.0 ** -6 * 1.0001, 448.0)]
    kept = sorted(set(range(0, nbins, 64)) | set(straddle))
    xd = torch.empty(nbins * group, dtype=torch.float32, device="cuda")
    keep = {}
    slab = 64
    for b0 in range(0, nbins, slab):
        xs, edges = workloads.log_bins(nbins, group, seed=5, bins=range(b0, b0 + slab))
        xd[b0 * group:(b0 + slab) * group] = torch.from_numpy(xs).cuda()
        for b in kept:
            if b0 <= b < b0 + slab:
                keep[b] = xs[(b - b0) * group:(b - b0 + 1) * group].copy()
        if b0 % 1024 == 0:
            print("generated bins up to %d" % (b0 + slab), flush=True)
    assert edges[straddle[0]] <= 2.0 ** -6 < edges[straddle[0] + 1] and edges[straddle[1]] <= 448.0 < edges[straddle[1] + 1]
    assert sum(1 for b in kept if edges[b + 1] <= 2.0 ** -6) >= 13 and sum(1 for b in kept if edges[b] > 448.0) >= 3
    ws = torch.empty(fbsr.bias_stats_workspace_bytes(nbins * group, nbins) // 8 + 1, dtype=torch.float64, device="cuda")
    for fmt in (E4M3, BF16):
        for variant in (SRFF, SRF, SRC):
            for nbits in range(1, 13):
                print("case fmt=%d variant=%d nbits=%d" % (fmt, variant, nbits), flush=True)
                stats, _ = fbsr.fbsr_bias_stats(xd, fmt, variant, nbits, 5, 0, group, 0, nbins, workspace=ws)
                s = stats.cpu().numpy()

                def one(b):
                    st, _ = oracle.bias_stats(keep[b], fmt, variant, nbits, 5, b * group, group, b, 1)
                    return st[0]
                with ThreadPoolExecutor(THREADS) as pool:
                    want = np.array(list(pool.map(one, kept)))
                assert_stats_close(s[kept], want)
                assert np.all(s[:, 0] == group)
                mean_e = s[:, 2] / s[:, 0]
                in_range = edges[1:] <= (448.0 if fmt == E4M3 else 3e38)
                assert np.all(np.abs(mean_e[in_range]) < 1.0)
                # A bin is far narrower than one E4M3 ulp, so a single bin sees only a slice of delta:
                # its bias is a point on the sawtooth (SRFF in [-2^-N, 0], SRF / SRC within +-2^-(N+1)),
                # plus sampling noise ~ 0.5 / sqrt(2^18) ~ 1e-3.  Averaged over all in-range bins the
                # sawtooth integrates to the closed forms of Sec. III-D / III-E.
                me = mean_e[in_range]
                half = 2.0 ** -(nbits + 1)
                if variant == SRFF:
                    assert np.all(me < 6e-3) and np.all(me > -2 * half - 6e-3), (me.min(), me.max())
                    assert abs(me.mean() + half) < 5e-3, me.mean()
                else:
                    assert np.all(np.abs(me) < half + 6e-3), (me.min(), me.max())
                    assert abs(me.mean()) < 5e-3, me.mean()


def test_more_than_2_32_elements(fbsr, oracle):
    """One call over 2^32 + 5000 elements (16 GiB in, 4 GiB out): element indices, byte offsets and the
    launch cut all pass 2^32.  The input repeats a 2^28-element host buffer; windows at the start, across
    every launch cut, across 2^32 and in the ragged tail are compared with the oracle."""
    from paper_2504_20634_amd import workloads
    base_n = 1 << 28
    n = (1 << 32) + 5000
    base = workloads.full_range(base_n, "e4m3", seed=11)
    bd = dev(base)
    xd = torch.empty(n, dtype=torch.float32, device="cuda")
    for k in range(16):
        xd[k * base_n:(k + 1) * base_n] = bd
    xd[16 * base_n:] = bd[:5000]
    del bd
    out = fbsr.fbsr_round(xd, E4M3, SRC, 3, seed=21, offset=0)
    width = 1 << 14
    starts = [0, (1 << 31) - 777, (1 << 32) - width // 2, n - width, (1 << 33) // 2 + 12345] + \
             [k * (1 << 22) * 2048 - 100 for k in range(1, 1 + n // ((1 << 22) * 2048))]
    for s in starts:
        s = max(0, min(int(s), n - width))
        idx = (s + np.arange(width)) % base_n if s + width <= (1 << 32) else None
        xs = xd[s:s + width].cpu().numpy()
        want = oracle.round_(xs, E4M3, SRC, 3, seed=21, offset=s)
        assert first_mismatch(host(out[s:s + width]), want) is None, s
    # the bf16-source path at the same scale shares the launch cut logic; check its last window too
    del out
    src = xd.view(torch.int16)[: n]           # any 16-bit patterns will do
    o2 = fbsr.fbsr_round_from16(src, 0, E5M2, SRF, 4, seed=3, offset=7)
    s = n - width
    want = oracle.round_from16(src[s:].cpu().numpy().view(np.uint16), 0, E5M2, SRF, 4, seed=3, offset=7 + s)
    assert first_mismatch(host(o2[s:]), want) is None


def test_workload4_sgd_1000_steps_drift(fbsr):
    """The fourth workload at full scale on the GPU: 2^27 bf16 weights ~ U(-1,1), lr = 1e-3, fresh
    gradients N(0, (1e-3)^2) per step, 1000 steps, N in {2, 4, 8} against nearest-even.  Updates are far
    below one ulp, so (Sec. IV) nearest-even stagnates -- and so do SRF and SRC, whose predicates never
    fire for |update| << ulp -- while SRFF loses 2^-(N+1) ulp of |w| per step (App. A-A), i.e. the
    weights drift toward zero.  Prints mean |w| every 250 steps."""
    n, lr, steps = 1 << 27, 1e-3, 1000
    from paper_2504_20634_amd import workloads
    w0 = dev(workloads.sgd_weights(n, seed=3))
    as_f = lambda w: (w.to(torch.int32) << 16).view(torch.float32)
    a0 = as_f(w0).abs()
    ulp0 = torch.exp2(torch.floor(torch.log2(a0.clamp_min(2.0 ** -120))) - 7)
    m0 = a0.double().mean().item()
    # the per-step rate is read on weights of at least 2^-6: relative to its own ulp a weight near zero moves
    # by an unbounded amount, so a mean over all weights is set by the few smallest ones
    big = a0 >= 2.0 ** -6
    gen = torch.Generator(device="cuda")
    g = torch.empty(n, dtype=torch.float32, device="cuda")
    print("start   mean|w| = %.6f" % m0, flush=True)
    for variant, nbits in ((RNE, 0), (SRF, 2), (SRC, 2), (SRFF, 8), (SRFF, 4), (SRFF, 2)):
        w = w0.clone()
        gen.manual_seed(1234)
        track = []
        for t in range(steps):
            g.normal_(0.0, 1e-3, generator=gen)
            fbsr.fbsr_sgd_update(w, g, lr, variant, nbits, seed=9, step=t)
            if t + 1 == 20:
                rate = (((as_f(w).abs() - a0) / ulp0)[big].double().mean().item()) / 20.0
            if (t + 1) % 250 == 0:
                track.append(as_f(w).abs().double().mean().item())
        moved = (w != w0).double().mean().item()
        print("variant=%d N=%d  ulp/step over the first 20 steps %+.5f  moved %.4f  mean|w| at 250..1000: %s"
              % (variant, nbits, rate, moved, " ".join("%.6f" % v for v in track)), flush=True)
        if variant == SRFF:
            assert abs(rate + 2.0 ** -(nbits + 1)) < 0.1 * 2.0 ** -(nbits + 1), (nbits, rate)
            # one ulp is between 2^-8 and 2^-7 of |w|, so |w| decays by a factor between these two per step
            loss = steps * 2.0 ** -(nbits + 1)
            assert m0 * np.exp(-loss / 128) < track[-1] < m0 * np.exp(-loss / 256), track
        else:
            # only weights so small that 1e-6 is not << their ulp (|w| < 2^-12: a few in a thousand) can move
            assert moved < 1e-2 and abs(track[-1] - m0) < 1e-5 * m0, (variant, moved, track)


def test_other_entry_points_at_bench_sizes(fbsr, oracle):
    """The paths bench.py times beside the headline, at its sizes (2^28 elements; 2^27 for the fused steps), each
    compared with the oracle on 24 sampled windows of 2^14: narrow-source, block-scaled, generic-format rounding
    (P3109 binary8p4 from fp32 and from bf16, the latter through the table kernel), the flavours with more than 16
    random bits, binary16 as a target, the statistics by descriptor (28 sampled bins) and both fused QAT steps."""
    from paper_2504_20634_amd import workloads
    n = 1 << 28
    width = 1 << 14
    x = workloads.full_range(n, "e4m3", seed=2)
    xd = dev(x)
    x16 = workloads.sgd_weights(n, seed=30)
    x16d = dev(x16)
    p4 = (8, 4, 8, 0x7E, 0x7F, 0x80, 0, 0)
    wins = [s - s % 32 for s in _windows(n, 24, width, seed=9)]      # block-scaled windows start on a block
    print("case narrow source", flush=True)
    out = fbsr.fbsr_round_from16(x16d, 0, E4M3, SRC, 3, seed=2)
    for s in wins:
        assert first_mismatch(host(out[s:s + width]), oracle.round_from16(x16[s:s + width], 0, E4M3, SRC, 3, seed=2, offset=s)) is None, s
    print("case block scaled", flush=True)
    out, sc = fbsr.fbsr_round_block_scaled(xd, E5M2, SRF, 8, seed=2)
    for s in wins:
        wc, wsc = oracle.round_block_scaled(x[s:s + width], E5M2, SRF, 8, seed=2, offset=s)
        assert first_mismatch(host(out[s:s + width]), wc) is None and first_mismatch(host(sc[s // 32:(s + width) // 32]), wsc) is None, s
    for src, data, datad, variant, nbits in ((2, x, xd, SRC, 3), (2, x, xd, 4, 3), (0, x16, x16d, SRFF, 3), (0, x16, x16d, SRC, 3)):
        print("case generic src=%d variant=%d" % (src, variant), flush=True)
        out = fbsr.fbsr_round_format8(datad, src, p4, variant, nbits, seed=2)
        for s in wins:
            assert first_mismatch(host(out[s:s + width]), oracle.round_format8(data[s:s + width], src, p4, variant, nbits, 2, s)) is None, s
    print("case more than 16 bits", flush=True)
    for fmt, variant, nbits in ((E4M3, SRFF, 20), (E4M3, SRC, 24)):
        out = fbsr.fbsr_round(xd, fmt, variant, nbits, seed=2)
        for s in wins:
            assert first_mismatch(host(out[s:s + width]), oracle.round_(x[s:s + width], fmt, variant, nbits, seed=2, offset=s)) is None, s
    out = fbsr.fbsr_round_from16(x16d, 0, E4M3, SRFF, 20, seed=2)
    for s in wins:
        assert first_mismatch(host(out[s:s + width]), oracle.round_from16(x16[s:s + width], 0, E4M3, SRFF, 20, seed=2, offset=s)) is None, s
    out = fbsr.fbsr_round_format8(xd, 2, p4, SRFF, 20, seed=2)
    for s in wins:
        assert first_mismatch(host(out[s:s + width]), oracle.round_format8(x[s:s + width], 2, p4, SRFF, 20, 2, s)) is None, s
    out, sc = fbsr.fbsr_round_block_scaled(xd, E4M3, SRFF, 20, seed=2)
    for s in wins:
        wc, wsc = oracle.round_block_scaled(x[s:s + width], E4M3, SRFF, 20, seed=2, offset=s)
        assert first_mismatch(host(out[s:s + width]), wc) is None and first_mismatch(host(sc[s // 32:(s + width) // 32]), wsc) is None, s
    print("case binary16 target", flush=True)
    b16 = (16, 11, 15, 0x7BFF, 0x7C00, 0x7E00, 1, 1)
    for variant, nbits in ((SRC, 3), (SRF, 8)):
        out = fbsr.fbsr_round_format16(xd, 2, b16, variant, nbits, seed=2)
        for s in wins:
            assert first_mismatch(host(out[s:s + width]), oracle.round_format16(x[s:s + width], 2, b16, variant, nbits, 2, s)) is None, s
    print("case statistics by descriptor", flush=True)
    group = 1 << 18
    xs, _ = workloads.log_bins(n // group, group, seed=5)
    xsd = dev(xs)
    for variant, nbits in ((SRF, 3), (SRC, 3)):
        stats, _ = fbsr.fbsr_bias_stats_format8(xsd, p4, variant, nbits, 5, 0, group, 0, n // group)
        got = stats.cpu().numpy()
        for b in range(0, n // group, 37):       # 28 of the 1024 bins, subnormal and above-M bins among them
            want, _ = oracle.bias_stats_format8(xs[b * group:(b + 1) * group], p4, variant, nbits, 5, b * group, group, b, 1)
            assert_stats_close(got[b:b + 1], want)
    del out, xd, x16d, xsd
    nq = 1 << 27
    w8 = (workloads.sgd_weights(nq, seed=40) & 0x7777).view(np.uint8)[:nq].copy()
    g16 = workloads.sgd_weights(nq, seed=50)
    m16 = workloads.sgd_weights(nq, seed=51) & 0x3FFF        # moments of modest size, second one non-negative
    v16 = workloads.sgd_weights(nq, seed=52) & 0x3FFF
    params = (1e-3, 0.9, 0.999, 1e-8, 0.01, 1 - 0.9 ** 2, 1 - 0.999 ** 2)
    qwins = _windows(nq, 24, width, seed=10)
    for generic in (False, True):
        print("case qat generic=%d" % generic, flush=True)
        wd, gd, md, vd = dev(w8), dev(g16), dev(m16), dev(v16)
        if generic:
            fbsr.fbsr_qat_adamw_step_format8(wd, gd, md, vd, p4, params, SRC, 3, seed=6, step=2)
        else:
            fbsr.fbsr_qat_adamw_step(wd, gd, md, vd, E4M3, params, SRC, 3, seed=6, step=2)
        for s in qwins:
            sl = slice(s, s + width)
            if generic:
                ww, mm, vv = oracle.qat_adamw_step_format8(w8[sl], g16[sl], m16[sl], v16[sl], p4, params, SRC, 3, 6, 2, s)
            else:
                ww, mm, vv = oracle.qat_adamw_step(w8[sl], g16[sl], m16[sl], v16[sl], E4M3, params, SRC, 3, 6, 2, s)
            assert first_mismatch(host(wd[sl]), ww) is None and first_mismatch(host(md[sl]), mm) is None and first_mismatch(host(vd[sl]), vv) is None, s
