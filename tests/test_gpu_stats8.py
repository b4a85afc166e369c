"""GPU parity: fbsr_bias_stats_format8 (the per-bin statistics of Figs. 1-2 for a target format given by its
descriptor, every rounding mode of fbsr_round_format8) against the oracle: counts exact, sums within 1e-6 relative
(fp64 accumulation on both sides, different orders), codes byte-identical."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from gpu_util import assert_stats_close, dev, first_mismatch, host
from test_gpu_format8 import FORMATS, _inputs

pytestmark = pytest.mark.gpu
RNE, SRFF, SRF, SRC, SRC_ODD, RNO, RNA = range(7)


def _run_both(fbsr, oracle, x, d, variant, nbits, seed, offset, group, first_bin, nbins, with_out):
    xd = dev(x)
    out = torch.empty(x.size, dtype=torch.uint8, device="cuda") if with_out else None
    stats, out = fbsr.fbsr_bias_stats_format8(xd, d, variant, nbits, seed, offset, group, first_bin, nbins, out=out)
    want, wout = oracle.bias_stats_format8(x, d, variant, nbits, seed, offset, group, first_bin, nbins, want_out=with_out)
    assert_stats_close(stats.cpu().numpy(), want)
    if with_out:
        assert first_mismatch(host(out), wout) is None
    return stats


@pytest.mark.parametrize("name", ["binary8p4", "ocp_e2m3", "binary8p1", "ocp_e5m2", "inf_apart"])
def test_groups_of_every_size(fbsr, oracle, name):
    """Bins smaller than, equal to and larger than a row, a span and a chunk; ragged ends; offsets; bins that the call
    only partly covers; every slot width, the modes that draw no bits, and more than 16 bits."""
    d = FORMATS[name]
    rng = np.random.default_rng(len(name))
    n = 5 * 8192 + 700
    x = _inputs(rng, d, n)[:n]
    x = np.where(np.isfinite(x), x, np.float32(1.0)).astype(np.float32)
    for variant, nbits in ((SRFF, 2), (SRF, 8), (SRC, 3), (RNE, 0), (SRC_ODD, 16), (RNA, 0), (SRFF, 1), (SRC, 20)):
        for group, offset in ((1, 0), (7, 3), (1000, 0), (1024, 0), (5000, 0), (5000, 1234), (8192, 8192), (20000, 16),
                              (1 << 20, 5), (512, 0), (513, 128)):
            first_bin = offset // group
            nbins = (offset + n - 1) // group - first_bin + 1
            print("case fmt=%s variant=%d nbits=%d group=%d offset=%d" % (name, variant, nbits, group, offset), flush=True)
            _run_both(fbsr, oracle, x, d, variant, nbits, 6, offset, group, first_bin, nbins, with_out=(group in (7, 5000, 513)))


@pytest.mark.parametrize("name", ["binary8p4", "binary8p3", "ocp_e4m3", "ocp_e5m2", "ocp_e2m3", "ocp_e2m1", "binary8p7", "bias96", "k2"])
def test_rows_of_ordinary_values_take_the_integer_path(fbsr, oracle, name):
    """Every row holds only values with |x| <= M that are zero or at least 2^(1 - B - P) -- normal and subnormal
    targets mixed, both signs, zeros, M itself, the smallest value without lost bits -- so the kernel's integer path
    serves them (a row that a bin boundary cuts, and the rows of the last block, which hold values one step outside
    either limit, go the general way)."""
    d = FORMATS[name]
    K, P, B, mx = d[:4]
    t_max = mx & ((1 << (P - 1)) - 1)
    M = np.float32((1.0 + t_max * 2.0 ** (1 - P)) * 2.0 ** ((mx >> (P - 1)) - B)) if (mx >> (P - 1)) else np.float32(t_max * 2.0 ** (2 - P - B))
    lo = np.float32(2.0 ** (1 - B - P))
    rng = np.random.default_rng(K * 100 + P)
    n = 6 * 16384
    mag = np.exp(rng.uniform(np.log(float(lo)), np.log(float(M)), n)).astype(np.float32)
    mag = np.clip(mag, lo, M)
    mag[::97] = 0.0
    mag[1::97] = M
    mag[2::97] = lo
    x = (mag * np.where(rng.integers(0, 2, n) == 1, np.float32(-1), np.float32(1))).astype(np.float32)
    x[5 * 16384::64] = np.nextafter(M, np.float32(np.inf))
    x[5 * 16384 + 1::64] = np.nextafter(lo, np.float32(0))
    for variant, nbits in ((SRFF, 2), (SRF, 3), (SRC, 3), (SRC_ODD, 4), (RNE, 0), (RNO, 0), (RNA, 0), (SRC, 16), (SRFF, 9)):
        for group, offset in ((1 << 14, 0), (5000, 0), (20000, 64)):
            first_bin = offset // group
            nbins = (offset + n - 1) // group - first_bin + 1
            print("case fmt=%s variant=%d nbits=%d group=%d offset=%d" % (name, variant, nbits, group, offset), flush=True)
            _run_both(fbsr, oracle, x, d, variant, nbits, 4, offset, group, first_bin, nbins, with_out=(group == 5000))


def test_under_ocp_descriptors_the_fixed_format_statistics_come_back(fbsr):
    """E4M3 and E5M2 by descriptor against fbsr_bias_stats with the format ids: same codes, sums equal to the last
    few bits (two kernels, two summation orders)."""
    from paper_2504_20634_amd import workloads
    n = 3 * 16384 + 512
    for fmt, name in ((1, "ocp_e4m3"), (2, "ocp_e5m2")):
        x = dev(workloads.full_range(n, {1: "e4m3", 2: "e5m2"}[fmt], seed=5, specials_every=0))
        for variant, nbits in ((SRFF, 3), (SRC, 4), (RNE, 0)):
            a, ca = fbsr.fbsr_bias_stats_format8(x, FORMATS[name], variant, nbits, 8, 0, 4096, 0, n // 4096 + 1,
                                                 out=torch.empty(n, dtype=torch.uint8, device="cuda"))
            b, cb = fbsr.fbsr_bias_stats(x, fmt, variant, nbits, 8, 0, 4096, 0, n // 4096 + 1,
                                         out=torch.empty(n, dtype=torch.uint8, device="cuda"))
            assert torch.equal(ca, cb)
            assert_stats_close(a.cpu().numpy(), b.cpu().numpy(), rel=1e-12)


def test_accumulates_and_is_reproducible(fbsr):
    from paper_2504_20634_amd import workloads
    n, group = 4 * 8192, 5000
    d = FORMATS["binary8p4"]
    xd = dev(workloads.scaled_normal(n, seed=2))
    nbins = (n - 1) // group + 1
    s1, _ = fbsr.fbsr_bias_stats_format8(xd, d, SRF, 4, 9, 0, group, 0, nbins)
    s2, _ = fbsr.fbsr_bias_stats_format8(xd, d, SRF, 4, 9, 0, group, 0, nbins)
    assert torch.equal(s1, s2), "reduction order is not fixed"
    s3 = s1.clone()
    fbsr.fbsr_bias_stats_format8(xd, d, SRF, 4, 9, 0, group, 0, nbins, stats=s3)
    assert torch.equal(s3, 2 * s1)
    half = 2 * 8192
    sa = torch.zeros_like(s1)
    fbsr.fbsr_bias_stats_format8(xd[:half], d, SRF, 4, 9, 0, group, 0, nbins, stats=sa)
    fbsr.fbsr_bias_stats_format8(xd[half:], d, SRF, 4, 9, half, group, 0, nbins, stats=sa)
    assert_stats_close(sa.cpu().numpy(), s1.cpu().numpy(), rel=1e-12)


def test_non_finite_values_propagate(fbsr, oracle):
    """Overflow to the infinity code, NaN inputs and saturation follow IEEE arithmetic in the sums."""
    n, group = 3 * 8192, 8192
    for name in ("binary8p4", "ocp_e5m2", "ocp_e4m3", "ocp_e2m1"):
        d = FORMATS[name]
        rng = np.random.default_rng(3)
        x = _inputs(rng, d, n)[:n]
        x = np.where(np.isfinite(x), x, np.float32(0.5)).astype(np.float32)
        x[100] = np.float32(np.nan)
        x[8192 + 5] = np.float32(np.inf)
        x[2 * 8192 + 9] = np.float32(-3.0e38)
        print("case fmt=%s" % name, flush=True)
        _run_both(fbsr, oracle, x, d, SRF, 4, 3, 0, group, 0, 3, with_out=True)


def test_sec3_closed_forms_at_2_24(fbsr, oracle):
    """2^24 elements: all bf16 values of [1, 2) (D = 4 excess bits for binary8p4) over many draws, three bits; the
    per-bin means land on (2^-D - 2^-N)/2 for SRFF, 2^-(D+1) for SRF and 0 for SRC (Sec. III-E), and the sums agree
    with the oracle's (threads over bins)."""
    d = FORMATS["binary8p4"]
    n, group = 1 << 24, 1 << 20
    x = np.tile((np.arange(0x3F80, 0x4000, dtype=np.uint32) << 16).view(np.float32), n // 128)
    xd = dev(x)
    want_bias = {SRFF: (2.0 ** -4 - 2.0 ** -3) / 2, SRF: 2.0 ** -5, SRC: 0.0}
    for variant in (SRFF, SRF, SRC):
        stats, _ = fbsr.fbsr_bias_stats_format8(xd, d, variant, 3, 11, 0, group, 0, n // group)
        got = stats.cpu().numpy()
        assert np.all(got[:, 0] == group)
        assert np.max(np.abs(got[:, 2] / group - want_bias[variant])) < 2e-3
        with ThreadPoolExecutor(16) as pool:
            parts = list(pool.map(lambda b: oracle.bias_stats_format8(x[b * group:(b + 1) * group], d, variant, 3, 11, b * group, group,
                                                                      b, 1)[0], range(n // group)))
        assert_stats_close(got, np.concatenate(parts))


def test_rejects_bad_arguments(fbsr):
    x = torch.ones(4096, dtype=torch.float32, device="cuda")
    d = FORMATS["binary8p4"]
    for bad in (lambda: fbsr.fbsr_bias_stats_format8(x, (9, 4, 7, 0x7E, -1, 0x7F, 1, 1), SRFF, 2, 1, 0, 512, 0, 8),
                lambda: fbsr.fbsr_bias_stats_format8(x, d, SRFF, 0, 1, 0, 512, 0, 8),
                lambda: fbsr.fbsr_bias_stats_format8(x, d, SRFF, 25, 1, 0, 512, 0, 8),
                lambda: fbsr.fbsr_bias_stats_format8(x, d, 7, 2, 1, 0, 512, 0, 8),
                lambda: fbsr.fbsr_bias_stats_format8(x, d, SRFF, 2, 1, 0, 0, 0, 8),
                lambda: fbsr.fbsr_bias_stats_format8(x, d, SRFF, 2, 1, 0, 512, 0, 7),
                lambda: fbsr.fbsr_bias_stats_format8(x, d, SRFF, 2, 1, 0, 512, 1, 8),
                lambda: fbsr.fbsr_bias_stats_format8(x, d, SRFF, 2, 1, 0, 512, 0, 8,
                                                     workspace=torch.empty(1, dtype=torch.float64, device="cuda"))):
        with pytest.raises(fbsr.FbsrError):
            bad()
