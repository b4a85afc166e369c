"""GPU parity: fbsr_bias_stats (per-bin mean / bias reduction of Figs. 1-2) against the oracle:
counts exact, sums within 1e-6 relative (fp64 accumulation on both sides), codes byte-identical."""
import numpy as np
import pytest
import torch

from gpu_util import assert_stats_close, dev, first_mismatch, host

pytestmark = pytest.mark.gpu
BF16, E4M3, E5M2 = 0, 1, 2
RNE, SRFF, SRF, SRC = 0, 1, 2, 3


def _run_both(fbsr, oracle, x, fmt, variant, nbits, seed, offset, group, first_bin, nbins, with_out):
    xd = dev(x)
    out = torch.empty(x.size, dtype=fbsr.binding.code_dtype(fmt), device="cuda") if with_out else None
    stats, out = fbsr.fbsr_bias_stats(xd, fmt, variant, nbits, seed, offset, group, first_bin, nbins, out=out)
    want, wout = oracle.bias_stats(x, fmt, variant, nbits, seed, offset, group, first_bin, nbins, want_out=with_out)
    assert_stats_close(stats.cpu().numpy(), want)
    if with_out:
        assert first_mismatch(host(out), wout) is None
    return stats


@pytest.mark.parametrize("fmt", [BF16, E4M3, E5M2, 3])
def test_groups_of_every_size(fbsr, oracle, fmt):
    """Bins smaller than, equal to and larger than a tile; ragged ends; offsets; bins that the
    call only partly covers."""
    from paper_2504_20634_amd import workloads
    n = 5 * 8192 + 700
    x = workloads.scaled_normal(n, seed=14 + fmt)
    for variant, nbits in ((SRFF, 2), (SRF, 8), (SRC, 3), (RNE, 0), (SRC, 16), (SRFF, 1)):
        for group, offset in ((1, 0), (7, 3), (1000, 0), (1024, 0), (5000, 0), (5000, 1234), (8192, 8192), (20000, 16),
                              (1 << 20, 5)):
            first_bin = offset // group
            nbins = (offset + n - 1) // group - first_bin + 1
            print("case fmt=%d variant=%d nbits=%d group=%d offset=%d" % (fmt, variant, nbits, group, offset), flush=True)
            _run_both(fbsr, oracle, x, fmt, variant, nbits, 6, offset, group, first_bin, nbins,
                      with_out=(group in (7, 5000)))


def test_accumulates_and_is_reproducible(fbsr, oracle):
    from paper_2504_20634_amd import workloads
    n, group = 4 * 8192, 5000
    x = workloads.scaled_normal(n, seed=2)
    xd = dev(x)
    nbins = (n - 1) // group + 1
    s1, _ = fbsr.fbsr_bias_stats(xd, E4M3, SRF, 4, 9, 0, group, 0, nbins)
    s2, _ = fbsr.fbsr_bias_stats(xd, E4M3, SRF, 4, 9, 0, group, 0, nbins)
    assert torch.equal(s1, s2), "reduction order is not fixed"
    s3 = s1.clone()
    fbsr.fbsr_bias_stats(xd, E4M3, SRF, 4, 9, 0, group, 0, nbins, stats=s3)
    assert torch.equal(s3, 2 * s1)
    # two half calls accumulate to the whole
    half = 2 * 8192
    sa = torch.zeros_like(s1)
    fbsr.fbsr_bias_stats(xd[:half], E4M3, SRF, 4, 9, 0, group, 0, nbins, stats=sa)
    fbsr.fbsr_bias_stats(xd[half:], E4M3, SRF, 4, 9, half, group, 0, nbins, stats=sa)
    assert_stats_close(sa.cpu().numpy(), s1.cpu().numpy(), rel=1e-12)


def test_non_finite_values_propagate(fbsr, oracle):
    """Overflow to infinity, NaN inputs and saturation follow IEEE arithmetic in the sums."""
    from paper_2504_20634_amd import workloads
    n, group = 3 * 8192, 8192
    for fmt in (BF16, E5M2, E4M3, 3):
        x = workloads.full_range(n, {BF16: "bf16", E5M2: "e5m2", E4M3: "e4m3", 3: "e4m3"}[fmt], seed=77, specials_every=0)
        x[100] = np.float32(np.nan)
        x[8192 + 5] = np.float32(np.inf)
        x[2 * 8192 + 9] = np.float32(-3.0e38)
        print("case fmt=%d" % fmt, flush=True)
        _run_both(fbsr, oracle, x, fmt, SRF, 4, 3, 0, group, 0, 3, with_out=True)


def test_fig1_grid_reproduces_the_papers_bias(fbsr, oracle):
    """Workload 1 (Fig. 1 style): 1024 X values x 5000 samples, bf16, N = 2.  GPU statistics
    match the oracle and land on the closed forms at D = 6: SRFF -0.1171875, SRF +0.0078125,
    SRC 0 (Sec. III-E); rounded codes are byte-identical."""
    from paper_2504_20634_amd import workloads
    x, X = workloads.fig1_grid()
    xd = dev(x)
    for variant, expect in ((SRFF, -0.1171875), (SRF, 0.0078125), (SRC, 0.0)):
        print("case variant=%d" % variant, flush=True)
        out = torch.empty(x.size, dtype=torch.uint16, device="cuda")
        stats, _ = fbsr.fbsr_bias_stats(xd, BF16, variant, 2, 0, 0, 5000, 0, 1024, out=out)
        want, wout = oracle.bias_stats(x, BF16, variant, 2, 0, 0, 5000, 0, 1024, want_out=True)
        assert_stats_close(stats.cpu().numpy(), want)
        assert first_mismatch(host(out), wout) is None
        rounded = fbsr.fbsr_round(xd, BF16, variant, 2, seed=0)
        assert torch.equal(rounded.view(torch.int16), out.view(torch.int16))
        s = stats.cpu().numpy()
        bias = s[:, 2].sum() / s[:, 0].sum()
        assert abs(bias - expect) < 1e-3, (variant, bias)
