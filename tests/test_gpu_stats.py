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


@pytest.mark.parametrize("fmt", [BF16, E4M3, E5M2, 3])
def test_every_path_of_the_vector_kernel(fbsr, oracle, fmt):
    """The vector kernel picks, per wave and per 512 elements, among integer paths (all positive and in the normal
    range; either sign; with zeros and target-subnormal values; the same without a sign bit) and the general fp64
    path (NaN, infinities, |x| > M, values far below the subnormal grid).  One input holds runs of 512 of every
    kind, in an order that also mixes kinds inside a wave's span; statistics and codes against the oracle."""
    rng = np.random.default_rng(100 + fmt)
    P, B, M = {BF16: (8, 127, 3.38e38), E4M3: (4, 7, 448.0), E5M2: (3, 15, 57344.0), 3: (4, 8, 224.0)}[fmt]
    tiny = 2.0 ** (1 - B)             # smallest normal value of the target
    spacing = 2.0 ** (2 - B - P)      # spacing of its subnormals

    def run(kind, n=512):
        if fmt == BF16:
            lo, hi = 1e-30, 1e30
        else:
            lo, hi = tiny, M * 0.99
        mag = np.exp(rng.uniform(np.log(lo), np.log(hi), n)).astype(np.float32)
        sign = np.where(rng.integers(0, 2, n) == 1, np.float32(-1), np.float32(1))
        if kind == "positive":
            return mag
        if kind == "signed":
            return mag * sign
        # target-subnormal values from half a subnormal spacing up: those the 24-bit code space places exactly
        sub = rng.uniform(0.505 * spacing, tiny, n).astype(np.float32)
        if kind == "positive_mixed":
            return np.where(rng.integers(0, 2, n) == 1, mag, sub).astype(np.float32)
        if kind == "mixed":
            v = np.where(rng.integers(0, 2, n) == 1, mag, sub).astype(np.float32) * sign
            v[::9] = 0.0
            v[4::18] = -0.0
            return v
        if kind == "deep":
            v = (rng.uniform(2.0 ** -40, 2.0 ** -20, n) * spacing).astype(np.float32) * sign
            v[::5] = np.float32(spacing * 2.0 ** -26 * (1 + 2.0 ** -23))
            return v
        if kind == "over":
            return (np.float32(M) * rng.uniform(1.0, 4.0, n).astype(np.float32) * sign) if fmt != BF16 else \
                np.full(n, 3.4e38, np.float32) * sign
        if kind == "special":
            v = mag * sign
            v[::7] = np.nan
            v[3::11] = np.inf
            v[5::13] = -np.inf
            return v
        raise ValueError(kind)
    kinds = ["positive", "signed", "positive_mixed", "mixed", "deep", "over", "special"]
    order = [kinds[i] for i in rng.integers(0, len(kinds), 8 * 8 * 3)] + kinds * 2
    x = np.concatenate([run(k) for k in order] + [run("signed", 300)]).astype(np.float32)
    n = x.size
    for variant, nbits in ((SRFF, 2), (SRF, 3), (SRC, 3), (RNE, 0), (SRC, 8), (SRF, 12), (SRFF, 20)):
        for group, offset in ((2048, 0), (700, 64), (1 << 20, 0)):
            first_bin = offset // group
            nbins = (offset + n - 1) // group - first_bin + 1
            print("case fmt=%d variant=%d nbits=%d group=%d offset=%d" % (fmt, variant, nbits, group, offset), flush=True)
            _run_both(fbsr, oracle, x, fmt, variant, nbits, 17, offset, group, first_bin, nbins, with_out=True)


@pytest.mark.parametrize("fmt", [E4M3, E5M2, 3])
def test_inputs_far_below_the_subnormal_grid(fbsr, oracle, fmt):
    """Replicated values below half the smallest subnormal (the Fig. 1 methodology in the range where y - x is not
    exact in fp32): every error in a bin has the same sign, so a rounding of single errors would add up.  The sum of
    e must agree with the oracle's fp64 arithmetic to the absolute floor 1e-6."""
    P, B = {E4M3: (4, 7), E5M2: (3, 15), 3: (4, 8)}[fmt]
    spacing = 2.0 ** (2 - B - P)
    X = np.array([spacing * 2.0 ** -3 * (1 + 2.0 ** -23), spacing * 2.0 ** -2 * (1 + 3 * 2.0 ** -23), spacing * 0.4999999,
                  spacing * 2.0 ** -5 * 1.5000001, spacing * 2.0 ** -1 * (1 - 2.0 ** -24), -spacing * 2.0 ** -3 * (1 + 2.0 ** -22)],
                 dtype=np.float32)
    group = 5000
    x = np.repeat(X, group)
    for variant, nbits in ((SRC, 3), (SRF, 3), (SRFF, 2), (SRF, 8), (SRC, 1)):
        print("case fmt=%d variant=%d nbits=%d" % (fmt, variant, nbits), flush=True)
        stats = _run_both(fbsr, oracle, x, fmt, variant, nbits, 23, 0, group, 0, X.size, with_out=True)
        assert np.all(stats.cpu().numpy()[:, 0] == group)
