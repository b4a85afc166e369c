"""GPU parity: fbsr_round_from16 (bf16 / binary16 -> fp8, the narrow-source setting of Sec. III-E
and Fig. 2) against the CPU oracle, byte for byte."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from gpu_util import assert_stats_close, dev, first_mismatch, host

pytestmark = pytest.mark.gpu
E4M3, E5M2, P4 = 1, 2, 3
RNE, SRFF, SRF, SRC = 0, 1, 2, 3
SRC_BF16, SRC_FP16 = 0, 1


def _oracle_from16(oracle, x, src, fmt, variant, nbits, seed, offset, threads=16):
    cuts = np.linspace(0, x.size, threads + 1).astype(np.int64)
    with ThreadPoolExecutor(threads) as pool:
        parts = list(pool.map(lambda ab: oracle.round_from16(x[ab[0]:ab[1]], src, fmt, variant, nbits, seed,
                                                             offset + int(ab[0])), zip(cuts[:-1], cuts[1:])))
    return np.concatenate(parts)


@pytest.mark.parametrize("src", [SRC_BF16, SRC_FP16])
@pytest.mark.parametrize("fmt", [E4M3, E5M2, P4])
def test_every_source_code_many_draws(fbsr, oracle, src, fmt):
    """All 65536 source codes (every normal, subnormal, zero, infinity, NaN), each drawn 64 times at
    different global indices, every variant, N below, at and above the number of excess bits."""
    codes = np.tile(np.arange(65536, dtype=np.uint16), 64)
    xd = dev(codes)
    for variant, nbits in [(RNE, 0)] + [(v, nb) for v in (SRFF, SRF, SRC) for nb in (1, 2, 3, 4, 5, 8, 11, 16)]:
        print("case src=%d fmt=%d variant=%d nbits=%d" % (src, fmt, variant, nbits), flush=True)
        got = host(fbsr.fbsr_round_from16(xd, src, fmt, variant, nbits, seed=13, offset=0))
        want = _oracle_from16(oracle, codes, src, fmt, variant, nbits, 13, 0)
        assert first_mismatch(got, want) is None, (src, fmt, variant, nbits, first_mismatch(got, want))


@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 127, 2047, 2048, 2049, 3 * 2048 + 100, 4 * 2048, 5 * 2048 + 9])
def test_sizes_offsets_alignment(fbsr, oracle, n):
    rng = np.random.default_rng(n)
    codes = rng.integers(0, 1 << 16, n + 8, dtype=np.uint16)
    xd = dev(codes)
    for src, fmt, variant, nbits in ((SRC_BF16, E4M3, SRFF, 3), (SRC_FP16, E5M2, SRC, 6), (SRC_BF16, E5M2, SRF, 2),
                                     (SRC_FP16, E4M3, RNE, 0)):
        for offset in (0, 3, 128, (1 << 36) + 5):
            for shift in (0, 1):
                print("case n=%d src=%d fmt=%d variant=%d nbits=%d offset=%d shift=%d" % (n, src, fmt, variant, nbits, offset, shift), flush=True)
                xs = xd[shift:shift + n] if n else torch.empty(0, dtype=torch.int16, device="cuda")
                got = host(fbsr.fbsr_round_from16(xs, src, fmt, variant, nbits, seed=2, offset=offset))
                want = oracle.round_from16(codes[shift:shift + n], src, fmt, variant, nbits, seed=2, offset=offset)
                assert first_mismatch(got, want) is None


def test_matches_the_fp32_path_on_widened_values(fbsr):
    """Rounding a bf16 source equals rounding its exact fp32 widening with fbsr_round."""
    codes = np.tile(np.arange(65536, dtype=np.uint16), 4)
    xd = dev(codes)
    wide = (xd.view(torch.int16).to(torch.int32) << 16).view(torch.float32)
    for fmt in (E4M3, E5M2, P4):
        for variant, nbits in ((SRFF, 2), (SRF, 4), (SRC, 3), (RNE, 0)):
            a = fbsr.fbsr_round_from16(xd, SRC_BF16, fmt, variant, nbits, seed=8, offset=4096)
            b = fbsr.fbsr_round(wide, fmt, variant, nbits, seed=8, offset=4096)
            assert torch.equal(a, b)


def test_rejects_bad_arguments(fbsr):
    x = torch.zeros(16, dtype=torch.int16, device="cuda")
    for src, fmt in ((2, E4M3), (-1, E5M2), (SRC_BF16, 0), (SRC_FP16, 4)):
        with pytest.raises(fbsr.FbsrError):
            fbsr.fbsr_round_from16(x, src, fmt, SRFF, 2, seed=0)


def test_fig2_experiment(fbsr, oracle):
    """Fig. 2: every bf16 value of one target interval, 100000 samples each, rounded to a
    precision-3 format (E5M2, D = 5 excess bits) with N = 3 random bits.  The rounded codes match the
    oracle and the measured bias lands on the printed -0.046875 / +0.015625 / 0.000 (noise of the
    draws ~ 0.4 / sqrt(3.2e6) ~ 2.5e-4 ulp).  The statistics run on the exact fp32 widening of the
    same values (identical rounding)."""
    samples = 100000
    codes16 = np.repeat((0x4000 + np.arange(32)).astype(np.uint16), samples)       # bf16 values in [2, 2.5)
    xd16 = dev(codes16)
    wide = (codes16.astype(np.uint32) << 16).view(np.float32)
    xd32 = dev(wide)
    for variant, printed in ((SRFF, -0.046875), (SRF, 0.015625), (SRC, 0.0)):
        got = host(fbsr.fbsr_round_from16(xd16, SRC_BF16, E5M2, variant, 3, seed=0))
        want = _oracle_from16(oracle, codes16, SRC_BF16, E5M2, variant, 3, 0, 0)
        assert first_mismatch(got, want) is None
        stats, out = fbsr.fbsr_bias_stats(xd32, E5M2, variant, 3, 0, 0, samples, 0, 32,
                                          out=torch.empty(wide.size, dtype=torch.uint8, device="cuda"))
        assert np.array_equal(host(out), got)
        s = stats.cpu().numpy()
        assert np.all(s[:, 0] == samples)
        bias = s[:, 2].sum() / s[:, 0].sum()
        assert abs(bias - printed) < 1.5e-3, (variant, bias)
