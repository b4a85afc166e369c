"""GPU parity for more than 16 random bits per element (17..24; every entry point but the fused updates): enough bits to
reach classical SR from fp32 (E4M3 and binary8p4 drop D = 20 bits, E5M2 21, bf16 16).  Aligned bodies run on the
tile kernels (32-bit slots; the hardware converts where they are exact, else the 24-bit code space with the
subnormal positions taken from a float product), heads and tails on the per-element kernels with 32 fraction bits;
the oracle is the same one, which takes any N <= 32."""
import numpy as np
import pytest
import torch

from gpu_util import assert_stats_close, dev, first_mismatch, host

pytestmark = pytest.mark.gpu

BF16, E4M3, E5M2, P4 = 0, 1, 2, 3
RNE, SRFF, SRF, SRC = 0, 1, 2, 3
TARGET = {BF16: "bf16", E4M3: "e4m3", E5M2: "e5m2", P4: "e4m3"}


def _inputs(n, fmt, seed):
    """Full-range patterns with specials, half of them pushed far below the target's smallest normal (where the
    fixed subnormal grid drops more bits than the 24 fraction bits of the tile kernels' code space hold)."""
    from paper_2504_20634_amd import workloads
    x = workloads.full_range(n, TARGET[fmt], seed=seed, specials_every=89)
    rng = np.random.default_rng(seed + 100)
    tiny = rng.integers(0, 1 << 32, n // 2, dtype=np.uint32)
    field = rng.integers(40, 125, n // 2, dtype=np.uint32)         # 2^-87 .. 2^-3
    x[: n // 2] = ((tiny & np.uint32(0x807FFFFF)) | (field << np.uint32(23))).view(np.float32)
    x[: n // 8].view(np.uint32)[:] &= np.uint32(0xFFFF0000)        # short significands: ties of the inner rounding
    return x


@pytest.mark.parametrize("fmt", [BF16, E4M3, E5M2, P4])
def test_round_with_17_to_24_bits(fbsr, oracle, fmt):
    n = 3 * 8192 + 517
    x = _inputs(n, fmt, seed=60 + fmt)
    xd = dev(x)
    for variant in (SRFF, SRF, SRC):
        for nbits in range(17, 25):
            for offset in (0, 3, (1 << 35) + 1):
                print("case fmt=%d variant=%d nbits=%d offset=%d" % (fmt, variant, nbits, offset), flush=True)
                got = host(fbsr.fbsr_round(xd, fmt, variant, nbits, seed=31, offset=offset))
                want = oracle.round_(x, fmt, variant, nbits, seed=31, offset=offset, nthreads=8)
                assert first_mismatch(got, want) is None, (fmt, variant, nbits, offset, first_mismatch(got, want))


def test_all_variants_are_exact_sr_once_every_dropped_bit_is_covered(fbsr):
    """N at or above the number of dropped bits (App. A-C): the three variants give the same codes on inputs in
    the target's normal range, where D = 24 - P bits are dropped (E4M3: 20, E5M2: 21)."""
    rng = np.random.default_rng(7)
    n = 1 << 18
    for fmt, nbits, lo, hi in ((E4M3, 20, -6, 8), (E5M2, 21, -14, 15), (E4M3, 24, -6, 8), (BF16, 16, -100, 100), (BF16, 22, -100, 100)):
        x = (rng.uniform(1.0, 2.0, n) * np.exp2(rng.integers(lo, hi + 1, n)) * rng.choice([-1.0, 1.0], n)).astype(np.float32)
        xd = dev(x)
        a = fbsr.fbsr_round(xd, fmt, SRFF, nbits, seed=3)
        b = fbsr.fbsr_round(xd, fmt, SRF, nbits, seed=3)
        c = fbsr.fbsr_round(xd, fmt, SRC, nbits, seed=3)
        assert torch.equal(a, b) and torch.equal(a, c), (fmt, nbits)
    # with fewer bits than are dropped they differ (about one element in 2^(N+1))
    x = (rng.uniform(1.0, 2.0, n) * np.exp2(rng.integers(-6, 9, n))).astype(np.float32)
    xd = dev(x)
    assert not torch.equal(fbsr.fbsr_round(xd, E4M3, SRFF, 8, seed=3), fbsr.fbsr_round(xd, E4M3, SRF, 8, seed=3))


def test_narrow_source_and_generic_formats_with_many_bits(fbsr, oracle):
    n = 2 * 8192 + 99
    rng = np.random.default_rng(11)
    codes = rng.integers(0, 1 << 16, n, dtype=np.uint16)
    cd = dev(codes)
    for src, fmt, variant, nbits in ((0, E4M3, SRC, 17), (0, E5M2, SRF, 24), (1, E4M3, SRFF, 20), (1, P4, SRC, 24), (0, P4, SRF, 19)):
        print("case from16 src=%d fmt=%d variant=%d nbits=%d" % (src, fmt, variant, nbits), flush=True)
        got = host(fbsr.fbsr_round_from16(cd, src, fmt, variant, nbits, seed=5, offset=6))
        assert first_mismatch(got, oracle.round_from16(codes, src, fmt, variant, nbits, seed=5, offset=6)) is None
    x = _inputs(n, E4M3, seed=70)
    xd = dev(x)
    formats = {"ocp_e2m1": (4, 2, 1, 0x7, -1, -1, 0, 1), "ocp_e3m2": (6, 3, 3, 0x1F, -1, -1, 0, 1), "binary8p4": (8, 4, 8, 0x7E, 0x7F, 0x80, 0, 0),
               "binary8p1": (8, 1, 64, 0x7E, 0x7F, 0x80, 0, 0), "binary8p7": (8, 7, 1, 0x7E, 0x7F, 0x80, 0, 0)}
    for name, d in formats.items():
        for variant, nbits in ((SRFF, 17), (SRF, 24), (SRC, 23), (4, 24), (4, 18), (SRC, 24)):       # 4: SRC with ties to odd
            print("case generic %s variant=%d nbits=%d" % (name, variant, nbits), flush=True)
            got = host(fbsr.fbsr_round_format8(xd, 2, d, variant, nbits, seed=9, offset=2))
            assert first_mismatch(got, oracle.round_format8(x, 2, d, variant, nbits, 9, 2)) is None, (name, variant, nbits)
        got = host(fbsr.fbsr_round_format8(cd, 0, d, SRC, 21, seed=9, offset=0))
        assert first_mismatch(got, oracle.round_format8(codes, 0, d, SRC, 21, 9, 0)) is None, name


def test_block_scaled_with_many_bits(fbsr, oracle):
    n = 3 * 2048 + 77
    x = _inputs(n, E4M3, seed=81)
    x[:64] = 0.0                                                # an all-zero block
    xd = dev(x)
    for fmt, variant, nbits, offset in ((E4M3, SRC, 17, 0), (E5M2, SRF, 24, 0), (P4, SRFF, 20, 32 * 5), (E4M3, SRC, 24, 64)):
        print("case block-scaled fmt=%d variant=%d nbits=%d offset=%d" % (fmt, variant, nbits, offset), flush=True)
        codes, scales = fbsr.fbsr_round_block_scaled(xd, fmt, variant, nbits, seed=12, offset=offset)
        wc, ws = oracle.round_block_scaled(x, fmt, variant, nbits, seed=12, offset=offset)
        assert first_mismatch(host(codes), wc) is None and first_mismatch(host(scales), ws) is None


@pytest.mark.parametrize("fmt", [BF16, E4M3, E5M2, P4])
def test_statistics_with_many_bits(fbsr, oracle, fmt):
    """Bins larger than a tile (the chunked kernel, whose strip of random bits is refilled half-way through a chunk),
    bins smaller than one (the per-bin kernel), ragged ends, an offset that starts inside a bin; codes written too."""
    n = 21 * 2048 + 300                                         # two whole chunks of 8 tiles, a part of a third, a tail
    x = _inputs(n, fmt, seed=90 + fmt)
    x = np.where(np.isfinite(x), x, np.float32(1.5)).astype(np.float32)
    xd = dev(x)
    for variant, nbits, group, offset in ((SRFF, 20, 4096, 0), (SRC, 24, 5000, 1234), (SRF, 17, 1 << 14, 8), (SRC, 21, 100, 0)):
        first_bin = offset // group
        nbins = (offset + n - 1) // group - first_bin + 1
        print("case stats fmt=%d variant=%d nbits=%d group=%d offset=%d" % (fmt, variant, nbits, group, offset), flush=True)
        out = torch.empty(n, dtype=fbsr.binding.code_dtype(fmt), device="cuda")
        stats, out = fbsr.fbsr_bias_stats(xd, fmt, variant, nbits, 6, offset, group, first_bin, nbins, out=out)
        want, wout = oracle.bias_stats(x, fmt, variant, nbits, 6, offset, group, first_bin, nbins, want_out=True)
        assert_stats_close(stats.cpu().numpy(), want)
        assert first_mismatch(host(out), wout) is None


def test_limits(fbsr):
    w = torch.zeros(64, dtype=torch.int16, device="cuda")
    g = torch.zeros(64, dtype=torch.float32, device="cuda")
    with pytest.raises(fbsr.FbsrError):
        fbsr.fbsr_sgd_update(w, g, 1e-3, SRC, 17, seed=1, step=0)
    with pytest.raises(fbsr.FbsrError):
        fbsr.fbsr_round_block_scaled(g, E4M3, SRC, 25, seed=1)
    with pytest.raises(fbsr.FbsrError):
        fbsr.fbsr_round(g, E4M3, SRC, 25, seed=1)
