"""GPU parity: fbsr_round through the C ABI against the CPU oracle, byte for byte."""
import numpy as np
import pytest
import torch

from gpu_util import dev, first_mismatch, host

pytestmark = pytest.mark.gpu

BF16, E4M3, E5M2, P4 = 0, 1, 2, 3        # P4: P3109 binary8p4
RNE, SRFF, SRF, SRC = 0, 1, 2, 3
FMT_TARGET = {BF16: "bf16", E4M3: "e4m3", E5M2: "e5m2", P4: "e4m3"}   # binary8p4 spans E4M3's range, one binade lower


def _mixed_inputs(n, fmt, seed):
    """Full-range patterns with specials sprinkled in, plus a band of scaled normals."""
    from paper_2504_20634_amd import workloads
    x = workloads.full_range(n, FMT_TARGET[fmt], seed=seed, specials_every=97)
    m = min(n // 3, 5000)
    if m:
        x[-m:] = workloads.scaled_normal(m, seed=seed + 1)
    return x


@pytest.mark.parametrize("fmt", [BF16, E4M3, E5M2, P4])
def test_all_variants_and_bit_counts(fbsr, oracle, fmt):
    """Several tiles plus ragged head and tail, every variant, every N in 1..16."""
    n = 3 * 8192 + 1024 + 333
    x = _mixed_inputs(n, fmt, seed=40 + fmt)
    xd = dev(x)
    cases = [(RNE, 0)] + [(v, nb) for v in (SRFF, SRF, SRC) for nb in range(1, 17)]
    for variant, nbits in cases:
        for offset in (0, 5):
            print("case fmt=%d variant=%d nbits=%d offset=%d n=%d" % (fmt, variant, nbits, offset, n), flush=True)
            got = host(fbsr.fbsr_round(xd, fmt, variant, nbits, seed=17, offset=offset))
            want = oracle.round_(x, fmt, variant, nbits, seed=17, offset=offset, nthreads=8)
            assert first_mismatch(got, want) is None, (fmt, variant, nbits, offset, first_mismatch(got, want))


@pytest.mark.parametrize("n", [0, 1, 3, 15, 16, 17, 127, 128, 1023, 1024, 1025, 4095, 4096, 8191, 8192, 8193, 20000])
def test_sizes_and_offsets(fbsr, oracle, n):
    """Empty, tiny and ragged sizes; offsets that do and do not start a Philox block."""
    x = _mixed_inputs(max(n, 1), E4M3, seed=3)[:n]
    xd = dev(x) if n else torch.empty(0, dtype=torch.float32, device="cuda")
    for fmt, variant, nbits in ((E4M3, SRFF, 2), (E5M2, SRC, 8), (BF16, SRF, 1), (BF16, SRC, 16), (E4M3, RNE, 0)):
        for offset in (0, 1, 64, 1000, (1 << 40) + 3):
            print("case n=%d fmt=%d variant=%d nbits=%d offset=%d" % (n, fmt, variant, nbits, offset), flush=True)
            got = host(fbsr.fbsr_round(xd, fmt, variant, nbits, seed=99, offset=offset))
            want = oracle.round_(x, fmt, variant, nbits, seed=99, offset=offset)
            assert got.shape == want.shape
            assert first_mismatch(got, want) is None, (n, fmt, variant, nbits, offset, first_mismatch(got, want))


def test_unaligned_buffers_take_the_element_path(fbsr, oracle):
    """x or out not 16-byte aligned: same bytes as the aligned call."""
    n = 2 * 8192 + 77
    x = _mixed_inputs(n + 8, E5M2, seed=8)
    xd = dev(x)
    for shift in (1, 2, 3):
        for fmt, variant, nbits in ((E5M2, SRF, 4), (BF16, SRFF, 2), (E4M3, SRC, 3)):
            print("case shift=%d fmt=%d variant=%d nbits=%d" % (shift, fmt, variant, nbits), flush=True)
            xs = xd[shift:shift + n]
            want = oracle.round_(x[shift:shift + n], fmt, variant, nbits, seed=5, offset=11)
            got = host(fbsr.fbsr_round(xs, fmt, variant, nbits, seed=5, offset=11))
            assert first_mismatch(got, want) is None
            # misaligned output, aligned input
            big = torch.zeros(n + 8, dtype=fbsr.binding.code_dtype(fmt), device="cuda")
            o = big[shift:shift + n]
            fbsr.fbsr_round(xd[:n], fmt, variant, nbits, seed=5, offset=11, out=o)
            want2 = oracle.round_(x[:n], fmt, variant, nbits, seed=5, offset=11)
            assert first_mismatch(host(o), want2) is None
            rest = host(big)
            assert not rest[:shift].any() and not rest[shift + n:].any(), "wrote outside the output range"


def test_chunked_calls_and_repeats_are_identical(fbsr):
    """Pure function of the arguments: a repeat gives the same bytes, and cutting the call into
    chunks whose offset continues the index gives the same bytes as the whole call."""
    n = 5 * 8192 + 100
    x = _mixed_inputs(n, E4M3, seed=12)
    xd = dev(x)
    for fmt, variant, nbits in ((E4M3, SRFF, 2), (E5M2, SRF, 6), (BF16, SRC, 12)):
        whole = fbsr.fbsr_round(xd, fmt, variant, nbits, seed=31, offset=256)
        again = fbsr.fbsr_round(xd, fmt, variant, nbits, seed=31, offset=256)
        assert torch.equal(whole.view(torch.uint8), again.view(torch.uint8))
        cuts = [0, 100, 100 + 8192, 100 + 8192 + 4096 + 64, 30000, n]
        parts = [fbsr.fbsr_round(xd[a:b], fmt, variant, nbits, seed=31, offset=256 + a)
                 for a, b in zip(cuts[:-1], cuts[1:])]
        assert torch.equal(whole.view(torch.uint8), torch.cat(parts).view(torch.uint8))
        other = fbsr.fbsr_round(xd, fmt, variant, nbits, seed=32, offset=256)
        assert not torch.equal(whole.view(torch.uint8), other.view(torch.uint8))


def test_output_canaries(fbsr):
    """Nothing is written outside [out, out + n)."""
    for fmt in (BF16, E4M3):
        for n in (1024, 8192 * 2, 8192 * 2 + 5):
            x = dev(_mixed_inputs(n, fmt, seed=2))
            dt = fbsr.binding.code_dtype(fmt)
            pad = 64
            big = torch.full((n + 2 * pad,), 0x5A, dtype=torch.uint8, device="cuda") if fmt != BF16 else \
                torch.full((n + 2 * pad,), 0x5A5A, dtype=torch.int16, device="cuda").view(dt)
            fbsr.fbsr_round(x, fmt, SRF, 4, seed=1, offset=0, out=big[pad:pad + n])
            b = host(big)
            canary = 0x5A if fmt != BF16 else 0x5A5A
            assert (b[:pad] == canary).all() and (b[pad + n:] == canary).all()


def test_runs_on_a_side_stream(fbsr, oracle):
    n = 8192 * 3
    x = _mixed_inputs(n, E5M2, seed=6)
    xd = dev(x)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        out = fbsr.fbsr_round(xd, E5M2, SRC, 5, seed=4, offset=0, stream=s)
    s.synchronize()
    assert first_mismatch(host(out), oracle.round_(x, E5M2, SRC, 5, seed=4)) is None


@pytest.mark.parametrize("fmt,variant,nbits", [(E4M3, SRFF, 8), (E5M2, SRF, 4), (E4M3, SRC, 3), (E5M2, SRC, 8),
                                               (E5M2, SRFF, 2), (E4M3, SRF, 16), (P4, SRC, 3), (P4, SRFF, 8), (P4, SRF, 2),
                                               (E4M3, SRC, 24), (E5M2, SRF, 21), (P4, SRFF, 20),
                                               (E4M3, SRFF, 20), (E4M3, SRF, 19), (E5M2, SRC, 20), (P4, SRC, 17),
                                               (E4M3, SRF, 24), (E5M2, SRC, 23), (P4, SRF, 24)])
def test_every_fp32_pattern(fbsr, oracle, fmt, variant, nbits):
    """All 2^32 input patterns (every normal, subnormal, zero, infinity and NaN of both signs), in
    16 slabs of 2^28 consecutive patterns, through the tile kernel: byte-identical to the oracle.  This is what
    licenses the hardware stochastic-rounding converts inside the fp8 tile kernel, with up to 24 - P random bits on any
    input and with more on target-normal inputs (the cases with 17 and more bits cover both sides of that line)."""
    slab = 1 << 28
    for s_no in range(16):
        base = s_no * slab
        bits = np.arange(base, base + slab, dtype=np.uint32)
        x = bits.view(np.float32)
        xd = torch.arange(base - (1 << 32) if base >= (1 << 31) else base,
                          (base - (1 << 32) if base >= (1 << 31) else base) + slab,
                          dtype=torch.int64, device="cuda").to(torch.int32).view(torch.float32)
        got = host(fbsr.fbsr_round(xd, fmt, variant, nbits, seed=77, offset=base))
        del xd
        want = oracle.round_(x, fmt, variant, nbits, seed=77, offset=base, nthreads=16)
        print("case fmt=%d variant=%d nbits=%d slab=%d" % (fmt, variant, nbits, s_no), flush=True)
        assert first_mismatch(got, want) is None, (s_no, first_mismatch(got, want))


def test_fp32_subnormal_inputs_to_fp8(fbsr, oracle):
    """fp32 subnormals and the smallest normals are ordinary (tiny) values for the fp8 targets."""
    rng = np.random.default_rng(5)
    n = 3 * 2048 + 40
    bits = rng.integers(0, 1 << 25, n, dtype=np.uint32) | (rng.integers(0, 2, n, dtype=np.uint32) << np.uint32(31))
    x = bits.view(np.float32)
    xd = dev(x)
    for fmt in (E4M3, E5M2, P4):
        for variant, nbits in ((SRFF, 4), (SRF, 8), (SRC, 2), (RNE, 0)):
            got = host(fbsr.fbsr_round(xd, fmt, variant, nbits, seed=1))
            assert first_mismatch(got, oracle.round_(x, fmt, variant, nbits, seed=1)) is None


def test_stream_probe_copies_top_bytes(fbsr):
    """The measurement aid writes the top byte of every pattern and nothing else."""
    n = 7 * 4096
    bits = torch.randint(-2 ** 31, 2 ** 31 - 1, (n,), dtype=torch.int64, device="cuda").to(torch.int32)
    out = torch.full((n + 16,), 0xA5, dtype=torch.uint8, device="cuda")
    fbsr.binding.fbsr_probe_stream41(bits.view(torch.float32), out[:n])
    assert torch.equal(out[:n], ((bits >> 24) & 0xFF).to(torch.uint8)) and bool((out[n:] == 0xA5).all())
    with pytest.raises(fbsr.FbsrError):
        fbsr.binding.fbsr_probe_stream41(bits.view(torch.float32)[:100], out[:100])
