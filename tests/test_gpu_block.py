"""GPU parity: fbsr_round_block_scaled (power-of-two scale per block of 32, Sec. I-A) against the CPU
oracle: element codes and scale bytes identical."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from gpu_util import dev, first_mismatch, host

pytestmark = pytest.mark.gpu
E4M3, E5M2 = 1, 2
RNE, SRFF, SRF, SRC = 0, 1, 2, 3


def _inputs(n, seed):
    """Blocks of very different magnitude, zeros, fp32 subnormals, a few NaN / inf blocks."""
    rng = np.random.default_rng(seed)
    nb = (n + 31) // 32
    scale = np.repeat(np.exp2(rng.integers(-140, 120, nb).astype(np.float64)), 32)[:n]
    x = (rng.standard_normal(n) * np.exp2(rng.integers(-12, 1, n)) * scale).astype(np.float32)
    for b in range(3, nb, 17):
        x[32 * b:32 * b + 32] = 0.0
    for b in range(5, nb, 23):
        x[min(n - 1, 32 * b + int(rng.integers(0, 32)))] = [np.nan, np.inf, -np.inf][b % 3]
    return x


def _oracle(oracle, x, fmt, variant, nbits, seed, offset, threads=16):
    n = x.size
    if n < 1 << 16:
        return oracle.round_block_scaled(x, fmt, variant, nbits, seed, offset)
    cuts = (np.linspace(0, n, threads + 1).astype(np.int64) // 32) * 32
    cuts[-1] = n
    with ThreadPoolExecutor(threads) as pool:
        parts = list(pool.map(lambda ab: oracle.round_block_scaled(x[ab[0]:ab[1]], fmt, variant, nbits, seed, offset + int(ab[0])),
                              zip(cuts[:-1], cuts[1:])))
    return np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])


@pytest.mark.parametrize("fmt", [E4M3, E5M2, 3])
def test_sizes_variants_offsets(fbsr, oracle, fmt):
    for n in (0, 1, 31, 32, 33, 2047, 2048, 2049, 5 * 2048 + 77):
        x = _inputs(max(n, 1), 7 + n)[:n]
        xd = dev(x) if n else torch.empty(0, dtype=torch.float32, device="cuda")
        for variant, nbits in [(RNE, 0)] + [(v, nb) for v in (SRFF, SRF, SRC) for nb in (1, 2, 3, 4, 8, 16)]:
            for offset in (0, 128, 5):
                print("case fmt=%d n=%d variant=%d nbits=%d offset=%d" % (fmt, n, variant, nbits, offset), flush=True)
                codes, scales = fbsr.fbsr_round_block_scaled(xd, fmt, variant, nbits, seed=19, offset=offset)
                wc, ws = _oracle(oracle, x, fmt, variant, nbits, 19, offset)
                assert first_mismatch(host(scales), ws) is None, "scales"
                assert first_mismatch(host(codes), wc) is None, "codes"


def test_unaligned_input_and_canaries(fbsr, oracle):
    n = 3 * 2048 + 40
    x = _inputs(n + 4, 3)
    xd = dev(x)
    for shift in (0, 1, 3):
        big = torch.full((n + 16,), 0x5A, dtype=torch.uint8, device="cuda")
        sc = torch.full(((n + 31) // 32 + 16,), 0x5A, dtype=torch.uint8, device="cuda")
        fbsr.fbsr_round_block_scaled(xd[shift:shift + n], E4M3, SRC, 3, seed=2, offset=0, out=big[8:8 + n],
                                     scales=sc[8:8 + (n + 31) // 32])
        wc, ws = _oracle(oracle, x[shift:shift + n], E4M3, SRC, 3, 2, 0)
        b, s = host(big), host(sc)
        assert first_mismatch(b[8:8 + n], wc) is None and first_mismatch(s[8:8 + ws.size], ws) is None
        assert (b[:8] == 0x5A).all() and (b[8 + n:] == 0x5A).all() and (s[:8] == 0x5A).all() and (s[8 + ws.size:] == 0x5A).all()


def test_2_26_elements_full(fbsr, oracle):
    """A large tensor of weight-like values (scaled normals), every byte, N = 3 and 8."""
    from paper_2504_20634_amd import workloads
    n = 1 << 26
    x = workloads.scaled_normal(n, seed=4)
    xd = dev(x)
    for fmt, variant, nbits in ((E4M3, SRC, 3), (E5M2, SRF, 8), (E4M3, SRFF, 2)):
        print("case fmt=%d variant=%d nbits=%d" % (fmt, variant, nbits), flush=True)
        codes, scales = fbsr.fbsr_round_block_scaled(xd, fmt, variant, nbits, seed=4)
        wc, ws = _oracle(oracle, x, fmt, variant, nbits, 4, 0)
        assert first_mismatch(host(scales), ws) is None and first_mismatch(host(codes), wc) is None
