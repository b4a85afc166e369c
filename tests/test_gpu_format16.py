"""GPU parity: fbsr_round_format16 (generic (K, P, B; M) targets with codes of up to 16 bits, IEEE binary16 among
them; every rounding mode of fbsr_round_format8) against the CPU oracle, code for code."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from gpu_util import dev, first_mismatch, host
from test_gpu_format8 import FROM_BF16, FROM_FP16, FROM_FP32, RNA, RNE, RNO, SRC, SRC_ODD, SRF, SRFF, _inputs

pytestmark = pytest.mark.gpu
MODES = [(RNE, 0), (RNO, 0), (RNA, 0)] + [(v, nb) for v in (SRFF, SRF, SRC, SRC_ODD) for nb in (1, 3, 8, 13, 14, 16)]
FORMATS = {"ieee_binary16": (16, 11, 15, 0x7BFF, 0x7C00, 0x7E00, 1, 1),
           "e6m9": (16, 10, 31, (62 << 9) | 0x1FF, 63 << 9, (63 << 9) | 0x100, 1, 1),
           "e8m7_low": (16, 8, 127, (253 << 7) | 0x7F, 254 << 7, (254 << 7) | 0x40, 1, 1),
           "e5m6_sat": (12, 7, 15, (31 << 6) | 0x3F, -1, -1, 0, 1),
           "ocp_e4m3": (8, 4, 7, 0x7E, -1, 0x7F, 1, 1)}      # a narrow format through the 16-bit entry point


def _oracle(oracle, x, src, d, variant, nbits, seed, offset, threads=16):
    cuts = np.linspace(0, x.size, threads + 1).astype(np.int64)
    with ThreadPoolExecutor(threads) as pool:
        parts = list(pool.map(lambda ab: oracle.round_format16(x[ab[0]:ab[1]], src, d, variant, nbits, seed, offset + int(ab[0])),
                              zip(cuts[:-1], cuts[1:])))
    return np.concatenate(parts)


@pytest.mark.parametrize("name", sorted(FORMATS))
def test_every_mode_from_fp32(fbsr, oracle, name):
    d = FORMATS[name]
    assert fbsr.format16_check(d) and oracle.format16_check(d)
    rng = np.random.default_rng(sum(map(ord, name)))
    x = _inputs(rng, d, 5 * 2048 + 333)
    xd = dev(x)
    for variant, nbits in MODES:
        if nbits > min(16, 30 - d[0]):      # the entry point's limit
            continue
        print("case %s variant=%d nbits=%d" % (name, variant, nbits), flush=True)
        got = host(fbsr.fbsr_round_format16(xd, FROM_FP32, d, variant, nbits, seed=21, offset=0))
        want = _oracle(oracle, x, FROM_FP32, d, variant, nbits, 21, 0)
        assert first_mismatch(got, want) is None, (name, variant, nbits, first_mismatch(got, want))


@pytest.mark.parametrize("src", [FROM_BF16, FROM_FP16])
def test_every_16_bit_source_code(fbsr, oracle, src):
    """All 65536 source codes (NaNs and infinities included), repeated so that tiles and a ragged tail occur."""
    codes = np.tile(np.arange(1 << 16, dtype=np.uint16), 2)[:2 * 65536 - 77]
    cd = dev(codes)
    for name in ("ieee_binary16", "e6m9", "e5m6_sat"):
        d = FORMATS[name]
        for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 2), (SRC, 3), (SRC_ODD, 5), (RNA, 0)):
            print("case src=%d %s variant=%d nbits=%d" % (src, name, variant, nbits), flush=True)
            got = host(fbsr.fbsr_round_format16(cd, src, d, variant, nbits, seed=5, offset=0))
            want = _oracle(oracle, codes, src, d, variant, nbits, 5, 0)
            assert first_mismatch(got, want) is None, (src, name, variant, nbits, first_mismatch(got, want))


def test_offsets_alignment_and_chunks(fbsr, oracle):
    """Unaligned buffers, offsets off the block grid, sizes around a tile: the vector and the per-element kernel give
    the same codes, and chunked calls continue the index."""
    d = FORMATS["ieee_binary16"]
    rng = np.random.default_rng(3)
    host_x = _inputs(rng, d, 3 * 2048 + 500)
    big = dev(np.concatenate([host_x, host_x[:8]]))
    for variant, nbits in ((SRF, 3), (SRC, 14), (RNE, 0)):
        for shift in (0, 1, 3):
            for offset in (0, 5, 64, 4099):
                n = host_x.size - 16
                xs = big[shift:shift + n]
                out = torch.empty(n + 1, dtype=torch.uint16, device="cuda")[1 if shift == 3 else 0:][:n]
                print("case variant=%d shift=%d offset=%d" % (variant, shift, offset), flush=True)
                got = host(fbsr.fbsr_round_format16(xs, FROM_FP32, d, variant, nbits, seed=2, offset=offset, out=out))
                want = oracle.round_format16(host_x[shift:shift + n] if shift + n <= host_x.size else
                                             np.concatenate([host_x, host_x[:8]])[shift:shift + n], FROM_FP32, d, variant, nbits, 2, offset)
                assert first_mismatch(got, want) is None, (variant, shift, offset, first_mismatch(got, want))
    x = dev(host_x)
    whole = fbsr.fbsr_round_format16(x, FROM_FP32, d, SRC, 3, seed=11, offset=1000)
    cut = 2048 + 77
    a = fbsr.fbsr_round_format16(x[:cut], FROM_FP32, d, SRC, 3, seed=11, offset=1000)
    b = fbsr.fbsr_round_format16(x[cut:], FROM_FP32, d, SRC, 3, seed=11, offset=1000 + cut)
    assert torch.equal(whole.view(torch.int16), torch.cat([a, b]).view(torch.int16))


def test_named_binary16_and_library_cast(fbsr):
    """The named descriptor; nearest-even through it equals torch's own fp32 -> float16 conversion on the device
    (a library routine outside this build) for every non-NaN input."""
    d = fbsr.format8_named("ieee_binary16")
    assert d.astuple() == FORMATS["ieee_binary16"]
    rng = np.random.default_rng(9)
    x = dev(_inputs(rng, FORMATS["ieee_binary16"], 1 << 20))
    got = fbsr.fbsr_round_format16(x, FROM_FP32, d, RNE, 0, seed=0)
    want = x.to(torch.float16).view(torch.int16)
    ok = ~torch.isnan(x)
    assert torch.equal(got.view(torch.int16)[ok], want[ok])


def test_argument_errors(fbsr):
    x = torch.zeros(64, dtype=torch.float32, device="cuda")
    with pytest.raises(fbsr.FbsrError):
        fbsr.fbsr_round_format16(x, FROM_FP32, (16, 7, 15, 0x7BFF, -1, -1, 0, 1), RNE, 0, seed=0)     # P < K - 8
    with pytest.raises(fbsr.FbsrError):
        fbsr.fbsr_round_format16(x, FROM_FP32, FORMATS["ieee_binary16"], SRFF, 15, seed=0)            # more than 30 - K bits
    with pytest.raises(fbsr.FbsrError):
        fbsr.fbsr_round_format16(x, FROM_FP32, FORMATS["e5m6_sat"], SRFF, 17, seed=0)                 # more than 16 bits
    with pytest.raises(fbsr.FbsrError):
        fbsr.fbsr_round_format8(x, FROM_FP32, FORMATS["ieee_binary16"], RNE, 0, seed=0)               # 16-bit codes do not fit a byte
