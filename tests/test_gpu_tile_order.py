"""GPU parity at a size where the tile kernels' XCD-aware workgroup -> tile map is in force: two whole chunks
of 2048 tiles, a part of a third that keeps the identity order, and a ragged tail, every byte compared with the
oracle for each entry point that runs a tile kernel."""
import numpy as np
import pytest

from gpu_util import dev, first_mismatch, host

pytestmark = pytest.mark.gpu

BF16, E4M3, E5M2, P4 = 0, 1, 2, 3
RNE, SRFF, SRF, SRC = 0, 1, 2, 3
N = (2 * 2048 + 300) * 2048 + 77


def test_round_every_byte(fbsr, oracle):
    from paper_2504_20634_amd import workloads
    x = workloads.full_range(N, "e4m3", seed=71, specials_every=1009)
    xd = dev(x)
    for fmt, variant, nbits, offset in ((E4M3, SRC, 3, 0), (E5M2, SRFF, 8, 1 << 33), (BF16, SRF, 5, 0), (P4, SRC, 2, 0), (E4M3, RNE, 0, 0)):
        print("case round fmt=%d variant=%d nbits=%d offset=%d n=%d" % (fmt, variant, nbits, offset, N), flush=True)
        got = host(fbsr.fbsr_round(xd, fmt, variant, nbits, seed=23, offset=offset))
        want = oracle.round_(x, fmt, variant, nbits, seed=23, offset=offset, nthreads=8)
        assert first_mismatch(got, want) is None, (fmt, variant, nbits, first_mismatch(got, want))


def test_narrow_source_block_scaled_and_generic_every_byte(fbsr, oracle):
    from paper_2504_20634_amd import workloads
    x = workloads.full_range(N, "e5m2", seed=72, specials_every=2003)
    x16 = workloads.sgd_weights(N, seed=73)
    xd, x16d = dev(x), dev(x16)
    print("case from16 n=%d" % N, flush=True)
    got = host(fbsr.fbsr_round_from16(x16d, 0, E4M3, SRC, 3, seed=4))
    assert first_mismatch(got, oracle.round_from16(x16, 0, E4M3, SRC, 3, seed=4)) is None
    print("case block scaled n=%d" % N, flush=True)
    codes, scales = fbsr.fbsr_round_block_scaled(xd, E4M3, SRF, 4, seed=5)
    wc, ws = oracle.round_block_scaled(x, E4M3, SRF, 4, seed=5)
    assert first_mismatch(host(codes), wc) is None and first_mismatch(host(scales), ws) is None
    e2m1 = (4, 2, 1, 0x7, -1, -1, 0, 1)
    for src, data, datad in ((2, x, xd), (0, x16, x16d)):
        print("case generic src=%d n=%d" % (src, N), flush=True)
        got = host(fbsr.fbsr_round_format8(datad, src, e2m1, SRC, 3, seed=6))
        assert first_mismatch(got, oracle.round_format8(data, src, e2m1, SRC, 3, 6, 0)) is None


def test_fused_updates_every_byte(fbsr, oracle):
    from paper_2504_20634_amd import workloads
    w16 = workloads.sgd_weights(N, seed=74)
    g = workloads.sgd_grads(N, step=3, seed=75)
    print("case sgd n=%d" % N, flush=True)
    wd = dev(w16)
    fbsr.fbsr_sgd_update(wd, dev(g), 1e-2, SRC, 4, seed=7, step=3)
    assert first_mismatch(host(wd), oracle.sgd_update(w16, g, 1e-2, SRC, 4, 7, 3)) is None
    w8 = (workloads.sgd_weights(N, seed=76) & 0x7777).view(np.uint8)[:N].copy()
    g16 = workloads.sgd_weights(N, seed=77)
    m16 = workloads.sgd_weights(N, seed=78) & 0x3FFF
    v16 = workloads.sgd_weights(N, seed=79) & 0x3FFF
    params = (1e-3, 0.9, 0.999, 1e-8, 0.01, 1 - 0.9 ** 2, 1 - 0.999 ** 2)
    p4 = (8, 4, 8, 0x7E, 0x7F, 0x80, 0, 0)
    for generic in (False, True):
        print("case qat generic=%d n=%d" % (generic, N), flush=True)
        wd, gd, md, vd = dev(w8), dev(g16), dev(m16), dev(v16)
        if generic:
            fbsr.fbsr_qat_adamw_step_format8(wd, gd, md, vd, p4, params, SRC, 3, seed=8, step=2)
            ww, mm, vv = oracle.qat_adamw_step_format8(w8, g16, m16, v16, p4, params, SRC, 3, 8, 2, 0)
        else:
            fbsr.fbsr_qat_adamw_step(wd, gd, md, vd, E4M3, params, SRC, 3, seed=8, step=2)
            ww, mm, vv = oracle.qat_adamw_step(w8, g16, m16, v16, E4M3, params, SRC, 3, 8, 2, 0)
        assert first_mismatch(host(wd), ww) is None and first_mismatch(host(md), mm) is None and first_mismatch(host(vd), vv) is None
