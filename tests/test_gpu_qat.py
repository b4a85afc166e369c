"""GPU parity: fbsr_qat_adamw_step (the fused step of Alg. 1) against the CPU oracle: new 8-bit
weights and both bf16 moments byte-identical."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from gpu_util import dev, first_mismatch, host

pytestmark = pytest.mark.gpu
E4M3, E5M2 = 1, 2
RNE, SRFF, SRF, SRC = 0, 1, 2, 3


def _bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _state(n, seed, wild=False):
    rng = np.random.default_rng(seed)
    w8 = rng.integers(0, 256, n).astype(np.uint8)
    g = _bf16(rng.standard_normal(n) * 0.3)
    m = _bf16(rng.standard_normal(n) * 0.05)
    v = _bf16(rng.random(n) * 0.02)
    if wild:   # raw patterns: negative second moments, infinities, NaNs, subnormals, huge gradients
        k = n // 4
        g[:k] = rng.integers(0, 1 << 16, k).astype(np.uint16)
        m[k:2 * k] = rng.integers(0, 1 << 16, k).astype(np.uint16)
        v[2 * k:3 * k] = rng.integers(0, 1 << 16, k).astype(np.uint16)
    return w8, g, m, v


def _oracle_step(oracle, w8, g, m, v, fmt, params, variant, nbits, seed, step, offset, threads=16):
    n = w8.size
    if n < 4096:
        return oracle.qat_adamw_step(w8, g, m, v, fmt, params, variant, nbits, seed, step, offset)
    cuts = np.linspace(0, n, threads + 1).astype(np.int64)
    with ThreadPoolExecutor(threads) as pool:
        parts = list(pool.map(lambda ab: oracle.qat_adamw_step(w8[ab[0]:ab[1]], g[ab[0]:ab[1]], m[ab[0]:ab[1]], v[ab[0]:ab[1]],
                                                               fmt, params, variant, nbits, seed, step, offset + int(ab[0])),
                              zip(cuts[:-1], cuts[1:])))
    return tuple(np.concatenate([p[i] for p in parts]) for i in range(3))


PARAMS = [(1e-3, 0.9, 0.999, 1e-8, 0.01, 1 - 0.9, 1 - 0.999),
          (3e-2, 0.9, 0.95, 1e-8, 0.1, 1 - 0.9 ** 3, 1 - 0.95 ** 3),
          (0.5, 0.0, 0.5, 1e-3, 0.0, 1.0, 0.5)]


@pytest.mark.parametrize("fmt", [E4M3, E5M2, 3])
def test_single_step(fbsr, oracle, fmt):
    for n in (0, 1, 7, 8, 2047, 2048, 5 * 2048 + 333):
        for wild in (False, True):
            w8, g, m, v = _state(max(n, 1), 100 + n, wild)
            w8, g, m, v = w8[:n], g[:n], m[:n], v[:n]
            for params in PARAMS:
                for variant, nbits, offset, step in ((RNE, 0, 0, 1), (SRFF, 3, 0, 2), (SRF, 3, 16, 7), (SRC, 4, 5, 1 << 33),
                                                     (SRC, 1, 0, 3), (SRF, 16, 128, 9)):
                    print("case fmt=%d n=%d wild=%d lr=%g variant=%d nbits=%d offset=%d" % (fmt, n, wild, params[0], variant, nbits, offset), flush=True)
                    if n:
                        wd, gd, md, vd = dev(w8), dev(g), dev(m), dev(v)
                    else:
                        wd = torch.empty(0, dtype=torch.uint8, device="cuda")
                        gd = md = vd = torch.empty(0, dtype=torch.int16, device="cuda")
                        md, vd = md.clone(), vd.clone()
                    fbsr.fbsr_qat_adamw_step(wd, gd, md, vd, fmt, params, variant, nbits, seed=31, step=step, offset=offset)
                    ww, mm, vv = _oracle_step(oracle, w8, g, m, v, fmt, params, variant, nbits, 31, step, offset)
                    assert first_mismatch(host(md), mm) is None, "first moment"
                    assert first_mismatch(host(vd), vv) is None, "second moment"
                    assert first_mismatch(host(wd), ww) is None, "weights"
                    assert np.array_equal(host(gd), g), "gradient buffer was written"


@pytest.mark.parametrize("fmt", [E4M3, E5M2, 3])
def test_extreme_finite_values_without_nan(fbsr, oracle, fmt):
    """Raw bit patterns for the gradient and both moments -- zeros, subnormals, magnitudes up to 2^73, squares that
    overflow to infinity -- but no input that can produce a NaN, so that every wave stays on the kernel's main path
    (hardware bf16 and fp8 converts); a wave that meets a NaN takes another path, covered by test_single_step."""
    n = 64 * 2048 + 77
    rng = np.random.default_rng(41 + fmt)
    finite8 = np.array([c for c in range(256) if np.isfinite(oracle.decode(c, fmt))], dtype=np.uint8)
    w8 = finite8[rng.integers(0, finite8.size, n)]

    def raw(signed):
        field = rng.integers(0, 201, n).astype(np.uint16)
        code = (field << 7) | rng.integers(0, 128, n).astype(np.uint16)
        return code | (rng.integers(0, 2, n).astype(np.uint16) << 15) if signed else code
    g, m, v = raw(True), raw(True), raw(False)
    # signed zeros everywhere (the sign of a zero moment can reach the sign of a zero weight), and moments around
    # 2^-103: far below the limits of the kernel's short paths (first moments below 2^-40 hand the wave over to the
    # full division; second moments below 2^-125 read a zero root), next to ordinary values in the same waves
    k = 512
    g[:k] = rng.choice(np.array([0x0000, 0x8000], dtype=np.uint16), k)
    m[:k] = rng.choice(np.array([0x0000, 0x8000], dtype=np.uint16), k)
    v[:k] = 0
    w8[:k] = rng.choice(np.array([0x00, 0x01, 0x81] + ([0x80] if fmt != 3 else []), dtype=np.uint8), k)
    edge = ((127 - 103 + rng.integers(-6, 7, k)).astype(np.uint16) << 7) | rng.integers(0, 128, k).astype(np.uint16)
    m[k:2 * k] = edge | (rng.integers(0, 2, k).astype(np.uint16) << 15)
    v[2 * k:3 * k] = edge
    g[k:3 * k] = 0
    for params in PARAMS:
        for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 2), (SRC, 4), (SRC, 16)):
            print("case fmt=%d lr=%g variant=%d nbits=%d" % (fmt, params[0], variant, nbits), flush=True)
            wd, gd, md, vd = dev(w8), dev(g), dev(m), dev(v)
            fbsr.fbsr_qat_adamw_step(wd, gd, md, vd, fmt, params, variant, nbits, seed=19, step=4, offset=0)
            ww, mm, vv = _oracle_step(oracle, w8, g, m, v, fmt, params, variant, nbits, 19, 4, 0)
            assert np.all((mm & 0x7FFF) <= 0x7F80) and np.all((vv & 0x7FFF) <= 0x7F80), "the recipe produced a NaN moment"
            assert not np.isnan([oracle.decode(int(c), fmt) for c in np.unique(ww)]).any(), "the recipe produced a NaN weight"
            assert first_mismatch(host(md), mm) is None, "first moment"
            assert first_mismatch(host(vd), vv) is None, "second moment"
            assert first_mismatch(host(wd), ww) is None, "weights"


@pytest.mark.parametrize("fmt", [E4M3, 3])
def test_moments_at_the_limits_of_the_short_paths(fbsr, oracle, fmt):
    """The limits of the tile kernel's short paths.  Second moments: exponent fields 0 and 1 (zero, bf16 subnormals,
    2^-126: the tabulated root reads zero, which an eps of 2^-28 or more must make exact), 2 and 3 (the smallest the
    tables scale), around 233 (above it the corrected moment may overflow and the wave hands over).  First moments
    around 2^-40, below which the wave hands over too.  Scalars: eps at its limit 2^-28 and at 1e-8, bias corrections
    at both ends of [2^-20, 1], and an eps below the limit (the whole launch on the full sequences).  Zero gradient,
    and first moments of the size of the denominator so that the quotient decides the update.  Tiles alternate
    between staying inside every limit (each wave on the short paths) and mixing in values just outside."""
    tiles = 24
    n = tiles * 2048
    rng = np.random.default_rng(97 + fmt)
    finite8 = np.array([c for c in range(256) if np.isfinite(oracle.decode(c, fmt)) and abs(oracle.decode(c, fmt)) <= 4.0],
                       dtype=np.uint8)
    w8 = finite8[rng.integers(0, finite8.size, n)]
    g = rng.choice(np.array([0x0000, 0x8000], dtype=np.uint16), n)

    def fields(lo, hi, count):      # positive bf16 codes, exponent field uniform in [lo, hi], any significand
        return (rng.integers(lo, hi + 1, count).astype(np.uint16) << 7) | rng.integers(0, 128, count).astype(np.uint16)
    v = np.empty(n, dtype=np.uint16)
    m = np.empty(n, dtype=np.uint16)
    for t in range(tiles):
        a, b = t * 2048, (t + 1) * 2048
        kind = t % 6
        if kind == 0:      # fields 0..3: zero, subnormal, the smallest scaled values; the denominator is eps or near it
            v[a:b] = fields(0, 3, 2048)
            v[a:a + 256] = 0
            m[a:b] = fields(127 - 32, 127 - 26, 2048)
        elif kind == 1:    # the top of the tabulated range, inside
            v[a:b] = fields(226, 233, 2048)
            m[a:b] = fields(127 + 50, 127 + 62, 2048)
        elif kind == 2:    # ... and across it (fields 234 and up overflow for the smallest correction, 255 is infinity)
            v[a:b] = np.where(rng.random(2048) < 0.05, fields(234, 255, 2048) & 0xFF80, fields(226, 233, 2048))
            m[a:b] = fields(127 + 50, 127 + 62, 2048)
        elif kind == 3:    # first moments at and above 2^-40 with a denominator of eps
            v[a:b] = 0
            m[a:b] = fields(127 - 40, 127 - 34, 2048)
            m[a:a + 64] = (127 - 40) << 7
        elif kind == 4:    # ... and across it
            v[a:b] = fields(0, 1, 2048)
            m[a:b] = fields(127 - 44, 127 - 36, 2048)
        else:              # the middle of everything
            v[a:b] = fields(60, 140, 2048)
            m[a:b] = fields(90, 130, 2048)
    m |= rng.integers(0, 2, n).astype(np.uint16) << 15
    lo = 2.0 ** -20
    scalars = ((0.5, 0.9, 0.999, 2.0 ** -28, 0.01, 1 - 0.9, 1 - 0.999), (0.25, 0.9, 0.95, 1e-8, 0.0, 1 - 0.9 ** 3, 1 - 0.95 ** 3),
               (0.125, 0.9, 0.999, 1e-6, 0.0, lo, lo), (0.5, 0.5, 0.75, 2.0 ** -28, 0.0, 1.0, 1.0),
               (0.5, 0.9, 0.999, 2.0 ** -29, 0.01, 1 - 0.9, 1 - 0.999))
    for params in scalars:
        for variant, nbits in ((RNE, 0), (SRFF, 3), (SRC, 4)):
            print("case fmt=%d lr=%g eps=%g corr=%g variant=%d nbits=%d" % (fmt, params[0], params[3], params[6], variant, nbits), flush=True)
            wd, gd, md, vd = dev(w8), dev(g), dev(m), dev(v)
            fbsr.fbsr_qat_adamw_step(wd, gd, md, vd, fmt, params, variant, nbits, seed=23, step=6, offset=0)
            ww, mm, vv = _oracle_step(oracle, w8, g, m, v, fmt, params, variant, nbits, 23, 6, 0)
            assert np.count_nonzero(ww != w8) > n // 8, "the recipe leaves the weights where they are"
            assert first_mismatch(host(md), mm) is None, "first moment"
            assert first_mismatch(host(vd), vv) is None, "second moment"
            assert first_mismatch(host(wd), ww) is None, "weights"


def test_short_division_and_tabulated_root_on_the_device(fbsr):
    """The tile kernel's own device functions against the plain operations, on the GPU at hand: its division without
    operand scaling on 2^26 operand pairs drawn to favour all-ones and all-zeros significands plus every pairing of an
    all-ones divisor significand with a power-of-two numerator (the operands on which a reciprocal one ulp low would
    show), and its two-table root of the corrected second moment on all 65536 codes for 300 correction values."""
    rng = np.random.default_rng(5)
    n = 1 << 26
    md = rng.integers(0, 1 << 23, n, dtype=np.uint32)
    mn = rng.integers(0, 1 << 23, n, dtype=np.uint32)
    kind = rng.integers(0, 8, n)
    md = np.where(kind == 0, 0x7FFFFF - rng.integers(0, 4, n, dtype=np.uint32), md)
    md = np.where(kind == 1, rng.integers(0, 4, n, dtype=np.uint32), md)
    mn = np.where(kind == 2, mn & 0x7F0000, mn)
    mn = np.where(kind == 3, 0, mn)
    ed = rng.integers(-28, 65, n)
    en = np.minimum(rng.integers(-40, 101, n), ed + 126)        # the quotient stays finite
    den = (((ed + 127).astype(np.uint32) << 23) | md.astype(np.uint32)).view(np.float32)
    num = (((en + 127).astype(np.uint32) << 23) | mn.astype(np.uint32) | (rng.integers(0, 2, n).astype(np.uint32) << 31)).view(np.float32)
    num[::1001] = 0.0
    num[1::1001] = -0.0
    dd, nn = np.meshgrid(np.arange(-28, 65), np.arange(-40, 101), indexing="ij")
    ok = (nn - dd) <= 126
    grid_d = ((dd[ok] + 127).astype(np.uint32) << 23)[:, None] | (0x7FFFFF - np.arange(8, dtype=np.uint32))[None, :]
    grid_n = np.broadcast_to(((nn[ok] + 127).astype(np.uint32) << 23)[:, None], grid_d.shape)
    den = np.concatenate([den, grid_d.reshape(-1).view(np.float32), grid_d.reshape(-1).view(np.float32)])
    num = np.concatenate([num, grid_n.reshape(-1).view(np.float32), -grid_n.reshape(-1).view(np.float32)])
    counts = torch.zeros(2, dtype=torch.int64, device="cuda")
    fbsr.binding.fbsr_check_qat_division(dev(num), dev(den), counts)
    corrections = [1.0, 2.0 ** -20, 1 - 0.999, 1 - 0.95 ** 3, float(np.float32(0.1))]
    corrections += [float(c) for c in np.exp(rng.uniform(np.log(2.0 ** -20), 0.0, 295)).astype(np.float32)]
    for c in corrections:
        fbsr.binding.fbsr_check_qat_root(c, counts)
    assert counts.tolist() == [0, 0], counts.tolist()
    with pytest.raises(fbsr.FbsrError):
        fbsr.binding.fbsr_check_qat_root(2.0, counts)


def test_stream_probe_of_the_step_is_a_plain_exclusive_or(fbsr):
    """The measurement aid in the step's launch shape: every word combined with the gradient's, nothing else touched,
    and a second call restores the buffers."""
    n = 5 * 2048
    g = torch.randint(0, 1 << 16, (n,), dtype=torch.int32, device="cuda").to(torch.int16)
    w = torch.randint(0, 256, (n + 16,), dtype=torch.int32, device="cuda").to(torch.uint8)
    m = torch.randint(0, 1 << 16, (n + 16,), dtype=torch.int32, device="cuda").to(torch.int16)
    v = torch.randint(0, 1 << 16, (n + 16,), dtype=torch.int32, device="cuda").to(torch.int16)
    w0, m0, v0, g0 = w.clone(), m.clone(), v.clone(), g.clone()
    fbsr.binding.fbsr_probe_stream75(w[:n], g, m[:n], v[:n])
    assert torch.equal(g, g0) and torch.equal(w[n:], w0[n:]) and torch.equal(m[n:], m0[n:]) and torch.equal(v[n:], v0[n:])
    assert torch.equal(m[:n], m0[:n] ^ g)
    assert torch.equal(v[:n].view(-1, 8), v0[:n].view(-1, 8) ^ g.view(-1, 4, 2).flip(1).reshape(-1, 8))
    assert not torch.equal(w[:n], w0[:n]) and bool((((w[:n] ^ w0[:n]) & 0xFE) == 0).all())
    fbsr.binding.fbsr_probe_stream75(w[:n], g, m[:n], v[:n])
    assert torch.equal(w, w0) and torch.equal(m, m0) and torch.equal(v, v0)
    with pytest.raises(fbsr.FbsrError):
        fbsr.binding.fbsr_probe_stream75(w[:100], g[:100], m[:100], v[:100])


def test_unaligned_buffers(fbsr, oracle):
    n = 3 * 2048 + 50
    w8, g, m, v = _state(n + 8, 9)
    for shift in (1, 3):
        wd, gd, md, vd = dev(w8), dev(g), dev(m), dev(v)
        sl = slice(shift, shift + n)
        fbsr.fbsr_qat_adamw_step(wd[sl], gd[sl], md[sl], vd[sl], E4M3, PARAMS[1], SRC, 3, seed=1, step=1)
        ww, mm, vv = _oracle_step(oracle, w8[sl], g[sl], m[sl], v[sl], E4M3, PARAMS[1], SRC, 3, 1, 1, 0)
        for got, want, orig in ((wd, ww, w8), (md, mm, m), (vd, vv, v)):
            full = host(got)
            assert first_mismatch(full[sl], want) is None
            assert np.array_equal(full[:shift], orig[:shift]) and np.array_equal(full[shift + n:], orig[shift + n:])


def test_ten_steps_at_2_22(fbsr, oracle):
    """A short training run: 2^22 weights, 10 steps with fresh gradients, N = 3 (the paper's setting),
    every variant: the GPU trajectory stays identical to the oracle's."""
    n = 1 << 22
    lr, b1, b2, eps, wdecay = 2e-2, 0.9, 0.99, 1e-8, 0.01
    for variant in (RNE, SRFF, SRF, SRC):
        w8, _, m, v = _state(n, 77)
        m[:] = 0
        v[:] = 0
        w8 &= 0x77          # moderate magnitudes, no NaN codes
        wd, md, vd = dev(w8), dev(m), dev(v)
        rng = np.random.default_rng(5)
        for t in range(1, 11):
            g = _bf16(rng.standard_normal(n) * 0.2)
            params = (lr, b1, b2, eps, wdecay, 1 - b1 ** t, 1 - b2 ** t)
            fbsr.fbsr_qat_adamw_step(wd, dev(g), md, vd, E4M3, params, variant, 3, seed=8, step=t)
            w8, m, v = _oracle_step(oracle, w8, g, m, v, E4M3, params, variant, 3, 8, t, 0)
        print("case variant=%d" % variant, flush=True)
        assert first_mismatch(host(md), m) is None and first_mismatch(host(vd), v) is None
        assert first_mismatch(host(wd), w8) is None


# ------------------------------------------------------------------ generic 8-bit formats ----
def p3109(P):
    return (8, P, 1 << (7 - P), 0x7E, 0x7F, 0x80, 0, 0)


FORMATS8 = {"binary8p4": p3109(4), "binary8p3": p3109(3), "binary8p5": p3109(5), "ocp_e4m3": (8, 4, 7, 0x7E, -1, 0x7F, 1, 1),
            "ocp_e5m2": (8, 3, 15, 0x7B, 0x7C, 0x7E, 1, 1), "ocp_e2m3": (6, 4, 1, 0x1F, -1, -1, 0, 1), "ocp_e2m1": (4, 2, 1, 0x07, -1, -1, 0, 1)}
SRC_ODD, RNO, RNA = 4, 5, 6


def _oracle_step8(oracle, w8, g, m, v, d, params, variant, nbits, seed, step, offset, threads=16):
    n = w8.size
    if n < 4096:
        return oracle.qat_adamw_step_format8(w8, g, m, v, d, params, variant, nbits, seed, step, offset)
    cuts = np.linspace(0, n, threads + 1).astype(np.int64)
    with ThreadPoolExecutor(threads) as pool:
        parts = list(pool.map(lambda ab: oracle.qat_adamw_step_format8(w8[ab[0]:ab[1]], g[ab[0]:ab[1]], m[ab[0]:ab[1]], v[ab[0]:ab[1]],
                                                                       d, params, variant, nbits, seed, step, offset + int(ab[0])),
                              zip(cuts[:-1], cuts[1:])))
    return tuple(np.concatenate([p[i] for p in parts]) for i in range(3))


@pytest.mark.parametrize("name", sorted(FORMATS8))
def test_format8_single_step(fbsr, oracle, name):
    """Every weight byte (NaN, infinity and unused encodings, bits above K included), tame and wild moments,
    every variant, sizes around the tile, shifted offsets."""
    d = FORMATS8[name]
    for n in (0, 1, 9, 2048, 5 * 2048 + 333):
        for wild in (False, True):
            w8, g, m, v = _state(max(n, 1), 200 + n, wild)
            w8, g, m, v = w8[:n], g[:n], m[:n], v[:n]
            for params in PARAMS[:2]:
                for variant, nbits, offset, step in ((RNE, 0, 0, 1), (SRFF, 3, 0, 2), (SRF, 3, 16, 7), (SRC, 4, 5, 1 << 33),
                                                     (SRC_ODD, 3, 0, 3), (RNO, 0, 7, 1), (RNA, 0, 0, 9), (SRF, 16, 128, 9)):
                    print("case fmt=%s n=%d wild=%d lr=%g variant=%d nbits=%d offset=%d" % (name, n, wild, params[0], variant, nbits, offset), flush=True)
                    if n:
                        wd, gd, md, vd = dev(w8), dev(g), dev(m), dev(v)
                    else:
                        wd = torch.empty(0, dtype=torch.uint8, device="cuda")
                        gd = torch.empty(0, dtype=torch.int16, device="cuda")
                        md, vd = gd.clone(), gd.clone()
                    fbsr.fbsr_qat_adamw_step_format8(wd, gd, md, vd, d, params, variant, nbits, seed=31, step=step, offset=offset)
                    ww, mm, vv = _oracle_step8(oracle, w8, g, m, v, d, params, variant, nbits, 31, step, offset)
                    assert first_mismatch(host(md), mm) is None, "first moment"
                    assert first_mismatch(host(vd), vv) is None, "second moment"
                    assert first_mismatch(host(wd), ww) is None, "weights"


def test_format8_main_path_without_nan(fbsr, oracle):
    """Finite binary8p4 weights and finite raw moments: no wave leaves the kernel's main path."""
    d = FORMATS8["binary8p4"]
    n = 32 * 2048 + 5
    rng = np.random.default_rng(61)
    finite8 = np.array([c for c in range(256) if np.isfinite(oracle.decode_format8(c, d))], dtype=np.uint8)
    w8 = finite8[rng.integers(0, finite8.size, n)]

    def raw(signed):
        code = (rng.integers(0, 201, n).astype(np.uint16) << 7) | rng.integers(0, 128, n).astype(np.uint16)
        return code | (rng.integers(0, 2, n).astype(np.uint16) << 15) if signed else code
    g, m, v = raw(True), raw(True), raw(False)
    for params in PARAMS:
        for variant, nbits in ((RNE, 0), (SRFF, 3), (SRF, 2), (SRC, 4), (SRC_ODD, 16), (RNA, 0)):
            print("case lr=%g variant=%d nbits=%d" % (params[0], variant, nbits), flush=True)
            wd, gd, md, vd = dev(w8), dev(g), dev(m), dev(v)
            fbsr.fbsr_qat_adamw_step_format8(wd, gd, md, vd, d, params, variant, nbits, seed=19, step=4, offset=0)
            ww, mm, vv = _oracle_step8(oracle, w8, g, m, v, d, params, variant, nbits, 19, 4, 0)
            assert np.all((mm & 0x7FFF) <= 0x7F80) and np.all((vv & 0x7FFF) <= 0x7F80) and not np.any(ww == 0x80), "the recipe produced a NaN"
            assert first_mismatch(host(md), mm) is None and first_mismatch(host(vd), vv) is None
            assert first_mismatch(host(wd), ww) is None, "weights"


def test_sec4_setting_binary8p4_three_bits(fbsr, oracle):
    """Sec. IV's configuration at small scale: binary8p4 weights, bf16 AdamW updates, 3 random bits, 10 steps
    over 2^21 weights with fresh gradients; the GPU trajectory equals the oracle's for every variant, and
    with an OCP E4M3 descriptor it equals fbsr_qat_adamw_step's."""
    n = 1 << 21
    lr, b1, b2, eps, wdecay = 2e-2, 0.9, 0.99, 1e-8, 0.01
    d = FORMATS8["binary8p4"]
    for variant in (RNE, SRFF, SRF, SRC):
        w8, _, m, v = _state(n, 78)
        m[:] = 0
        v[:] = 0
        w8 &= 0x77
        wd, md, vd = dev(w8), dev(m), dev(v)
        wd_a, md_a, vd_a = dev(w8), dev(m), dev(v)
        wd_b, md_b, vd_b = dev(w8), dev(m), dev(v)
        rng = np.random.default_rng(6)
        for t in range(1, 11):
            g = _bf16(rng.standard_normal(n) * 0.2)
            gd = dev(g)
            params = (lr, b1, b2, eps, wdecay, 1 - b1 ** t, 1 - b2 ** t)
            fbsr.fbsr_qat_adamw_step_format8(wd, gd, md, vd, d, params, variant, 3, seed=8, step=t)
            w8, m, v = _oracle_step8(oracle, w8, g, m, v, d, params, variant, 3, 8, t, 0)
            fbsr.fbsr_qat_adamw_step(wd_a, gd, md_a, vd_a, E4M3, params, variant, 3, seed=8, step=t)
            fbsr.fbsr_qat_adamw_step_format8(wd_b, gd, md_b, vd_b, FORMATS8["ocp_e4m3"], params, variant, 3, seed=8, step=t)
        print("case variant=%d" % variant, flush=True)
        assert first_mismatch(host(md), m) is None and first_mismatch(host(vd), v) is None
        assert first_mismatch(host(wd), w8) is None
        assert torch.equal(wd_a, wd_b) and torch.equal(md_a, md_b) and torch.equal(vd_a, vd_b)


def test_sec4_behaviour_on_a_noisy_quadratic(fbsr, oracle):
    """Sec. IV in miniature, on the fused step itself: 2^20 binary8p4 weights pulled toward targets by the noisy
    gradient of a quadratic, AdamW in bf16, updates of about an eighth of an 8-bit ulp.  Nearest-even stagnates (no
    update crosses half an ulp).  With 3 random bits and D = 4 excess bits SRFF's bias (2^-4 - 2^-3)/2 = -1/32 ulp per
    rounding pulls the weights toward zero and SRF's residual 2^-(D+1) = +1/32 ulp pushes them away by as much
    (Sec. III-E), both ending near the starting error; SRC, with either tie rule, has no bias and ends well below.
    With 4 bits (N = D, "the ideal number" of Sec. IV) all three are exact SR and agree."""
    d = FORMATS8["binary8p4"]
    n, steps, lr, sigma = 1 << 20, 1500, 5e-4, 0.05
    lut = torch.tensor([oracle.decode_format8(c, d) for c in range(256)], dtype=torch.float32, device="cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    t = torch.randn(n, device="cuda", generator=gen) * 0.05
    start = t + torch.randn(n, device="cuda", generator=gen) * 0.01
    w0 = fbsr.fbsr_round_format8(start, 2, d, RNE, 0, seed=0)
    mse0 = ((lut[w0.long()] - t) ** 2).mean().item()
    print("start           mse %.3e" % mse0, flush=True)
    result = {}
    for variant, nbits, name in ((RNE, 0, "rne"), (SRFF, 3, "srff_3"), (SRF, 3, "srf_3"), (SRC, 3, "src_3"), (SRC_ODD, 3, "src_ties_odd_3"),
                                 (SRFF, 4, "srff_4"), (SRF, 4, "srf_4"), (SRC, 4, "src_4")):
        w = w0.clone()
        m = torch.zeros(n, dtype=torch.int16, device="cuda")
        v = torch.zeros(n, dtype=torch.int16, device="cuda")
        gen.manual_seed(11)
        track = []
        for k in range(1, steps + 1):
            g = (lut[w.long()] - t + sigma * torch.randn(n, device="cuda", generator=gen)).to(torch.bfloat16).view(torch.int16)
            fbsr.fbsr_qat_adamw_step_format8(w, g, m, v, d, (lr, 0.9, 0.999, 1e-8, 0.0, 1 - 0.9 ** k, 1 - 0.999 ** k), variant, nbits, seed=5, step=k)
            if k % 500 == 0:
                track.append(((lut[w.long()] - t) ** 2).mean().item())
        shrink = (lut[w.long()].abs() - t.abs()).mean().item()
        moved = (w != w0).double().mean().item()
        result[name] = (track[-1], shrink, moved)
        print("%-15s mse at 500/1000/1500 %s  mean(|w| - |t|) %+.2e  weights moved %.3f" %
              (name, " ".join("%.3e" % x for x in track), shrink, moved), flush=True)
    assert result["rne"][0] > 0.9 * mse0 and result["rne"][2] < 0.25
    assert result["srff_3"][1] < -3e-3 and result["srf_3"][1] > 3e-3
    for name in ("src_3", "src_ties_odd_3", "srff_4", "srf_4", "src_4"):
        assert result[name][0] < 0.6 * mse0 and abs(result[name][1]) < 1.5e-3, name
    assert result["srff_3"][0] > 1.5 * result["src_3"][0] and result["srf_3"][0] > 1.5 * result["src_3"][0]
    assert max(result[k][0] for k in ("srff_4", "srf_4", "src_4")) < 1.1 * min(result[k][0] for k in ("srff_4", "srf_4", "src_4"))
