"""GPU parity on randomly drawn calls: every entry point with random sizes (empty, tiny, ragged, several tiles),
element shifts of the buffers (so that the vector kernels' alignment conditions fail or hold by chance), offsets up to
2^40, all variants, every allowed bit count, random seeds -- each compared with the oracle, bytes exactly and
statistics to 1e-6.  Seeded: the same cases every run."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
TARGET = {0: "bf16", 1: "e4m3", 2: "e5m2", 3: "e4m3"}


def dev(a):
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


def host(t):
    a = t.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


@pytest.mark.parametrize("run_seed", [11, 12, 13])
def test_random_calls(fbsr, oracle, run_seed):
    from paper_2504_20634_amd import workloads
    rng = np.random.default_rng(run_seed)
    cases = 700
    bad = 0
    for c in range(cases):
        kind = rng.choice(["round", "from16", "block", "format8", "sgd", "qat", "stats"])
        n = int(rng.choice([rng.integers(0, 300), rng.integers(0, 70000), 2048 * int(rng.integers(1, 30)) + int(rng.integers(0, 40))]))
        shift = int(rng.integers(0, 8))
        offset = int(rng.choice([0, rng.integers(0, 4096), rng.integers(0, 1 << 40)]))
        variant = int(rng.integers(0, 4))
        maxn = 16 if kind in ("sgd", "qat") else 24
        nbits = int(rng.integers(1, maxn + 1))
        seed = int(rng.integers(0, 1 << 62))
        fmt = int(rng.integers(0, 4))
        desc = "%s n=%d shift=%d offset=%d variant=%d nbits=%d fmt=%d seed=%d" % (kind, n, shift, offset, variant, nbits, fmt, seed)
        print("case", c, desc, flush=True)
        ok = True
        if kind == "round":
            x = workloads.full_range(n + 8, TARGET[fmt], seed=c, specials_every=53)
            xd = dev(x)[shift:shift + n]
            got = host(fbsr.fbsr_round(xd, fmt, variant, nbits, seed=seed, offset=offset))
            ok = np.array_equal(got, oracle.round_(x[shift:shift + n], fmt, variant, nbits, seed=seed, offset=offset))
        elif kind == "from16":
            fmt = max(fmt, 1); src = int(rng.integers(0, 2))
            x = rng.integers(0, 1 << 16, n + 8, dtype=np.uint16)
            got = host(fbsr.fbsr_round_from16(dev(x)[shift:shift + n], src, fmt, variant, nbits, seed=seed, offset=offset))
            ok = np.array_equal(got, oracle.round_from16(x[shift:shift + n], src, fmt, variant, nbits, seed=seed, offset=offset))
        elif kind == "block":
            fmt = max(fmt, 1)
            x = workloads.full_range(n + 8, TARGET[fmt], seed=c, specials_every=997)
            offset -= offset % 32
            codes, scales = fbsr.fbsr_round_block_scaled(dev(x)[shift:shift + n], fmt, variant, nbits, seed=seed, offset=offset)
            wc, ws = oracle.round_block_scaled(x[shift:shift + n], fmt, variant, nbits, seed=seed, offset=offset)
            ok = np.array_equal(host(codes), wc) and np.array_equal(host(scales), ws)
        elif kind == "format8":
            P = int(rng.integers(1, 8)); d = (8, P, 1 << (7 - P), 0x7E, 0x7F, 0x80, 0, 0)
            if rng.random() < 0.3: d = (4, 2, 1, 0x7, -1, -1, 0, 1)
            variant = int(rng.integers(0, 7)); src = int(rng.integers(0, 3))
            if src == 2:
                x = workloads.full_range(n + 8, "e4m3", seed=c, specials_every=53)
            else:
                x = rng.integers(0, 1 << 16, n + 8, dtype=np.uint16)
            got = host(fbsr.fbsr_round_format8(dev(x)[shift:shift + n], src, d, variant, nbits, seed=seed, offset=offset))
            ok = np.array_equal(got, oracle.round_format8(x[shift:shift + n], src, d, variant, nbits, seed, offset))
        elif kind == "sgd":
            w = workloads.sgd_weights(n + 8, seed=c); g = workloads.sgd_grads(n + 8, c, seed=3, std=1e-2)
            wd = dev(w); gd = dev(g)
            fbsr.fbsr_sgd_update(wd[shift:shift + n], gd[shift:shift + n], 1e-2, variant, nbits, seed=seed, step=c, offset=offset)
            full = host(wd)
            ok = np.array_equal(full[shift:shift + n], oracle.sgd_update(w[shift:shift + n], g[shift:shift + n], 1e-2, variant, nbits, seed, c, offset)) \
                and np.array_equal(full[:shift], w[:shift]) and np.array_equal(full[shift + n:], w[shift + n:])
        elif kind == "qat":
            fmt = max(fmt, 1)
            w8 = (workloads.sgd_weights(n + 8, seed=c) & 0x7777).view(np.uint8)[:n + 8].copy()
            if fmt == 3: w8[w8 == 0x80] = 0
            g16 = workloads.sgd_weights(n + 8, seed=c + 1); m16 = workloads.sgd_weights(n + 8, seed=c + 2) & 0xBFFF; v16 = workloads.sgd_weights(n + 8, seed=c + 3) & 0x3FFF
            params = (1e-3, 0.9, 0.999, 1e-8, 0.01, 1 - 0.9 ** 3, 1 - 0.999 ** 3)
            sl = slice(shift, shift + n)
            wd, gd, md, vd = dev(w8), dev(g16), dev(m16), dev(v16)
            fbsr.fbsr_qat_adamw_step(wd[sl], gd[sl], md[sl], vd[sl], fmt, params, variant, nbits, seed=seed, step=c, offset=offset)
            ww, mm, vv = oracle.qat_adamw_step(w8[sl], g16[sl], m16[sl], v16[sl], fmt, params, variant, nbits, seed, c, offset)
            ok = np.array_equal(host(wd)[sl], ww) and np.array_equal(host(md)[sl], mm) and np.array_equal(host(vd)[sl], vv)
        else:
            x = workloads.scaled_normal(n + 8, seed=c)
            group = int(rng.choice([1, 7, 100, 2048, 5000, 1 << 14, 1 << 20]))
            if n == 0: continue
            first_bin = offset // group; nbins = (offset + n - 1) // group - first_bin + 1
            if nbins > 200000: continue
            stats, out = fbsr.fbsr_bias_stats(dev(x)[shift:shift + n], fmt, variant, nbits, seed, offset, group, first_bin, nbins,
                                              out=torch.empty(n, dtype=fbsr.binding.code_dtype(fmt), device="cuda"))
            want, wout = oracle.bias_stats(x[shift:shift + n], fmt, variant, nbits, seed, offset, group, first_bin, nbins, want_out=True)
            s = stats.cpu().numpy()
            ok = np.array_equal(host(out), wout) and np.array_equal(s[:, 0], want[:, 0]) and np.allclose(s, want, rtol=1e-6, atol=1e-6, equal_nan=True)
        if not ok:
            bad += 1
            print("MISMATCH", desc, flush=True)
    assert bad == 0
