"""GPU parity on randomly drawn calls: every entry point (the 16-bit-code, descriptor-statistics, static-workspace and
descriptor-QAT ones included) with random sizes (empty, tiny, ragged, several tiles),
element shifts of the buffers (so that the vector kernels' alignment conditions fail or hold by chance), offsets up to
2^40, all variants, every allowed bit count, random seeds, random AdamW scalars (eps on both sides of the short paths' limit) -- each compared with the oracle, bytes exactly and
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
    cases = 900
    bad = 0
    for c in range(cases):
        kind = rng.choice(["round", "from16", "block", "format8", "sgd", "qat", "stats", "format16", "stats8", "qat8", "stats"])
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
            t = int(rng.integers(1, 2000))
            params = (float(rng.choice([1e-3, 0.05, 0.5])), 0.9, float(rng.choice([0.999, 0.95])), float(rng.choice([1e-8, 2.0 ** -28, 1e-10, 1e-3, 0.0])),
                      float(rng.choice([0.0, 0.01])), 1 - 0.9 ** t, 1 - float(rng.choice([0.999, 0.95])) ** t)
            if rng.random() < 0.3:
                v16 = rng.integers(0, 1 << 15, n + 8).astype(np.uint16); m16 = rng.integers(0, 1 << 16, n + 8).astype(np.uint16)
                m16[(m16 & 0x7F80) == 0x7F80] = 0; v16[(v16 & 0x7F80) == 0x7F80] = 0
            sl = slice(shift, shift + n)
            wd, gd, md, vd = dev(w8), dev(g16), dev(m16), dev(v16)
            fbsr.fbsr_qat_adamw_step(wd[sl], gd[sl], md[sl], vd[sl], fmt, params, variant, nbits, seed=seed, step=c, offset=offset)
            ww, mm, vv = oracle.qat_adamw_step(w8[sl], g16[sl], m16[sl], v16[sl], fmt, params, variant, nbits, seed, c, offset)
            ok = np.array_equal(host(wd)[sl], ww) and np.array_equal(host(md)[sl], mm) and np.array_equal(host(vd)[sl], vv)
        elif kind == "qat8":
            P = int(rng.integers(2, 6)); d = (8, P, 1 << (7 - P), 0x7E, 0x7F, 0x80, 0, 0)
            variant = int(rng.integers(0, 7)); nbits = int(rng.integers(1, 17))
            w8 = (workloads.sgd_weights(n + 8, seed=c) & 0x7777).view(np.uint8)[:n + 8].copy(); w8[w8 == 0x80] = 0
            g16 = workloads.sgd_weights(n + 8, seed=c + 1); m16 = workloads.sgd_weights(n + 8, seed=c + 2) & 0xBFFF; v16 = workloads.sgd_weights(n + 8, seed=c + 3) & 0x3FFF
            params = (1e-3, 0.9, 0.999, 1e-8, 0.01, 1 - 0.9 ** 3, 1 - 0.999 ** 3)
            sl = slice(shift, shift + n)
            wd, gd, md, vd = dev(w8), dev(g16), dev(m16), dev(v16)
            fbsr.fbsr_qat_adamw_step_format8(wd[sl], gd[sl], md[sl], vd[sl], d, params, variant, nbits, seed=seed, step=c, offset=offset)
            ww, mm, vv = oracle.qat_adamw_step_format8(w8[sl], g16[sl], m16[sl], v16[sl], d, params, variant, nbits, seed, c, offset)
            ok = np.array_equal(host(wd)[sl], ww) and np.array_equal(host(md)[sl], mm) and np.array_equal(host(vd)[sl], vv)
        elif kind == "format16":
            d = [(16, 11, 15, 0x7BFF, 0x7C00, 0x7E00, 1, 1), (16, 10, 31, (61 << 9) | 0x1FF, -1, -1, 0, 1), (12, 6, 31, (62 << 5) | 0x1F, (63 << 5), -1, 0, 1)][int(rng.integers(0, 3))]
            variant = int(rng.integers(0, 7)); src = int(rng.integers(0, 3)); nbits = int(rng.integers(1, min(16, 30 - d[0]) + 1))
            x = workloads.full_range(n + 8, "e5m2", seed=c, specials_every=53) if src == 2 else rng.integers(0, 1 << 16, n + 8, dtype=np.uint16)
            if not oracle.format16_check(d): continue
            got = host(fbsr.fbsr_round_format16(dev(x)[shift:shift + n], src, d, variant, nbits, seed=seed, offset=offset))
            ok = np.array_equal(got, oracle.round_format16(x[shift:shift + n], src, d, variant, nbits, seed, offset))
        elif kind == "stats8":
            P = int(rng.integers(1, 8)); d = (8, P, 1 << (7 - P), 0x7E, 0x7F, 0x80, 0, 0)
            if rng.random() < 0.3: d = (8, 4, 7, 0x7E, -1, 0x7F, 1, 1)
            variant = int(rng.integers(0, 7))
            x = workloads.full_range(n + 8, "e4m3", seed=c, specials_every=int(rng.choice([0, 997]))) if rng.random() < 0.5 else workloads.scaled_normal(n + 8, seed=c)
            group = int(rng.choice([1, 7, 100, 512, 2048, 5000, 1 << 14, 1 << 20]))
            if n == 0: continue
            first_bin = offset // group; nbins = (offset + n - 1) // group - first_bin + 1
            if nbins > 200000: continue
            stats, out = fbsr.fbsr_bias_stats_format8(dev(x)[shift:shift + n], d, variant, nbits, seed, offset, group, first_bin, nbins,
                                                      out=torch.empty(n, dtype=torch.uint8, device="cuda"))
            want, wout = oracle.bias_stats_format8(x[shift:shift + n], d, variant, nbits, seed, offset, group, first_bin, nbins, want_out=True)
            s = stats.cpu().numpy()
            fin = np.isfinite(want)
            ok = np.array_equal(host(out), wout) and np.array_equal(s[:, 0], want[:, 0]) and np.array_equal(np.isnan(s), np.isnan(want)) \
                and np.allclose(s[fin], want[fin], rtol=1e-6, atol=1e-6) and np.array_equal(s[~fin & ~np.isnan(want)], want[~fin & ~np.isnan(want)])
        else:
            x = workloads.scaled_normal(n + 8, seed=c) if rng.random() < 0.4 else workloads.full_range(n + 8, TARGET[fmt], seed=c, specials_every=int(rng.choice([0, 0, 997])))
            group = int(rng.choice([1, 7, 100, 2048, 5000, 1 << 14, 1 << 20]))
            if n == 0: continue
            first_bin = offset // group; nbins = (offset + n - 1) // group - first_bin + 1
            if nbins > 200000: continue
            if rng.random() < 0.3:
                stats, out = fbsr.fbsr_bias_stats_static(dev(x)[shift:shift + n], fmt, variant, nbits, seed, offset, group, first_bin, nbins,
                                                         torch.zeros((nbins, 4), dtype=torch.float64, device="cuda"),
                                                         out=torch.empty(n, dtype=fbsr.binding.code_dtype(fmt), device="cuda"))
            else:
                stats, out = fbsr.fbsr_bias_stats(dev(x)[shift:shift + n], fmt, variant, nbits, seed, offset, group, first_bin, nbins,
                                                  out=torch.empty(n, dtype=fbsr.binding.code_dtype(fmt), device="cuda"))
            want, wout = oracle.bias_stats(x[shift:shift + n], fmt, variant, nbits, seed, offset, group, first_bin, nbins, want_out=True)
            s = stats.cpu().numpy()
            fin = np.isfinite(want)
            ok = np.array_equal(host(out), wout) and np.array_equal(s[:, 0], want[:, 0]) and np.array_equal(np.isnan(s), np.isnan(want)) \
                and np.allclose(s[fin], want[fin], rtol=1e-6, atol=1e-6) and np.array_equal(s[~fin & ~np.isnan(want)], want[~fin & ~np.isnan(want)])
        if not ok:
            bad += 1
            print("MISMATCH", desc, flush=True)
    assert bad == 0
