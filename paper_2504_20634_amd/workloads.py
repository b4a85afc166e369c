"""Seeded synthetic inputs for the five benchmark workloads.

This module is shared by the GPU tests, the benchmark and the CPU oracle's tests, so it
holds NO rounding arithmetic and no random-bit generator of the method: it only builds
fp32 / bf16 input arrays with numpy (PCG64 streams), as plain bytes that are handed
unchanged to whichever side consumes them.  It imports neither the GPU binding nor the
oracle.

The paper's own experiments use analytic grids (Fig. 1, Fig. 2) and language-model weights
and updates (Alg. 1, Sec. IV); the generators below stand in for those: a Fig.-1 style grid,
scaled-normal tensors like weights/activations to be cast to fp8, full-range log-uniform
tensors, weight/gradient pairs for the fused update, and a log-spaced bin sweep.
"""
import numpy as np

# exponent-field ranges (fp32 biased exponent) for the full-range workload, per target:
# from two binades below the target's smallest subnormal to one binade above its largest
# finite value.
_FULL_RANGE_FIELDS = {
    "e5m2": (127 - 16 - 2, 127 + 16),   # min subnormal 2^-16, max 1.75 * 2^15
    "e4m3": (127 - 9 - 2, 127 + 9),     # min subnormal 2^-9,  max 1.75 * 2^8
    "bf16": (0, 254),                   # bf16 shares fp32's exponent range
}


def fig1_grid(points=1024, samples=5000, ulps=16, dtype=np.float32):
    """Workload 1 (Fig. 1 style): `points` values evenly spaced over [1, 1 + ulps * 2^-7),
    each replicated `samples` times, bin-major (element k * samples + r holds X_k).
    Returns (x, X) with X the distinct values.  2^-7 is one bf16 ulp in [1, 2)."""
    step = ulps * 2.0 ** -7 / points
    X = (1.0 + np.arange(points, dtype=np.float64) * step).astype(dtype)
    assert np.all(X.astype(np.float64) == 1.0 + np.arange(points) * step), "grid not exact in fp32"
    return np.repeat(X, samples), X


def scaled_normal(n, seed=1):
    """Workload 2: z * 2^k * s with z ~ N(0,1), k uniform integer in [-6, 6], s = +-1."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal(n, dtype=np.float32)
    k = rng.integers(-6, 7, size=n, dtype=np.int32)
    s = rng.integers(0, 2, size=n, dtype=np.int32) * 2 - 1
    return (z * np.ldexp(np.float32(1.0), k) * s.astype(np.float32)).astype(np.float32)


def full_range(n, target, seed=2, specials_every=0):
    """Workload 3: random sign, fp32 exponent field uniform over the target's whole range
    (subnormals below, overflow above), 23 random trailing bits: piecewise log-uniform
    magnitudes.  specials_every > 0 overwrites every such element with +-inf / NaN in turn."""
    lo, hi = _FULL_RANGE_FIELDS[target]
    rng = np.random.default_rng(seed)
    bits = rng.integers(0, 1 << 32, size=n, dtype=np.uint32)
    field = rng.integers(lo, hi + 1, size=n, dtype=np.uint32)
    bits = (bits & np.uint32(0x807FFFFF)) | (field << np.uint32(23))
    if specials_every:
        idx = np.arange(0, n, specials_every)
        pattern = np.array([0x7F800000, 0xFF800000, 0x7FC00000, 0xFFC00001, 0x7F800001],
                           dtype=np.uint32)
        bits[idx] = pattern[np.arange(idx.size) % pattern.size]
    return bits.view(np.float32)


def sgd_weights(n, seed=3):
    """Workload 4 weights: U(-1,1) fp32 samples cut to their upper 16 bits (a bf16 code)."""
    rng = np.random.default_rng(seed)
    w = rng.uniform(-1.0, 1.0, size=n).astype(np.float32)
    return (w.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def sgd_grads(n, step, seed=3, std=1e-3):
    """Workload 4 gradients for one step: fp32 N(0, std^2), fresh per (seed, step)."""
    rng = np.random.default_rng([seed, step, 0x5EED])
    return (rng.standard_normal(n, dtype=np.float32) * np.float32(std)).astype(np.float32)


def log_bins(nbins=4096, group=1 << 18, lo_exp=-10.0, hi_exp=10.0, seed=5, bins=None):
    """Workload 5: nbins log-spaced bins spanning [2^lo_exp, 2^hi_exp); bin b holds `group`
    fp32 values uniform in [edge_b, edge_{b+1}), bin-major.  `bins` (an iterable of bin
    numbers) restricts the output to those bins, each with its own stream, so any subset
    can be regenerated without the rest.  Returns (x, edges)."""
    edges = np.exp2(lo_exp + (hi_exp - lo_exp) * np.arange(nbins + 1, dtype=np.float64) / nbins)
    edges = edges.astype(np.float32)
    which = range(nbins) if bins is None else list(bins)
    out = np.empty(len(which) * group, dtype=np.float32)
    for k, b in enumerate(which):
        rng = np.random.default_rng([seed, b])
        u = rng.random(group, dtype=np.float64)
        lo, hi = np.float64(edges[b]), np.float64(edges[b + 1])
        v = (lo + u * (hi - lo)).astype(np.float32)
        # the fp32 cast may land exactly on the upper edge; fold it back inside the bin
        v = np.where(v >= edges[b + 1], edges[b], v)
        out[k * group:(k + 1) * group] = v
    return out, edges
