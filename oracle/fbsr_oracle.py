"""ctypes access to the CPU oracle (oracle/fbsr_oracle.cpp).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It never imports the GPU package, and the GPU package never imports it.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(_HERE, "fbsr_oracle.cpp")
LIB = os.path.join(_HERE, "liboracle_fbsr.so")
# A test that plants a mistake in a COPY of the oracle points this at the mutated build.
_OVERRIDE = os.environ.get("FBSR_ORACLE_LIB")

FMT_BF16, FMT_E4M3, FMT_E5M2, FMT_BINARY8P4 = 0, 1, 2, 3
SRC_BF16, SRC_FP16 = 0, 1
FROM_BF16, FROM_FP16, FROM_FP32 = 0, 1, 2  # source types of the generic-format entry points
RNE, SRFF, SRF, SRC = 0, 1, 2, 3
SRC_ODD, TNO, TA = 4, 5, 6                        # generic-format entry points only
FMT_NAMES = {FMT_BF16: "bf16", FMT_E4M3: "e4m3", FMT_E5M2: "e5m2", FMT_BINARY8P4: "binary8p4"}
VARIANT_NAMES = {RNE: "rne", SRFF: "srff", SRF: "srf", SRC: "src"}


def build(force=False):
    """Compile the oracle with the host compiler (no contraction: the SGD step's single
    fused multiply-add must stay the only fused operation)."""
    if _OVERRIDE:
        return _OVERRIDE
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SOURCE):
        subprocess.check_call(
            ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
             "-o", LIB, SOURCE])
    return LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u64, u32, i32, f32, f64 = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int,
                                   ctypes.c_float, ctypes.c_double)
        vp = ctypes.c_void_p
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.oracle_philox4x32_10.restype = None
        L.oracle_random_bits.argtypes = [u64, u64, u64, i32]
        L.oracle_random_bits.restype = u64
        L.oracle_round_with_n.argtypes = [f32, i32, i32, i32, u64]
        L.oracle_round_with_n.restype = u32
        L.oracle_decode.argtypes = [u32, i32]
        L.oracle_decode.restype = f64
        L.oracle_ulp.argtypes = [f32, i32]
        L.oracle_ulp.restype = f64
        L.oracle_count_up.argtypes = [vp, u64, i32, i32, i32, vp]
        L.oracle_count_up.restype = i32
        L.oracle_round.argtypes = [vp, vp, u64, i32, i32, i32, u64, u64]
        L.oracle_round.restype = i32
        L.oracle_round_threads.argtypes = [vp, vp, u64, i32, i32, i32, u64, u64, i32]
        L.oracle_round_threads.restype = i32
        L.oracle_round_from16.argtypes = [vp, vp, u64, i32, i32, i32, i32, u64, u64]
        L.oracle_round_from16.restype = i32
        L.oracle_widen16.argtypes = [ctypes.c_uint16, i32]
        L.oracle_widen16.restype = u32
        L.oracle_qat_adamw_step.argtypes = [vp, vp, vp, vp, u64, i32, vp, i32, i32, u64, u64, u64]
        L.oracle_qat_adamw_step.restype = i32
        L.oracle_qat_adamw_step_format8.argtypes = [vp, vp, vp, vp, u64, vp, vp, i32, i32, u64, u64, u64]
        L.oracle_qat_adamw_step_format8.restype = i32
        L.oracle_round_block_scaled.argtypes = [vp, vp, vp, u64, i32, i32, i32, u64, u64]
        L.oracle_round_block_scaled.restype = i32
        L.oracle_format8_check.argtypes = [vp]
        L.oracle_format8_check.restype = i32
        L.oracle_decode_format8.argtypes = [u32, vp]
        L.oracle_decode_format8.restype = ctypes.c_double
        L.oracle_round_format8_with_n.argtypes = [f32, vp, i32, i32, u64]
        L.oracle_round_format8_with_n.restype = u32
        L.oracle_round_format8.argtypes = [vp, i32, vp, u64, vp, i32, i32, u64, u64]
        L.oracle_round_format8.restype = i32
        L.oracle_format16_check.argtypes = [vp]
        L.oracle_format16_check.restype = i32
        L.oracle_decode_format16.argtypes = [u32, vp]
        L.oracle_decode_format16.restype = ctypes.c_double
        L.oracle_round_format16_with_n.argtypes = [f32, vp, i32, i32, u64]
        L.oracle_round_format16_with_n.restype = u32
        L.oracle_round_format16.argtypes = [vp, i32, vp, u64, vp, i32, i32, u64, u64]
        L.oracle_round_format16.restype = i32
        L.oracle_sgd_update.argtypes = [vp, vp, u64, f32, i32, i32, u64, u64, u64]
        L.oracle_sgd_update.restype = i32
        L.oracle_bias_stats.argtypes = [vp, vp, u64, i32, i32, i32, u64, u64, u64, u64, u32, vp]
        L.oracle_bias_stats.restype = i32
        L.oracle_bias_stats_format8.argtypes = [vp, vp, u64, vp, i32, i32, u64, u64, u64, u64, u32, vp]
        L.oracle_bias_stats_format8.restype = i32
        _lib = L
    return _lib


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def code_dtype(fmt):
    return np.uint16 if fmt == FMT_BF16 else np.uint8


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def random_bits(seed, step, index, nbits):
    return int(lib().oracle_random_bits(seed, step, index, nbits))


def round_with_n(x, fmt, variant, nbits, n):
    code = lib().oracle_round_with_n(float(np.float32(x)), fmt, variant, nbits, n)
    if code == 0xFFFFFFFF:
        raise ValueError("oracle_round_with_n: bad arguments")
    return int(code)


def decode(code, fmt):
    return float(lib().oracle_decode(int(code), fmt))


def ulp(x, fmt):
    return float(lib().oracle_ulp(float(np.float32(x)), fmt))


def count_up(x, fmt, variant, nbits):
    """For each x: how many of the 2^nbits draws round it away from zero."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    ups = np.zeros(x.size, dtype=np.uint64)
    rc = lib().oracle_count_up(_ptr(x), x.size, fmt, variant, nbits, _ptr(ups))
    if rc != 0:
        raise ValueError("oracle_count_up: status %d" % rc)
    return ups


def round_(x, fmt, variant, nbits, seed, offset=0, nthreads=1):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.size, dtype=code_dtype(fmt))
    if nthreads > 1:
        rc = lib().oracle_round_threads(_ptr(x), _ptr(out), x.size, fmt, variant, nbits, seed,
                                        offset, nthreads)
    else:
        rc = lib().oracle_round(_ptr(x), _ptr(out), x.size, fmt, variant, nbits, seed, offset)
    if rc != 0:
        raise ValueError("oracle_round: status %d" % rc)
    return out


def round_from16(x, src_fmt, fmt, variant, nbits, seed, offset=0):
    """x: uint16 codes of the source format (0 = bf16, 1 = IEEE binary16) -> fp8 codes."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    out = np.empty(x.size, dtype=np.uint8)
    rc = lib().oracle_round_from16(_ptr(x), _ptr(out), x.size, src_fmt, fmt, variant, nbits, seed, offset)
    if rc != 0:
        raise ValueError("oracle_round_from16: status %d" % rc)
    return out


def widen16(code, src_fmt):
    """fp32 bit pattern of the exact value of a 16-bit source code."""
    return int(lib().oracle_widen16(int(code), src_fmt))


def round_block_scaled(x, fmt, variant, nbits, seed, offset=0):
    """Blocks of 32 share a power-of-two scale.  Returns (codes uint8[n], scales uint8[ceil(n/32)])."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.size, dtype=np.uint8)
    scales = np.empty((x.size + 31) // 32, dtype=np.uint8)
    rc = lib().oracle_round_block_scaled(_ptr(x), _ptr(out), _ptr(scales), x.size, fmt, variant, nbits, seed, offset)
    if rc != 0:
        raise ValueError("oracle_round_block_scaled: status %d" % rc)
    return out, scales


def _desc(desc):
    d = np.asarray(desc, dtype=np.int32)
    assert d.shape == (8,), "descriptor = (K, P, B, max_code, inf_code, nan_code, nan_signed, neg_zero)"
    return np.ascontiguousarray(d)


def format8_check(desc):
    return lib().oracle_format8_check(_ptr(_desc(desc))) == 0


def decode_format8(code, desc):
    return float(lib().oracle_decode_format8(int(code), _ptr(_desc(desc))))


def round_format8_with_n(x, desc, variant, nbits, n):
    code = lib().oracle_round_format8_with_n(float(np.float32(x)), _ptr(_desc(desc)), variant, nbits, n)
    if code == 0xFFFFFFFF:
        raise ValueError("oracle_round_format8_with_n: bad arguments")
    return int(code)


def round_format8(x, src, desc, variant, nbits, seed, offset=0):
    """x: fp32 values (src = 2) or uint16 codes of bf16 (src = 0) / IEEE binary16 (src = 1); desc as in
    _desc.  Returns one code per byte."""
    x = np.ascontiguousarray(x, dtype=np.float32 if src == FROM_FP32 else np.uint16)
    out = np.empty(x.size, dtype=np.uint8)
    rc = lib().oracle_round_format8(_ptr(x), src, _ptr(out), x.size, _ptr(_desc(desc)), variant, nbits, seed, offset)
    if rc != 0:
        raise ValueError("oracle_round_format8: status %d" % rc)
    return out


def bias_stats_format8(x, desc, variant, nbits, seed, offset, group, first_bin, nbins, stats=None, want_out=False):
    """bias_stats for a format given by its descriptor: (stats[nbins,4], byte codes or None)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if stats is None:
        stats = np.zeros((nbins, 4), dtype=np.float64)
    assert stats.dtype == np.float64 and stats.shape == (nbins, 4) and stats.flags.c_contiguous
    out = np.empty(x.size, dtype=np.uint8) if want_out else None
    rc = lib().oracle_bias_stats_format8(_ptr(x), _ptr(out) if want_out else None, x.size, _ptr(_desc(desc)), variant, nbits,
                                         seed, offset, group, first_bin, nbins, _ptr(stats))
    if rc != 0:
        raise ValueError("oracle_bias_stats_format8: status %d" % rc)
    return stats, out


def format16_check(desc):
    return lib().oracle_format16_check(_ptr(_desc(desc))) == 0


def decode_format16(code, desc):
    return float(lib().oracle_decode_format16(int(code), _ptr(_desc(desc))))


def round_format16_with_n(x, desc, variant, nbits, n):
    code = lib().oracle_round_format16_with_n(float(np.float32(x)), _ptr(_desc(desc)), variant, nbits, n)
    if code == 0xFFFFFFFF:
        raise ValueError("oracle_round_format16_with_n: bad arguments")
    return int(code)


def round_format16(x, src, desc, variant, nbits, seed, offset=0):
    """round_format8 for a format of up to 16 bits: one code per uint16."""
    x = np.ascontiguousarray(x, dtype=np.float32 if src == FROM_FP32 else np.uint16)
    out = np.empty(x.size, dtype=np.uint16)
    rc = lib().oracle_round_format16(_ptr(x), src, _ptr(out), x.size, _ptr(_desc(desc)), variant, nbits, seed, offset)
    if rc != 0:
        raise ValueError("oracle_round_format16: status %d" % rc)
    return out


def sgd_update(w, g, lr, variant, nbits, seed, step, offset=0):
    """Returns the updated bf16 codes (the input array is not modified)."""
    w = np.array(w, dtype=np.uint16, copy=True)
    g = np.ascontiguousarray(g, dtype=np.float32)
    assert w.size == g.size
    rc = lib().oracle_sgd_update(_ptr(w), _ptr(g), w.size, float(np.float32(lr)), variant, nbits,
                                 seed, step, offset)
    if rc != 0:
        raise ValueError("oracle_sgd_update: status %d" % rc)
    return w


def qat_adamw_step(w8, g16, m16, v16, fmt, params, variant, nbits, seed, step, offset=0):
    """One fused QAT step.  params = (lr, beta1, beta2, eps, weight_decay, 1 - beta1^t, 1 - beta2^t).
    Returns new (w8, m16, v16); the inputs are not modified."""
    w8 = np.array(w8, dtype=np.uint8, copy=True)
    m16 = np.array(m16, dtype=np.uint16, copy=True)
    v16 = np.array(v16, dtype=np.uint16, copy=True)
    g16 = np.ascontiguousarray(g16, dtype=np.uint16)
    p = np.asarray(params, dtype=np.float32)
    assert p.size == 7 and w8.size == g16.size == m16.size == v16.size
    rc = lib().oracle_qat_adamw_step(_ptr(w8), _ptr(g16), _ptr(m16), _ptr(v16), w8.size, fmt, _ptr(p), variant,
                                     nbits, seed, step, offset)
    if rc != 0:
        raise ValueError("oracle_qat_adamw_step: status %d" % rc)
    return w8, m16, v16


def qat_adamw_step_format8(w8, g16, m16, v16, desc, params, variant, nbits, seed, step, offset=0):
    """qat_adamw_step with the 8-bit weights in a generic format (descriptor as in round_format8)."""
    w8 = np.array(w8, dtype=np.uint8, copy=True)
    m16 = np.array(m16, dtype=np.uint16, copy=True)
    v16 = np.array(v16, dtype=np.uint16, copy=True)
    g16 = np.ascontiguousarray(g16, dtype=np.uint16)
    p = np.asarray(params, dtype=np.float32)
    assert p.size == 7 and w8.size == g16.size == m16.size == v16.size
    rc = lib().oracle_qat_adamw_step_format8(_ptr(w8), _ptr(g16), _ptr(m16), _ptr(v16), w8.size, _ptr(_desc(desc)), _ptr(p),
                                             variant, nbits, seed, step, offset)
    if rc != 0:
        raise ValueError("oracle_qat_adamw_step_format8: status %d" % rc)
    return w8, m16, v16


def bias_stats(x, fmt, variant, nbits, seed, offset, group, first_bin, nbins, stats=None,
               want_out=False):
    """Returns (stats[nbins,4], out or None); accumulates into `stats` when given."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if stats is None:
        stats = np.zeros((nbins, 4), dtype=np.float64)
    assert stats.dtype == np.float64 and stats.shape == (nbins, 4) and stats.flags.c_contiguous
    out = np.empty(x.size, dtype=code_dtype(fmt)) if want_out else None
    rc = lib().oracle_bias_stats(_ptr(x), _ptr(out) if want_out else None, x.size, fmt, variant,
                                 nbits, seed, offset, group, first_bin, nbins, _ptr(stats))
    if rc != 0:
        raise ValueError("oracle_bias_stats: status %d" % rc)
    return stats, out
