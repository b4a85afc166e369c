"""ctypes binding of the C ABI in include/fbsr.h.  Argument marshalling only: every step of
the computation runs in the library's HIP kernels.  Tensors are torch tensors on the GPU
(torch is used for device memory and streams, nothing else).

The binding loads the in-tree libfbsr.so and raises if it is missing: there is no fallback.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfbsr.so")

FMT_BF16, FMT_E4M3, FMT_E5M2, FMT_BINARY8P4 = 0, 1, 2, 3
RNE, SRFF, SRF, SRC = 0, 1, 2, 3
SRC_TIES_ODD, RNO, RNA = 4, 5, 6          # fbsr_round_format8 only
SRC_BF16, SRC_FP16 = 0, 1
FROM_BF16, FROM_FP16, FROM_FP32 = 0, 1, 2  # source types of fbsr_round_format8
OK, EINVAL, EALIGN, ERANGE, EDEVICE = 0, 1, 2, 3, 4
MAX_NBITS = 16            # the fused updates (SGD, QAT steps)
MAX_NBITS_ROUND = 24      # every other entry point
FMT_NAMES = {FMT_BF16: "bf16", FMT_E4M3: "e4m3", FMT_E5M2: "e5m2", FMT_BINARY8P4: "binary8p4"}
VARIANT_NAMES = {RNE: "rne", SRFF: "srff", SRF: "srf", SRC: "src"}
EXPORTS = ("fbsr_round", "fbsr_round_from16", "fbsr_round_format8", "fbsr_round_format16", "fbsr_format16_check", "fbsr_format8_named", "fbsr_format8_check", "fbsr_qat_adamw_step_format8", "fbsr_round_block_scaled", "fbsr_qat_adamw_step", "fbsr_sgd_update", "fbsr_bias_stats", "fbsr_bias_stats_format8", "fbsr_bias_stats_static", "fbsr_bias_stats_workspace_bytes",
           "fbsr_probe_stream41", "fbsr_probe_stream75", "fbsr_check_qat_division", "fbsr_check_qat_root", "fbsr_strerror", "fbsr_version")


class FbsrError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (status %d)" % (what, strerror(status), status))


_lib = None


def lib():
    """The loaded library.  Raises OSError if libfbsr.so has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("libfbsr.so is not built: run `python -m paper_2504_20634_amd.build` "
                          "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        u64, u32, i32, f32, vp = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_float,
                                  ctypes.c_void_p)
        L.fbsr_round.argtypes = [vp, vp, u64, i32, i32, i32, u64, u64, vp]
        L.fbsr_round.restype = i32
        L.fbsr_round_from16.argtypes = [vp, vp, u64, i32, i32, i32, i32, u64, u64, vp]
        L.fbsr_round_from16.restype = i32
        L.fbsr_round_block_scaled.argtypes = [vp, vp, vp, u64, i32, i32, i32, u64, u64, vp]
        L.fbsr_round_block_scaled.restype = i32
        L.fbsr_qat_adamw_step.argtypes = [vp, vp, vp, vp, u64, i32, vp, i32, i32, u64, u64, u64, vp]
        L.fbsr_qat_adamw_step.restype = i32
        L.fbsr_sgd_update.argtypes = [vp, vp, u64, f32, i32, i32, u64, u64, u64, vp]
        L.fbsr_sgd_update.restype = i32
        L.fbsr_bias_stats.argtypes = [vp, vp, u64, i32, i32, i32, u64, u64, u64, u64, u32, vp, vp, u64, vp]
        L.fbsr_bias_stats.restype = i32
        L.fbsr_bias_stats_format8.argtypes = [vp, vp, u64, vp, i32, i32, u64, u64, u64, u64, u32, vp, vp, u64, vp]
        L.fbsr_bias_stats_format8.restype = i32
        L.fbsr_bias_stats_static.argtypes = [vp, vp, u64, i32, i32, i32, u64, u64, u64, u64, u32, vp, vp]
        L.fbsr_bias_stats_static.restype = i32
        L.fbsr_bias_stats_workspace_bytes.argtypes = [u64, u32]
        L.fbsr_bias_stats_workspace_bytes.restype = u64
        L.fbsr_format8_named.argtypes = [ctypes.c_char_p, vp]
        L.fbsr_format8_named.restype = i32
        L.fbsr_format8_check.argtypes = [vp]
        L.fbsr_format8_check.restype = i32
        L.fbsr_round_format8.argtypes = [vp, i32, vp, u64, vp, i32, i32, u64, u64, vp]
        L.fbsr_round_format8.restype = i32
        L.fbsr_round_format16.argtypes = [vp, i32, vp, u64, vp, i32, i32, u64, u64, vp]
        L.fbsr_round_format16.restype = i32
        L.fbsr_format16_check.argtypes = [vp]
        L.fbsr_format16_check.restype = i32
        L.fbsr_qat_adamw_step_format8.argtypes = [vp, vp, vp, vp, u64, vp, vp, i32, i32, u64, u64, u64, vp]
        L.fbsr_qat_adamw_step_format8.restype = i32
        L.fbsr_probe_stream41.argtypes = [vp, vp, u64, vp]
        L.fbsr_probe_stream41.restype = i32
        L.fbsr_probe_stream75.argtypes = [vp, vp, vp, vp, u64, vp]
        L.fbsr_probe_stream75.restype = i32
        L.fbsr_check_qat_division.argtypes = [vp, vp, u64, vp, vp]
        L.fbsr_check_qat_division.restype = i32
        L.fbsr_check_qat_root.argtypes = [ctypes.c_float, vp, vp]
        L.fbsr_check_qat_root.restype = i32
        L.fbsr_strerror.argtypes = [i32]
        L.fbsr_strerror.restype = ctypes.c_char_p
        L.fbsr_version.argtypes = []
        L.fbsr_version.restype = i32
        _lib = L
    return _lib


def strerror(status):
    return lib().fbsr_strerror(int(status)).decode()


def _check(status, what):
    if status != OK:
        raise FbsrError(status, what)


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def code_dtype(fmt):
    import torch
    return torch.uint16 if fmt == FMT_BF16 else torch.uint8


def fbsr_round(x, fmt, variant, nbits, seed, offset=0, out=None, stream=None):
    """out[j] = FBSR(x[j]) with the random bits of global element offset + j.
    x: float32 CUDA tensor (contiguous).  Returns the code tensor (uint16 for bf16, uint8 for
    fp8), allocated with torch unless `out` is given."""
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    n = x.numel()
    if out is None:
        out = torch.empty(n, dtype=code_dtype(fmt), device=x.device)
    assert out.is_cuda and out.is_contiguous() and out.numel() == n and out.dtype == code_dtype(fmt)
    _check(lib().fbsr_round(x.data_ptr(), out.data_ptr(), n, fmt, variant, nbits, seed, offset,
                            _stream_handle(stream)), "fbsr_round")
    return out


def fbsr_round_from16(x, src_fmt, fmt, variant, nbits, seed, offset=0, out=None, stream=None):
    """Narrow-source rounding: x holds 16-bit codes of src_fmt (SRC_BF16 / SRC_FP16) as a uint16 /
    int16 / bfloat16 / float16 CUDA tensor; returns the fp8 code tensor (uint8)."""
    import torch
    assert x.is_cuda and x.element_size() == 2 and x.is_contiguous()
    n = x.numel()
    if out is None:
        out = torch.empty(n, dtype=torch.uint8, device=x.device)
    assert out.is_cuda and out.is_contiguous() and out.numel() == n and out.dtype == torch.uint8
    _check(lib().fbsr_round_from16(x.data_ptr(), out.data_ptr(), n, src_fmt, fmt, variant, nbits, seed,
                                   offset, _stream_handle(stream)), "fbsr_round_from16")
    return out


class Format8(ctypes.Structure):
    """Mirror of the C struct fbsr_format8: a format (K, P, B; M) with K <= 8 and its special codes."""
    _fields_ = [(k, ctypes.c_int32) for k in ("width", "precision", "bias", "max_code", "inf_code", "nan_code",
                                             "nan_signed", "neg_zero")]

    def astuple(self):
        return tuple(getattr(self, k) for k, _ in self._fields_)


def _format8(fmt):
    return fmt if isinstance(fmt, Format8) else Format8(*[int(v) for v in fmt])


def format8_named(name):
    """The descriptor of a published format ("ocp_e4m3", "ocp_e2m1", "p3109_binary8p4", ...).  Host-only."""
    f = Format8()
    _check(lib().fbsr_format8_named(name.encode(), ctypes.byref(f)), "fbsr_format8_named(%r)" % name)
    return f


def format8_check(fmt):
    """True when the descriptor (a Format8 or an 8-tuple) is acceptable.  Host-only."""
    return lib().fbsr_format8_check(ctypes.byref(_format8(fmt))) == OK


def fbsr_round_format8(x, src, fmt, variant, nbits, seed, offset=0, out=None, stream=None):
    """Rounds to a generic format (a Format8 or an 8-tuple), one code per output byte.  x: float32 CUDA tensor
    (src = FROM_FP32) or a tensor of 16-bit codes (FROM_BF16 / FROM_FP16)."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.element_size() == (4 if src == FROM_FP32 else 2)
    if src == FROM_FP32:
        assert x.dtype == torch.float32
    n = x.numel()
    if out is None:
        out = torch.empty(n, dtype=torch.uint8, device=x.device)
    assert out.is_cuda and out.is_contiguous() and out.numel() == n and out.dtype == torch.uint8
    f = _format8(fmt)
    _check(lib().fbsr_round_format8(x.data_ptr(), src, out.data_ptr(), n, ctypes.byref(f), variant, nbits, seed, offset,
                                    _stream_handle(stream)), "fbsr_round_format8")
    return out


def format16_check(fmt):
    """True when the descriptor is acceptable to fbsr_round_format16 (K <= 16, P >= K - 8).  Host-only."""
    return lib().fbsr_format16_check(ctypes.byref(_format8(fmt))) == OK


def fbsr_round_format16(x, src, fmt, variant, nbits, seed, offset=0, out=None, stream=None):
    """fbsr_round_format8 for formats of up to 16 bits: one code per uint16."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.element_size() == (4 if src == FROM_FP32 else 2)
    if src == FROM_FP32:
        assert x.dtype == torch.float32
    n = x.numel()
    if out is None:
        out = torch.empty(n, dtype=torch.uint16, device=x.device)
    assert out.is_cuda and out.is_contiguous() and out.numel() == n and out.element_size() == 2
    f = _format8(fmt)
    _check(lib().fbsr_round_format16(x.data_ptr(), src, out.data_ptr(), n, ctypes.byref(f), variant, nbits, seed, offset,
                                     _stream_handle(stream)), "fbsr_round_format16")
    return out


def fbsr_probe_stream41(x, out, stream=None):
    """Measurement aid: out[j] = top byte of x[j]'s pattern, in the rounding kernels' launch shape."""
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and out.is_cuda and out.dtype == torch.uint8
    assert out.numel() == x.numel()
    _check(lib().fbsr_probe_stream41(x.data_ptr(), out.data_ptr(), x.numel(), _stream_handle(stream)), "fbsr_probe_stream41")
    return out


def fbsr_probe_stream75(w8, g16, m16, v16, stream=None):
    """Measurement aid: the fused training step's loads and stores with no arithmetic (buffers updated in place)."""
    n = w8.numel()
    assert all(t.is_cuda and t.is_contiguous() for t in (w8, g16, m16, v16)) and w8.element_size() == 1
    assert all(t.numel() == n and t.element_size() == 2 for t in (g16, m16, v16))
    _check(lib().fbsr_probe_stream75(w8.data_ptr(), g16.data_ptr(), m16.data_ptr(), v16.data_ptr(), n, _stream_handle(stream)),
           "fbsr_probe_stream75")


def fbsr_check_qat_division(num, den, counts, stream=None):
    """Device self-check: counts[0] += pairs where the fused step's short division differs from num / den."""
    import torch
    assert num.is_cuda and den.is_cuda and num.dtype == torch.float32 and den.dtype == torch.float32 and num.numel() == den.numel()
    assert num.is_contiguous() and den.is_contiguous() and counts.is_cuda and counts.dtype == torch.int64 and counts.numel() == 2
    _check(lib().fbsr_check_qat_division(num.data_ptr(), den.data_ptr(), num.numel(), counts.data_ptr(), _stream_handle(stream)),
           "fbsr_check_qat_division")


def fbsr_check_qat_root(bias_corr2, counts, stream=None):
    """Device self-check: counts[1] += second-moment codes whose tabulated root differs from sqrt(v / bias_corr2)."""
    import torch
    assert counts.is_cuda and counts.dtype == torch.int64 and counts.numel() == 2
    _check(lib().fbsr_check_qat_root(float(bias_corr2), counts.data_ptr(), _stream_handle(stream)), "fbsr_check_qat_root")


SCALE_BLOCK = 32


def fbsr_round_block_scaled(x, fmt, variant, nbits, seed, offset=0, out=None, scales=None, stream=None):
    """Blocks of 32 share a power-of-two scale.  x: float32 CUDA tensor.  Returns (codes uint8[n],
    scales uint8[ceil(n / 32)])."""
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    n = x.numel()
    nb = (n + SCALE_BLOCK - 1) // SCALE_BLOCK
    if out is None:
        out = torch.empty(n, dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty(nb, dtype=torch.uint8, device=x.device)
    assert out.is_cuda and out.is_contiguous() and out.numel() == n and out.dtype == torch.uint8
    assert scales.is_cuda and scales.is_contiguous() and scales.numel() == nb and scales.dtype == torch.uint8
    _check(lib().fbsr_round_block_scaled(x.data_ptr(), out.data_ptr(), scales.data_ptr(), n, fmt, variant, nbits,
                                         seed, offset, _stream_handle(stream)), "fbsr_round_block_scaled")
    return out, scales


class AdamW(ctypes.Structure):
    """Mirror of the C struct fbsr_adamw."""
    _fields_ = [(k, ctypes.c_float) for k in ("lr", "beta1", "beta2", "eps", "weight_decay", "bias_corr1", "bias_corr2")]


def fbsr_qat_adamw_step(w8, g16, m16, v16, fmt, params, variant, nbits, seed, step, offset=0, stream=None):
    """One fused step of Alg. 1, in place on w8 (uint8 fp8 codes), m16, v16 (bf16 codes); g16 is read.
    params = (lr, beta1, beta2, eps, weight_decay, 1 - beta1^t, 1 - beta2^t)."""
    import torch
    for t in (w8, g16, m16, v16):
        assert t.is_cuda and t.is_contiguous()
    assert w8.dtype == torch.uint8 and g16.element_size() == m16.element_size() == v16.element_size() == 2
    n = w8.numel()
    assert g16.numel() == m16.numel() == v16.numel() == n
    p = AdamW(*[float(x) for x in params])
    _check(lib().fbsr_qat_adamw_step(w8.data_ptr(), g16.data_ptr(), m16.data_ptr(), v16.data_ptr(), n, fmt,
                                     ctypes.byref(p), variant, nbits, seed, step, offset, _stream_handle(stream)),
           "fbsr_qat_adamw_step")
    return w8, m16, v16


def fbsr_qat_adamw_step_format8(w8, g16, m16, v16, fmt, params, variant, nbits, seed, step, offset=0, stream=None):
    """fbsr_qat_adamw_step with the 8-bit weights in a generic format (a Format8 or an 8-tuple)."""
    import torch
    for t in (w8, g16, m16, v16):
        assert t.is_cuda and t.is_contiguous()
    assert w8.dtype == torch.uint8 and g16.element_size() == m16.element_size() == v16.element_size() == 2
    n = w8.numel()
    assert g16.numel() == m16.numel() == v16.numel() == n
    p = AdamW(*[float(x) for x in params])
    f = _format8(fmt)
    _check(lib().fbsr_qat_adamw_step_format8(w8.data_ptr(), g16.data_ptr(), m16.data_ptr(), v16.data_ptr(), n, ctypes.byref(f),
                                             ctypes.byref(p), variant, nbits, seed, step, offset, _stream_handle(stream)),
           "fbsr_qat_adamw_step_format8")
    return w8, m16, v16


def fbsr_sgd_update(w, g, lr, variant, nbits, seed, step, offset=0, stream=None):
    """In place: w <- FBSR_bf16(fma(-lr, g, float(w))).  w: uint16 / int16 / bfloat16 CUDA tensor
    holding bf16 codes; g: float32 CUDA tensor of the same length."""
    import torch
    assert w.is_cuda and g.is_cuda and w.is_contiguous() and g.is_contiguous()
    assert w.element_size() == 2 and g.dtype == torch.float32 and w.numel() == g.numel()
    _check(lib().fbsr_sgd_update(w.data_ptr(), g.data_ptr(), w.numel(), float(lr), variant, nbits,
                                 seed, step, offset, _stream_handle(stream)), "fbsr_sgd_update")
    return w


def bias_stats_workspace_bytes(n, nbins):
    return int(lib().fbsr_bias_stats_workspace_bytes(n, nbins))


def fbsr_bias_stats(x, fmt, variant, nbits, seed, offset, group, first_bin, nbins, stats=None,
                    out=None, workspace=None, stream=None):
    """Accumulates {count, sum y, sum e, sum e^2} per bin into stats[nbins, 4] (float64 CUDA
    tensor, created zeroed if None).  Returns (stats, out)."""
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    n = x.numel()
    if stats is None:
        stats = torch.zeros((nbins, 4), dtype=torch.float64, device=x.device)
    assert stats.is_cuda and stats.dtype == torch.float64 and stats.is_contiguous()
    assert stats.numel() == 4 * nbins
    need = bias_stats_workspace_bytes(n, nbins)
    if workspace is None:
        workspace = torch.empty((need + 7) // 8, dtype=torch.float64, device=x.device)
    wbytes = workspace.numel() * workspace.element_size()
    if out is not None:
        assert out.is_cuda and out.is_contiguous() and out.numel() == n and out.dtype == code_dtype(fmt)
    _check(lib().fbsr_bias_stats(x.data_ptr(), out.data_ptr() if out is not None else None, n, fmt,
                                 variant, nbits, seed, offset, group, first_bin, nbins,
                                 stats.data_ptr(), workspace.data_ptr(), wbytes,
                                 _stream_handle(stream)), "fbsr_bias_stats")
    return stats, out


def fbsr_bias_stats_format8(x, fmt, variant, nbits, seed, offset, group, first_bin, nbins, stats=None, out=None,
                            workspace=None, stream=None):
    """fbsr_bias_stats for a format given by its descriptor (a tuple as for fbsr_round_format8 or an fbsr_format8);
    out: uint8 codes or None.  Returns (stats, out)."""
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    n = x.numel()
    if stats is None:
        stats = torch.zeros((nbins, 4), dtype=torch.float64, device=x.device)
    assert stats.is_cuda and stats.dtype == torch.float64 and stats.is_contiguous() and stats.numel() == 4 * nbins
    if workspace is None:
        workspace = torch.empty((bias_stats_workspace_bytes(n, nbins) + 7) // 8, dtype=torch.float64, device=x.device)
    if out is not None:
        assert out.is_cuda and out.is_contiguous() and out.numel() == n and out.dtype == torch.uint8
    f = _format8(fmt)
    _check(lib().fbsr_bias_stats_format8(x.data_ptr(), out.data_ptr() if out is not None else None, n, ctypes.byref(f), variant,
                                         nbits, seed, offset, group, first_bin, nbins, stats.data_ptr(), workspace.data_ptr(),
                                         workspace.numel() * workspace.element_size(), _stream_handle(stream)),
           "fbsr_bias_stats_format8")
    return stats, out


BIAS_STATS_STATIC_MAX_ELEMS = 1 << 28


def fbsr_bias_stats_static(x, fmt, variant, nbits, seed, offset, group, first_bin, nbins, stats, out=None, stream=None):
    """fbsr_bias_stats without a workspace argument (the library's built-in one is used) and without any
    allocation: `stats` (float64 [nbins, 4], accumulated into) and `out` (or None) are the caller's."""
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    assert stats.is_cuda and stats.dtype == torch.float64 and stats.is_contiguous() and stats.numel() == 4 * nbins
    n = x.numel()
    if out is not None:
        assert out.is_cuda and out.is_contiguous() and out.numel() == n and out.dtype == code_dtype(fmt)
    _check(lib().fbsr_bias_stats_static(x.data_ptr(), out.data_ptr() if out is not None else None, n, fmt, variant, nbits,
                                        seed, offset, group, first_bin, nbins, stats.data_ptr(), _stream_handle(stream)),
           "fbsr_bias_stats_static")
    return stats, out
