"""GPU: fbsr_bias_stats_static (the entry point for callers that cannot allocate: its workspace is an array
inside the library) against fbsr_bias_stats, through the C ABI: statistics bit for bit, codes byte for byte, on
two calls in a row of which the second is smaller (the array keeps the first call's records)."""
import ctypes

import numpy as np
import pytest
import torch

from gpu_util import dev, host

pytestmark = pytest.mark.gpu
BF16, E4M3, E5M2 = 0, 1, 2
SRFF, SRF, SRC = 1, 2, 3


def _both(fbsr, L, x, fmt, variant, nbits, seed, offset, group):
    n = x.numel()
    first_bin = offset // group
    nbins = (offset + n - 1) // group - first_bin + 1
    cd = fbsr.binding.code_dtype(fmt)
    ref_stats = torch.zeros((nbins, 4), dtype=torch.float64, device="cuda")
    ref_out = torch.empty(n, dtype=cd, device="cuda")
    ws = torch.empty(L.fbsr_bias_stats_workspace_bytes(n, nbins) // 8 + 1, dtype=torch.float64, device="cuda")
    stats = torch.full((nbins, 4), 0.0, dtype=torch.float64, device="cuda")
    out = torch.empty(n, dtype=cd, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.fbsr_bias_stats(x.data_ptr(), ref_out.data_ptr(), n, fmt, variant, nbits, seed, offset, group, first_bin, nbins,
                           ref_stats.data_ptr(), ws.data_ptr(), ws.numel() * 8, stream)
    assert rc == 0
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = L.fbsr_bias_stats_static(x.data_ptr(), out.data_ptr(), n, fmt, variant, nbits, seed, offset, group, first_bin, nbins,
                                  stats.data_ptr(), stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(stats, ref_stats), "statistics differ from fbsr_bias_stats"
    assert np.array_equal(host(out), host(ref_out)), "codes differ from fbsr_bias_stats"
    return stats


def test_static_workspace_matches_the_workspace_entry_point(fbsr, oracle):
    from paper_2504_20634_amd import workloads
    L = fbsr.binding.lib()
    big = dev(workloads.scaled_normal(40 * 16384 + 777, seed=31))
    small = dev(workloads.scaled_normal(3 * 16384 + 5, seed=32))
    for fmt, variant, nbits, group in ((E4M3, SRC, 3, 5000), (BF16, SRFF, 2, 1 << 16), (E5M2, SRF, 20, 2048)):
        print("case fmt=%d variant=%d nbits=%d group=%d: large call" % (fmt, variant, nbits, group), flush=True)
        _both(fbsr, L, big, fmt, variant, nbits, 11, 16, group)
        print("   then a smaller one", flush=True)
        s = _both(fbsr, L, small, fmt, variant, nbits, 12, 0, group)
        # and against the oracle, for the smaller call
        want, _ = oracle.bias_stats(small.cpu().numpy(), fmt, variant, nbits, 12, 0, group, 0, s.shape[0])
        from gpu_util import assert_stats_close
        assert_stats_close(s.cpu().numpy(), want)


def test_static_workspace_limits(fbsr):
    """Sizes beyond the built-in workspace are refused on the host, before anything is launched."""
    L = fbsr.binding.lib()
    p = ctypes.c_void_p
    good = 0x7F0000001000
    too_many = fbsr.binding.BIAS_STATS_STATIC_MAX_ELEMS + 1
    assert L.fbsr_bias_stats_static(p(good), None, too_many, 1, 1, 2, 0, 0, 1 << 20, 0, 1024, p(good), None) == fbsr.binding.ERANGE
    assert L.fbsr_bias_stats_static(None, None, 0, 1, 1, 2, 0, 0, 1, 0, 1, None, None) == fbsr.binding.OK
    assert L.fbsr_bias_stats_static(p(good), None, 8, 1, 1, 2, 0, 0, 4, 0, 2, None, None) == fbsr.binding.EINVAL
