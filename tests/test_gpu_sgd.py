"""GPU parity: fbsr_sgd_update (the fused weight update of Alg. 1) against the CPU oracle."""
import numpy as np
import pytest
import torch

from gpu_util import dev, first_mismatch, host

pytestmark = pytest.mark.gpu
RNE, SRFF, SRF, SRC = 0, 1, 2, 3


def _weights_and_grads(n, seed):
    from paper_2504_20634_amd import workloads
    w = workloads.sgd_weights(n, seed=seed)
    g = workloads.sgd_grads(n, 0, seed=seed, std=1.0)
    # a few extreme cases: huge weights that overflow to inf, NaN/inf weights, subnormal results
    w[::1001] = 0x7F7F
    w[1::1001] = 0x0001
    w[2::1001] = 0x7FC0
    w[3::1001] = 0xFF80
    g[::1001] = -3.0e38
    return w, g


@pytest.mark.parametrize("n", [0, 1, 7, 1024, 8192 + 3, 3 * 8192 + 1024 + 50])
def test_single_step_matches_oracle(fbsr, oracle, n):
    w, g = _weights_and_grads(max(n, 4), seed=5)
    w, g = w[:n], g[:n]
    for variant, nbits in ((RNE, 0), (SRFF, 1), (SRFF, 2), (SRF, 4), (SRC, 8), (SRC, 3), (SRF, 16)):
        for lr, offset, step in ((1e-3, 0, 0), (0.37, 48, 7), (2.5, 3, (1 << 35) + 1)):
            print("case n=%d variant=%d nbits=%d lr=%g offset=%d step=%d" % (n, variant, nbits, lr, offset, step), flush=True)
            wd = dev(w) if n else torch.empty(0, dtype=torch.int16, device="cuda")
            gd = dev(g) if n else torch.empty(0, dtype=torch.float32, device="cuda")
            fbsr.fbsr_sgd_update(wd, gd, lr, variant, nbits, seed=21, step=step, offset=offset)
            want = oracle.sgd_update(w, g, lr, variant, nbits, seed=21, step=step, offset=offset)
            assert first_mismatch(host(wd), want) is None, (n, variant, nbits, lr, offset, step)


def test_twenty_steps_at_2_20_weights(fbsr, oracle):
    """The benchmark workload at reduced scale: 2^20 weights, 20 steps, fresh gradients per step."""
    from paper_2504_20634_amd import workloads
    n, lr = 1 << 20, 1e-3
    for variant, nbits in ((SRFF, 2), (SRF, 4), (SRC, 8), (RNE, 0)):
        w = workloads.sgd_weights(n, seed=3)
        wd = dev(w)
        for t in range(20):
            g = workloads.sgd_grads(n, t, seed=3)
            fbsr.fbsr_sgd_update(wd, dev(g), lr, variant, nbits, seed=4, step=t)
            w = oracle.sgd_update(w, g, lr, variant, nbits, seed=4, step=t)
        print("case variant=%d nbits=%d" % (variant, nbits), flush=True)
        assert first_mismatch(host(wd), w) is None, (variant, nbits)


def test_resume_is_bit_identical(fbsr):
    """State is (weights, seed, step): 6 steps in a row equal 3 + 3 from a copy of the weights."""
    from paper_2504_20634_amd import workloads
    n = 8192 * 4 + 17
    w = dev(workloads.sgd_weights(n, seed=9))
    gs = [dev(workloads.sgd_grads(n, t, seed=9, std=0.05)) for t in range(6)]
    a = w.clone()
    for t in range(6):
        fbsr.fbsr_sgd_update(a, gs[t], 0.1, SRF, 3, seed=2, step=t)
    b = w.clone()
    for t in range(3):
        fbsr.fbsr_sgd_update(b, gs[t], 0.1, SRF, 3, seed=2, step=t)
    c = b.clone()
    for t in range(3, 6):
        fbsr.fbsr_sgd_update(c, gs[t], 0.1, SRF, 3, seed=2, step=t)
    assert torch.equal(a, c)
