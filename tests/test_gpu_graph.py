"""The library allocates nothing and never synchronises, so its calls can be recorded into a HIP graph:
a captured sequence of every kind of entry point is replayed several times, with eager work and
synchronisations in between, and every replay is compared with the eager result."""
import numpy as np
import pytest
import torch

from gpu_util import dev

pytestmark = pytest.mark.gpu
E4M3, P4, BF16 = 1, 3, 0
SRFF, SRF, SRC = 1, 2, 3


def test_entry_points_replay_from_a_graph(fbsr):
    from paper_2504_20634_amd import workloads
    n = 5 * 2048 + 321                      # tiles plus a ragged tail: several kernels per call
    group, nbins = 4096, (n + 4095) // 4096
    x = torch.empty(n, dtype=torch.float32, device="cuda")
    x16 = torch.empty(n, dtype=torch.int16, device="cuda")
    out8 = torch.empty(n, dtype=torch.uint8, device="cuda")
    out8b = torch.empty(n, dtype=torch.uint8, device="cuda")
    out8c = torch.empty(n, dtype=torch.uint8, device="cuda")
    outbs = torch.empty(n, dtype=torch.uint8, device="cuda")
    scales = torch.empty((n + 31) // 32, dtype=torch.uint8, device="cuda")
    w = torch.empty(n, dtype=torch.int16, device="cuda")
    g = torch.empty(n, dtype=torch.float32, device="cuda")
    w8 = torch.empty(n, dtype=torch.uint8, device="cuda")
    m16 = torch.zeros(n, dtype=torch.int16, device="cuda")
    v16 = torch.zeros(n, dtype=torch.int16, device="cuda")
    stats = torch.zeros((nbins, 4), dtype=torch.float64, device="cuda")
    stats8 = torch.zeros((nbins, 4), dtype=torch.float64, device="cuda")
    stats_static = torch.zeros((nbins, 4), dtype=torch.float64, device="cuda")
    out16 = torch.empty(n, dtype=torch.int16, device="cuda")
    w8b = torch.empty(n, dtype=torch.uint8, device="cuda")
    m16b = torch.zeros(n, dtype=torch.int16, device="cuda")
    v16b = torch.zeros(n, dtype=torch.int16, device="cuda")
    ws8 = torch.empty(fbsr.bias_stats_workspace_bytes(n, nbins) // 8 + 1, dtype=torch.float64, device="cuda")
    b16 = fbsr.format8_named("ieee_binary16")
    ws = torch.empty(fbsr.bias_stats_workspace_bytes(n, nbins) // 8 + 1, dtype=torch.float64, device="cuda")
    p4 = fbsr.format8_named("p3109_binary8p4")
    params = (1e-2, 0.9, 0.999, 1e-8, 0.01, 0.1, 0.001)

    def fill(seed):
        x.copy_(dev(workloads.scaled_normal(n, seed=seed)))
        x16.copy_(dev(workloads.sgd_weights(n, seed=seed + 1)))
        w.copy_(dev(workloads.sgd_weights(n, seed=seed + 2)))
        g.copy_(dev(workloads.sgd_grads(n, seed, seed=3)))
        w8.copy_(dev((workloads.sgd_weights(n, seed=seed + 3) & 0x7777).view(np.uint8)[:n].copy()))
        w8b.copy_(w8)
        w8b[w8b == 0x80] = 0                    # binary8p4's NaN code
        for t in (m16, v16, m16b, v16b, stats, stats8, stats_static):
            t.zero_()

    def sequence():
        fbsr.fbsr_round(x, E4M3, SRC, 3, seed=1, offset=7, out=out8)
        fbsr.fbsr_round_from16(x16, 0, P4, SRF, 3, seed=2, out=out8b)
        fbsr.fbsr_round_format8(x, 2, p4, 4, 3, seed=3, out=out8c)
        fbsr.fbsr_round_block_scaled(x, E4M3, SRFF, 2, seed=4, out=outbs, scales=scales)
        fbsr.fbsr_sgd_update(w, g, 1e-3, SRF, 4, seed=5, step=9)
        fbsr.fbsr_qat_adamw_step(w8, x16, m16, v16, P4, params, SRC, 3, seed=6, step=2)
        fbsr.fbsr_bias_stats(x, BF16, SRFF, 2, 7, 0, group, 0, nbins, stats=stats, workspace=ws)
        fbsr.fbsr_round_format16(x, 2, b16, SRC, 3, seed=8, out=out16)
        fbsr.fbsr_qat_adamw_step_format8(w8b, x16, m16b, v16b, p4, params, SRC, 3, seed=9, step=2)
        fbsr.fbsr_bias_stats_format8(x, p4, SRF, 3, 10, 0, group, 0, nbins, stats=stats8, workspace=ws8)
        fbsr.fbsr_bias_stats_static(x, E4M3, SRC, 3, 11, 0, group, 0, nbins, stats_static)

    def snapshot():
        return [t.clone() for t in (out8, out8b, out8c, outbs, scales, w, w8, m16, v16, stats, out16, w8b, m16b, v16b, stats8,
                                    stats_static)]

    fill(10)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sequence()                              # warm-up on the capture stream's side, as torch asks
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    fill(10)
    with torch.cuda.graph(graph):
        sequence()
    for seed in (10, 20, 30):
        fill(seed)
        sequence()
        torch.cuda.synchronize()
        eager = snapshot()
        fill(seed)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replayed = snapshot()
        for a, b in zip(eager, replayed):
            assert torch.equal(a, b), seed
        # unrelated eager work between replays
        (x * 2.0).sum().item()


def test_table_kernel_replays_from_a_graph(fbsr):
    """A 16-bit source of 2^26 elements to a descriptor format goes through the kernel that tabulates the source
    magnitudes per workgroup (its launch asks the device for two attributes, cached after the first call): captured
    once, replayed twice on changed inputs."""
    n = (1 << 26) + 4096
    p4 = fbsr.format8_named("p3109_binary8p4")
    x16 = torch.empty(n, dtype=torch.int16, device="cuda")
    out = torch.empty(n, dtype=torch.uint8, device="cuda")

    def fill(seed):
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
        x16.copy_(torch.randint(-32768, 32767, (n,), dtype=torch.int16, device="cuda", generator=gen))

    def sequence():
        fbsr.fbsr_round_format8(x16, 0, p4, SRC, 3, seed=3, out=out)

    fill(1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sequence()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence()
    for seed in (2, 3):
        fill(seed)
        sequence()
        torch.cuda.synchronize()
        eager = out.clone()
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), seed
