"""bench.py's MFMA issue-rate probe (bench_probe.py): argument checks on the CPU, one counted run
on the GPU."""
import ctypes as C

import pytest

import bench_probe

FAKE = 0x10000


def _rc(dtype, operands, blocks, iters, sink):
    return bench_probe.lib().bench_mfma_probe(dtype, operands, blocks, iters, sink, None, None)


def test_probe_validation():
    assert bench_probe.operand_bytes() == 1 << 20
    assert _rc(1, None, 4, 1, FAKE) == 1
    assert _rc(1, FAKE, 4, 1, None) == 1
    assert _rc(1, FAKE + 2, 4, 1, FAKE) == 1
    assert _rc(1, FAKE, 0, 1, FAKE) == 1
    assert _rc(1, FAKE, 4, 0, FAKE) == 1
    assert _rc(7, FAKE, 4, 1, FAKE) == 1


@pytest.mark.gpu
def test_probe_counts_and_runs():
    """Constant operands 1.0 make every accumulator element equal to the number of multiply-adds
    along k, so the sink holds 16 x (iters x 64 / 4 chains) x 16 x 4."""
    import torch
    n = bench_probe.operand_bytes() // 2
    ops = torch.full((n,), 1.0, dtype=torch.bfloat16, device="cuda:0")
    sink = torch.zeros(8 * 256, dtype=torch.float32, device="cuda:0")
    iters = 3
    flops = bench_probe.mfma_probe(1, ops, 8, iters, sink, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert flops == 8 * 4 * iters * 64 * 2 * 32 * 32 * 16
    expect = 4 * 16 * (iters * 64 // 4) * 16
    assert torch.all(sink == float(expect)), (sink[:4], expect)
