"""The library's measurement aids (the denominators of the rooflines) run and give sane figures:
they are timing loops with no result to compare, so the checks are on ranges and on the order
that must hold between their modes."""
import pytest
import torch

import paper_2511_18793_amd as nz
from _gpu_common import device

pytestmark = pytest.mark.gpu


def test_tile_step_modes_are_ordered():
    both, clk = nz.bench_tile_step(2, iters=4000)
    matrix, _ = nz.bench_tile_step(0, iters=4000)
    vector, _ = nz.bench_tile_step(1, iters=4000)
    assert 300.0 < clk < 3000.0                       # MHz
    # a SIMD at 2.4 GHz cannot issue four 16-cycle MFMAs in less than 26 ns
    assert 1e5 < both < 1.0 / 26e-9
    # the loop with both kinds of work is no faster than either alone, no slower than their sum
    assert both < 1.05 * min(matrix, vector)
    assert 1.0 / both < 1.1 * (1.0 / matrix + 1.0 / vector)


def test_matrix_rate_and_gather_run():
    x = torch.randn(1 << 16, device=device()).to(torch.bfloat16)
    tflops, clk = nz.bench_mfma_rate(x, iters=500)
    assert 100.0 < tflops < 2600.0 and 300.0 < clk < 3000.0
    buf = torch.zeros(1 << 24, dtype=torch.uint8, device=device())
    nz.bench_random_gather(buf, 1 << 20, 64, 3)
    torch.cuda.synchronize()
