"""The benchmark's calibration kernels (not part of the layer): the plain copy copies, and the register-only
MFMA loops run on both kinds of operand data, report the operation count their launch performs and leave
the sink untouched (it is only written if a sum takes one particular value)."""
import pytest
import torch

import paper_2505_18663_amd as dvdq

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("nbytes", [16, 4096 - 16, 16384, (1 << 20) + 4096, (1 << 20) + 16 * 1021, 40 << 20])
def test_copy_kernel_copies(nbytes):
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    buf = torch.randint(0, 256, (nbytes + 512,), device=DEV, dtype=torch.uint8, generator=g)
    out = torch.full((nbytes + 512,), 0xA5, device=DEV, dtype=torch.uint8)
    src, dst = buf[256:256 + nbytes], out[256:256 + nbytes]
    dvdq.bench_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert bool((out[:256] == 0xA5).all()) and bool((out[256 + nbytes:] == 0xA5).all())   # nothing written outside


@pytest.mark.parametrize("data", [0, 1])
def test_mfma_loops_report_their_operation_count(data):
    sink = torch.zeros((4,), dtype=torch.int32, device=DEV)
    iters = 50
    waves = 2 * 256 * 4   # two 4-wave workgroups per compute unit
    ops8 = dvdq.bench_mfma_i8(iters, sink, data=data)
    ops6 = dvdq.bench_mfma_fp6(iters, sink, data=data)
    torch.cuda.synchronize()
    assert ops8 == 2.0 * 32 * 32 * 32 * 16 * iters * waves
    assert ops6 == 2.0 * 32 * 32 * 64 * 8 * iters * waves
    assert int(sink.abs().sum()) == 0
