"""The layer's C calls enqueue kernels and nothing else (no allocation, no synchronization, no
memset), so a caller may record them into a HIP graph.  Replays are checked against the eager
result several times, with eager work and synchronizations in between."""
import numpy as np
import pytest
import torch

import dvdq_inputs as di
import paper_2505_18663_amd as dvdq

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("container,with_zero", [("int8", False), ("packed4", True), ("fp6", False), ("fp6", True)])
def test_qlinear_and_controller_replay_from_a_graph(container, with_zero):
    wl = di.WORKLOADS[0]
    M, K, N, B, bits = wl.M, wl.K, wl.N, wl.had_block, wl.act_bits
    rng = np.random.default_rng(3)
    wp, ws, _ = di.make_weights(wl)
    if container == "fp6":
        w_native, lay, fmt = dvdq.w4_prepack_fp6(torch.from_numpy(wp).to(DEV)), dvdq.W_NATIVE_FP6, dvdq.CODES_FP6
    else:
        w_native, lay = dvdq.w4_prepack(torch.from_numpy(wp).to(DEV)), dvdq.W_NATIVE
        fmt = dvdq.CODES_PACKED4 if container == "packed4" else dvdq.CODES_INT8
    ws_dev = torch.from_numpy(ws).to(DEV)
    wz = torch.from_numpy(rng.integers(-3, 4, N).astype(np.int8)).to(DEV) if with_zero else None
    xs = [torch.from_numpy(di.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)).view(np.int16))
          .view(torch.bfloat16).to(DEV) for _ in range(3)]
    x_in = xs[0].clone()
    y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    wsp = torch.empty((dvdq.qlinear_workspace_bytes(M, K, fmt),), dtype=torch.uint8, device=DEV)
    f_prev = torch.randn((4096,), device=DEV).to(torch.bfloat16)
    ctl = dvdq.GbsController(delta=0.5)

    def layer():
        dvdq.qlinear(x_in, w_native, ws_dev, B, bits, lay, y=y, workspace=wsp, codes_format=fmt, w_zero=wz)
        ctl.step(y.view(-1)[:4096], f_prev)

    layer()                       # first launches outside the capture (one-time kernel attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            layer()
    torch.cuda.synchronize()
    for rep, x_new in enumerate(xs + xs[:1]):
        # eager reference on separate buffers
        y_ref, _ = dvdq.qlinear(x_new, w_native, ws_dev, B, bits, lay, codes_format=fmt, w_zero=wz)
        ctl_ref = dvdq.GbsController(delta=0.5)
        ctl_ref.step(y_ref.view(-1)[:4096], f_prev)
        torch.cuda.synchronize()
        x_in.copy_(x_new)
        ctl.reset()
        y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), f"replay {rep}"
        assert ctl.read() == ctl_ref.read(), f"replay {rep}: controller state"
