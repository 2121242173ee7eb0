"""The library's calls captured into a HIP graph: every replay must reproduce the eager result bit
for bit.  The replays are separated by eager work and synchronisations of the program's own, and the
inputs change between replays (the graph reads the same buffers, refilled in place)."""
import numpy as np
import pytest
import torch

from paper_2502_08141_amd import lowra, synth
from tests.gpu_util import DeviceLayer

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    L = synth.make_custom(520, 1024, 64, 16, seed=61)
    D = DeviceLayer(L)
    lay = D.layout
    ws = torch.empty(max(lay.workspace_bytes(lowra.OP_LINEAR_FWD, 64, L.r), lay.workspace_bytes(lowra.OP_LINEAR_BWD_INPUT, 64, L.r),
                         lay.workspace_bytes(lowra.OP_ADAPTER_GRADS, 64, L.r)), dtype=torch.uint8, device="cuda")
    ws4 = torch.empty_like(ws)
    packed = torch.empty(lay.packed_bytes, dtype=torch.uint8, device="cuda")
    absmax = torch.empty((L.N, L.K // 64), dtype=torch.float32, device="cuda")
    What = torch.empty((L.N, L.K), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((64, L.N), dtype=torch.bfloat16, device="cuda")
    y4 = torch.empty((4, L.N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((64, L.K), dtype=torch.bfloat16, device="cuda")
    W, x, dY = D.W.clone(), D.x.clone(), D.dY.clone()

    pb = [torch.empty_like(packed) for _ in range(2)]
    ab = [torch.empty_like(absmax) for _ in range(2)]

    def calls(side=None):
        lowra.lowra_quantize(lay, W, D.thr, packed, absmax)
        lowra.lowra_quantize_batch([lay, lay], [W, W], [D.thr, D.thr], pb, ab)     # descriptors are kernel arguments: capturable
        lowra.lowra_dequantize(lay, packed, absmax, D.mp, out=What)
        if side is not None:                                    # the small-token call on a parallel branch
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                lowra.lowra_linear_fwd(lay, packed, absmax, D.mp, x[:4], D.A, D.B, L.s, y=y4, workspace=ws4)
        else:
            lowra.lowra_linear_fwd(lay, packed, absmax, D.mp, x[:4], D.A, D.B, L.s, y=y4, workspace=ws4)
        lowra.lowra_linear_fwd(lay, packed, absmax, D.mp, x, D.A, D.B, L.s, y=y, workspace=ws)
        lowra.lowra_linear_bwd_input(lay, packed, absmax, D.mp, dY, D.A, D.B, L.s, dX=dX, workspace=ws)
        if side is not None:
            torch.cuda.current_stream().wait_stream(side)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (packed, absmax, What, y, y4, dX, *pb, *ab)]

    calls()                                                     # eager first: one-time set-up happens outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        calls(side)
    gen = torch.Generator(device="cuda").manual_seed(7)
    for rep in range(4):
        print(f"[graph replay {rep}]", flush=True)
        if rep:                                                 # new inputs in the same buffers
            W.normal_(0.0, 0.02, generator=gen)
            x.copy_(torch.randn(x.shape, generator=gen, device="cuda").bfloat16())
            dY.copy_(torch.randn(dY.shape, generator=gen, device="cuda").bfloat16())
        calls()
        want = snapshot()
        assert torch.equal(pb[1], packed) and torch.equal(ab[0], absmax)
        for t in (packed, absmax, What, y, y4, dX, *pb, *ab):
            t.zero_()
        scratch = torch.randn(1 << 20, device="cuda").sum()     # eager work of the program's own between replays
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
        assert np.isfinite(float(scratch))


@pytest.mark.parametrize("scale_dtype", [torch.float32, torch.bfloat16])
def test_small_token_calls_in_a_graph(scale_dtype):
    """The streaming small-token kernels as single calls (forward under LOWRA_PATH_GEMV, input gradient under
    LOWRA_PATH_AUTO): their set-up kernels write the descriptors on the device from kernel arguments, so the calls
    copy nothing from the host and a captured sequence replays bit for bit on new inputs."""
    L = synth.make_custom(520, 4096, 5, 16, fractions=(0.4, 0.3, 0.3), seed=62)
    D = DeviceLayer(L)
    lay = D.layout.set_scale_dtype(scale_dtype)
    packed, absmax = lowra.lowra_quantize(lay, D.W, D.thr)
    wsf = torch.empty(lay.workspace_bytes(lowra.OP_LINEAR_FWD, L.M, L.r), dtype=torch.uint8, device="cuda")
    wsb = torch.empty(lay.workspace_bytes(lowra.OP_LINEAR_BWD_INPUT, L.M, L.r), dtype=torch.uint8, device="cuda")
    y = torch.empty((L.M, L.N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((L.M, L.K), dtype=torch.bfloat16, device="cuda")
    x, dY = D.x.clone(), D.dY.clone()

    def calls():
        lowra.lowra_set_linear_path(lowra.PATH_GEMV)
        try:
            lowra.lowra_linear_fwd(lay, packed, absmax, D.mp, x, D.A, D.B, L.s, y=y, workspace=wsf)
        finally:
            lowra.lowra_set_linear_path(lowra.PATH_AUTO)
        lowra.lowra_linear_bwd_input(lay, packed, absmax, D.mp, dY, D.A, D.B, L.s, dX=dX, workspace=wsb)

    calls()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        calls()
    gen = torch.Generator(device="cuda").manual_seed(8)
    for rep in range(3):
        x.copy_(torch.randn(x.shape, generator=gen, device="cuda").bfloat16())
        dY.copy_(torch.randn(dY.shape, generator=gen, device="cuda").bfloat16())
        calls()
        torch.cuda.synchronize()
        want = [y.clone(), dX.clone()]
        y.zero_(); dX.zero_(); wsf.zero_(); wsb.zero_()            # the workspace holds nothing a replay depends on
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), want[0].view(torch.int16))
        assert torch.equal(dX.view(torch.int16), want[1].view(torch.int16))
