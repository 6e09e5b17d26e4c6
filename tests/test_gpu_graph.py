"""The library's calls captured in a HIP graph (how bench.py times the small-token passes): every replay must give the
bits the eager calls give, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from parity import announce, small_inputs

pytestmark = pytest.mark.gpu


def _snapshot(layer, sib=None):
    out = [layer.host_y().copy(), layer.host_dx().copy(), layer.host_dA().copy(), layer.host_dB().copy()]
    if sib is not None:
        out.append(sib.host_dx().copy())
    return out


@pytest.mark.parametrize("M,K", [(16, 512), (28, 1024), (300, 512), (300, 2048)],
                         ids=["weight_streaming", "two_token_blocks", "tiled", "tiled_split"])
def test_graph_replays_match_eager(M, K):
    import torch
    from paper_2306_08162_amd.device import DeviceLayer, DeviceSiblings
    announce(f"graph replay M={M} K={K}")   # K = 2048: the forward GEMM's contraction is split over 4 workgroups per tile
    inp = small_inputs(123 + M, M, K, 264, 4, 128, 8, "f16")
    layer = DeviceLayer(inp)
    other = DeviceLayer(small_inputs(124 + M, M, K, 136, 4, 128, 8, "f16"))
    other.x = layer.x
    sib = DeviceSiblings([layer, other]) if M <= 16 else None
    if M == 28:     # ... and the zero-points handed over bit-packed (packed on the device, before anything is captured)
        layer.use_packed_zeros()

    def run():
        layer.forward()
        layer.backward()
        if sib is not None:
            sib.forward()
            sib.backward()

    run()
    torch.cuda.synchronize()
    eager = _snapshot(layer, sib)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(4):
        # scribble over the outputs, do some eager work of the same kind, then replay
        for t in (layer.y, layer.dx, layer.dA, layer.dB):
            t.fill_(7)
        other.forward()
        other.backward()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, _snapshot(layer, sib)):
            assert np.array_equal(a, b), f"replay {rep} differs from the eager result"
