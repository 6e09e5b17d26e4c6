"""GPU parity of the stacked-adapter backward pass (a frozen pair and a trainable pair on one projection, App. D)."""
import numpy as np
import pytest

import oracle
from paper_2306_08162_amd import binding as ql
from parity import TOL, announce, make_oracle, rel_fro, small_inputs

pytestmark = pytest.mark.gpu

CASES = [
    # (M, K, N, bits, G, rank, frozen, dtype): weight-streaming backward, tiled backward at small and large M
    (6, 256, 72, 4, 64, 16, 8, "f16"),
    (16, 1376, 520, 2, 32, 40, 32, "bf16"),
    (40, 384, 264, 3, 128, 40, 32, "f16"),
    (300, 640, 392, 4, 128, 40, 32, "f16"),
    (257, 1024, 520, 8, 128, 64, 32, "bf16"),
    (131, 512, 136, 4, 64, 24, 16, "f16"),
    (9, 512, 200, 8, 128, 64, 56, "f16"),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "M{}_K{}_N{}_b{}_G{}_r{}_f{}_{}".format(*c))
@pytest.mark.parametrize("beta", [0.0, 1.0])
def test_stacked_backward(case, beta):
    import torch
    from paper_2306_08162_amd.device import DeviceLayer
    M, K, N, bits, G, r, f, dtype = case
    inp = small_inputs(5 * M + K + r + f, M, K, N, bits, G, r, dtype)
    c = inp.cfg
    announce(f"stacked {c.name}: frozen={f} beta={beta}")
    layer = DeviceLayer(inp)
    layer.forward()
    if beta:
        layer.backward_stacked(f)                 # allocate, then preset what is accumulated into
        layer.dA_train.fill_(0.5)
        layer.dB_train.fill_(-1.5)
    dA_t, dB_t = layer.backward_stacked(f, beta=beta, use_saved_t=(M % 2 == 0))
    torch.cuda.synchronize()
    lo = make_oracle(inp)
    dx_ref = lo.backward_dx(inp.dy)
    x, dy = oracle.widen(inp.x, dtype), oracle.widen(inp.dy, dtype)
    A, B = oracle.widen(inp.A, dtype), oracle.widen(inp.B, dtype)
    dA_ref, dB_ref = oracle.backward_adapters_stacked(dy, x, A, B, c.alpha, f)
    errs = {"dx": rel_fro(oracle.widen(layer.host_dx(), dtype), dx_ref),
            "dA": rel_fro(dA_t.cpu().numpy(), beta * 0.5 + dA_ref),
            "dB": rel_fro(dB_t.cpu().numpy(), beta * -1.5 + dB_ref)}
    announce(" ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    for k, v in errs.items():
        assert np.isfinite(v) and v <= TOL, f"{c.name}: rel. Frobenius error of {k} = {v:.3e} > {TOL}"


def test_stacked_with_nothing_frozen_is_the_plain_backward():
    import torch
    from paper_2306_08162_amd.device import DeviceLayer
    inp = small_inputs(321, 70, 256, 136, 4, 64, 16, "f16")
    layer = DeviceLayer(inp)
    layer.forward()
    layer.backward()
    dA_t, dB_t = layer.backward_stacked(0)
    torch.cuda.synchronize()
    assert np.array_equal(dA_t.cpu().numpy(), layer.host_dA()) and np.array_equal(dB_t.cpu().numpy(), layer.host_dB())
