"""GPU parity of the stacked-adapter backward pass (a frozen pair and a trainable pair on one projection, App. D)."""
import numpy as np
import pytest

import oracle
from paper_2306_08162_amd import binding as ql
from parity import Report, announce, layer_bounds, make_oracle, small_inputs

pytestmark = pytest.mark.gpu

CASES = [
    # (M, K, N, bits, G, rank, frozen, dtype): weight-streaming backward, tiled backward at small and large M
    (6, 256, 72, 4, 64, 16, 8, "f16"),
    (16, 1376, 520, 2, 32, 40, 32, "bf16"),
    (20, 512, 136, 2, 128, 40, 32, "bf16"),      # two token blocks in the staged backward kernel
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
    sc = c.alpha / r
    t_ref, u_ref = oracle.lora_down(x, A), oracle.lora_u(dy, B)
    bounds = layer_bounds(lo.Wd, A, B, sc, dy=dy, t=t_ref, u=u_ref, x_adapter=x)
    rep = Report(f"stacked {c.name} f={f} beta={beta}", dtype)
    rep.add("dx", oracle.widen(layer.host_dx(), dtype), dx_ref, lines="rows", bound=bounds["dx"])
    rep.add("dA", dA_t.cpu().numpy(), beta * 0.5 + dA_ref, bound=bounds["dA"][f:, :] + 1e-3 * beta)
    rep.add("dB", dB_t.cpu().numpy(), beta * -1.5 + dB_ref, bound=bounds["dB"][:, f:] + 1e-3 * beta)
    rep.add("dA_new", dA_t.cpu().numpy() - beta * 0.5, dA_ref, lines="rows")
    rep.add("dB_new", dB_t.cpu().numpy() - beta * -1.5, dB_ref, lines="cols")
    rep.finish()


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


# ---------------------------------------------------------------- stacked adapters trained with LoRA dropout
# (App. B's dropout rate on App. D's stacking).  The oracle has no function of its own for the combination: the
# gradients of the trainable pair are the rows / columns frozen.. of the full-stack gradients under the mask, and dX
# is the masked full-stack dX.

DROPOUT_CASES = [
    # (M, K, N, bits, G, rank, frozen, dtype, p): weight-streaming backward, tiled backward with the masked product in
    # the GEMM's epilogue (ranks up to 32) and added afterwards (above), 256-row tiles
    (6, 256, 72, 4, 64, 16, 8, "f16", 0.05),
    (16, 1024, 520, 2, 128, 40, 32, "bf16", 0.3),
    (29, 1024, 264, 4, 128, 24, 16, "f16", 0.3),          # 17 to 32 token rows: the staged backward kernel, two token blocks
    (40, 384, 264, 3, 128, 24, 16, "f16", 0.05),
    (300, 640, 392, 4, 128, 40, 32, "f16", 0.3),
    (257, 1024, 264, 8, 128, 32, 24, "bf16", 0.05),
    (2048, 512, 136, 4, 128, 16, 8, "f16", 0.05),
]


@pytest.mark.parametrize("case", DROPOUT_CASES, ids=lambda c: "M{}_K{}_N{}_b{}_G{}_r{}_f{}_{}_p{}".format(*c))
@pytest.mark.parametrize("beta", [0.0, 1.0])
def test_stacked_backward_with_dropout(case, beta):
    import torch
    from paper_2306_08162_amd import workloads as wl
    from paper_2306_08162_amd.device import DeviceLayer
    M, K, N, bits, G, r, f, dtype, p = case
    inp = small_inputs(7 * M + K + r + f, M, K, N, bits, G, r, dtype)
    c = inp.cfg
    announce(f"stacked + dropout {c.name}: frozen={f} p={p} beta={beta}")
    u01 = wl.splitmix64(c.seed + 91, 0, M * K).astype(np.float64) / 2.0 ** 64
    keep = (u01 >= p).astype(np.uint8).reshape(M, K)
    bits32 = keep.reshape(M, K // 32, 32).astype(np.uint64)
    words = (bits32 << np.arange(32, dtype=np.uint64)).sum(axis=2).astype(np.uint32)
    ks = 1.0 / (1.0 - p)
    layer = DeviceLayer(inp)
    km = torch.from_numpy(words.view(np.int32)).to(layer.device)
    saved = M % 2 == 0
    layer.forward_dropout(km, ks, save_t=saved)
    if beta:
        layer.backward_dropout_stacked(km, ks, f)          # allocate, then preset what is accumulated into
        layer.dA_train.fill_(0.5)
        layer.dB_train.fill_(-1.5)
    dA_t, dB_t = layer.backward_dropout_stacked(km, ks, f, beta=beta, use_saved_t=saved)
    torch.cuda.synchronize()
    lo = make_oracle(inp)
    _, t_ref = lo.forward_dropout(inp.x, keep, ks)
    dx_ref = lo.backward_dx_dropout(inp.dy, keep, ks)
    dA_full, dB_full = lo.backward_adapters_dropout(inp.dy, inp.x, keep, ks)
    dA_ref, dB_ref = dA_full[f:, :], dB_full[:, f:]
    x, dy = oracle.widen(inp.x, dtype), oracle.widen(inp.dy, dtype)
    sc = c.alpha / r
    xt = x * keep * ks
    u_ref = oracle.lora_u(dy, lo.B)
    bounds = layer_bounds(lo.Wd, lo.A * ks, lo.B, sc, dy=dy, t=t_ref, u=u_ref, x_adapter=xt)
    rep = Report(f"stacked + dropout {c.name} f={f} beta={beta}", dtype)
    rep.add("dx", oracle.widen(layer.host_dx(), dtype), dx_ref, lines="rows", bound=bounds["dx"])
    rep.add("dA", dA_t.cpu().numpy(), beta * 0.5 + dA_ref, bound=bounds["dA"][f:, :] + 1e-3 * beta)
    rep.add("dB", dB_t.cpu().numpy(), beta * -1.5 + dB_ref, bound=bounds["dB"][:, f:] + 1e-3 * beta)
    rep.add("dA_new", dA_t.cpu().numpy() - beta * 0.5, dA_ref, lines="rows")
    rep.add("dB_new", dB_t.cpu().numpy() - beta * -1.5, dB_ref, lines="cols")
    rep.finish()


def test_stacked_dropout_without_mask_is_the_stacked_backward():
    import torch
    from paper_2306_08162_amd.device import DeviceLayer
    inp = small_inputs(322, 70, 256, 136, 4, 64, 24, "f16")
    layer = DeviceLayer(inp)
    layer.forward()
    dA_t, dB_t = layer.backward_stacked(8)
    torch.cuda.synchronize()
    a0, b0, x0 = dA_t.cpu().numpy().copy(), dB_t.cpu().numpy().copy(), layer.host_dx().copy()
    dA_t, dB_t = layer.backward_dropout_stacked(None, 1.0, 8)
    torch.cuda.synchronize()
    assert np.array_equal(dA_t.cpu().numpy(), a0) and np.array_equal(dB_t.cpu().numpy(), b0)
    assert np.array_equal(layer.host_dx(), x0)
