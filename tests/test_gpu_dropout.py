"""GPU parity of the LoRA-dropout entry points against the fp64 oracle (the mask is an input to both)."""
import numpy as np
import pytest

import oracle
from paper_2306_08162_amd import workloads as wl
from parity import Report, announce, layer_bounds, make_oracle, small_inputs

pytestmark = pytest.mark.gpu


def _mask(seed, M, K, p):
    """keep [M,K] in {0,1} (seeded) and its bit-packed form [M, K/32] (bit k % 32 of word k / 32)."""
    u = wl.splitmix64(seed, 0, M * K).astype(np.float64) / 2.0 ** 64
    keep = (u >= p).astype(np.uint8).reshape(M, K)
    bits = keep.reshape(M, K // 32, 32).astype(np.uint64)
    words = (bits << np.arange(32, dtype=np.uint64)).sum(axis=2).astype(np.uint32)
    return keep, words


def _check(inp, p, recompute_t=False, beta=0.0):
    import torch
    from paper_2306_08162_amd.device import DeviceLayer
    c = inp.cfg
    announce(f"dropout {c.name}: p={p} recompute_t={recompute_t} beta={beta}")
    keep, words = _mask(c.seed + 77, c.M, c.K, p)
    ks = 1.0 / (1.0 - p)
    layer = DeviceLayer(inp)
    km = torch.from_numpy(words.view(np.int32)).to(layer.device)
    if beta:
        layer.dA.fill_(1.0)
        layer.dB.fill_(-2.0)
    layer.forward_dropout(km, ks, save_t=not recompute_t)
    layer.backward_dropout(km, ks, use_saved_t=not recompute_t, beta=beta)
    torch.cuda.synchronize()
    lo = make_oracle(inp)
    y_ref, t_ref = lo.forward_dropout(inp.x, keep, ks)
    dx_ref = lo.backward_dx_dropout(inp.dy, keep, ks)
    x, dy = oracle.widen(inp.x, c.dtype), oracle.widen(inp.dy, c.dtype)
    sc = c.alpha / c.rank if c.rank else 0.0
    xt = x * keep * ks                                   # what the adapter branch sees
    u_ref = oracle.lora_u(dy, lo.B) if c.rank else None
    # element scales as in parity.py; the adapter's share of dX is at most keep_scale times the unmasked one
    bounds = layer_bounds(lo.Wd, lo.A * ks, lo.B, sc, x=x, dy=dy, t=t_ref if c.rank else None, u=u_ref, x_adapter=xt)
    rep = Report(f"dropout {c.name}", c.dtype)
    rep.add("y", oracle.widen(layer.host_y(), c.dtype), y_ref, lines="rows", bound=bounds["y"])
    rep.add("dx", oracle.widen(layer.host_dx(), c.dtype), dx_ref, lines="rows", bound=bounds["dx"])
    if c.rank:
        dA_ref, dB_ref = lo.backward_adapters_dropout(inp.dy, inp.x, keep, ks)
        # accumulation adds beta * (the preset constant), itself exact in fp32, to both sides
        rep.add("dA", layer.host_dA(), beta * 1.0 + dA_ref, bound=bounds["dA"] + 1e-3 * beta)
        rep.add("dB", layer.host_dB(), beta * -2.0 + dB_ref, bound=bounds["dB"] + 1e-3 * beta)
        rep.add("dA_new", layer.host_dA() - beta * 1.0, dA_ref, lines="rows")
        rep.add("dB_new", layer.host_dB() - beta * -2.0, dB_ref, lines="cols")
        if not recompute_t:
            rep.add("t", oracle.widen(layer.host_t(), c.dtype), t_ref, lines="cols",
                    bound=np.outer(np.linalg.norm(xt, axis=1), np.linalg.norm(lo.A, axis=1)))
    rep.finish()


CASES = [
    # (M, K, N, bits, G, r, dtype, p): weight-streaming (M <= 16), forward-only streaming (17..64), tiled
    (7, 256, 72, 4, 64, 8, "f16", 0.05),
    (16, 1376, 520, 2, 32, 24, "bf16", 0.5),
    (3, 512, 136, 8, 128, 64, "f16", 0.05),
    (27, 1024, 264, 4, 128, 16, "f16", 0.3),             # 17 to 32 token rows: the staged kernels with two token blocks
    (32, 512, 136, 2, 128, 8, "bf16", 0.05),
    (40, 384, 264, 3, 128, 16, "f16", 0.3),
    (300, 640, 392, 4, 128, 8, "f16", 0.05),
    (257, 1024, 520, 2, 128, 32, "bf16", 0.5),
    (130, 96, 40, 8, 32, 64, "bf16", 0.05),
    (200, 384, 264, 4, 128, 24, "f16", 0.3),             # rank 24 in the 32-wide one-pass gradient kernel, masked
    (90, 512, 136, 2, 128, 56, "bf16", 0.05),            # rank 56 in the 64-wide one
    (65, 256, 1000, 4, 64, 0, "f16", 0.05),              # no adapter: the mask has nothing to act on
    (2048, 4096, 264, 4, 128, 16, "f16", 0.05),          # 256-row tiles: masked product added in the GEMM's epilogue
    (2050, 4128, 136, 2, 96, 32, "bf16", 0.3),           # the same with ragged last tiles and two 16-column groups
    (4100, 512, 136, 4, 128, 56, "f16", 0.05),           # 16 token rows per workgroup of the t kernel would not fit
    (4096, 384, 72, 8, 128, 64, "bf16", 0.3),            #   the LDS at these ranks under a mask: 8-row workgroups
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "M{}_K{}_N{}_b{}_G{}_r{}_{}_p{}".format(*c))
def test_dropout_shapes(case):
    M, K, N, bits, G, r, dtype, p = case
    inp = small_inputs(3 * M + K + bits, M, K, N, bits, G, r, dtype)
    _check(inp, p)
    if r:
        _check(inp, p, recompute_t=True, beta=0.5)


def test_dropout_extremes():
    inp = small_inputs(5, 33, 256, 136, 4, 64, 8, "f16")
    _check(inp, 0.0)            # nothing dropped: the plain layer
    _check(inp, 0.999999)       # (almost surely) everything dropped: the adapter is gone
