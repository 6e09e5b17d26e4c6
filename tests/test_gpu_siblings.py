"""GPU parity of the sibling entry points (projections that share x, small token counts) against the CPU oracle.

The oracle knows single layers only: y_i, dA_i, dB_i are compared per projection, dX with the sum of the layers' dX
(the rule is pinned on the CPU in test_oracle_pins.py).  The same calls are also checked against the per-layer entry
points of the library itself.
"""
import dataclasses

import numpy as np
import pytest

import oracle
from paper_2306_08162_amd import workloads as wl
from parity import TOL, Report, announce, layer_bounds, make_oracle, rel_fro, small_inputs

pytestmark = pytest.mark.gpu


def _siblings(seed, M, K, Ns, bits, G, r, dtype):
    """Projections with their own weights, adapters and dY, all fed the first one's x."""
    inps = [small_inputs(seed + 31 * i, M, K, N, bits, G, r, dtype) for i, N in enumerate(Ns)]
    x = inps[0].x
    return [dataclasses.replace(inp, x=x) for inp in inps]


def _check(inps, recompute_t=False):
    import torch
    from paper_2306_08162_amd.device import DeviceLayer, DeviceSiblings

    c = inps[0].cfg
    announce(f"siblings N={[i.cfg.N for i in inps]} M={c.M} K={c.K} bits={c.bits} G={c.group_size} r={c.rank} {c.dtype} "
             f"recompute_t={recompute_t}")
    layers = [DeviceLayer(inp) for inp in inps]
    sib = DeviceSiblings(layers)
    sib.forward(save_t=not recompute_t)
    sib.backward(use_saved_t=not recompute_t)
    torch.cuda.synchronize()
    rep = Report(f"siblings N={[i.cfg.N for i in inps]} M={c.M}", c.dtype)
    dx_ref, dx_bound = 0.0, 0.0
    sc = c.alpha / c.rank if c.rank else 0.0
    for i, (inp, layer) in enumerate(zip(inps, layers)):
        lo = make_oracle(inp)
        y_ref, t_ref = lo.forward(inp.x)
        dx_ref = dx_ref + lo.backward_dx(inp.dy)
        x, dy = oracle.widen(inp.x, c.dtype), oracle.widen(inp.dy, c.dtype)
        u_ref = oracle.lora_u(dy, lo.B) if c.rank else None
        b = layer_bounds(lo.Wd, lo.A, lo.B, sc, x=x, dy=dy, t=t_ref if c.rank else None, u=u_ref, x_adapter=x)
        dx_bound = dx_bound + b["dx"]
        rep.add(f"y{i}", oracle.widen(layer.host_y(), c.dtype), y_ref, lines="rows", bound=b["y"])
        if c.rank:
            dA_ref, dB_ref = lo.backward_adapters(inp.dy, inp.x)
            rep.add(f"dA{i}", layer.host_dA(), dA_ref, lines="rows", bound=b["dA"])
            rep.add(f"dB{i}", layer.host_dB(), dB_ref, lines="cols", bound=b["dB"])
            if not recompute_t:
                rep.add(f"t{i}", oracle.widen(layer.host_t(), c.dtype), t_ref, lines="cols")
    rep.add("dx", oracle.widen(sib.host_dx(), c.dtype), dx_ref, lines="rows", bound=dx_bound)
    rep.finish()
    return layers, sib


CASES = [
    # (M, K, Ns, bits, G, r, dtype)
    (5, 256, (72, 40, 136), 4, 64, 8, "f16"),
    (16, 512, (1000, 520), 2, 128, 16, "bf16"),
    (1, 128, (64, 64, 64, 64), 8, 32, 0, "f16"),           # four projections, no adapters
    (9, 320, (264, 48), 3, 32, 64, "bf16"),                # rank 64: t from its own launches
    (16, 4096, (136, 264, 72), 4, 128, 40, "f16"),         # rank 40: ... which split the contraction over workgroups
    (13, 1376, (520, 2056, 8), 2, 32, 24, "f16"),          # very different sizes, K not a multiple of 128
    (16, 160, (4200, 4104), 8, 32, 8, "f16"),              # many row slices, ragged column block
    (7, 96, (12312,), 4, 96, 8, "f16"),                    # a single projection through the sibling entry points
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "M{}_K{}_N{}_b{}_G{}_r{}_{}".format(c[0], c[1], "x".join(map(str, c[2])), *c[3:]))
def test_sibling_shapes(case):
    M, K, Ns, bits, G, r, dtype = case
    inps = _siblings(5 * M + K + bits, M, K, Ns, bits, G, r, dtype)
    _check(inps)
    if r:
        _check(inps, recompute_t=True)


def test_siblings_agree_with_per_layer_calls():
    """y, dA, dB bit for bit (the same kernels do the same sums); dX within rounding of the sum of the layers' dX."""
    import torch
    inps = _siblings(99, 16, 512, (264, 136, 392), 4, 128, 8, "f16")
    layers, sib = _check(inps)
    got = [(l.host_y().copy(), l.host_dA().copy(), l.host_dB().copy()) for l in layers]
    dx_sum = 0.0
    for l in layers:
        l.forward()
        l.backward()
        torch.cuda.synchronize()
        dx_sum = dx_sum + oracle.widen(l.host_dx(), "f16")
    for l, (y, dA, dB) in zip(layers, got):
        assert np.array_equal(l.host_y(), y)
        assert np.array_equal(l.host_dB(), dB)
        assert rel_fro(l.host_dA(), dA) <= 1e-6          # u is summed over a different slicing
    assert rel_fro(oracle.widen(sib.host_dx(), "f16"), dx_sum) <= 2e-3


def test_siblings_are_bitwise_reproducible():
    import torch
    inps = _siblings(7, 16, 256, (520, 264), 2, 64, 8, "f16")
    layers, sib = _check(inps)
    first = [sib.host_dx().copy()] + [l.host_y().copy() for l in layers] + [l.host_dA().copy() for l in layers]
    for _ in range(2):
        sib.forward()
        sib.backward()
        torch.cuda.synchronize()
        again = [sib.host_dx()] + [l.host_y() for l in layers] + [l.host_dA() for l in layers]
        for a, b in zip(first, again):
            assert np.array_equal(a, b)


@pytest.mark.parametrize("bits", [2, 8])
def test_decoder_block_siblings_full_size(bits):
    """q/k/v and gate/up of a LLaMA-7B block at M = 16, the grouping bench.py times."""
    block = {c.name.split("_")[1]: c for c in wl.config5(bits, 16)}
    for names in (("q", "k", "v"), ("gate", "up")):
        inps = [wl.make_inputs(block[n]) for n in names]
        x = inps[0].x
        _check([dataclasses.replace(i, x=x) for i in inps])


@pytest.mark.parametrize("case", [(100, 512, (264, 136), 4, 128, 8, "f16"), (300, 1024, (520, 264, 72), 2, 64, 8, "bf16")],
                         ids=["two_f16", "three_bf16"])
def test_siblings_above_16_rows_as_one_concatenated_layer(case):
    """Above 16 token rows siblings need no entry point of their own: packed rows, scales and zeros of the siblings
    laid one after the other along N are themselves a valid weight, the stacked A with a block-structured B a valid
    adapter of rank (count * r), so one call of the ordinary entry points serves them all.  Checked per projection
    against the single-layer oracle (dX against the sum of the layers' dX)."""
    import torch
    from paper_2306_08162_amd.device import DeviceLayer

    M, K, Ns, bits, G, r, dtype = case
    inps = _siblings(11 * M + K, M, K, Ns, bits, G, r, dtype)
    c0, count, Ntot = inps[0].cfg, len(Ns), sum(Ns)
    B = np.zeros((Ntot, count * r), dtype=np.uint16)            # bit pattern 0 is +0.0 in both formats
    row = 0
    for i, inp in enumerate(inps):
        B[row:row + inp.cfg.N, i * r:(i + 1) * r] = inp.B
        row += inp.cfg.N
    cat = wl.LayerInputs(
        cfg=dataclasses.replace(c0, name="concatenated", N=Ntot, rank=count * r, alpha=c0.alpha * count),  # same alpha/r
        codes=np.concatenate([i.codes for i in inps]), scales=np.concatenate([i.scales for i in inps]),
        zeros=np.concatenate([i.zeros for i in inps]), A=np.concatenate([i.A for i in inps]), B=B, x=inps[0].x,
        dy=np.ascontiguousarray(np.concatenate([i.dy for i in inps], axis=1)))
    announce(f"concatenated siblings N={Ns} M={M} K={K} bits={bits} G={G} r={r} {dtype}")
    layer = DeviceLayer(cat)
    layer.forward()
    layer.backward()
    torch.cuda.synchronize()
    y, dA, dB = oracle.widen(layer.host_y(), dtype), layer.host_dA(), layer.host_dB()
    rep = Report(f"concatenated siblings N={Ns} M={M}", dtype)
    dx_ref, dx_bound, row = 0.0, 0.0, 0
    sc = c0.alpha / r
    for i, inp in enumerate(inps):
        lo, n = make_oracle(inp), inp.cfg.N
        y_ref, t_ref = lo.forward(inp.x)
        dx_ref = dx_ref + lo.backward_dx(inp.dy)
        dA_ref, dB_ref = lo.backward_adapters(inp.dy, inp.x)
        xw, dyw = oracle.widen(inp.x, dtype), oracle.widen(inp.dy, dtype)
        b = layer_bounds(lo.Wd, lo.A, lo.B, sc, x=xw, dy=dyw, t=t_ref, u=oracle.lora_u(dyw, lo.B), x_adapter=xw)
        dx_bound = dx_bound + b["dx"]
        rep.add(f"y{i}", y[:, row:row + n], y_ref, lines="rows", bound=b["y"])
        rep.add(f"dA{i}", dA[i * r:(i + 1) * r], dA_ref, lines="rows", bound=b["dA"])
        rep.add(f"dB{i}", dB[row:row + n, i * r:(i + 1) * r], dB_ref, lines="cols", bound=b["dB"])
        row += n
    rep.add("dx", oracle.widen(layer.host_dx(), dtype), dx_ref, lines="rows", bound=dx_bound)
    rep.finish()
