"""The allocation-free forward entry point (scratch in a static device array) against qlora_linear_fwd with a caller's
workspace: the same kernels run on the same inputs, so every output must agree bit for bit -- on two calls in a row, the
second on a smaller problem that finds the first one's leftovers in the scratch -- and both against the fp64 oracle."""
import numpy as np
import pytest

import oracle
from paper_2306_08162_amd import binding as ql
from parity import Report, announce, layer_bounds, make_oracle, small_inputs

pytestmark = pytest.mark.gpu


def _both_ways(inp):
    """y and t from qlora_linear_fwd (workspace) and from qlora_linear_fwd_static; t is not saved in the static call of
    the pair that checks y (it then lives in the scratch), and saved in a second static call."""
    import torch
    from paper_2306_08162_amd.device import DeviceLayer
    c = inp.cfg
    layer = DeviceLayer(inp)
    layer.forward(save_t=True)
    torch.cuda.synchronize()
    y_ws, t_ws = layer.host_y().copy(), layer.host_t().copy()
    layer.y.fill_(0x7e7e)
    layer.t.fill_(0x7e7e)
    args = (layer.x, layer.packed, layer.scales, layer.zeros, layer.A, layer.B, layer.y)
    tail = (c.M, c.N, c.K, c.bits, c.group_size, c.rank, c.alpha, layer.dtype_flag)
    ql.qlora_linear_fwd_static(*args, None, *tail)                     # t in the static scratch
    torch.cuda.synchronize()
    y_st = layer.host_y().copy()
    layer.y.fill_(0x7e7e)
    ql.qlora_linear_fwd_static(*args, layer.t if c.rank else None, *tail)   # t handed back to the caller
    torch.cuda.synchronize()
    return y_ws, t_ws, y_st, layer.host_y().copy(), layer.host_t().copy()


def _check(inp):
    c = inp.cfg
    announce(f"static-scratch forward {c.name}: M={c.M} K={c.K} N={c.N} bits={c.bits} r={c.rank} {c.dtype}")
    y_ws, t_ws, y_st, y_st2, t_st = _both_ways(inp)
    assert np.array_equal(y_st, y_ws), "static-scratch forward differs from the workspace forward"
    assert np.array_equal(y_st2, y_ws) and (c.rank == 0 or np.array_equal(t_st, t_ws))
    lo = make_oracle(inp)
    y_ref, t_ref = lo.forward(inp.x)
    x = oracle.widen(inp.x, c.dtype)
    b = layer_bounds(lo.Wd, lo.A, lo.B, c.alpha / c.rank if c.rank else 0.0, x=x, t=t_ref if c.rank else None)
    rep = Report(f"static {c.name}", c.dtype)
    rep.add("y", oracle.widen(y_st, c.dtype), y_ref, lines="rows", bound=b["y"])
    rep.finish()


def test_two_calls_in_a_row_the_second_smaller():
    # tiled path with the contraction split over 4 workgroups per tile (fp32 planes and t in the scratch), then a
    # smaller problem of the same kind, then the weight-streaming path (t in the scratch) and an unsplit tiled call
    _check(small_inputs(901, 100, 2048, 512, 4, 128, 8, "f16"))
    _check(small_inputs(902, 70, 1024, 264, 4, 128, 8, "f16"))
    _check(small_inputs(903, 300, 640, 392, 2, 128, 24, "bf16"))
    _check(small_inputs(904, 16, 512, 264, 8, 128, 64, "f16"))      # rank 64: t from its own launch, into the scratch
    _check(small_inputs(905, 9, 256, 72, 3, 32, 16, "bf16"))
    _check(small_inputs(907, 28, 1024, 136, 4, 128, 32, "f16"))     # two token blocks, rank 32 formed in the kernel


def test_llama_block_shapes_fit_and_oversized_problems_are_refused():
    import torch
    # every projection of the decoder block at the token counts of the sweep fits the static array
    inp = small_inputs(906, 256, 4096, 4096, 2, 128, 8, "f16")     # 4 planes of 256 x 4096 floats: 16 MiB
    _check(inp)
    # The planes of a split contraction never exceed 256 tiles' worth of floats (16 MiB); what can outgrow the array
    # is t = x A^T of a very long token batch.  Such a call is refused before anything is launched, with its own status.
    M, N, K, r = 300000, 8, 32, 64                                  # t alone: 300000 x 64 x 2 bytes = 36.6 MiB
    assert M * r * 2 > ql.STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    st = ql.qlora_linear_fwd_static(dummy, dummy, dummy, dummy, dummy, dummy, dummy, None, M, N, K, 4, 32, r, 16.0,
                                    ql.QLORA_F16, check=False)
    assert ql.STATUS_NAMES[st] == "QLORA_E_STATIC"
    assert "static" in ql.status_string(st)
    # with t saved by the caller the same shape needs no scratch to speak of, but its buffers would have to be real:
    # only the refusal is exercised here
