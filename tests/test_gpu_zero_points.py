"""GPU parity of the layer with its zero-points left bit-packed (Sec. 3.2 counts `bits` bits of zero-point per group;
Sec. 2.2 / App. A: that is how the quantized checkpoints store them).  The packed rows are written by the oracle and
the results are compared with the oracle's on the unpacked zero-points: y, dX, dA, dB to the layer's bars, and bit
for bit on inputs whose every product and sum is a small integer."""
import numpy as np
import pytest

import oracle
from parity import announce, check_layer, integer_inputs, small_inputs

pytestmark = pytest.mark.gpu

# (M, K, N, bits, G, rank, dtype)
STREAMED = [
    # both weight-streaming kernels read the packed rows themselves (up to 16 token rows, K and G multiples of 128)
    (7, 512, 136, 2, 128, 8, "f16"),           # one word per row, two groups per backward column block
    (16, 1024, 264, 2, 128, 16, "bf16"),
    (16, 8192, 144, 2, 128, 8, "f16"),         # four words per row: the backward windows move along the row
    (5, 1024, 200, 4, 128, 8, "f16"),          # one group per backward column block
    (16, 4096, 264, 4, 128, 8, "bf16"),        # four words per row, a ragged last block of weight rows
    (12, 2048, 136, 8, 128, 16, "f16"),
    (16, 4096, 72, 8, 256, 8, "f16"),          # groups wider than a column block
    (3, 1280, 80, 8, 128, 0, "bf16"),          # no adapter; 10 groups: rows of 2.5 words padded to 3
    (1, 3072, 96, 2, 128, 8, "f16"),           # 24 groups of 2 bits: 1.5 words
]
MIXED = [
    # one pass reads the packed rows, the other (or both) has them unpacked into the workspace first
    (9, 1408, 80, 3, 128, 8, "f16"),           # 3 bits: a field straddles two words; the backward kernel unpacks
    (16, 1024, 72, 3, 128, 16, "bf16"),
    (8, 512, 136, 4, 64, 8, "f16"),            # G = 64: forward unpacks, backward reads two groups per block
    (11, 1024, 200, 8, 64, 8, "f16"),
    (6, 256, 72, 4, 32, 16, "f16"),            # four groups per column block: both unpack
    (14, 384, 56, 2, 128, 8, "f16"),           # N * groups not in whole 16-byte pieces
    (27, 1024, 136, 4, 128, 8, "f16"),         # 17 to 32 token rows, two token blocks: both passes read the packed rows
    (20, 1024, 72, 3, 128, 8, "f16"),          # ... 3 bits: both unpack
    (32, 2048, 200, 8, 128, 8, "bf16"),        # ... 8 bits: forward reads them, the tiled backward kernel unpacks
    (16, 512, 136, 4, 128, 40, "f16"),         # rank above what the forward kernel computes t for
    (40, 512, 136, 4, 128, 8, "f16"),          # more than 16 token rows
    (200, 640, 264, 2, 128, 16, "bf16"),       # the tiled kernels
    (300, 512, 136, 3, 64, 8, "f16"),
]


@pytest.mark.parametrize("case", STREAMED + MIXED, ids=lambda c: "M{}_K{}_N{}_b{}_G{}_r{}_{}".format(*c))
def test_packed_zero_points(case):
    M, K, N, bits, G, r, dtype = case
    inp = small_inputs(3 * M + K + N + bits, M, K, N, bits, G, r, dtype)
    check_layer(inp, packed_zeros=True, recompute_t=(M % 2 == 1))


EXACT = [
    (16, 1024, 136, 2, 128, 8, "f16"),
    (13, 4096, 72, 4, 128, 8, "f16"),
    (16, 2048, 80, 8, 128, 8, "bf16"),
    (8, 1408, 80, 3, 128, 8, "f16"),
    (64, 512, 72, 4, 64, 8, "f16"),
]


@pytest.mark.parametrize("case", EXACT, ids=lambda c: "M{}_K{}_N{}_b{}_G{}_r{}_{}".format(*c))
def test_packed_zero_points_exact(case):
    M, K, N, bits, G, r, dtype = case
    inp = integer_inputs(17 + M + K + bits, M, K, N, bits, G, r, dtype, density=0.05 if K > 1024 else 0.2)
    check_layer(inp, packed_zeros=True, exact=True)


def test_packed_and_unpacked_zero_points_give_the_same_bits():
    """Same kernels, same order of operations: the two forms of the zero-points must not differ in a single bit."""
    import torch
    from paper_2306_08162_amd.device import DeviceLayer
    for M, K, N, bits, G, r, dtype in (STREAMED[1], STREAMED[4], STREAMED[5], (9, 1408, 80, 3, 128, 8, "f16"),
                                       (8, 512, 136, 4, 64, 8, "f16"), (27, 1024, 136, 4, 128, 8, "f16"),
                                       (200, 640, 264, 2, 128, 16, "bf16")):
        inp = small_inputs(91 + M + K, M, K, N, bits, G, r, dtype)
        announce(f"packed vs unpacked zero-points {inp.cfg.name}")
        plain, zp = DeviceLayer(inp), DeviceLayer(inp)
        zp.use_packed_zeros(oracle.pack_zeros(inp.zeros, bits))
        for layer in (plain, zp):
            layer.forward()
            layer.backward()
        torch.cuda.synchronize()
        assert np.array_equal(plain.host_y(), zp.host_y())
        assert np.array_equal(plain.host_dx(), zp.host_dx())
        if r:
            assert np.array_equal(plain.host_t(), zp.host_t())
            assert np.array_equal(plain.host_dA(), zp.host_dA())
            assert np.array_equal(plain.host_dB(), zp.host_dB())


def test_streamed_shapes_read_the_packed_rows_in_the_kernels():
    """Where the weight-streaming kernels take the shape nothing is unpacked: the room for the unpacked zero-points at
    the end of the workspace keeps what the caller left there.  Where a pass falls back it holds them afterwards."""
    import torch
    from paper_2306_08162_amd import binding as ql
    from paper_2306_08162_amd.device import DeviceLayer
    fallback = [(6, 256, 72, 4, 32, 16, "f16"), (40, 512, 136, 4, 128, 8, "f16")]      # narrow groups; the tiled kernels
    for case, streamed in [(c, True) for c in STREAMED] + [(c, False) for c in fallback]:
        M, K, N, bits, G, r, dtype = case
        inp = small_inputs(7 + M + N, M, K, N, bits, G, r, dtype)
        c = inp.cfg
        announce(f"zero-points stay packed: {c.name} streamed={streamed}")
        layer = DeviceLayer(inp)
        layer.use_packed_zeros(oracle.pack_zeros(inp.zeros, bits))
        plain_bytes = ql.qlora_workspace_bytes(M, N, K, bits, G, r)
        layer.workspace.fill_(0xA5)
        layer.forward()
        layer.backward()
        torch.cuda.synchronize()
        room = layer.workspace[plain_bytes:plain_bytes + N * c.groups].cpu().numpy()
        if streamed:
            assert np.all(room == 0xA5), f"{c.name}: the zero-points were unpacked"
        else:
            assert np.array_equal(room.reshape(N, c.groups), inp.zeros)


def test_packed_zero_points_workspace_is_checked():
    import torch
    from paper_2306_08162_amd import binding as ql
    from paper_2306_08162_amd.device import DeviceLayer
    inp = small_inputs(5, 8, 512, 136, 4, 128, 8, "f16")
    c = inp.cfg
    layer = DeviceLayer(inp)
    plain_bytes = ql.qlora_workspace_bytes(c.M, c.N, c.K, c.bits, c.group_size, c.rank)
    layer.use_packed_zeros(oracle.pack_zeros(inp.zeros, c.bits))
    assert layer.workspace.numel() >= plain_bytes + c.N * c.groups
    E = ql.STATUS_NAMES.index
    small = torch.empty(plain_bytes, dtype=torch.uint8, device=layer.device)     # enough for the unpacked entry point
    st = ql.qlora_linear_fwd_zp(layer.x, layer.packed, layer.scales, layer.packed_zeros, layer.A, layer.B, layer.y,
                                None, c.M, c.N, c.K, c.bits, c.group_size, c.rank, c.alpha, layer.dtype_flag, small,
                                check=False)
    assert st == E("QLORA_E_WORKSPACE")
    st = ql.qlora_linear_bwd_zp(layer.dy, layer.x, layer.packed, layer.scales, None, layer.A, layer.B, None, layer.dx,
                                layer.dA, layer.dB, 0.0, c.M, c.N, c.K, c.bits, c.group_size, c.rank, c.alpha,
                                layer.dtype_flag, layer.workspace, check=False)
    assert st == E("QLORA_E_NULL")
