"""Device-side plumbing for one layer: torch allocates HBM buffers, the HIP library does all the work.

Used by the tests, the smoke check and the benchmark so that they all call the
C ABI the same way.  Nothing here computes anything.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as ql
from .workloads import LayerConfig, LayerInputs


def _dev(a: np.ndarray, device) -> torch.Tensor:
    """Upload raw bytes; 16-bit patterns travel as int16, words as int32."""
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def _host16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


class DeviceLayer:
    """One quantized LoRA projection resident in HBM."""

    def __init__(self, inp: LayerInputs, device: str = "cuda:0", upload_activations: bool = True):
        c: LayerConfig = inp.cfg
        self.cfg = c
        self.device = torch.device(device)
        self.dtype_flag = ql.QLORA_BF16 if c.dtype == "bf16" else ql.QLORA_F16
        self.codes = _dev(inp.codes, self.device)
        self.scales = _dev(inp.scales, self.device)
        self.zeros = _dev(inp.zeros, self.device)
        self.A = _dev(inp.A, self.device) if c.rank else None
        self.B = _dev(inp.B, self.device) if c.rank else None
        self.packed = torch.empty((c.N, c.words_per_row), dtype=torch.int32, device=self.device)
        ql.qlora_pack(self.codes, self.packed, c.N, c.K, c.bits)
        self.x = _dev(inp.x, self.device) if upload_activations else None
        self.dy = _dev(inp.dy, self.device) if upload_activations else None
        self.y = torch.empty((c.M, c.N), dtype=torch.int16, device=self.device)
        self.dx = torch.empty((c.M, c.K), dtype=torch.int16, device=self.device)
        self.t = torch.empty((c.M, max(c.rank, 1)), dtype=torch.int16, device=self.device)
        self.dA = torch.empty((max(c.rank, 1), c.K), dtype=torch.float32, device=self.device)
        self.dB = torch.empty((c.N, max(c.rank, 1)), dtype=torch.float32, device=self.device)
        nbytes = ql.qlora_workspace_bytes(c.M, c.N, c.K, c.bits, c.group_size, c.rank)
        if nbytes == 0:
            raise ValueError(f"shape not accepted by the library: {c}")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)

    @classmethod
    def drawn_on_device(cls, cfg: LayerConfig, device: str = "cuda:0", seed: int = 0) -> "DeviceLayer":
        """The same layer with every tensor drawn by torch's seeded generator on the GPU instead of uploaded from the
        host generators: same shapes, dtypes and value distributions (uniform codes and zero-points, uniform scales,
        A ~ N(0, 1/K), B ~ N(0, 0.01), x and dY ~ N(0, 1)).  For timing runs of the large shapes, where drawing
        10^8 numbers on the host would take longer than the measurement; the parity tests use the host generators."""
        self = cls.__new__(cls)
        c = cfg
        dev = torch.device(device)
        g = torch.Generator(device=dev)
        g.manual_seed(cfg.seed + seed)
        f16 = torch.bfloat16 if c.dtype == "bf16" else torch.float16

        def bits16(t, dt):
            return t.to(dt).view(torch.int16).contiguous()

        self.cfg, self.device = c, dev
        self.dtype_flag = ql.QLORA_BF16 if c.dtype == "bf16" else ql.QLORA_F16
        self.codes = torch.randint(0, 1 << c.bits, (c.N, c.K), dtype=torch.uint8, device=dev, generator=g)
        sc = torch.rand((c.N, c.groups), device=dev, generator=g) * (c.scale_hi - c.scale_lo) + c.scale_lo
        self.scales = bits16(sc, torch.float16)
        self.zeros = torch.randint(0, 1 << c.bits, (c.N, c.groups), dtype=torch.uint8, device=dev, generator=g)
        r = max(c.rank, 1)
        self.A = bits16(torch.randn((r, c.K), device=dev, generator=g) * c.K ** -0.5, f16) if c.rank else None
        self.B = bits16(torch.randn((c.N, r), device=dev, generator=g) * 0.1, f16) if c.rank else None
        self.packed = torch.empty((c.N, c.words_per_row), dtype=torch.int32, device=dev)
        ql.qlora_pack(self.codes, self.packed, c.N, c.K, c.bits)
        self.codes = None                                   # only the packed form stays resident
        self.x = bits16(torch.randn((c.M, c.K), device=dev, generator=g), f16)
        self.dy = bits16(torch.randn((c.M, c.N), device=dev, generator=g), f16)
        self.y = torch.empty((c.M, c.N), dtype=torch.int16, device=dev)
        self.dx = torch.empty((c.M, c.K), dtype=torch.int16, device=dev)
        self.t = torch.empty((c.M, r), dtype=torch.int16, device=dev)
        self.dA = torch.empty((r, c.K), dtype=torch.float32, device=dev)
        self.dB = torch.empty((c.N, r), dtype=torch.float32, device=dev)
        nbytes = ql.qlora_workspace_bytes(c.M, c.N, c.K, c.bits, c.group_size, c.rank)
        if nbytes == 0:
            raise ValueError(f"shape not accepted by the library: {c}")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        return self

    def use_packed_zeros(self, packed_zeros: Optional[np.ndarray] = None) -> None:
        """Hand the zero-points over in their bit-packed storage form ([N, ceil(groups * bits / 32)] uint32, packed
        by the caller; None: packed here from the resident ones by qlora_pack_zeros): forward() and backward() then
        go through qlora_linear_fwd_zp / qlora_linear_bwd_zp and the unpacked zero-points are dropped."""
        c = self.cfg
        want = (c.N, ql.qlora_packed_zero_words(c.N, c.groups, c.bits) // c.N)
        if packed_zeros is None:
            self.packed_zeros = torch.empty(want, dtype=torch.int32, device=self.device)
            ql.qlora_pack_zeros(self.zeros, self.packed_zeros, c.N, c.groups, c.bits)
            torch.cuda.synchronize(self.device)
        else:
            if packed_zeros.shape != want:
                raise ValueError(f"packed zero-points of shape {packed_zeros.shape}, expected {want}")
            self.packed_zeros = _dev(np.ascontiguousarray(packed_zeros).view(np.int32), self.device)
        self.zeros = None
        nbytes = ql.qlora_workspace_bytes_zp(c.M, c.N, c.K, c.bits, c.group_size, c.rank)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)

    # -- calls through the C ABI -------------------------------------------------
    def forward(self, save_t: bool = True, stream=None):
        c = self.cfg
        if getattr(self, "packed_zeros", None) is not None:
            ql.qlora_linear_fwd_zp(self.x, self.packed, self.scales, self.packed_zeros, self.A, self.B, self.y,
                                   self.t if (save_t and c.rank) else None, c.M, c.N, c.K, c.bits, c.group_size,
                                   c.rank, c.alpha, self.dtype_flag, self.workspace, stream=stream)
            return
        ql.qlora_linear_fwd(self.x, self.packed, self.scales, self.zeros, self.A, self.B, self.y,
                            self.t if (save_t and c.rank) else None, c.M, c.N, c.K, c.bits, c.group_size, c.rank,
                            c.alpha, self.dtype_flag, self.workspace, stream=stream)

    def backward(self, use_saved_t: bool = True, stream=None):
        c = self.cfg
        if getattr(self, "packed_zeros", None) is not None:
            return self.backward_accumulate(0.0, use_saved_t, stream)
        ql.qlora_linear_bwd(self.dy, self.x, self.packed, self.scales, self.zeros, self.A, self.B,
                            self.t if (use_saved_t and c.rank) else None, self.dx,
                            self.dA if c.rank else None, self.dB if c.rank else None,
                            c.M, c.N, c.K, c.bits, c.group_size, c.rank, c.alpha, self.dtype_flag, self.workspace,
                            stream=stream)

    def backward_accumulate(self, beta: float, use_saved_t: bool = True, stream=None):
        c = self.cfg
        if getattr(self, "packed_zeros", None) is not None:
            ql.qlora_linear_bwd_zp(self.dy, self.x, self.packed, self.scales, self.packed_zeros, self.A, self.B,
                                   self.t if (use_saved_t and c.rank) else None, self.dx,
                                   self.dA if c.rank else None, self.dB if c.rank else None, beta,
                                   c.M, c.N, c.K, c.bits, c.group_size, c.rank, c.alpha, self.dtype_flag,
                                   self.workspace, stream=stream)
            return
        ql.qlora_linear_bwd_accumulate(self.dy, self.x, self.packed, self.scales, self.zeros, self.A, self.B,
                                       self.t if (use_saved_t and c.rank) else None, self.dx,
                                       self.dA if c.rank else None, self.dB if c.rank else None, beta,
                                       c.M, c.N, c.K, c.bits, c.group_size, c.rank, c.alpha, self.dtype_flag,
                                       self.workspace, stream=stream)

    def backward_stacked(self, frozen_rank: int, beta: float = 0.0, use_saved_t: bool = True, stream=None):
        """Gradients for the trainable pair only: returns (dA_train [r - f, K], dB_train [N, r - f]) device tensors."""
        c = self.cfg
        rt = c.rank - frozen_rank
        if not hasattr(self, "dA_train") or self.dA_train.shape[0] != rt:
            self.dA_train = torch.zeros((rt, c.K), dtype=torch.float32, device=self.device)
            self.dB_train = torch.zeros((c.N, rt), dtype=torch.float32, device=self.device)
        ql.qlora_linear_bwd_stacked(self.dy, self.x, self.packed, self.scales, self.zeros, self.A, self.B,
                                    self.t if use_saved_t else None, self.dx, self.dA_train, self.dB_train, beta,
                                    frozen_rank, c.M, c.N, c.K, c.bits, c.group_size, c.rank, c.alpha, self.dtype_flag,
                                    self.workspace, stream=stream)
        return self.dA_train, self.dB_train

    def backward_dropout_stacked(self, keep_mask, keep_scale: float, frozen_rank: int, beta: float = 0.0,
                                 use_saved_t: bool = True, stream=None):
        """backward_stacked with the keep mask of the dropout pass: returns (dA_train, dB_train) device tensors."""
        c = self.cfg
        rt = c.rank - frozen_rank
        if not hasattr(self, "dA_train") or self.dA_train.shape[0] != rt:
            self.dA_train = torch.zeros((rt, c.K), dtype=torch.float32, device=self.device)
            self.dB_train = torch.zeros((c.N, rt), dtype=torch.float32, device=self.device)
        ql.qlora_linear_bwd_dropout_stacked(self.dy, self.x, self.packed, self.scales, self.zeros, self.A, self.B,
                                            keep_mask, keep_scale, self.t if use_saved_t else None, self.dx,
                                            self.dA_train, self.dB_train, beta, frozen_rank, c.M, c.N, c.K, c.bits,
                                            c.group_size, c.rank, c.alpha, self.dtype_flag, self.workspace,
                                            stream=stream)
        return self.dA_train, self.dB_train

    def forward_dropout(self, keep_mask, keep_scale: float, save_t: bool = True, stream=None):
        """keep_mask: int32 tensor [M, K/32] of keep bits (bit k % 32 of word k / 32)."""
        c = self.cfg
        ql.qlora_linear_fwd_dropout(self.x, self.packed, self.scales, self.zeros, self.A, self.B, keep_mask,
                                    keep_scale, self.y, self.t if (save_t and c.rank) else None, c.M, c.N, c.K,
                                    c.bits, c.group_size, c.rank, c.alpha, self.dtype_flag, self.workspace,
                                    stream=stream)

    def backward_dropout(self, keep_mask, keep_scale: float, use_saved_t: bool = True, beta: float = 0.0, stream=None):
        c = self.cfg
        ql.qlora_linear_bwd_dropout(self.dy, self.x, self.packed, self.scales, self.zeros, self.A, self.B, keep_mask,
                                    keep_scale, self.t if (use_saved_t and c.rank) else None, self.dx,
                                    self.dA if c.rank else None, self.dB if c.rank else None, beta,
                                    c.M, c.N, c.K, c.bits, c.group_size, c.rank, c.alpha, self.dtype_flag,
                                    self.workspace, stream=stream)

    def unpack(self) -> np.ndarray:
        c = self.cfg
        out = torch.empty((c.N, c.K), dtype=torch.uint8, device=self.device)
        ql.qlora_unpack(self.packed, out, c.N, c.K, c.bits)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    # -- downloads (raw 16-bit patterns / fp32) ------------------------------------
    def host_packed(self) -> np.ndarray:
        return self.packed.cpu().numpy().view(np.uint32)

    def host_y(self) -> np.ndarray:
        return _host16(self.y)

    def host_dx(self) -> np.ndarray:
        return _host16(self.dx)

    def host_t(self) -> np.ndarray:
        return _host16(self.t)

    def host_dA(self) -> np.ndarray:
        return self.dA.cpu().numpy()

    def host_dB(self) -> np.ndarray:
        return self.dB.cpu().numpy()


class ActOrderLayer(DeviceLayer):
    """A projection whose checkpoint was quantized in activation order (per-column group index g_idx).

    `inp.codes`, `inp.x` and the returned dX are in the checkpoint's column order; scales and zeros are indexed by
    group as always; the adapter A is held in the sorted column order.  Load time: columns sorted by group and packed.
    Run time: x gathered into the sorted order before the forward call, dX gathered back after the backward call.
    """

    def __init__(self, inp: LayerInputs, g_idx: np.ndarray, device: str = "cuda:0"):
        super().__init__(inp, device=device)
        c = self.cfg
        g_idx = np.ascontiguousarray(g_idx, dtype=np.int32)
        perm = np.empty(c.K, dtype=np.int32)
        inv = np.empty(c.K, dtype=np.int32)
        ql.qlora_actorder_perm(g_idx, perm, inv, c.K, c.group_size)
        self.perm = _dev(perm, self.device)
        self.inv_perm = _dev(inv, self.device)
        ql.qlora_pack_permuted(self.codes, self.perm, self.packed, c.N, c.K, c.bits)
        self.x_checkpoint_order = self.x
        self.x = torch.empty_like(self.x_checkpoint_order)
        self.dx_checkpoint_order = torch.empty_like(self.dx)

    def forward(self, save_t: bool = True, stream=None):
        c = self.cfg
        ql.qlora_gather_columns(self.x_checkpoint_order, self.perm, self.x, c.M, c.K, stream=stream)
        super().forward(save_t=save_t, stream=stream)

    def backward(self, use_saved_t: bool = True, stream=None):
        c = self.cfg
        if getattr(self, "packed_zeros", None) is not None:
            return self.backward_accumulate(0.0, use_saved_t, stream)
        super().backward(use_saved_t=use_saved_t, stream=stream)
        ql.qlora_gather_columns(self.dx, self.inv_perm, self.dx_checkpoint_order, c.M, c.K, stream=stream)

    def host_dx(self) -> np.ndarray:
        return _host16(self.dx_checkpoint_order)


class DeviceSiblings:
    """Several projections that read the same x (q/k/v, gate/up), called together through the sibling entry points.

    Built from DeviceLayer objects of equal M, K, bits, group size, rank, alpha and dtype; the first one's x is the
    shared input.  dx receives the sum of the projections' dX.
    """

    def __init__(self, layers):
        c0 = layers[0].cfg
        for l in layers[1:]:
            c = l.cfg
            if (c.M, c.K, c.bits, c.group_size, c.rank, c.alpha, c.dtype) != (c0.M, c0.K, c0.bits, c0.group_size,
                                                                              c0.rank, c0.alpha, c0.dtype):
                raise ValueError("sibling projections must share everything but N")
        self.layers = list(layers)
        self.cfg = c0
        self.N = [l.cfg.N for l in layers]
        self.x = layers[0].x
        self.dx = torch.empty((c0.M, c0.K), dtype=torch.int16, device=layers[0].device)
        nbytes = ql.qlora_siblings_workspace_bytes(self.N, c0.M, c0.K, c0.bits, c0.group_size, c0.rank)
        if nbytes == 0:
            raise ValueError(f"shapes not accepted by the sibling entry points: {self.N}, {c0}")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=layers[0].device)

    def _each(self, name):
        return [getattr(l, name) for l in self.layers]

    def forward(self, save_t: bool = True, stream=None):
        c = self.cfg
        ql.qlora_linear_fwd_siblings(self.x, self._each("packed"), self._each("scales"), self._each("zeros"),
                                     self._each("A") if c.rank else None, self._each("B") if c.rank else None,
                                     self._each("y"), self._each("t") if (save_t and c.rank) else None, self.N,
                                     c.M, c.K, c.bits, c.group_size, c.rank, c.alpha, self.layers[0].dtype_flag,
                                     self.workspace, stream=stream)

    def backward(self, use_saved_t: bool = True, stream=None):
        c = self.cfg
        if getattr(self, "packed_zeros", None) is not None:
            return self.backward_accumulate(0.0, use_saved_t, stream)
        ql.qlora_linear_bwd_siblings(self._each("dy"), self.x, self._each("packed"), self._each("scales"),
                                     self._each("zeros"), self._each("A") if c.rank else None,
                                     self._each("B") if c.rank else None,
                                     self._each("t") if (use_saved_t and c.rank) else None, self.dx,
                                     self._each("dA") if c.rank else None, self._each("dB") if c.rank else None,
                                     self.N, c.M, c.K, c.bits, c.group_size, c.rank, c.alpha,
                                     self.layers[0].dtype_flag, self.workspace, stream=stream)

    def host_dx(self) -> np.ndarray:
        return _host16(self.dx)
