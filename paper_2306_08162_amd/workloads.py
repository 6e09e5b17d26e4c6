"""Seeded synthetic inputs for the quantized LoRA linear layer.

This module only draws numbers. It holds none of the layer's arithmetic (no
packing, no dequantisation, no matrix products) so that the CPU oracle and the
HIP library can both be fed from it without sharing any code of the method.

Every tensor is a pure function of (seed, element index): a counter-based
splitmix64 stream, so a slice of a big tensor can be regenerated on its own and
the bytes do not depend on the platform or on numpy's global RNG.

Shapes and value ranges stand in for the workloads of the paper's experiments:
LLaMA-7B projection shapes (Experimental Setup), GPTQ-style grouped affine
quantisation with group size 128 (Appendix B, "Quantization Parameters") and
LoRA pairs with r = 8 and a linear stretch of 16 (Appendix B, "Adaptation
Parameters").  The real tensors (LLaMA weights, GPTQ checkpoints, Alpaca / C4
activations) are not available; uniform codes and N(0,1) activations replace
them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

BASE_SEED = 0x230608162000

# tensor ids (added to the per-config seed)
T_CODES, T_SCALES, T_ZEROS, T_A, T_B, T_X, T_DY = range(7)
T_GIDX = 11


def splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    """uint64[count]: element i is the splitmix64 output for counter start+i."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + 1 + count, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, start: int, count: int) -> np.ndarray:
    """float64 in [0, 1) with 53 random bits."""
    return (splitmix64(seed, start, count) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def uniform_ints(seed: int, count: int, n_values: int, start: int = 0) -> np.ndarray:
    """uint8[count], uniform in [0, n_values) (n_values <= 256)."""
    hi = splitmix64(seed, start, count) >> np.uint64(32)
    return ((hi * np.uint64(n_values)) >> np.uint64(32)).astype(np.uint8)


def uniform_range(seed: int, count: int, lo: float, hi: float, start: int = 0) -> np.ndarray:
    return lo + (hi - lo) * uniform01(seed, start, count)


def normal(seed: int, count: int, std: float = 1.0, start: int = 0) -> np.ndarray:
    """float64[count] ~ N(0, std^2) by Box-Muller; element i uses counters 2i, 2i+1."""
    u = uniform01(seed, 2 * start, 2 * count)
    u1 = 1.0 - u[0::2]          # (0, 1]
    u2 = u[1::2]
    return std * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def to_f16_bits(v: np.ndarray) -> np.ndarray:
    """Round fp64 values once (RNE) to IEEE half; returned as raw uint16 bits."""
    return v.astype(np.float16).view(np.uint16)


def to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (RNE on the fp32 image); returned as raw uint16 bits."""
    f = v.astype(np.float32).view(np.uint32)
    bias = ((f >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((f + bias) >> np.uint32(16)).astype(np.uint16)


def to_bits(v: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f16":
        return to_f16_bits(v)
    if dtype == "bf16":
        return to_bf16_bits(v)
    raise ValueError(dtype)


@dataclass(frozen=True)
class LayerConfig:
    """One quantized-LoRA linear problem."""
    name: str
    cfg_id: int          # seed offset
    M: int               # tokens
    K: int               # in features
    N: int               # out features
    bits: int            # 2, 3, 4 or 8
    group_size: int      # along K
    rank: int
    alpha: float
    dtype: str           # "f16" | "bf16" for x, dY, A, B, y, dX
    scale_lo: float
    scale_hi: float

    @property
    def seed(self) -> int:
        return BASE_SEED + 16 * self.cfg_id

    @property
    def groups(self) -> int:
        return self.K // self.group_size

    @property
    def words_per_row(self) -> int:
        return self.K * self.bits // 32

    @property
    def flops_fwd_bwd(self) -> int:
        """Counted work of one forward plus one backward (dequantisation not counted)."""
        return 4 * self.M * self.N * self.K + 6 * self.M * self.rank * (self.K + self.N)

    @property
    def weight_side_bytes(self) -> int:
        """Packed codes + fp16 scales + uint8 zeros: what one pass must stream."""
        return self.N * self.K * self.bits // 8 + 3 * self.N * self.groups

    def with_tokens(self, M: int) -> "LayerConfig":
        return replace(self, M=M, name=f"{self.name}_M{M}")


@dataclass
class LayerInputs:
    cfg: LayerConfig
    codes: np.ndarray    # uint8  [N, K]   integer codes in [0, 2^bits)
    scales: np.ndarray   # uint16 [N, K/G] fp16 bits
    zeros: np.ndarray    # uint8  [N, K/G] zero-point codes
    A: np.ndarray        # uint16 [r, K]   16-bit float bits (cfg.dtype)
    B: np.ndarray        # uint16 [N, r]
    x: np.ndarray        # uint16 [M, K]
    dy: np.ndarray       # uint16 [M, N]


def make_inputs(cfg: LayerConfig) -> LayerInputs:
    s = cfg.seed
    nq = 1 << cfg.bits
    codes = uniform_ints(s + T_CODES, cfg.N * cfg.K, nq).reshape(cfg.N, cfg.K)
    scales = to_f16_bits(uniform_range(s + T_SCALES, cfg.N * cfg.groups, cfg.scale_lo, cfg.scale_hi))
    zeros = uniform_ints(s + T_ZEROS, cfg.N * cfg.groups, nq)
    r = max(cfg.rank, 0)
    A = to_bits(normal(s + T_A, r * cfg.K, std=cfg.K ** -0.5), cfg.dtype)
    B = to_bits(normal(s + T_B, cfg.N * r, std=0.1), cfg.dtype)
    x = to_bits(normal(s + T_X, cfg.M * cfg.K), cfg.dtype)
    dy = to_bits(normal(s + T_DY, cfg.M * cfg.N), cfg.dtype)
    return LayerInputs(
        cfg=cfg,
        codes=codes,
        scales=scales.reshape(cfg.N, cfg.groups),
        zeros=zeros.reshape(cfg.N, cfg.groups),
        A=A.reshape(r, cfg.K),
        B=B.reshape(cfg.N, r),
        x=x.reshape(cfg.M, cfg.K),
        dy=dy.reshape(cfg.M, cfg.N),
    )


def actorder_g_idx(seed: int, K: int, G: int) -> np.ndarray:
    """Per-column group index of a checkpoint quantized in activation order (App. A): the columns are visited in a
    data-dependent order (here a seeded random one) and every G consecutive visits form a group.  int32 [K]."""
    keys = splitmix64(seed + T_GIDX, 0, K)
    order = np.argsort(keys, kind="stable")          # order[i] = column visited i-th
    g_idx = np.empty(K, dtype=np.int32)
    g_idx[order] = (np.arange(K) // G).astype(np.int32)
    return g_idx


# --- the named workloads ---------------------------------------------------

def config1() -> LayerConfig:
    """Small layer the oracle finishes in well under a second."""
    return LayerConfig("c1_small", 1, M=64, K=256, N=256, bits=4, group_size=64, rank=8,
                       alpha=16.0, dtype="f16", scale_lo=0.005, scale_hi=0.02)


def config2() -> LayerConfig:
    """LLaMA-7B q_proj, batch 4 x seq 512, INT4: the headline workload."""
    return LayerConfig("c2_qproj_int4", 2, M=2048, K=4096, N=4096, bits=4, group_size=128, rank=8,
                       alpha=16.0, dtype="f16", scale_lo=0.002, scale_hi=0.02)


def config3() -> LayerConfig:
    """LLaMA-7B gate/up_proj, INT2, bf16 activations, r = 16."""
    return LayerConfig("c3_gateup_int2", 3, M=2048, K=4096, N=11008, bits=2, group_size=128, rank=16,
                       alpha=32.0, dtype="bf16", scale_lo=0.01, scale_hi=0.05)


def config4() -> LayerConfig:
    """LLaMA-7B down_proj, INT3 bit stream, batch 8 x seq 512."""
    return LayerConfig("c4_down_int3", 4, M=4096, K=11008, N=4096, bits=3, group_size=128, rank=8,
                       alpha=16.0, dtype="f16", scale_lo=0.005, scale_hi=0.03)


_BLOCK_SHAPES = [  # (name, K, N) of the seven projections of one LLaMA-7B decoder block
    ("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
    ("gate", 4096, 11008), ("up", 4096, 11008), ("down", 11008, 4096),
]


def config5(bits: int, M: int) -> List[LayerConfig]:
    """All seven projections of one decoder block at `bits` in {2, 8} and M tokens.

    Scales are U[0.01, 0.05] * 3 / (2^bits - 1) so the dequantised weights have
    the same spread at both widths.
    """
    f = 3.0 / ((1 << bits) - 1)
    out = []
    for i, (nm, K, N) in enumerate(_BLOCK_SHAPES):
        out.append(LayerConfig(f"c5_{nm}_int{bits}_M{M}", 5 + 8 * (bits == 8) + i, M=M, K=K, N=N,
                               bits=bits, group_size=128, rank=8, alpha=16.0, dtype="f16",
                               scale_lo=0.01 * f, scale_hi=0.05 * f))
    return out


def named_configs() -> Dict[str, LayerConfig]:
    return {c.name: c for c in (config1(), config2(), config3(), config4())}
