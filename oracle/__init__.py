"""ctypes front end of the fp64 CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of
`bench.py` may import this package.  It shares nothing with the HIP library:
its arithmetic lives in `qlora_oracle.c` (plain C, fp64), this file only
widens 16-bit inputs to double (exactly) and marshals numpy arrays.

Paper passages each entry follows are cited in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qlora_oracle.c")
_LIB = os.path.join(_HERE, "libqlora_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.qo_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().qo_num_threads())


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _l(v) -> ctypes.c_long:
    return ctypes.c_long(int(v))


def widen(bits16: np.ndarray, dtype: str) -> np.ndarray:
    """Exact conversion of raw fp16 / bf16 bit patterns (uint16) to float64."""
    b = np.ascontiguousarray(bits16, dtype=np.uint16)
    if dtype == "f16":
        return b.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


# ------------------------------------------------------------------ codes

def pack(codes: np.ndarray, bits: int) -> np.ndarray:
    codes = _c(codes, np.uint8)
    N, K = codes.shape
    assert (K * bits) % 32 == 0
    P = np.empty((N, K * bits // 32), dtype=np.uint32)
    _load().qo_pack(_p(codes), _p(P), _l(N), _l(K), ctypes.c_int(bits))
    return P


def unpack(P: np.ndarray, K: int, bits: int) -> np.ndarray:
    P = _c(P, np.uint32)
    N = P.shape[0]
    assert P.shape[1] == K * bits // 32
    codes = np.empty((N, K), dtype=np.uint8)
    _load().qo_unpack(_p(P), _p(codes), _l(N), _l(K), ctypes.c_int(bits))
    return codes


def dequant(P: np.ndarray, scales: np.ndarray, zeros: np.ndarray, K: int, bits: int, G: int) -> np.ndarray:
    """Wd [N,K] float64.  `scales` float64 [N,K/G], `zeros` uint8 [N,K/G]."""
    P = _c(P, np.uint32)
    s = _c(scales, np.float64)
    z = _c(zeros, np.uint8)
    N = P.shape[0]
    assert s.shape == (N, K // G) and z.shape == (N, K // G) and K % G == 0
    Wd = np.empty((N, K), dtype=np.float64)
    _load().qo_dequant(_p(P), _p(s), _p(z), _p(Wd), _l(N), _l(K), ctypes.c_int(bits), _l(G))
    return Wd


def zero_words(groups: int, bits: int) -> int:
    """Words per row of the packed zero-points: the row's bit stream rounded up to whole 32-bit words."""
    return (groups * bits + 31) // 32


def pack_zeros(zeros: np.ndarray, bits: int) -> np.ndarray:
    """Zero-points [N, groups] (uint8, each < 2^bits) as checkpoints store them: `bits` wide, bit-packed per row in
    group order with the same little-endian stream as the codes (Sec. 3.1), the last word zero-padded."""
    z = _c(zeros, np.uint8)
    N, groups = z.shape
    per_word_run = 32                      # 32 fields of any width fill whole words
    padded = (groups + per_word_run - 1) // per_word_run * per_word_run
    zp = np.zeros((N, padded), dtype=np.uint8)
    zp[:, :groups] = z
    return np.ascontiguousarray(pack(zp, bits)[:, :zero_words(groups, bits)])


def unpack_zeros(packed_zeros: np.ndarray, groups: int, bits: int) -> np.ndarray:
    P = _c(packed_zeros, np.uint32)
    N = P.shape[0]
    padded = (groups + 31) // 32 * 32
    full = np.zeros((N, padded * bits // 32), dtype=np.uint32)
    full[:, :P.shape[1]] = P
    return np.ascontiguousarray(unpack(full, padded, bits)[:, :groups])


# ------------------------------------------- activation-order checkpoints

def dequant_actorder(codes: np.ndarray, scales: np.ndarray, zeros: np.ndarray, g_idx: np.ndarray) -> np.ndarray:
    """Wd[n,k] = s[n, g_idx[k]] * (q[n,k] - z[n, g_idx[k]]) in float64.

    Eq. 1 with the per-column group index a GPTQ checkpoint quantized with the
    "activation order" option carries (App. A): the columns of one group are no
    longer a run of consecutive columns.  Plain definition, numpy indexing only.
    """
    q = _c(codes, np.uint8).astype(np.float64)
    s = _c(scales, np.float64)
    z = _c(zeros, np.uint8).astype(np.float64)
    g = _c(g_idx, np.int64)
    assert q.shape[1] == g.shape[0] and s.shape == z.shape and s.shape[0] == q.shape[0]
    return s[:, g] * (q - z[:, g])


def actorder_perm(g_idx: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Stable sort of the columns by group: perm[j] = column that moves to place j, and its inverse."""
    g = _c(g_idx, np.int64)
    perm = np.argsort(g, kind="stable").astype(np.int32)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size, dtype=np.int32)
    return perm, inv


# ------------------------------------------------------------ layer passes

def lora_down(x: np.ndarray, A: np.ndarray) -> np.ndarray:
    x = _c(x, np.float64)
    A = _c(A, np.float64)
    M, K = x.shape
    r = A.shape[0]
    t = np.zeros((M, r), dtype=np.float64)
    if r:
        _load().qo_lora_down(_p(x), _p(A), _p(t), _l(M), _l(K), _l(r))
    return t


def lora_u(dy: np.ndarray, B: np.ndarray) -> np.ndarray:
    dy = _c(dy, np.float64)
    B = _c(B, np.float64)
    M, N = dy.shape
    r = B.shape[1]
    u = np.zeros((M, r), dtype=np.float64)
    if r:
        _load().qo_lora_u(_p(dy), _p(B), _p(u), _l(M), _l(N), _l(r))
    return u


def forward(x, Wd, A, B, alpha: float) -> Tuple[np.ndarray, np.ndarray]:
    """y [M,N] and t = x A^T [M,r], all float64.  Rows of x are independent."""
    x = _c(x, np.float64)
    Wd = _c(Wd, np.float64)
    A = _c(A, np.float64)
    B = _c(B, np.float64)
    M, K = x.shape
    N = Wd.shape[0]
    r = A.shape[0]
    assert Wd.shape == (N, K) and A.shape == (r, K) and B.shape == (N, r)
    t = lora_down(x, A)
    y = np.empty((M, N), dtype=np.float64)
    _load().qo_forward(_p(x), _p(Wd), _p(t), _p(B), ctypes.c_double(alpha), _p(y),
                       _l(M), _l(N), _l(K), _l(r))
    return y, t


def backward_dx(dy, Wd, A, B, alpha: float) -> np.ndarray:
    """dX [M,K] float64.  Rows of dY are independent."""
    dy = _c(dy, np.float64)
    Wd = _c(Wd, np.float64)
    A = _c(A, np.float64)
    B = _c(B, np.float64)
    M, N = dy.shape
    K = Wd.shape[1]
    r = A.shape[0]
    assert Wd.shape == (N, K) and A.shape == (r, K) and B.shape == (N, r)
    u = lora_u(dy, B)
    dx = np.empty((M, K), dtype=np.float64)
    _load().qo_backward_dx(_p(dy), _p(Wd), _p(u), _p(A), ctypes.c_double(alpha), _p(dx),
                           _l(M), _l(N), _l(K), _l(r))
    return dx


def backward_adapters(dy, x, A, B, alpha: float) -> Tuple[np.ndarray, np.ndarray]:
    """(dA [r,K], dB [N,r]) float64; needs every row m (sums over tokens)."""
    dy = _c(dy, np.float64)
    x = _c(x, np.float64)
    A = _c(A, np.float64)
    B = _c(B, np.float64)
    M, N = dy.shape
    K = x.shape[1]
    r = A.shape[0]
    assert x.shape == (M, K) and A.shape == (r, K) and B.shape == (N, r)
    t = lora_down(x, A)
    u = lora_u(dy, B)
    dA = np.zeros((r, K), dtype=np.float64)
    dB = np.zeros((N, r), dtype=np.float64)
    if r:
        _load().qo_backward_adapters(_p(dy), _p(x), _p(t), _p(u), ctypes.c_double(alpha),
                                     _p(dA), _p(dB), _l(M), _l(N), _l(K), _l(r))
    return dA, dB


def backward_adapters_stacked(dy, x, A, B, alpha: float, frozen_rank: int) -> Tuple[np.ndarray, np.ndarray]:
    """Stacked adapters (App. D: a recovery adapter trained by LREC stays on the layer, frozen, while a second pair is
    trained on the task): A = [A_frozen; A_train] (r rows), B = [B_frozen, B_train] (r columns), scaling alpha / r
    for the whole stack.  Only the trainable pair has gradients: the rows frozen_rank.. of dA and the columns
    frozen_rank.. of dB of the full-stack gradient; dX is that of the full stack.  Returns (dA_train [r-f, K],
    dB_train [N, r-f])."""
    dA, dB = backward_adapters(dy, x, A, B, alpha)
    return np.ascontiguousarray(dA[frozen_rank:, :]), np.ascontiguousarray(dB[:, frozen_rank:])


# ------------------------------------------------------------ LoRA dropout
# Appendix B trains with a dropout rate of 0.05.  Reading: as in the LoRA method the paper builds on, dropout acts on
# the input of the low-rank branch only, with inverted scaling; the frozen quantized path sees x itself:
#     x~ = x * keep * keep_scale   (keep in {0,1} per element of x, keep_scale = 1 / (1 - p))
#     y  = x Wd^T + sc (x~ A^T) B^T
#     dX = dY Wd + (sc (dY B) A) * keep * keep_scale,   dA = sc (dY B)^T x~,   dB = sc dY^T (x~ A^T)
# The mask is an input (the caller draws it); the functions below are the plain ones applied to x~ where x~ stands.

def forward_dropout(x, Wd, A, B, alpha: float, keep, keep_scale: float) -> Tuple[np.ndarray, np.ndarray]:
    x = _c(x, np.float64)
    xt = x * _c(keep, np.float64) * float(keep_scale)
    base, _ = forward(x, Wd, np.zeros_like(_c(A, np.float64)), B, alpha)          # x Wd^T
    lora, t = forward(xt, np.zeros_like(_c(Wd, np.float64)), A, B, alpha)         # sc (x~ A^T) B^T
    return base + lora, t


def backward_dx_dropout(dy, Wd, A, B, alpha: float, keep, keep_scale: float) -> np.ndarray:
    Wd = _c(Wd, np.float64)
    base = backward_dx(dy, Wd, A, np.zeros_like(_c(B, np.float64)), alpha)        # dY Wd
    lora = backward_dx(dy, np.zeros_like(Wd), A, B, alpha)                         # sc (dY B) A
    return base + lora * _c(keep, np.float64) * float(keep_scale)


def backward_adapters_dropout(dy, x, A, B, alpha: float, keep, keep_scale: float) -> Tuple[np.ndarray, np.ndarray]:
    xt = _c(x, np.float64) * _c(keep, np.float64) * float(keep_scale)
    return backward_adapters(dy, xt, A, B, alpha)


class LayerOracle:
    """The layer on one set of stored inputs (raw 16-bit patterns + codes).

    Widening and dequantisation are done once; forward / backward can then be
    asked for any subset of token rows.
    """

    def __init__(self, codes, scales_f16_bits, zeros, A_bits, B_bits, *, bits: int, group_size: int,
                 alpha: float, dtype: str):
        codes = _c(codes, np.uint8)
        self.N, self.K = codes.shape
        self.bits, self.G, self.alpha, self.dtype = bits, group_size, float(alpha), dtype
        self.P = pack(codes, bits)
        self.s = widen(scales_f16_bits, "f16")
        self.z = _c(zeros, np.uint8)
        self.Wd = dequant(self.P, self.s, self.z, self.K, bits, group_size)
        self.A = widen(A_bits, dtype).reshape(-1, self.K)
        self.B = widen(B_bits, dtype).reshape(self.N, -1)
        self.r = self.A.shape[0]

    def forward(self, x_bits, rows: Optional[np.ndarray] = None):
        x = widen(x_bits if rows is None else np.asarray(x_bits)[rows], self.dtype)
        return forward(x, self.Wd, self.A, self.B, self.alpha)

    def backward_dx(self, dy_bits, rows: Optional[np.ndarray] = None):
        dy = widen(dy_bits if rows is None else np.asarray(dy_bits)[rows], self.dtype)
        return backward_dx(dy, self.Wd, self.A, self.B, self.alpha)

    def backward_adapters(self, dy_bits, x_bits):
        return backward_adapters(widen(dy_bits, self.dtype), widen(x_bits, self.dtype),
                                 self.A, self.B, self.alpha)

    # the same with LoRA dropout (keep: {0,1} [M,K] for the rows asked for, keep_scale = 1 / (1 - p))
    def forward_dropout(self, x_bits, keep, keep_scale: float, rows: Optional[np.ndarray] = None):
        x = widen(x_bits if rows is None else np.asarray(x_bits)[rows], self.dtype)
        k = keep if rows is None else np.asarray(keep)[rows]
        return forward_dropout(x, self.Wd, self.A, self.B, self.alpha, k, keep_scale)

    def backward_dx_dropout(self, dy_bits, keep, keep_scale: float, rows: Optional[np.ndarray] = None):
        dy = widen(dy_bits if rows is None else np.asarray(dy_bits)[rows], self.dtype)
        k = keep if rows is None else np.asarray(keep)[rows]
        return backward_dx_dropout(dy, self.Wd, self.A, self.B, self.alpha, k, keep_scale)

    def backward_adapters_dropout(self, dy_bits, x_bits, keep, keep_scale: float):
        return backward_adapters_dropout(widen(dy_bits, self.dtype), widen(x_bits, self.dtype), self.A, self.B,
                                         self.alpha, keep, keep_scale)
