"""Thin ctypes binding of libqlora.so: argument marshalling only.

Function names and argument order mirror `include/qlora.h`.  Tensors are torch
tensors used as plain device buffers (torch supplies memory and the stream, all
arithmetic runs in the HIP kernels).  There is no fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libqlora.so")

QLORA_F16, QLORA_BF16 = 0, 1
STATUS_NAMES = ["QLORA_OK", "QLORA_E_NULL", "QLORA_E_BITS", "QLORA_E_SHAPE", "QLORA_E_GROUP", "QLORA_E_RANK",
                "QLORA_E_DTYPE", "QLORA_E_ALIGN", "QLORA_E_WORKSPACE", "QLORA_E_HIP", "QLORA_E_GIDX", "QLORA_E_STATIC"]
STATIC_SCRATCH_BYTES = 32 << 20
EXPORTS = ["qlora_status_string", "qlora_packed_words", "qlora_workspace_bytes", "qlora_pack", "qlora_unpack",
           "qlora_actorder_perm", "qlora_pack_permuted", "qlora_gather_columns",
           "qlora_packed_zero_words", "qlora_pack_zeros", "qlora_unpack_zeros",
           "qlora_linear_fwd", "qlora_linear_bwd", "qlora_linear_bwd_accumulate", "qlora_linear_fwd_dropout",
           "qlora_linear_bwd_dropout", "qlora_linear_bwd_stacked", "qlora_linear_bwd_dropout_stacked", "qlora_siblings_workspace_bytes", "qlora_linear_fwd_siblings",
           "qlora_linear_bwd_siblings", "qlora_lrec_workspace_bytes", "qlora_lrec_loss", "qlora_lrec_loss_scaled", "qlora_linear_fwd_static",
           "qlora_workspace_bytes_zp", "qlora_linear_fwd_zp", "qlora_linear_bwd_zp"]
BENCH_EXPORTS = ["qlora_profile_gemm", "qlora_profile_gemm_span", "qlora_stream_probe", "qlora_mfma_probe"]        # include/qlora_bench.h
STREAM_PROBE_WORDS = 1024
MFMA_PROBE_FLOATS = 256 * 512              # floats of the probe's output
MFMA_PROBE_FLOP_PER_ITER = 256 * 8 * 8 * 32768   # per round: workgroups x waves x MFMAs x flop of a 32x32x16 MFMA
MAX_SIBLINGS, SIBLINGS_MAX_M = 4, 16

_lib = None


class QLoraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{where}: {name}: {status_string(status)}")


def load() -> ctypes.CDLL:
    """Load libqlora.so (building it first only if it is not there)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2306_08162_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_sz, vp, f32 = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_float
    lib.qlora_status_string.restype = ctypes.c_char_p
    lib.qlora_status_string.argtypes = [c_int]
    lib.qlora_packed_words.restype = c_sz
    lib.qlora_packed_words.argtypes = [c_int] * 3
    lib.qlora_workspace_bytes.restype = c_sz
    lib.qlora_workspace_bytes.argtypes = [c_int] * 6
    lib.qlora_pack.restype = c_int
    lib.qlora_pack.argtypes = [vp, vp, c_int, c_int, c_int, vp]
    lib.qlora_unpack.restype = c_int
    lib.qlora_unpack.argtypes = [vp, vp, c_int, c_int, c_int, vp]
    lib.qlora_packed_zero_words.restype = c_sz
    lib.qlora_packed_zero_words.argtypes = [c_int, c_int, c_int]
    lib.qlora_pack_zeros.restype = c_int
    lib.qlora_pack_zeros.argtypes = [vp, vp, c_int, c_int, c_int, vp]
    lib.qlora_unpack_zeros.restype = c_int
    lib.qlora_unpack_zeros.argtypes = [vp, vp, c_int, c_int, c_int, vp]
    lib.qlora_actorder_perm.restype = c_int
    lib.qlora_actorder_perm.argtypes = [vp, vp, vp, c_int, c_int]
    lib.qlora_pack_permuted.restype = c_int
    lib.qlora_pack_permuted.argtypes = [vp, vp, vp, c_int, c_int, c_int, vp]
    lib.qlora_gather_columns.restype = c_int
    lib.qlora_gather_columns.argtypes = [vp, vp, vp, c_int, c_int, vp]
    lib.qlora_linear_fwd.restype = c_int
    lib.qlora_linear_fwd.argtypes = [vp] * 8 + [c_int] * 6 + [f32, c_int, vp, c_sz, vp]
    lib.qlora_linear_bwd.restype = c_int
    lib.qlora_linear_bwd.argtypes = [vp] * 11 + [c_int] * 6 + [f32, c_int, vp, c_sz, vp]
    lib.qlora_linear_fwd_static.restype = c_int
    lib.qlora_linear_fwd_static.argtypes = [vp] * 8 + [c_int] * 6 + [f32, c_int, vp]
    lib.qlora_profile_gemm.restype = c_int
    lib.qlora_profile_gemm.argtypes = [vp, vp]
    lib.qlora_profile_gemm_span.restype = c_int
    lib.qlora_profile_gemm_span.argtypes = [c_int]
    lib.qlora_stream_probe.restype = c_int
    lib.qlora_stream_probe.argtypes = [vp, ctypes.c_ulonglong, vp, vp]
    lib.qlora_mfma_probe.restype = c_int
    lib.qlora_mfma_probe.argtypes = [vp, c_int, c_int, vp]
    lib.qlora_workspace_bytes_zp.restype = c_sz
    lib.qlora_workspace_bytes_zp.argtypes = [c_int] * 6
    lib.qlora_linear_fwd_zp.restype = c_int
    lib.qlora_linear_fwd_zp.argtypes = lib.qlora_linear_fwd.argtypes
    lib.qlora_linear_bwd_zp.restype = c_int
    lib.qlora_linear_bwd_zp.argtypes = [vp] * 11 + [f32] + [c_int] * 6 + [f32, c_int, vp, c_sz, vp]
    lib.qlora_linear_bwd_accumulate.restype = c_int
    lib.qlora_linear_bwd_accumulate.argtypes = [vp] * 11 + [f32] + [c_int] * 6 + [f32, c_int, vp, c_sz, vp]
    lib.qlora_linear_fwd_dropout.restype = c_int
    lib.qlora_linear_fwd_dropout.argtypes = [vp] * 7 + [f32] + [vp] * 2 + [c_int] * 6 + [f32, c_int, vp, c_sz, vp]
    lib.qlora_linear_bwd_dropout.restype = c_int
    lib.qlora_linear_bwd_dropout.argtypes = [vp] * 8 + [f32] + [vp] * 4 + [f32] + [c_int] * 6 + [f32, c_int, vp, c_sz, vp]
    lib.qlora_linear_bwd_stacked.restype = c_int
    lib.qlora_linear_bwd_stacked.argtypes = [vp] * 11 + [f32, c_int] + [c_int] * 6 + [f32, c_int, vp, c_sz, vp]
    lib.qlora_linear_bwd_dropout_stacked.restype = c_int
    lib.qlora_linear_bwd_dropout_stacked.argtypes = ([vp] * 8 + [f32] + [vp] * 4 + [f32, c_int] + [c_int] * 6 +
                                                     [f32, c_int, vp, c_sz, vp])
    lib.qlora_siblings_workspace_bytes.restype = c_sz
    lib.qlora_siblings_workspace_bytes.argtypes = [c_int, vp] + [c_int] * 5
    lib.qlora_linear_fwd_siblings.restype = c_int
    lib.qlora_linear_fwd_siblings.argtypes = [c_int] + [vp] * 9 + [c_int] * 5 + [f32, c_int, vp, c_sz, vp]
    lib.qlora_linear_bwd_siblings.restype = c_int
    lib.qlora_linear_bwd_siblings.argtypes = [c_int] + [vp] * 12 + [c_int] * 5 + [f32, c_int, vp, c_sz, vp]
    lib.qlora_lrec_workspace_bytes.restype = c_sz
    lib.qlora_lrec_workspace_bytes.argtypes = [c_int]
    lib.qlora_lrec_loss.restype = c_int
    lib.qlora_lrec_loss.argtypes = [vp] * 3 + [f32, f32] + [vp] * 4 + [c_int] * 3 + [vp, c_sz, vp]
    lib.qlora_lrec_loss_scaled.restype = c_int
    lib.qlora_lrec_loss_scaled.argtypes = [vp] * 3 + [f32, f32, f32] + [vp] * 4 + [c_int] * 3 + [vp, c_sz, vp]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device (or raw integer) pointer of a buffer; None stays NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("qlora buffers must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def status_string(status: int) -> str:
    return load().qlora_status_string(int(status)).decode()


def qlora_packed_words(N: int, K: int, bits: int) -> int:
    return int(load().qlora_packed_words(N, K, bits))


def qlora_workspace_bytes(M: int, N: int, K: int, bits: int, group_size: int, rank: int) -> int:
    return int(load().qlora_workspace_bytes(M, N, K, bits, group_size, rank))


def qlora_profile_gemm(ev_before: Optional[int], ev_after: Optional[int]) -> int:
    """Set (or clear with None, None) the raw hipEvent_t handles recorded around the GEMM kernel."""
    return int(load().qlora_profile_gemm(ev_before, ev_after))


def qlora_profile_gemm_span(span: int) -> int:
    """0: the events enclose the GEMM alone; 1: the adapter kernel before it and the GEMM; 2: that kernel alone."""
    return int(load().qlora_profile_gemm_span(span))


def qlora_stream_probe(src, nbytes: int, out, stream=None, check: bool = True) -> int:
    """STREAM_PROBE_WORDS partial exclusive-ors of the 32-bit words of `nbytes` bytes at src: a kernel that only
    streams the buffer."""
    st = load().qlora_stream_probe(_ptr(src), nbytes, _ptr(out), _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_stream_probe")
    return st


def qlora_mfma_probe(out, iters: int, random: bool, stream=None, check: bool = True) -> int:
    """Register-resident MFMAs and nothing else (MFMA_PROBE_FLOP_PER_ITER flop per round); out: MFMA_PROBE_FLOATS floats."""
    st = load().qlora_mfma_probe(_ptr(out), iters, 1 if random else 0, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_mfma_probe")
    return st


def qlora_pack(codes, packed, N: int, K: int, bits: int, stream=None, check: bool = True) -> int:
    st = load().qlora_pack(_ptr(codes), _ptr(packed), N, K, bits, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_pack")
    return st


def qlora_unpack(packed, codes, N: int, K: int, bits: int, stream=None, check: bool = True) -> int:
    st = load().qlora_unpack(_ptr(packed), _ptr(codes), N, K, bits, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_unpack")
    return st


def qlora_packed_zero_words(N: int, groups: int, bits: int) -> int:
    return int(load().qlora_packed_zero_words(N, groups, bits))


def qlora_pack_zeros(zeros, packed_zeros, N: int, groups: int, bits: int, stream=None, check: bool = True) -> int:
    st = load().qlora_pack_zeros(_ptr(zeros), _ptr(packed_zeros), N, groups, bits, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_pack_zeros")
    return st


def qlora_unpack_zeros(packed_zeros, zeros, N: int, groups: int, bits: int, stream=None, check: bool = True) -> int:
    st = load().qlora_unpack_zeros(_ptr(packed_zeros), _ptr(zeros), N, groups, bits, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_unpack_zeros")
    return st


def qlora_actorder_perm(g_idx, perm, inv_perm, K: int, group_size: int, check: bool = True) -> int:
    """Host arrays (numpy int32, or None): stable sort of the columns by group and its inverse."""
    def host(a):
        return None if a is None else a.ctypes.data_as(ctypes.c_void_p)
    st = load().qlora_actorder_perm(host(g_idx), host(perm), host(inv_perm), K, group_size)
    if check and st != 0:
        raise QLoraError(st, "qlora_actorder_perm")
    return st


def qlora_pack_permuted(codes, perm, packed, N: int, K: int, bits: int, stream=None, check: bool = True) -> int:
    st = load().qlora_pack_permuted(_ptr(codes), _ptr(perm), _ptr(packed), N, K, bits, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_pack_permuted")
    return st


def qlora_gather_columns(src, index, dst, M: int, K: int, stream=None, check: bool = True) -> int:
    st = load().qlora_gather_columns(_ptr(src), _ptr(index), _ptr(dst), M, K, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_gather_columns")
    return st


def qlora_linear_fwd(x, packed, scales, zeros, A, B, y, t_save, M: int, N: int, K: int, bits: int, group_size: int,
                     rank: int, alpha: float, dtype: int, workspace, workspace_bytes: Optional[int] = None,
                     stream=None, check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_fwd(_ptr(x), _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(A), _ptr(B), _ptr(y),
                                 _ptr(t_save), M, N, K, bits, group_size, rank, float(alpha), dtype,
                                 _ptr(workspace), workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_fwd")
    return st


def qlora_linear_fwd_static(x, packed, scales, zeros, A, B, y, t_save, M: int, N: int, K: int, bits: int,
                            group_size: int, rank: int, alpha: float, dtype: int, stream=None, check: bool = True) -> int:
    st = load().qlora_linear_fwd_static(_ptr(x), _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(A), _ptr(B), _ptr(y),
                                        _ptr(t_save), M, N, K, bits, group_size, rank, float(alpha), dtype,
                                        _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_fwd_static")
    return st


def qlora_linear_bwd(dy, x, packed, scales, zeros, A, B, t_saved, dx, dA, dB, M: int, N: int, K: int, bits: int,
                     group_size: int, rank: int, alpha: float, dtype: int, workspace,
                     workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_bwd(_ptr(dy), _ptr(x), _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(A), _ptr(B),
                                 _ptr(t_saved), _ptr(dx), _ptr(dA), _ptr(dB), M, N, K, bits, group_size, rank,
                                 float(alpha), dtype, _ptr(workspace), workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_bwd")
    return st


def _ptr_array(items, count: int):
    """Host array of `count` device pointers (None entries are NULL); None stays a NULL array."""
    if items is None:
        return None
    if len(items) != count:
        raise ValueError("one entry per sibling projection is needed")
    return (ctypes.c_void_p * count)(*[_ptr(t) for t in items])


def _int_array(values):
    return (ctypes.c_int * len(values))(*[int(v) for v in values])


def qlora_linear_bwd_stacked(dy, x, packed, scales, zeros, A, B, t_saved, dx, dA_train, dB_train, beta: float,
                             frozen_rank: int, M: int, N: int, K: int, bits: int, group_size: int, rank: int,
                             alpha: float, dtype: int, workspace, workspace_bytes: Optional[int] = None, stream=None,
                             check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_bwd_stacked(_ptr(dy), _ptr(x), _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(A), _ptr(B),
                                         _ptr(t_saved), _ptr(dx), _ptr(dA_train), _ptr(dB_train), float(beta),
                                         frozen_rank, M, N, K, bits, group_size, rank, float(alpha), dtype,
                                         _ptr(workspace), workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_bwd_stacked")
    return st


def qlora_linear_bwd_dropout_stacked(dy, x, packed, scales, zeros, A, B, keep_mask, keep_scale: float, t_saved, dx,
                                     dA_train, dB_train, beta: float, frozen_rank: int, M: int, N: int, K: int,
                                     bits: int, group_size: int, rank: int, alpha: float, dtype: int, workspace,
                                     workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_bwd_dropout_stacked(_ptr(dy), _ptr(x), _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(A),
                                                 _ptr(B), _ptr(keep_mask), float(keep_scale), _ptr(t_saved), _ptr(dx),
                                                 _ptr(dA_train), _ptr(dB_train), float(beta), frozen_rank, M, N, K,
                                                 bits, group_size, rank, float(alpha), dtype, _ptr(workspace),
                                                 workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_bwd_dropout_stacked")
    return st


def qlora_siblings_workspace_bytes(N, M: int, K: int, bits: int, group_size: int, rank: int) -> int:
    return int(load().qlora_siblings_workspace_bytes(len(N), _int_array(N), M, K, bits, group_size, rank))


def qlora_linear_fwd_siblings(x, packed, scales, zeros, A, B, y, t_save, N, M: int, K: int, bits: int,
                              group_size: int, rank: int, alpha: float, dtype: int, workspace,
                              workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    """packed, scales, zeros, A, B, y, t_save: sequences with one buffer per sibling projection; N: their out-features."""
    n = len(N)
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_fwd_siblings(n, _ptr(x), _ptr_array(packed, n), _ptr_array(scales, n),
                                          _ptr_array(zeros, n), _ptr_array(A, n), _ptr_array(B, n), _ptr_array(y, n),
                                          _ptr_array(t_save, n), _int_array(N), M, K, bits, group_size, rank,
                                          float(alpha), dtype, _ptr(workspace), workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_fwd_siblings")
    return st


def qlora_linear_bwd_siblings(dy, x, packed, scales, zeros, A, B, t_saved, dx, dA, dB, N, M: int, K: int, bits: int,
                              group_size: int, rank: int, alpha: float, dtype: int, workspace,
                              workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    n = len(N)
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_bwd_siblings(n, _ptr_array(dy, n), _ptr(x), _ptr_array(packed, n), _ptr_array(scales, n),
                                          _ptr_array(zeros, n), _ptr_array(A, n), _ptr_array(B, n),
                                          _ptr_array(t_saved, n), _ptr(dx), _ptr_array(dA, n), _ptr_array(dB, n),
                                          _int_array(N), M, K, bits, group_size, rank, float(alpha), dtype,
                                          _ptr(workspace), workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_bwd_siblings")
    return st


def qlora_lrec_workspace_bytes(M: int) -> int:
    return int(load().qlora_lrec_workspace_bytes(M))


def qlora_lrec_loss(student_logits, teacher_logits, labels, lambda_kl: float, lambda_ce: float, kl, ce, loss_mean,
                    dlogits, M: int, V: int, dtype: int, workspace, workspace_bytes: Optional[int] = None,
                    stream=None, check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_lrec_loss(_ptr(student_logits), _ptr(teacher_logits), _ptr(labels), float(lambda_kl),
                                float(lambda_ce), _ptr(kl), _ptr(ce), _ptr(loss_mean), _ptr(dlogits), M, V, dtype,
                                _ptr(workspace), workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_lrec_loss")
    return st


def qlora_lrec_loss_scaled(student_logits, teacher_logits, labels, lambda_kl: float, lambda_ce: float,
                           grad_scale: float, kl, ce, loss_mean, dlogits, M: int, V: int, dtype: int, workspace,
                           workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_lrec_loss_scaled(_ptr(student_logits), _ptr(teacher_logits), _ptr(labels), float(lambda_kl),
                                       float(lambda_ce), float(grad_scale), _ptr(kl), _ptr(ce), _ptr(loss_mean),
                                       _ptr(dlogits), M, V, dtype, _ptr(workspace), workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_lrec_loss_scaled")
    return st


def qlora_linear_bwd_accumulate(dy, x, packed, scales, zeros, A, B, t_saved, dx, dA, dB, beta: float, M: int, N: int,
                                K: int, bits: int, group_size: int, rank: int, alpha: float, dtype: int, workspace,
                                workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_bwd_accumulate(_ptr(dy), _ptr(x), _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(A),
                                            _ptr(B), _ptr(t_saved), _ptr(dx), _ptr(dA), _ptr(dB), float(beta), M, N,
                                            K, bits, group_size, rank, float(alpha), dtype, _ptr(workspace),
                                            workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_bwd_accumulate")
    return st


def qlora_workspace_bytes_zp(M: int, N: int, K: int, bits: int, group_size: int, rank: int) -> int:
    return int(load().qlora_workspace_bytes_zp(M, N, K, bits, group_size, rank))


def qlora_linear_fwd_zp(x, packed, scales, packed_zeros, A, B, y, t_save, M: int, N: int, K: int, bits: int,
                        group_size: int, rank: int, alpha: float, dtype: int, workspace,
                        workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_fwd_zp(_ptr(x), _ptr(packed), _ptr(scales), _ptr(packed_zeros), _ptr(A), _ptr(B),
                                    _ptr(y), _ptr(t_save), M, N, K, bits, group_size, rank, float(alpha), dtype,
                                    _ptr(workspace), workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_fwd_zp")
    return st


def qlora_linear_bwd_zp(dy, x, packed, scales, packed_zeros, A, B, t_saved, dx, dA, dB, beta: float, M: int, N: int,
                        K: int, bits: int, group_size: int, rank: int, alpha: float, dtype: int, workspace,
                        workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_bwd_zp(_ptr(dy), _ptr(x), _ptr(packed), _ptr(scales), _ptr(packed_zeros), _ptr(A),
                                    _ptr(B), _ptr(t_saved), _ptr(dx), _ptr(dA), _ptr(dB), float(beta), M, N, K, bits,
                                    group_size, rank, float(alpha), dtype, _ptr(workspace), workspace_bytes,
                                    _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_bwd_zp")
    return st


def qlora_linear_fwd_dropout(x, packed, scales, zeros, A, B, keep_mask, keep_scale: float, y, t_save, M: int, N: int,
                             K: int, bits: int, group_size: int, rank: int, alpha: float, dtype: int, workspace,
                             workspace_bytes: Optional[int] = None, stream=None, check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_fwd_dropout(_ptr(x), _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(A), _ptr(B),
                                         _ptr(keep_mask), float(keep_scale), _ptr(y), _ptr(t_save), M, N, K, bits,
                                         group_size, rank, float(alpha), dtype, _ptr(workspace), workspace_bytes,
                                         _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_fwd_dropout")
    return st


def qlora_linear_bwd_dropout(dy, x, packed, scales, zeros, A, B, keep_mask, keep_scale: float, t_saved, dx, dA, dB,
                             beta: float, M: int, N: int, K: int, bits: int, group_size: int, rank: int, alpha: float,
                             dtype: int, workspace, workspace_bytes: Optional[int] = None, stream=None,
                             check: bool = True) -> int:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    st = load().qlora_linear_bwd_dropout(_ptr(dy), _ptr(x), _ptr(packed), _ptr(scales), _ptr(zeros), _ptr(A), _ptr(B),
                                         _ptr(keep_mask), float(keep_scale), _ptr(t_saved), _ptr(dx), _ptr(dA),
                                         _ptr(dB), float(beta), M, N, K, bits, group_size, rank, float(alpha), dtype,
                                         _ptr(workspace), workspace_bytes, _stream(stream))
    if check and st != 0:
        raise QLoraError(st, "qlora_linear_bwd_dropout")
    return st
