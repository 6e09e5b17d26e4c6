"""Shared helpers of the GPU parity tests: run the HIP library and the CPU oracle on the same bytes."""
from __future__ import annotations

import sys

import numpy as np

import oracle
from paper_2306_08162_amd import workloads as wl

TOL = 5e-3   # relative Frobenius error allowed on y, dX, dA, dB (fp16/bf16 in, fp32 accumulate)


def rel_fro(got: np.ndarray, want: np.ndarray) -> float:
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    n = np.linalg.norm(want)
    d = np.linalg.norm(got - want)
    return float(d / n) if n > 0 else float(d)


def announce(msg: str) -> None:
    """Name the case before it touches the GPU, so a fault can be traced to it."""
    print(f"[parity] {msg}", flush=True)
    sys.stdout.flush()


def make_oracle(inp: wl.LayerInputs) -> oracle.LayerOracle:
    c = inp.cfg
    return oracle.LayerOracle(inp.codes, inp.scales, inp.zeros, inp.A, inp.B, bits=c.bits,
                              group_size=c.group_size, alpha=c.alpha, dtype=c.dtype)


def small_inputs(seed: int, M: int, K: int, N: int, bits: int, G: int, r: int, dtype: str = "f16",
                 alpha: float | None = None, scale_lo: float = 0.005, scale_hi: float = 0.03) -> wl.LayerInputs:
    cfg = wl.LayerConfig(f"case_s{seed}_M{M}_K{K}_N{N}_b{bits}_G{G}_r{r}_{dtype}", 1000 + seed, M=M, K=K, N=N,
                         bits=bits, group_size=G, rank=r, alpha=float(2 * r if alpha is None else alpha),
                         dtype=dtype, scale_lo=scale_lo, scale_hi=scale_hi)
    return wl.make_inputs(cfg)


def check_layer(inp: wl.LayerInputs, rows: np.ndarray | None = None, recompute_t: bool = False,
                device: str = "cuda:0") -> dict:
    """Forward + backward on the GPU, compared with the oracle.

    `rows`: token rows on which y / dX are compared (None = all).  dA, dB and
    the packed words are always compared in full.  Returns the error figures.
    """
    import torch
    from paper_2306_08162_amd.device import DeviceLayer

    c = inp.cfg
    announce(f"{c.name}: M={c.M} K={c.K} N={c.N} bits={c.bits} G={c.group_size} r={c.rank} {c.dtype} "
             f"recompute_t={recompute_t}")
    layer = DeviceLayer(inp, device)
    layer.forward(save_t=not recompute_t)
    layer.backward(use_saved_t=not recompute_t)
    torch.cuda.synchronize()

    lo = make_oracle(inp)
    out = {}
    assert np.array_equal(layer.host_packed(), lo.P), "packed words differ from the oracle's"
    y_ref, t_ref = lo.forward(inp.x, rows)
    dx_ref = lo.backward_dx(inp.dy, rows)
    sel = slice(None) if rows is None else rows
    out["y"] = rel_fro(oracle.widen(layer.host_y()[sel], c.dtype), y_ref)
    out["dx"] = rel_fro(oracle.widen(layer.host_dx()[sel], c.dtype), dx_ref)
    if c.rank:
        dA_ref, dB_ref = lo.backward_adapters(inp.dy, inp.x)
        out["dA"] = rel_fro(layer.host_dA(), dA_ref)
        out["dB"] = rel_fro(layer.host_dB(), dB_ref)
        if not recompute_t:
            out["t"] = rel_fro(oracle.widen(layer.host_t()[sel], c.dtype), t_ref)
    announce(f"{c.name}: " + " ".join(f"{k}={v:.2e}" for k, v in out.items()))
    for k, v in out.items():
        assert np.isfinite(v) and v <= TOL, f"{c.name}: rel. Frobenius error of {k} = {v:.3e} > {TOL}"
    return out
