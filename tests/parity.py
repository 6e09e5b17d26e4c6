"""Shared helpers of the GPU parity tests: run the HIP library and the CPU oracle on the same bytes.

Three bars are applied to every floating-point output, all against the fp64 oracle:

* the matrix-wide relative Frobenius error, at most TOL = 5e-3 (the bar the workload definition states);
* the same figure for every row (y, dX: token rows are independent problems; dA: one row per adapter column) or
  every column (dB, t: one column per adapter column) on its own, at most ROW_C * TOL, so that a block of wrong
  elements cannot hide in the norm of a large matrix;
* an element bound from the arithmetic: the GPU rounds the dequantised weight, t / u and the output to 16 bits
  (unit roundoff u = 2^-11 for fp16, 2^-8 for bf16) and accumulates in fp32, so by Cauchy-Schwarz
      |y_gpu[m,n] - y[m,n]|   <= ELEM_K u (|x_m| |Wd_n| + sc |t_m| |B_n|)
      |dX_gpu[m,k] - dX[m,k]| <= ELEM_K u (|dY_m| |Wd_:,k| + sc |u_m| |A_:,k|)
      |dA_gpu[j,k] - dA[j,k]| <= ELEM_K u sc |u_:,j| |x_:,k|,   |dB_gpu[n,j] - dB[n,j]| <= ELEM_K u sc |dY_:,n| |t_:,j|
  (norms over the contraction index).  Worst case by count: weight rounding u, output rounding u (twice under
  dropout), rounding of t or u and of sc * t: ELEM_K = 4 covers every path.  A typical element is ~ |x_m| |Wd_n| /
  sqrt(K), far above the fp16 bound, so a single wrong element fails it.
"""
from __future__ import annotations

import sys

import numpy as np

import oracle
from paper_2306_08162_amd import workloads as wl

TOL = 5e-3      # relative Frobenius error allowed on y, dX, dA, dB (fp16/bf16 in, fp32 accumulate)
ROW_C = 1.0     # per-row / per-column bar as a multiple of TOL
ELEM_K = 4.0    # element bound as a multiple of u * (Cauchy-Schwarz scale of the element)


def unit_roundoff(dtype: str) -> float:
    return 2.0 ** -11 if dtype == "f16" else 2.0 ** -8


def rel_fro(got: np.ndarray, want: np.ndarray) -> float:
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    n = np.linalg.norm(want)
    d = np.linalg.norm(got - want)
    return float(d / n) if n > 0 else float(d)


def worst_line(got: np.ndarray, want: np.ndarray, axis: int) -> float:
    """Largest relative error of a row (axis = 1: norms along the row) or column (axis = 0) taken alone.  Lines whose
    reference is all zero are left to the element bound."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    if want.size == 0:
        return 0.0
    d = np.linalg.norm(got - want, axis=axis)
    n = np.linalg.norm(want, axis=axis)
    live = n > 0
    return float(np.max(d[live] / n[live])) if np.any(live) else 0.0


def elem_excess(got: np.ndarray, want: np.ndarray, bound: np.ndarray, u: float) -> float:
    """max over elements of |got - want| / (ELEM_K u bound); at most 1 when the bound holds.  Where the bound is zero
    the element must be exact."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    if want.size == 0:
        return 0.0
    d = np.abs(got - want)
    lim = ELEM_K * u * np.asarray(bound, np.float64)
    if np.any(d[lim == 0] != 0):
        return float("inf")
    ok = lim > 0
    return float(np.max(d[ok] / lim[ok])) if np.any(ok) else 0.0


class Report:
    """Collects the error figures of one case, prints them, and applies the three bars."""

    def __init__(self, name: str, dtype: str):
        self.name, self.u = name, unit_roundoff(dtype)
        self.fro, self.line, self.elem = {}, {}, {}

    def add(self, key: str, got, want, *, lines: str | None = None, bound=None) -> None:
        """lines: 'rows' or 'cols' (which lines are judged one by one); bound: Cauchy-Schwarz scale per element."""
        got = np.asarray(got, np.float64)
        want = np.asarray(want, np.float64)
        assert got.shape == want.shape, f"{self.name}: {key} has shape {got.shape}, the oracle's {want.shape}"
        self.fro[key] = rel_fro(got, want)
        if lines is not None:
            self.line[key] = worst_line(got, want, 1 if lines == "rows" else 0)
        if bound is not None:
            self.elem[key] = elem_excess(got, want, bound, self.u)

    def finish(self) -> dict:
        announce(f"{self.name}: " + " ".join(
            f"{k}={v:.2e}/{self.line.get(k, float('nan')):.2e}/{self.elem.get(k, float('nan')):.2f}"
            for k, v in self.fro.items()) + "   (Frobenius / worst line / element bound used)")
        for k, v in self.fro.items():
            assert np.isfinite(v) and v <= TOL, f"{self.name}: rel. Frobenius error of {k} = {v:.3e} > {TOL}"
        for k, v in self.line.items():
            assert np.isfinite(v) and v <= ROW_C * TOL, f"{self.name}: worst row/column of {k} is off by {v:.3e} > {ROW_C * TOL}"
        for k, v in self.elem.items():
            assert v <= 1.0, f"{self.name}: an element of {k} exceeds its rounding bound {v:.2f} times"
        return dict(self.fro)


def layer_bounds(Wd, A, B, sc, x=None, dy=None, t=None, u=None, x_adapter=None):
    """Cauchy-Schwarz scales of the elements of y, dX, dA, dB (see the module header).  All arguments fp64 (the
    oracle's values); x_adapter is what the adapter branch sees of x (x itself unless dropout is on)."""
    out = {}
    nrm = np.linalg.norm
    if x is not None:
        out["y"] = np.outer(nrm(x, axis=1), nrm(Wd, axis=1))
        if t is not None and t.shape[1]:
            out["y"] = out["y"] + sc * np.outer(nrm(t, axis=1), nrm(B, axis=1))
    if dy is not None:
        out["dx"] = np.outer(nrm(dy, axis=1), nrm(Wd, axis=0))
        if u is not None and u.shape[1]:
            out["dx"] = out["dx"] + sc * np.outer(nrm(u, axis=1), nrm(A, axis=0))
    if u is not None and u.shape[1] and x_adapter is not None:
        out["dA"] = sc * np.outer(nrm(u, axis=0), nrm(x_adapter, axis=0))
    if t is not None and t.shape[1] and dy is not None:
        out["dB"] = sc * np.outer(nrm(dy, axis=0), nrm(t, axis=0))
    return out


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


def integer_inputs(seed: int, M: int, K: int, N: int, bits: int, G: int, r: int, dtype: str, *, spread: int = 3,
                   density: float = 1.0, adapter: bool = True) -> wl.LayerInputs:
    """Inputs on which every product and sum of the layer is a small integer, so that a correct implementation
    returns the oracle's values bit for bit whatever its summation order: scales 1, codes within `spread` of their
    group's zero-point, x and dY in {-1, 0, 1} (non-zero with probability `density`), A and B in {-1, 0, 1} with a
    few non-zeros per row (all zero when adapter is False), alpha = rank (branch scale 1)."""
    inp = small_inputs(seed, M, K, N, bits, G, r, dtype, alpha=float(max(r, 1)))
    one = wl.to_bits(np.ones(1), dtype)[0]
    qmax = (1 << bits) - 1
    z = inp.zeros.astype(np.int64)[:, np.arange(K) // G]
    delta = wl.uniform_ints(seed + 1, N * K, 2 * spread + 1).reshape(N, K).astype(np.int64) - spread
    inp.codes[...] = np.clip(z + delta, 0, qmax).astype(np.uint8)
    inp.scales[...] = np.float16(1.0).view(np.uint16)

    def ternary(s, count, p):
        v = wl.uniform_ints(s, count, 3).astype(np.float64) - 1.0
        keep = wl.uniform01(s + 7, 0, count) < p
        return wl.to_bits(v * keep, dtype)

    inp.x[...] = ternary(seed + 2, M * K, density).reshape(M, K)
    inp.dy[...] = ternary(seed + 3, M * N, density).reshape(M, N)
    if r:
        inp.A[...] = ternary(seed + 4, r * K, min(1.0, 6.0 / K) if adapter else 0.0).reshape(r, K)
        inp.B[...] = ternary(seed + 5, N * r, 0.5 if adapter else 0.0).reshape(N, r)
    assert one != 0
    return inp


def check_layer(inp: wl.LayerInputs, rows: np.ndarray | None = None, recompute_t: bool = False,
                device: str = "cuda:0", exact: bool = False, packed_zeros: bool = False) -> dict:
    """Forward + backward on the GPU, compared with the oracle.

    `rows`: token rows on which y / dX are compared (None = all).  dA, dB and
    the packed words are always compared in full.  `exact`: the inputs make every
    result an exactly representable integer (integer_inputs): demand equality.
    `packed_zeros`: the zero-points reach the library in their bit-packed storage form, packed by the oracle.
    Returns the Frobenius figures.
    """
    import torch
    from paper_2306_08162_amd.device import DeviceLayer

    c = inp.cfg
    announce(f"{c.name}: M={c.M} K={c.K} N={c.N} bits={c.bits} G={c.group_size} r={c.rank} {c.dtype} "
             f"recompute_t={recompute_t}" + (" exact" if exact else "") + (" packed zero-points" if packed_zeros else ""))
    layer = DeviceLayer(inp, device)
    if packed_zeros:
        layer.use_packed_zeros(oracle.pack_zeros(inp.zeros, c.bits))
    layer.forward(save_t=not recompute_t)
    layer.backward(use_saved_t=not recompute_t)
    torch.cuda.synchronize()

    lo = make_oracle(inp)
    assert np.array_equal(layer.host_packed(), lo.P), "packed words differ from the oracle's"
    y_ref, t_ref = lo.forward(inp.x, rows)
    dx_ref = lo.backward_dx(inp.dy, rows)
    sel = slice(None) if rows is None else rows
    got = {"y": oracle.widen(layer.host_y()[sel], c.dtype), "dx": oracle.widen(layer.host_dx()[sel], c.dtype)}
    want = {"y": y_ref, "dx": dx_ref}
    x = oracle.widen(inp.x, c.dtype)
    dy = oracle.widen(inp.dy, c.dtype)
    sc = c.alpha / c.rank if c.rank else 0.0
    t_all = oracle.lora_down(x, lo.A) if c.rank else None
    u_all = oracle.lora_u(dy, lo.B) if c.rank else None
    if c.rank:
        want["dA"], want["dB"] = lo.backward_adapters(inp.dy, inp.x)
        got["dA"], got["dB"] = layer.host_dA(), layer.host_dB()
        if not recompute_t:
            got["t"], want["t"] = oracle.widen(layer.host_t()[sel], c.dtype), t_ref
    if exact:
        lim = 2048 if c.dtype == "f16" else 256          # integers every 16-bit output must stay below
        for k in ("y", "dx", "t"):
            if k in want:
                assert np.all(want[k] == np.round(want[k])) and np.abs(want[k]).max() <= lim, f"{k} is not exactly representable"
        for k, w in want.items():
            assert np.abs(w).max() < 2 ** 24
            assert np.array_equal(got[k], w), f"{c.name}: {k} differs from the exact integer result in " \
                                              f"{int(np.sum(got[k] != w))} of {w.size} elements"
        announce(f"{c.name}: " + " ".join(f"{k}: exact, max |value| {np.abs(w).max():.0f}" for k, w in want.items()))
        return {k: 0.0 for k in want}
    bounds_sel = layer_bounds(lo.Wd, lo.A, lo.B, sc, x=x[sel], dy=dy[sel], t=None if t_all is None else t_all[sel],
                              u=None if u_all is None else u_all[sel])
    bounds_all = layer_bounds(lo.Wd, lo.A, lo.B, sc, x=None, dy=dy, t=t_all, u=u_all, x_adapter=x)
    rep = Report(c.name, c.dtype)
    rep.add("y", got["y"], want["y"], lines="rows", bound=bounds_sel["y"])
    rep.add("dx", got["dx"], want["dx"], lines="rows", bound=bounds_sel["dx"])
    if c.rank:
        rep.add("dA", got["dA"], want["dA"], lines="rows", bound=bounds_all["dA"])
        rep.add("dB", got["dB"], want["dB"], lines="cols", bound=bounds_all["dB"])
        if "t" in got:
            # t = round16(fp32 sum): one rounding of the result, plus fp32 accumulation
            rep.add("t", got["t"], want["t"], lines="cols",
                    bound=np.outer(np.linalg.norm(x[sel], axis=1), np.linalg.norm(lo.A, axis=1)))
    return rep.finish()
