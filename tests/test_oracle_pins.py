"""Pins for the CPU oracle: it is checked against things that are not itself.

hand-derived packed words, a big-integer bit-stream writer, numpy float64
products, pure-Python loops on tiny shapes, finite differences, adjoint
identities and the special cases the layer's definition implies
(Sec. 3.1 and Fig. 1 of the paper; Appendix B for the adapter shapes).
"""
import os

import numpy as np
import pytest

import oracle
from paper_2306_08162_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RTOL = 1e-11


def _rel(a, b):
    d = np.linalg.norm(np.asarray(a, np.float64) - np.asarray(b, np.float64))
    n = np.linalg.norm(np.asarray(b, np.float64))
    return d / n if n > 0 else d


def _read_pack_golden():
    rows = []
    with open(os.path.join(GOLDEN, "pack_words.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            b, codes, words = [p.strip() for p in line.split("|")]
            rows.append((int(b), np.array(codes.split(), dtype=np.uint8),
                         np.array([int(w, 16) for w in words.split()], dtype=np.uint32)))
    return rows


def _bigint_pack(row, b):
    """Independent writer: the row as one big little-endian integer."""
    stream = 0
    for k, q in enumerate(row.tolist()):
        stream |= int(q) << (b * k)
    nw = len(row) * b // 32
    return np.array([(stream >> (32 * w)) & 0xFFFFFFFF for w in range(nw)], dtype=np.uint32)


# ------------------------------------------------------------------ codes

@pytest.mark.parametrize("case", _read_pack_golden(), ids=lambda c: f"b{c[0]}_{c[2][0]:08X}")
def test_pack_matches_hand_derived_words(case):
    b, codes, words = case
    P = oracle.pack(codes[None, :], b)
    assert P.shape == (1, len(words))
    assert np.array_equal(P[0], words)
    assert np.array_equal(oracle.unpack(words[None, :], len(codes), b)[0], codes)


@pytest.mark.parametrize("b", [2, 3, 4, 8])
@pytest.mark.parametrize("K", [32, 96, 256, 11008])
def test_pack_matches_bigint_stream_and_roundtrips(b, K):
    N = 5
    codes = wl.uniform_ints(1234 + b * 100 + K, N * K, 1 << b).reshape(N, K)
    P = oracle.pack(codes, b)
    assert P.dtype == np.uint32 and P.shape == (N, K * b // 32)
    for n in range(N):
        assert np.array_equal(P[n], _bigint_pack(codes[n], b))
    assert np.array_equal(oracle.unpack(P, K, b), codes)


@pytest.mark.parametrize("b", [2, 3, 4, 8])
def test_pack_extreme_codes(b):
    K = 64
    top = (1 << b) - 1
    P = oracle.pack(np.full((2, K), top, np.uint8), b)
    assert np.all(P == 0xFFFFFFFF)
    assert np.all(oracle.pack(np.zeros((2, K), np.uint8), b) == 0)


def test_rows_are_independent_streams():
    # INT3 with K=32: each row is 3 whole words; row 1 must not leak into row 0.
    codes = np.zeros((2, 32), np.uint8)
    codes[1, :] = 7
    P = oracle.pack(codes, 3)
    assert np.all(P[0] == 0) and np.all(P[1] == 0xFFFFFFFF)


def test_adapter_shape_pin_from_paper():
    with open(os.path.join(GOLDEN, "shape_pins.txt")) as f:
        line = [l for l in f if l.strip() and not l.startswith("#")][0]
    L, d, r, total = [int(v) for v in line.split("|")]
    assert 2 * L * d * r == total
    cfg = wl.config2()                       # a 4096 -> 4096 projection with r = 8
    assert (cfg.K, cfg.N, cfg.rank) == (d, d, r)
    inp = wl.make_inputs(wl.config1())
    assert inp.A.shape == (inp.cfg.rank, inp.cfg.K) and inp.B.shape == (inp.cfg.N, inp.cfg.rank)
    per_projection = cfg.rank * (cfg.K + cfg.N)
    assert L * per_projection == total


# ---------------------------------------------------------------- dequant

def _np_dequant(codes, s, z, G):
    g = np.arange(codes.shape[1]) // G
    return s[:, g] * (codes.astype(np.float64) - z[:, g].astype(np.float64))


@pytest.mark.parametrize("b,G,K", [(2, 32, 96), (3, 32, 64), (4, 64, 256), (8, 128, 256), (3, 128, 384), (4, 96, 96)])
def test_dequant_is_scale_times_code_minus_zero(b, G, K):
    N = 7
    codes = wl.uniform_ints(77 + b, N * K, 1 << b).reshape(N, K)
    s = wl.uniform_range(78, N * (K // G), 0.002, 0.05).reshape(N, K // G)
    z = wl.uniform_ints(79 + b, N * (K // G), 1 << b).reshape(N, K // G)
    Wd = oracle.dequant(oracle.pack(codes, b), s, z, K, b, G)
    assert np.array_equal(Wd, _np_dequant(codes, s, z, G))      # same two fp64 ops: exact
    # scalar spot checks written out longhand
    for (n, k) in [(0, 0), (3, K - 1), (6, G % K), (2, G - 1)]:
        assert Wd[n, k] == s[n, k // G] * (float(codes[n, k]) - float(z[n, k // G]))


def test_widen_is_exact():
    h = np.array([0x3C00, 0xC000, 0x0001, 0x7BFF, 0x8000], np.uint16)   # 1, -2, 2^-24, 65504, -0
    assert oracle.widen(h, "f16").tolist() == [1.0, -2.0, 2.0 ** -24, 65504.0, -0.0]
    bf = np.array([0x3F80, 0xC000, 0x3F81, 0x0080], np.uint16)          # 1, -2, 1+2^-7, 2^-126
    assert oracle.widen(bf, "bf16").tolist() == [1.0, -2.0, 1.0 + 2.0 ** -7, 2.0 ** -126]


# ---------------------------------------------------------------- helpers

def _small_problem(seed, M, N, K, r, b, G, alpha=16.0):
    codes = wl.uniform_ints(seed, N * K, 1 << b).reshape(N, K)
    s = wl.uniform_range(seed + 1, N * (K // G), 0.005, 0.03).reshape(N, K // G)
    z = wl.uniform_ints(seed + 2, N * (K // G), 1 << b).reshape(N, K // G)
    A = wl.normal(seed + 3, r * K, K ** -0.5).reshape(r, K)
    B = wl.normal(seed + 4, N * r, 0.1).reshape(N, r)
    x = wl.normal(seed + 5, M * K).reshape(M, K)
    dy = wl.normal(seed + 6, M * N).reshape(M, N)
    Wd = oracle.dequant(oracle.pack(codes, b), s, z, K, b, G)
    return dict(codes=codes, s=s, z=z, A=A, B=B, x=x, dy=dy, Wd=Wd, alpha=alpha, r=r, G=G, b=b)


def _loops_forward(p):
    """Pure-Python triple loops straight from the definition (tiny shapes only)."""
    x, codes, s, z, A, B = p["x"], p["codes"], p["s"], p["z"], p["A"], p["B"]
    M, K = x.shape
    N = codes.shape[0]
    r, G = p["r"], p["G"]
    y = [[0.0] * N for _ in range(M)]
    for m in range(M):
        t = [sum(float(x[m, k]) * float(A[j, k]) for k in range(K)) for j in range(r)]
        for n in range(N):
            acc = 0.0
            for k in range(K):
                w = float(s[n, k // G]) * (float(codes[n, k]) - float(z[n, k // G]))
                acc += float(x[m, k]) * w
            lo = sum(t[j] * float(B[n, j]) for j in range(r))
            y[m][n] = acc + (p["alpha"] / r) * lo
    return np.array(y)


def _loops_backward(p):
    x, dy, codes, s, z, A, B = p["x"], p["dy"], p["codes"], p["s"], p["z"], p["A"], p["B"]
    M, K = x.shape
    N = codes.shape[0]
    r, G = p["r"], p["G"]
    sc = p["alpha"] / r
    dx = np.zeros((M, K))
    dA = np.zeros((r, K))
    dB = np.zeros((N, r))
    for m in range(M):
        t = [sum(float(x[m, k]) * float(A[j, k]) for k in range(K)) for j in range(r)]
        u = [sum(float(dy[m, n]) * float(B[n, j]) for n in range(N)) for j in range(r)]
        for k in range(K):
            acc = 0.0
            for n in range(N):
                w = float(s[n, k // G]) * (float(codes[n, k]) - float(z[n, k // G]))
                acc += float(dy[m, n]) * w
            acc += sc * sum(u[j] * float(A[j, k]) for j in range(r))
            dx[m, k] = acc
        for j in range(r):
            for k in range(K):
                dA[j, k] += sc * u[j] * float(x[m, k])
            for n in range(N):
                dB[n, j] += sc * float(dy[m, n]) * t[j]
    return dx, dA, dB


# ---------------------------------------------------------------- forward

@pytest.mark.parametrize("b,K,G", [(2, 32, 32), (3, 64, 32), (4, 96, 32), (8, 64, 32)])
def test_forward_matches_python_loops(b, K, G):
    p = _small_problem(100 + b, M=5, N=7, K=K, r=3, b=b, G=G)
    y, t = oracle.forward(p["x"], p["Wd"], p["A"], p["B"], p["alpha"])
    assert _rel(y, _loops_forward(p)) < RTOL
    assert _rel(t, p["x"] @ p["A"].T) < RTOL


def test_forward_with_B_zero_is_the_dequantised_gemm():
    p = _small_problem(200, M=33, N=40, K=256, r=8, b=4, G=64)
    y, _ = oracle.forward(p["x"], p["Wd"], p["A"], np.zeros_like(p["B"]), p["alpha"])
    assert _rel(y, p["x"] @ _np_dequant(p["codes"], p["s"], p["z"], p["G"]).T) < RTOL


def test_forward_full_against_numpy_float64():
    p = _small_problem(201, M=21, N=48, K=384, r=16, b=3, G=128, alpha=32.0)
    y, t = oracle.forward(p["x"], p["Wd"], p["A"], p["B"], p["alpha"])
    W = _np_dequant(p["codes"], p["s"], p["z"], p["G"])
    ref = p["x"] @ W.T + (p["alpha"] / p["r"]) * (p["x"] @ p["A"].T) @ p["B"].T
    assert _rel(y, ref) < RTOL


def test_forward_codes_equal_zero_point_leaves_only_the_lora_branch():
    p = _small_problem(202, M=9, N=16, K=64, r=8, b=2, G=32)
    g = np.arange(64) // 32
    codes = p["z"][:, g]                                    # q == z everywhere -> Wd == 0
    Wd = oracle.dequant(oracle.pack(codes, 2), p["s"], p["z"], 64, 2, 32)
    assert np.all(Wd == 0.0)
    y, _ = oracle.forward(p["x"], Wd, p["A"], p["B"], p["alpha"])
    assert _rel(y, 2.0 * (p["x"] @ p["A"].T) @ p["B"].T) < RTOL     # alpha/r = 16/8


def test_forward_rank_zero_is_plain_quantised_linear():
    p = _small_problem(203, M=6, N=8, K=64, r=8, b=4, G=32)
    y, t = oracle.forward(p["x"], p["Wd"], np.zeros((0, 64)), np.zeros((8, 0)), 16.0)
    assert t.shape == (6, 0)
    assert _rel(y, p["x"] @ p["Wd"].T) < RTOL


def test_forward_is_linear_in_x():
    p = _small_problem(204, M=12, N=24, K=128, r=8, b=4, G=64)
    x2 = wl.normal(999, 12 * 128).reshape(12, 128)
    f = lambda v: oracle.forward(v, p["Wd"], p["A"], p["B"], p["alpha"])[0]
    assert _rel(f(p["x"] + x2), f(p["x"]) + f(x2)) < RTOL
    assert _rel(f(3.0 * p["x"]), 3.0 * f(p["x"])) < RTOL


def test_forward_integer_exact_case():
    # s = 1, x in {-1,0,1}, no adapter contribution: y is an exactly representable integer.
    M, N, K, b, G = 8, 16, 256, 2, 64
    codes = wl.uniform_ints(300, N * K, 4).reshape(N, K)
    z = wl.uniform_ints(301, N * (K // G), 4).reshape(N, K // G)
    x = wl.uniform_ints(302, M * K, 3).reshape(M, K).astype(np.float64) - 1.0
    Wd = oracle.dequant(oracle.pack(codes, b), np.ones((N, K // G)), z, K, b, G)
    y, _ = oracle.forward(x, Wd, np.zeros((8, K)), wl.normal(5, N * 8).reshape(N, 8), 16.0)
    g = np.arange(K) // G
    want = x.astype(np.int64) @ (codes.astype(np.int64) - z[:, g].astype(np.int64)).T
    assert np.array_equal(y, want.astype(np.float64))
    assert np.abs(want).max() < 2048


# --------------------------------------------------------------- backward

@pytest.mark.parametrize("b,K,G", [(2, 32, 32), (3, 64, 32), (4, 96, 32), (8, 64, 32)])
def test_backward_matches_python_loops(b, K, G):
    p = _small_problem(400 + b, M=4, N=6, K=K, r=3, b=b, G=G)
    dx = oracle.backward_dx(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"])
    dA, dB = oracle.backward_adapters(p["dy"], p["x"], p["A"], p["B"], p["alpha"])
    ldx, ldA, ldB = _loops_backward(p)
    assert _rel(dx, ldx) < RTOL and _rel(dA, ldA) < RTOL and _rel(dB, ldB) < RTOL


def test_backward_against_numpy_float64():
    p = _small_problem(500, M=19, N=40, K=256, r=8, b=4, G=128)
    sc = p["alpha"] / p["r"]
    W = _np_dequant(p["codes"], p["s"], p["z"], p["G"])
    dx = oracle.backward_dx(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"])
    dA, dB = oracle.backward_adapters(p["dy"], p["x"], p["A"], p["B"], p["alpha"])
    assert _rel(dx, p["dy"] @ W + sc * (p["dy"] @ p["B"]) @ p["A"]) < RTOL
    assert _rel(dA, sc * (p["dy"] @ p["B"]).T @ p["x"]) < RTOL
    assert _rel(dB, sc * p["dy"].T @ (p["x"] @ p["A"].T)) < RTOL
    assert dA.shape == p["A"].shape and dB.shape == p["B"].shape and dx.shape == p["x"].shape


def test_backward_finite_differences():
    # L = <dY, y> is linear in each of x, A, B, so central differences are exact to rounding.
    p = _small_problem(600, M=5, N=9, K=64, r=4, b=3, G=32)
    L = lambda x, A, B: float(np.sum(p["dy"] * oracle.forward(x, p["Wd"], A, B, p["alpha"])[0]))
    dx = oracle.backward_dx(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"])
    dA, dB = oracle.backward_adapters(p["dy"], p["x"], p["A"], p["B"], p["alpha"])
    h = 1e-3
    rng = np.random.RandomState(0)
    for name, grad in (("x", dx), ("A", dA), ("B", dB)):
        for _ in range(12):
            idx = tuple(rng.randint(0, s) for s in grad.shape)
            args = {k: p[k].copy() for k in ("x", "A", "B")}
            args[name][idx] += h
            up = L(args["x"], args["A"], args["B"])
            args[name][idx] -= 2 * h
            dn = L(args["x"], args["A"], args["B"])
            fd = (up - dn) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-8 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])


def test_sibling_projections_dx_is_the_sum_of_their_dx():
    # Projections that read the same x (q/k/v, gate/up): the gradient of L = sum_i <dY_i, y_i(x)> w.r.t. x is what the
    # sibling entry points must return.  Central differences on the oracle's forward (L is linear in x) pin the rule
    # "dX = sum of the per-layer dX" that the GPU parity test of those entry points relies on.
    ps = [_small_problem(610 + i, M=4, N=n, K=64, r=4, b=b, G=32) for i, (n, b) in enumerate(((9, 3), (16, 4), (7, 2)))]
    x = ps[0]["x"]
    L = lambda xx: sum(float(np.sum(p["dy"] * oracle.forward(xx, p["Wd"], p["A"], p["B"], p["alpha"])[0])) for p in ps)
    dx = sum(oracle.backward_dx(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"]) for p in ps)
    h = 1e-3
    rng = np.random.RandomState(1)
    for _ in range(16):
        idx = tuple(rng.randint(0, s) for s in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd = (L(xp) - L(xm)) / (2 * h)
        assert abs(fd - dx[idx]) <= 1e-8 * max(1.0, abs(fd)), (idx, fd, dx[idx])


def test_lora_dropout_reduces_to_the_plain_layer_and_to_no_adapter():
    p = _small_problem(620, M=6, N=10, K=64, r=4, b=4, G=32)
    ones, zeros = np.ones_like(p["x"]), np.zeros_like(p["x"])
    y0, t0 = oracle.forward(p["x"], p["Wd"], p["A"], p["B"], p["alpha"])
    y1, t1 = oracle.forward_dropout(p["x"], p["Wd"], p["A"], p["B"], p["alpha"], ones, 1.0)
    assert np.allclose(y0, y1, rtol=0, atol=1e-12) and np.allclose(t0, t1, rtol=0, atol=1e-13)
    assert np.allclose(oracle.backward_dx(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"]),
                       oracle.backward_dx_dropout(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"], ones, 1.0), atol=1e-12)
    # everything dropped: the adapter is gone from y, dX and dA (dB = sc dY^T t with t = 0)
    y2, t2 = oracle.forward_dropout(p["x"], p["Wd"], p["A"], p["B"], p["alpha"], zeros, 1.0 / 0.95)
    assert _rel(y2, p["x"] @ p["Wd"].T) < RTOL and np.all(t2 == 0)
    assert _rel(oracle.backward_dx_dropout(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"], zeros, 1.0 / 0.95),
                p["dy"] @ p["Wd"]) < RTOL
    dA, dB = oracle.backward_adapters_dropout(p["dy"], p["x"], p["A"], p["B"], p["alpha"], zeros, 1.0 / 0.95)
    assert np.all(dA == 0) and np.all(dB == 0)
    # against the formulas written with numpy
    rng = np.random.RandomState(2)
    keep = (rng.rand(*p["x"].shape) > 0.3).astype(np.float64)
    ks, sc = 1.0 / 0.7, p["alpha"] / 4
    xt = p["x"] * keep * ks
    y3, _ = oracle.forward_dropout(p["x"], p["Wd"], p["A"], p["B"], p["alpha"], keep, ks)
    assert _rel(y3, p["x"] @ p["Wd"].T + sc * (xt @ p["A"].T) @ p["B"].T) < RTOL
    dx3 = oracle.backward_dx_dropout(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"], keep, ks)
    assert _rel(dx3, p["dy"] @ p["Wd"] + sc * ((p["dy"] @ p["B"]) @ p["A"]) * keep * ks) < RTOL


def test_lora_dropout_gradients_by_finite_differences():
    # with the mask fixed, L = <dY, y> is still linear in each of x, A, B
    p = _small_problem(630, M=5, N=9, K=64, r=4, b=3, G=32)
    rng = np.random.RandomState(3)
    keep = (rng.rand(*p["x"].shape) > 0.25).astype(np.float64)
    ks = 1.0 / 0.75
    L = lambda x, A, B: float(np.sum(p["dy"] * oracle.forward_dropout(x, p["Wd"], A, B, p["alpha"], keep, ks)[0]))
    dx = oracle.backward_dx_dropout(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"], keep, ks)
    dA, dB = oracle.backward_adapters_dropout(p["dy"], p["x"], p["A"], p["B"], p["alpha"], keep, ks)
    h = 1e-3
    for name, grad in (("x", dx), ("A", dA), ("B", dB)):
        for _ in range(12):
            idx = tuple(rng.randint(0, s) for s in grad.shape)
            args = {k: p[k].copy() for k in ("x", "A", "B")}
            args[name][idx] += h
            up = L(args["x"], args["A"], args["B"])
            args[name][idx] -= 2 * h
            dn = L(args["x"], args["A"], args["B"])
            fd = (up - dn) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-8 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])


def test_backward_adjoint_identities():
    p = _small_problem(700, M=11, N=24, K=128, r=8, b=4, G=64)
    fwd = lambda x, A, B: oracle.forward(x, p["Wd"], A, B, p["alpha"])[0]
    dx = oracle.backward_dx(p["dy"], p["Wd"], p["A"], p["B"], p["alpha"])
    dA, dB = oracle.backward_adapters(p["dy"], p["x"], p["A"], p["B"], p["alpha"])
    y0 = fwd(p["x"], p["A"], p["B"])
    v = wl.normal(701, p["x"].size).reshape(p["x"].shape)
    VA = wl.normal(702, p["A"].size).reshape(p["A"].shape)
    VB = wl.normal(703, p["B"].size).reshape(p["B"].shape)
    lhs_x = np.sum(p["dy"] * (fwd(p["x"] + v, p["A"], p["B"]) - y0))
    lhs_A = np.sum(p["dy"] * (fwd(p["x"], p["A"] + VA, p["B"]) - y0))
    lhs_B = np.sum(p["dy"] * (fwd(p["x"], p["A"], p["B"] + VB) - y0))
    assert abs(lhs_x - np.sum(dx * v)) < 1e-9 * abs(lhs_x)
    assert abs(lhs_A - np.sum(dA * VA)) < 1e-9 * abs(lhs_A)
    assert abs(lhs_B - np.sum(dB * VB)) < 1e-9 * abs(lhs_B)


def test_backward_special_cases():
    p = _small_problem(800, M=7, N=16, K=64, r=8, b=4, G=32)
    Z_B = np.zeros_like(p["B"])
    Z_A = np.zeros_like(p["A"])
    dA, dB = oracle.backward_adapters(p["dy"], p["x"], p["A"], Z_B, p["alpha"])
    assert np.all(dA == 0.0) and np.any(dB != 0.0)                  # B = 0  =>  dA = 0
    dx = oracle.backward_dx(p["dy"], p["Wd"], p["A"], Z_B, p["alpha"])
    assert _rel(dx, p["dy"] @ p["Wd"]) < RTOL                        # and dX is the pure dY Wd
    dA, dB = oracle.backward_adapters(p["dy"], p["x"], Z_A, p["B"], p["alpha"])
    assert np.all(dB == 0.0) and np.any(dA != 0.0)                  # A = 0  =>  dB = 0


def test_layer_oracle_row_subsets_equal_full_rows():
    inp = wl.make_inputs(wl.config1())
    c = inp.cfg
    lo = oracle.LayerOracle(inp.codes, inp.scales, inp.zeros, inp.A, inp.B, bits=c.bits,
                            group_size=c.group_size, alpha=c.alpha, dtype=c.dtype)
    y, t = lo.forward(inp.x)
    rows = np.array([3, 17, 63])
    ys, ts = lo.forward(inp.x, rows)
    assert np.array_equal(ys, y[rows]) and np.array_equal(ts, t[rows])
    dx = lo.backward_dx(inp.dy)
    assert np.array_equal(lo.backward_dx(inp.dy, rows), dx[rows])
    # config 1 against numpy on the widened stored values
    W = _np_dequant(inp.codes, oracle.widen(inp.scales, "f16"), inp.zeros, c.group_size)
    X = oracle.widen(inp.x, "f16")
    ref = X @ W.T + 2.0 * (X @ oracle.widen(inp.A, "f16").T) @ oracle.widen(inp.B, "f16").T
    assert _rel(y, ref) < RTOL


# ------------------------------------------------- activation-order checkpoints (App. A)

def _actorder_case(b=4, N=5, K=192, G=32, seed=901):
    codes = wl.uniform_ints(seed, N * K, 1 << b).reshape(N, K)
    s = wl.uniform_range(seed + 1, N * (K // G), 0.002, 0.05).reshape(N, K // G)
    z = wl.uniform_ints(seed + 2, N * (K // G), 1 << b).reshape(N, K // G)
    g_idx = wl.actorder_g_idx(seed + 3, K, G)
    return codes, s, z, g_idx


def test_actorder_generator_gives_full_groups_in_scattered_columns():
    g_idx = wl.actorder_g_idx(5, 256, 32)
    assert g_idx.dtype == np.int32 and np.array_equal(np.bincount(g_idx), np.full(8, 32))
    assert not np.array_equal(g_idx, np.arange(256) // 32)          # really out of order


def test_actorder_dequant_by_python_loops():
    codes, s, z, g_idx = _actorder_case()
    Wd = oracle.dequant_actorder(codes, s, z, g_idx)
    for n in range(codes.shape[0]):
        for k in range(codes.shape[1]):
            g = int(g_idx[k])
            assert Wd[n, k] == s[n, g] * (float(codes[n, k]) - float(z[n, g]))


def test_actorder_with_consecutive_groups_is_the_plain_dequant():
    codes, s, z, _ = _actorder_case()
    K, G = codes.shape[1], 32
    plain = oracle.dequant(oracle.pack(codes, 4), s, z, K, 4, G)
    assert np.array_equal(oracle.dequant_actorder(codes, s, z, np.arange(K) // G), plain)


def test_actorder_perm_sorts_columns_into_consecutive_groups_and_keeps_the_product():
    b, G = 3, 32
    codes, s, z, g_idx = _actorder_case(b=b, N=6, K=256, G=G, seed=911)
    K = codes.shape[1]
    perm, inv = oracle.actorder_perm(g_idx)
    assert np.array_equal(np.sort(perm), np.arange(K))                       # a permutation
    assert np.array_equal(g_idx[perm], np.arange(K) // G)                    # groups become runs of G columns
    assert np.array_equal(perm[inv], np.arange(K)) and np.array_equal(inv[perm], np.arange(K))
    for g in range(K // G):                                                  # stable: original order inside a group
        assert np.all(np.diff(perm[g * G:(g + 1) * G]) > 0)
    # the layer in sorted coordinates: same weight entries, so the same product up to summation order
    W_act = oracle.dequant_actorder(codes, s, z, g_idx)
    W_sorted = oracle.dequant(oracle.pack(codes[:, perm], b), s, z, K, b, G)
    assert np.array_equal(W_sorted, W_act[:, perm])
    x = wl.normal(912, 4 * K).reshape(4, K)
    np.testing.assert_allclose(x[:, perm] @ W_sorted.T, x @ W_act.T, rtol=1e-12, atol=1e-12)
    dy = wl.normal(913, 4 * 6).reshape(4, 6)
    np.testing.assert_allclose((dy @ W_sorted)[:, inv], dy @ W_act, rtol=1e-12, atol=1e-12)


# ------------------------------------------------- packed zero-points

def test_packed_zero_points_hand_derived():
    # INT4, 5 groups: fields 0x3, 0xA, 0xF, 0x0, 0x7 from bit 0 upwards -> 0x000 7 0 F A 3
    P = oracle.pack_zeros(np.array([[3, 10, 15, 0, 7]], np.uint8), 4)
    assert P.shape == (1, 1) and P[0, 0] == 0x00070FA3
    # INT3, 11 groups = 33 bits: the eleventh field (value 5 = 0b101) straddles the word boundary at bit 30
    z = np.array([[1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 5]], np.uint8)
    P = oracle.pack_zeros(z, 3)
    stream = sum(int(v) << (3 * i) for i, v in enumerate(z[0]))
    assert P.shape == (1, 2) and P[0, 0] == stream & 0xFFFFFFFF and P[0, 1] == stream >> 32 == 0b1
    # INT2: 0b11, 0b00, 0b10 -> 0b10_00_11 ; INT8: bytes in order
    assert oracle.pack_zeros(np.array([[3, 0, 2]], np.uint8), 2)[0, 0] == 0b100011
    assert oracle.pack_zeros(np.array([[0x12, 0x34, 0x56, 0x78, 0x9A]], np.uint8), 8).tolist() == [[0x78563412, 0x9A]]


@pytest.mark.parametrize("b", [2, 3, 4, 8])
@pytest.mark.parametrize("groups", [1, 7, 32, 33, 86, 344])
def test_packed_zero_points_match_bigint_stream_and_roundtrip(b, groups):
    N = 6
    z = wl.uniform_ints(4321 + 10 * b + groups, N * groups, 1 << b).reshape(N, groups)
    P = oracle.pack_zeros(z, b)
    assert P.shape == (N, oracle.zero_words(groups, b)) == (N, -(-groups * b // 32))
    for n in range(N):
        stream = sum(int(v) << (b * i) for i, v in enumerate(z[n]))
        assert P[n].tolist() == [(stream >> (32 * w)) & 0xFFFFFFFF for w in range(P.shape[1])]
    assert np.array_equal(oracle.unpack_zeros(P, groups, b), z)


# ------------------------------------------------- stacked adapters (App. D)

def test_stacked_adapters_forward_is_the_sum_of_the_two_branches_and_gradients_by_finite_differences():
    p = _small_problem(640, M=4, N=10, K=64, r=8, b=4, G=32)
    f = 6                                                       # frozen rows / columns of the stack
    A, B, x, dy, Wd, alpha = p["A"], p["B"], p["x"], p["dy"], p["Wd"], p["alpha"]
    sc = alpha / A.shape[0]
    # the stack is the sum of its two pairs, both scaled by alpha / (total rank)
    y, _ = oracle.forward(x, Wd, A, B, alpha)
    y_two = x @ Wd.T + sc * (x @ A[:f].T) @ B[:, :f].T + sc * (x @ A[f:].T) @ B[:, f:].T
    np.testing.assert_allclose(y, y_two, rtol=1e-12, atol=1e-12)
    dA_t, dB_t = oracle.backward_adapters_stacked(dy, x, A, B, alpha, f)
    assert dA_t.shape == (2, 64) and dB_t.shape == (10, 2)
    # central differences on trainable entries only (L = <dY, y> is linear in each of A and B)
    L = lambda A_, B_: float(np.sum(dy * oracle.forward(x, Wd, A_, B_, alpha)[0]))
    h = 1e-3
    rng = np.random.RandomState(3)
    for _ in range(10):
        j, k = rng.randint(f, 8), rng.randint(0, 64)
        Ap, Am = A.copy(), A.copy()
        Ap[j, k] += h
        Am[j, k] -= h
        fd = (L(Ap, B) - L(Am, B)) / (2 * h)
        assert abs(fd - dA_t[j - f, k]) <= 1e-8 * max(1.0, abs(fd))
        n = rng.randint(0, 10)
        Bp, Bm = B.copy(), B.copy()
        Bp[n, j] += h
        Bm[n, j] -= h
        fd = (L(A, Bp) - L(A, Bm)) / (2 * h)
        assert abs(fd - dB_t[n, j - f]) <= 1e-8 * max(1.0, abs(fd))
    # nothing frozen: the plain gradients
    dA, dB = oracle.backward_adapters(dy, x, A, B, alpha)
    dA0, dB0 = oracle.backward_adapters_stacked(dy, x, A, B, alpha, 0)
    assert np.array_equal(dA0, dA) and np.array_equal(dB0, dB)
