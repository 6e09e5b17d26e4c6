"""GPU parity of qlora_lrec_loss (the LREC objective and its gradient) against the fp64 oracle."""
import numpy as np
import pytest

import oracle
from oracle import lrec
from paper_2306_08162_amd import workloads as wl
from parity import announce, rel_fro

pytestmark = pytest.mark.gpu

# fp32 arithmetic on 16-bit inputs: the per-token values are compared to 2e-5 relative (sums of up to 128k fp32 terms,
# hardware exp2 / log2), the gradient, rounded to the 16-bit dtype (bf16: 2^-9 relative per element), to the layer's bar
TOL_SCALAR, TOL_GRAD = 2e-5, 5e-3


def _inputs(seed, M, V, dtype, spread=4.0, agree=0.7):
    """Teacher logits ~ N(0, spread^2); the student is the teacher plus noise (a quantized model tracks its teacher)."""
    zt = wl.normal(seed, M * V).reshape(M, V) * spread
    zs = agree * zt + wl.normal(seed + 1, M * V).reshape(M, V) * spread * (1 - agree)
    labels = (wl.splitmix64(seed + 2, 0, M) % np.uint64(V)).astype(np.int32)
    return wl.to_bits(zs.ravel(), dtype).reshape(M, V), wl.to_bits(zt.ravel(), dtype).reshape(M, V), labels


def _run(zs_bits, zt_bits, labels, lkl, lce, dtype, want_grad=True, want_parts=True, grad_scale=None):
    import torch
    from paper_2306_08162_amd import binding as ql
    M, V = zs_bits.shape
    dev = torch.device("cuda:0")
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a.view(np.int16))).to(dev)
    zs, zt = up(zs_bits), up(zt_bits)
    lab = torch.from_numpy(labels.astype(np.int32)).to(dev)
    kl = torch.empty(M, dtype=torch.float32, device=dev) if want_parts else None
    ce = torch.empty(M, dtype=torch.float32, device=dev) if want_parts else None
    mean = torch.empty(1, dtype=torch.float32, device=dev)
    grad = torch.empty((M, V), dtype=torch.int16, device=dev) if want_grad else None
    ws = torch.empty(ql.qlora_lrec_workspace_bytes(M), dtype=torch.uint8, device=dev)
    flag = ql.QLORA_BF16 if dtype == "bf16" else ql.QLORA_F16
    if grad_scale is None:
        ql.qlora_lrec_loss(zs, zt, lab, lkl, lce, kl, ce, mean, grad, M, V, flag, ws)
    else:
        ql.qlora_lrec_loss_scaled(zs, zt, lab, lkl, lce, grad_scale, kl, ce, mean, grad, M, V, flag, ws)
    torch.cuda.synchronize()
    return (kl.cpu().numpy() if want_parts else None, ce.cpu().numpy() if want_parts else None,
            float(mean.cpu().numpy()[0]), grad.cpu().numpy().view(np.uint16) if want_grad else None)


def _compare(what, zs, zt, lab, dtype, lkl, lce, grad_scale=None):
    """Run the library on raw 16-bit logits and hold it against the oracle: per-token KL and CE and the mean to
    TOL_SCALAR; the gradient to TOL_GRAD as a whole, row by row, and once more with the target entries left out (with
    lambda_CE = 120 they carry most of the norm, and would hide the other V - 1 entries of a row)."""
    M, V = zs.shape
    announce(f"lrec loss {what}: M={M} V={V} {dtype} lambda_kl={lkl} lambda_ce={lce} grad_scale={grad_scale}")
    kl, ce, mean, grad = _run(zs, zt, lab, lkl, lce, dtype, grad_scale=grad_scale)
    # the library treats a label that is not below V like a negative one; the oracle only knows the negative form
    lab_o = np.where(lab < V, lab, -1)
    okl, oce, omean, ograd = lrec.lrec_loss(oracle.widen(zs, dtype), oracle.widen(zt, dtype), lab_o, lkl, lce)
    g = oracle.widen(grad, dtype) / (1.0 if grad_scale is None else grad_scale)
    off = np.ones((M, V), dtype=bool)                         # everything but the target entries
    off[np.nonzero(lab_o >= 0)[0], lab_o[lab_o >= 0]] = False
    # Per token.  KL and CE come out of log-sum-exps of the size of the largest logit, formed in fp32: the error
    # of a value that happens to be much smaller than that (two nearly equal distributions) is relative to the
    # logits, not to the value.  Likewise a gradient row is a difference of probabilities times lambda / M: a row
    # that is almost zero (the target is the dominant logit) is held to an absolute error on that scale.
    zmax = 1.0 + np.abs(oracle.widen(zs, dtype).max(axis=1)) + np.abs(oracle.widen(zt, dtype).max(axis=1))   # size of the lse's
    nat = (abs(lkl) + abs(lce)) / M
    rows = np.linalg.norm(g - ograd, axis=1) / (np.linalg.norm(ograd, axis=1) + 1e-3 * nat)
    errs = {"kl": float(np.max(np.abs(kl - okl) / (np.abs(okl) + zmax))),
            "ce": float(np.max(np.abs(ce - oce) / (np.abs(oce) + zmax))),
            "mean": abs(mean - omean) / (abs(omean) + (abs(lkl) + abs(lce)) * float(zmax.mean())),
            "kl_all": rel_fro(kl, okl), "ce_all": rel_fro(ce, oce),
            "grad": rel_fro(g, ograd), "grad_worst_row": float(rows.max()),
            "grad_off_target": rel_fro(g * off, ograd * off)}
    announce(" ".join(f"{k}={v:.2e}" for k, v in errs.items()))
    assert np.all(np.isfinite(g))
    assert errs["kl"] <= TOL_SCALAR and errs["ce"] <= TOL_SCALAR and errs["mean"] <= TOL_SCALAR
    assert errs["grad"] <= TOL_GRAD and errs["grad_worst_row"] <= TOL_GRAD
    return grad, errs


def _check(seed, M, V, dtype, lkl, lce, labels=None):
    zs, zt, lab = _inputs(seed, M, V, dtype)
    if labels is not None:
        lab = labels
    # Without loss scaling the 1 / M of the mean leaves only part of an fp16 row representable: the off-target
    # figure is held to the bar only where the row count leaves the entries normal numbers.
    grad, errs = _compare("seeded", zs, zt, lab, dtype, lkl, lce)
    assert errs["kl_all"] <= TOL_SCALAR and errs["ce_all"] <= TOL_SCALAR      # over all tokens, relative to their norm
    if dtype == "bf16" or M <= 16:
        assert errs["grad_off_target"] <= TOL_GRAD
    return grad


CASES = [
    # (M, V, dtype, lambda_kl, lambda_ce): the factor pairs are rows of the paper's Appendix C table
    (5, 8, "f16", 1.0, 120.0),
    (3, 504, "bf16", 1.0, 40.0),
    (16, 4096, "f16", 1.0, 10.0),            # exactly one 8-element piece per thread
    (7, 4104, "f16", 0.5, 120.0),            # one piece more than that
    (9, 32000, "f16", 1.0, 120.0),           # LLaMA vocabulary: eight pieces per thread
    (4, 32000, "bf16", 1.0, 10.0),
    (2, 65536, "f16", 1.0, 40.0),            # sixteen pieces per thread: the most that stay in registers
    (2, 70000, "bf16", 1.0, 40.0),           # beyond: every sweep reads the rows again
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "M{}_V{}_{}".format(*c[:3]))
def test_lrec_loss_shapes(case):
    M, V, dtype, lkl, lce = case
    _check(100 * M + V % 97, M, V, dtype, lkl, lce)


def test_lrec_loss_edge_cases():
    M, V = 6, 1024
    zs, zt, lab = _inputs(11, M, V, "f16")
    # no targets at all, targets out of range: no CE term, gradient of the divergence only
    lab2 = np.array([-1, 5, V, 0, V - 1, -7], np.int32)
    _check(11, M, V, "f16", 1.0, 120.0, labels=lab2)
    # student == teacher: KL is zero (up to rounding of the log-sum-exp) and the gradient is that of the cross entropy
    kl, ce, mean, grad = _run(zs, zs, lab, 3.0, 1.0, "f16")
    assert np.all(np.abs(kl) <= 1e-5)
    p = np.exp(lrec.log_softmax(oracle.widen(zs, "f16")))
    want = (p - np.eye(V)[lab]) / M
    assert rel_fro(oracle.widen(grad, "f16"), want) <= TOL_GRAD
    # objective only (no gradient buffer, no per-token outputs): the same mean
    mean2 = _run(zs, zt, lab, 1.0, 120.0, "f16", want_grad=False, want_parts=False)[2]
    mean1 = _run(zs, zt, lab, 1.0, 120.0, "f16")[2]
    assert mean1 == mean2


def test_lrec_loss_hard_rows():
    """Rows unlike the seeded ones: a dominant logit (a confident language model), masked vocabulary entries at the
    most negative fp16 value, and a student far from its teacher."""
    M, V = 6, 4096
    for dtype in ("f16", "bf16"):
        zs, zt, lab = _inputs(41, M, V, dtype)
        # one logit 25 above everything else, the same one in both models, and it is the target in half of the rows
        top = (wl.splitmix64(42, 0, M) % np.uint64(V)).astype(np.int64)
        zs_f, zt_f = oracle.widen(zs, dtype), oracle.widen(zt, dtype)
        zs_f[np.arange(M), top] = zs_f.max(axis=1) + 25.0
        zt_f[np.arange(M), top] = zt_f.max(axis=1) + 25.0
        lab2 = lab.copy()
        lab2[::2] = top[::2]
        _compare("dominant logit", wl.to_bits(zs_f.ravel(), dtype).reshape(M, V),
                 wl.to_bits(zt_f.ravel(), dtype).reshape(M, V), lab2, dtype, 1.0, 120.0, grad_scale=1024.0)
        # the student disagrees: its dominant logit sits elsewhere
        zs_g = oracle.widen(zs, dtype)
        zs_g[np.arange(M), (top + 7) % V] = zs_g.max(axis=1) + 25.0
        _compare("dominant logits apart", wl.to_bits(zs_g.ravel(), dtype).reshape(M, V),
                 wl.to_bits(zt_f.ravel(), dtype).reshape(M, V), lab2, dtype, 1.0, 40.0, grad_scale=1024.0)
        # masked entries (the most negative fp16 number, exactly representable in bf16 too): in both models at the
        # same places, and in the student alone
        masked = (wl.splitmix64(43, 0, 64) % np.uint64(V)).astype(np.int64)
        zs_m, zt_m = oracle.widen(zs, dtype), oracle.widen(zt, dtype)
        low = -65504.0 if dtype == "f16" else -65280.0
        zs_m[:, masked] = low
        zt_m[:, masked] = low
        lab3 = np.where(np.isin(lab, masked), (lab + 1) % V, lab).astype(np.int32)
        lab3 = np.where(np.isin(lab3, masked), -1, lab3).astype(np.int32)
        _compare("masked in both", wl.to_bits(zs_m.ravel(), dtype).reshape(M, V),
                 wl.to_bits(zt_m.ravel(), dtype).reshape(M, V), lab3, dtype, 1.0, 120.0, grad_scale=256.0)
        _compare("masked in the student", wl.to_bits(zs_m.ravel(), dtype).reshape(M, V), zt, lab3, dtype, 1.0, 10.0,
                 grad_scale=256.0)
    # student and teacher unrelated, wide logits: KL of the order of the spread
    zt = wl.to_bits(wl.normal(51, M * V) * 8.0, "f16").reshape(M, V)
    zs = wl.to_bits(wl.normal(52, M * V) * 8.0, "f16").reshape(M, V)
    lab = (wl.splitmix64(53, 0, M) % np.uint64(V)).astype(np.int32)
    _compare("student far from teacher", zs, zt, lab, "f16", 1.0, 120.0, grad_scale=64.0)


def test_lrec_loss_scaling_keeps_the_small_entries():
    """2048 x 32000 in fp16: the mean's 1 / M makes a typical off-target entry ~1e-8, below the smallest normal fp16
    number.  With grad_scale = 2^14 the sampled rows match the oracle entry by entry, target entries left out."""
    M, V = 2048, 32000
    zs, zt, lab = _inputs(31, M, V, "f16")
    scale = 16384.0
    announce(f"lrec loss M={M} V={V} f16 grad_scale={scale} (sampled rows, off-target entries)")
    kl, ce, mean, grad = _run(zs, zt, lab, 1.0, 120.0, "f16", grad_scale=scale)
    kl1, ce1, mean1, _ = _run(zs, zt, lab, 1.0, 120.0, "f16", want_grad=False)
    assert np.array_equal(kl, kl1) and np.array_equal(ce, ce1) and mean == mean1      # the objective is not scaled
    rows = np.unique(np.concatenate([[0, M - 1], (wl.splitmix64(32, 0, 14) % np.uint64(M)).astype(np.int64)]))
    _, _, _, ograd = lrec.lrec_loss(oracle.widen(zs[rows], "f16"), oracle.widen(zt[rows], "f16"), lab[rows], 1.0, 120.0)
    ograd = ograd * len(rows) / M
    g = oracle.widen(grad[rows], "f16") / scale
    off = np.ones(g.shape, dtype=bool)
    off[np.arange(len(rows)), lab[rows]] = False
    e_all, e_off = rel_fro(g, ograd), rel_fro(g * off, ograd * off)
    announce(f"grad={e_all:.2e} grad_off_target={e_off:.2e}")
    assert e_all <= TOL_GRAD and e_off <= TOL_GRAD


def test_lrec_loss_is_bitwise_reproducible():
    zs, zt, lab = _inputs(21, 33, 32000, "f16")
    a = _run(zs, zt, lab, 1.0, 120.0, "f16")
    b = _run(zs, zt, lab, 1.0, 120.0, "f16")
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and a[2] == b[2] and np.array_equal(a[3], b[3])


def test_lrec_loss_full_size_sampled_rows():
    """The size bench.py times (2048 tokens x 32000 logits): the oracle checks a seeded sample of rows in full."""
    M, V = 2048, 32000
    zs, zt, lab = _inputs(31, M, V, "f16")
    announce(f"lrec loss M={M} V={V} f16 (sampled rows)")
    kl, ce, mean, grad = _run(zs, zt, lab, 1.0, 120.0, "f16")
    rows = np.unique(np.concatenate([[0, M - 1], (wl.splitmix64(32, 0, 30) % np.uint64(M)).astype(np.int64)]))
    okl, oce, _, ograd = lrec.lrec_loss(oracle.widen(zs[rows], "f16"), oracle.widen(zt[rows], "f16"), lab[rows], 1.0, 120.0)
    assert rel_fro(kl[rows], okl) <= TOL_SCALAR and rel_fro(ce[rows], oce) <= TOL_SCALAR
    # the oracle's gradient is scaled by 1 / (rows handed to it); the library's by 1 / M
    assert rel_fro(oracle.widen(grad[rows], "f16"), ograd * len(rows) / M) <= TOL_GRAD
    # the mean follows from the per-token values, which the sample pins: check the reduction itself in fp64
    assert abs(mean - float(np.mean(1.0 * kl.astype(np.float64) + 120.0 * ce.astype(np.float64)))) <= 1e-5 * abs(mean)
