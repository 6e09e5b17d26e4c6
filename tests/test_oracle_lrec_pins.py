"""Pins of the LREC-objective oracle (oracle/lrec.py) against things that do not depend on it: closed forms,
brute-force loops over probabilities, finite differences, invariances and the inequalities the definitions imply
(Sec. 3.2, Eq. 1 and 2 of the paper)."""
import math

import numpy as np
import pytest

from oracle import lrec


def _softmax_loops(z):
    e = [math.exp(v - max(z)) for v in z]
    s = sum(e)
    return [v / s for v in e]


def _brute(zs, zt, labels, lkl, lce):
    """Per-token KL and CE and the mean objective from explicit probabilities, pure Python."""
    kls, ces = [], []
    for row_s, row_t, lab in zip(zs, zt, labels):
        p, q = _softmax_loops(list(row_s)), _softmax_loops(list(row_t))
        kls.append(sum(pi * math.log(pi / qi) for pi, qi in zip(p, q)))
        ces.append(-math.log(p[lab]) if lab >= 0 else 0.0)
    loss = sum(lkl * k + lce * c for k, c in zip(kls, ces)) / len(kls)
    return kls, ces, loss


def test_two_class_closed_form():
    # V = 2: y_hat = (sigma(a), 1 - sigma(a)) with a = z0 - z1, likewise y with b: everything is a scalar formula
    a, b = 0.7, -1.3
    sig = lambda v: 1.0 / (1.0 + math.exp(-v))
    p, q = sig(a), sig(b)
    kl_want = p * math.log(p / q) + (1 - p) * math.log((1 - p) / (1 - q))
    kl, ce, loss, g = lrec.lrec_loss(np.array([[a, 0.0]]), np.array([[b, 0.0]]), np.array([1]), 2.0, 3.0)
    assert abs(kl[0] - kl_want) < 1e-14
    assert abs(ce[0] + math.log(1 - p)) < 1e-14
    assert abs(loss - (2.0 * kl_want + 3.0 * (-math.log(1 - p)))) < 1e-13
    # d/da of 2 KL + 3 CE, by hand: dKL/da = p (1-p) (log(p/q) - log((1-p)/(1-q))), dCE/da = p (label is class 1)
    want = 2.0 * p * (1 - p) * (math.log(p / q) - math.log((1 - p) / (1 - q))) + 3.0 * p
    assert abs(g[0, 0] - want) < 1e-13 and abs(g[0, 1] + want) < 1e-13


@pytest.mark.parametrize("M,V", [(3, 5), (4, 17), (1, 2)])
def test_matches_brute_force_probabilities(M, V):
    rng = np.random.RandomState(10 * M + V)
    zs, zt = rng.randn(M, V) * 3, rng.randn(M, V) * 3
    labels = rng.randint(0, V, M)
    if M > 2:
        labels[1] = -1          # a position without a target
    kl, ce, loss, _ = lrec.lrec_loss(zs, zt, labels, 1.0, 120.0)        # the 7B INT2 factors of Appendix C
    bk, bc, bl = _brute(zs, zt, labels, 1.0, 120.0)
    assert np.allclose(kl, bk, rtol=0, atol=1e-13) and np.allclose(ce, bc, rtol=0, atol=1e-13)
    assert abs(loss - bl) < 1e-11


def test_special_cases():
    rng = np.random.RandomState(3)
    z = rng.randn(6, 33) * 2
    lab = rng.randint(0, 33, 6)
    # equal distributions: the divergence and its gradient vanish, the gradient is that of the cross entropy alone
    kl, ce, loss, g = lrec.lrec_loss(z, z + 5.0, lab, 7.0, 1.0)        # a constant shift of the logits changes nothing
    assert np.all(np.abs(kl) < 1e-14)
    p = np.exp(lrec.log_softmax(z))
    onehot = np.eye(33)[lab]
    assert np.allclose(g, (p - onehot) / 6, atol=1e-15)
    # uniform student: CE = log V whatever the label; against a uniform teacher KL = 0
    kl, ce, _, _ = lrec.lrec_loss(np.zeros((2, 1000)), np.full((2, 1000), -4.0), np.array([0, 999]), 1.0, 1.0)
    assert np.all(np.abs(kl) < 1e-12) and np.allclose(ce, math.log(1000), atol=1e-12)
    # lambda_CE = 0 and no labels give the same thing
    a = lrec.lrec_loss(z, z[::-1], lab, 2.0, 0.0)
    b = lrec.lrec_loss(z, z[::-1], np.full(6, -1), 2.0, 9.0)
    assert np.allclose(a[0], b[0]) and abs(a[2] - b[2]) < 1e-15 and np.allclose(a[3], b[3], atol=1e-16)


def test_inequalities_and_invariances():
    rng = np.random.RandomState(4)
    zs, zt = rng.randn(9, 50) * 4, rng.randn(9, 50) * 4
    lab = rng.randint(0, 50, 9)
    kl, ce, loss, g = lrec.lrec_loss(zs, zt, lab, 1.0, 10.0)
    assert np.all(kl >= 0) and np.all(ce >= 0)                           # Gibbs' inequality; -log of a probability
    assert np.all(np.abs(g.sum(axis=1)) < 1e-15)                        # softmax: every row of the gradient sums to zero
    shift_s, shift_t = rng.randn(9, 1) * 10, rng.randn(9, 1) * 10
    kl2, ce2, loss2, g2 = lrec.lrec_loss(zs + shift_s, zt + shift_t, lab, 1.0, 10.0)
    assert np.allclose(kl, kl2, atol=1e-12) and np.allclose(ce, ce2, atol=1e-12) and np.allclose(g, g2, atol=1e-14)
    # KL is not symmetric: the order "student first" matters (Eq. 1 as printed)
    kl_rev = lrec.lrec_loss(zt, zs, lab, 1.0, 10.0)[0]
    assert not np.allclose(kl, kl_rev, rtol=1e-3)


def test_gradient_by_finite_differences():
    rng = np.random.RandomState(5)
    zs, zt = rng.randn(4, 12) * 2, rng.randn(4, 12) * 2
    lab = np.array([3, -1, 0, 11])
    f = lambda z: lrec.lrec_loss(z, zt, lab, 1.0, 40.0)[2]              # the 7B INT3 factors of Appendix C
    g = lrec.lrec_loss(zs, zt, lab, 1.0, 40.0)[3]
    h = 1e-5
    for m in range(4):
        for k in range(12):
            zp, zm = zs.copy(), zs.copy()
            zp[m, k] += h
            zm[m, k] -= h
            fd = (f(zp) - f(zm)) / (2 * h)
            assert abs(fd - g[m, k]) < 1e-8 * max(1.0, abs(fd)), (m, k, fd, g[m, k])
