"""fp64 oracle of the LREC objective and its gradient -- TEST INFRASTRUCTURE ONLY.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may import this module.  It shares
nothing with the HIP library.  Plain numpy, float64, the definitions written out; no blocking, no fusion.

What is computed (Sec. 3.2 "Optimization", Eq. 1 and Eq. 2 of the paper): for every token position the student's
(quantized, LoRA-injected model's) output distribution y_hat and the teacher's (full-precision model's) y over the
vocabulary, the divergence D_KL(y_hat || y) = sum_i y_hat_i log(y_hat_i / y_i) -- student first, as the paper writes
it -- and the cross entropy of y_hat against the true next token; the objective is the mean over the token positions
of lambda_KL * D_KL + lambda_CE * CE (Eq. 2, with the scaling factors of Appendix C).

Readings (the paper gives the formulas only):
  * y_hat and y are softmax distributions of the two models' logits; the cached teacher targets (Appendix C) are taken
    to be its logits.
  * CE is printed with its arguments in an unusual order (y_hat_i log y*_i, which is undefined for a one-hot y*); it
    is read as the usual next-token cross entropy, CE = -log y_hat[label].  A negative label means "no target
    here": that position contributes no CE term (it still counts in the mean).
  * the expectation is the mean over the M token positions handed in.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def log_softmax(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, np.float64)
    m = z.max(axis=-1, keepdims=True)
    return z - (m + np.log(np.exp(z - m).sum(axis=-1, keepdims=True)))


def lrec_loss(student_logits: np.ndarray, teacher_logits: np.ndarray, labels: np.ndarray, lambda_kl: float,
              lambda_ce: float) -> Tuple[np.ndarray, np.ndarray, float, np.ndarray]:
    """Returns (kl[M], ce[M], mean objective, d(mean objective)/d(student_logits)[M,V])."""
    ls = log_softmax(student_logits)                 # log y_hat
    lt = log_softmax(teacher_logits)                 # log y
    p = np.exp(ls)                                   # y_hat
    M, V = p.shape
    labels = np.asarray(labels, np.int64)
    kl = (p * (ls - lt)).sum(axis=1)                 # Eq. 1, left
    has = labels >= 0
    ce = np.zeros(M)
    ce[has] = -ls[np.nonzero(has)[0], labels[has]]   # Eq. 1, right (read as next-token cross entropy)
    loss = float((lambda_kl * kl + lambda_ce * ce).mean())          # Eq. 2
    # gradient with respect to the student logits z (y_hat = softmax(z)):
    #   d KL / d z_k = y_hat_k * ((log y_hat_k - log y_k) - KL)
    #   d CE / d z_k = y_hat_k - [k == label]
    g = lambda_kl * p * ((ls - lt) - kl[:, None])
    onehot = np.zeros_like(p)
    onehot[np.nonzero(has)[0], labels[has]] = 1.0
    g = g + lambda_ce * (p * has[:, None] - onehot)
    return kl, ce, loss, g / M
