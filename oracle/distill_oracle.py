"""TEST INFRASTRUCTURE ONLY: the united-expert distillation of the paper's section "United Expert Model",
written out plainly in numpy float64.  Nothing under the package imports it.

One student FFN (the united expert of a group) is fitted to its group of teacher FFNs (the original experts)
on calibration tokens X by minimising the section's MSE equation

    L = (1/k) sum_i || H_u - H_o^i ||^2          (squared norm summed over features, averaged over tokens)

with H = FFN(X) = (silu(X W1^T) * (X W3^T)) W2^T.  The paper fixes neither the optimiser nor its settings;
the reading taken here (and by the library) is full-batch Adam (beta1 0.9, beta2 0.999, eps 1e-8, bias
corrected), started from the student weights handed in (the library starts from the parameter mean).

Pinned by tests/test_oracle_distill.py: analytic gradients against central finite differences, the way = 1
fixed point (student = teacher: loss 0, gradients 0), the closed form of the minimiser over H_u (the mean
teacher output), and descent of the loss.
"""
import numpy as np


def silu(g):
    return g / (1.0 + np.exp(-g))


def ffn(x, w1, w3, w2):
    """x [n,d], w1/w3 [F,d], w2 [d,F] -> [n,d]"""
    return (silu(x @ w1.T) * (x @ w3.T)) @ w2.T


def loss(x, student, teachers):
    """The MSE equation: mean over the k teachers of ||H_u - H_o^i||^2, averaged over the n tokens."""
    hu = ffn(x, *student)
    n, k = x.shape[0], len(teachers)
    return sum(((hu - ffn(x, *t)) ** 2).sum() for t in teachers) / (k * n)


def loss_and_grads(x, student, teachers):
    """Loss and its gradients with respect to the student's (w1, w3, w2)."""
    w1, w3, w2 = student
    n, k = x.shape[0], len(teachers)
    g = x @ w1.T
    u = x @ w3.T
    sig = 1.0 / (1.0 + np.exp(-g))
    a = silu(g) * u
    hu = a @ w2.T
    targets = [ffn(x, *t) for t in teachers]
    val = sum(((hu - t) ** 2).sum() for t in targets) / (k * n)
    d_hu = (2.0 / (k * n)) * sum(hu - t for t in targets)             # [n,d]
    d_w2 = d_hu.T @ a                                                  # [d,F]
    d_a = d_hu @ w2                                                    # [n,F]
    d_g = d_a * u * (sig * (1.0 + g * (1.0 - sig)))
    d_u = d_a * (g * sig)
    return val, (d_g.T @ x, d_u.T @ x, d_w2)


def distill(x, student0, teachers, steps, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """Full-batch Adam from student0.  Returns the final student and the loss before every step and after
    the last one (steps + 1 values)."""
    w = [np.array(p, np.float64) for p in student0]
    m = [np.zeros_like(p) for p in w]
    v = [np.zeros_like(p) for p in w]
    hist = []
    for t in range(1, steps + 1):
        val, grads = loss_and_grads(x, tuple(w), teachers)
        hist.append(val)
        for p, gr, mm, vv in zip(w, grads, m, v):
            mm *= beta1
            mm += (1.0 - beta1) * gr
            vv *= beta2
            vv += (1.0 - beta2) * gr * gr
            p -= lr * (mm / (1.0 - beta1 ** t)) / (np.sqrt(vv / (1.0 - beta2 ** t)) + eps)
    hist.append(loss(x, tuple(w), teachers))
    return tuple(w), np.asarray(hist)
