"""Oracle: one decoupled-weight-decay Adam (AdamW) step in fp64 (test infrastructure only).

Alg. 1's commit step names no optimiser; the benchmark configuration names AdamW, so the
oracle is the textbook definition (Loshchilov & Hutter, "Decoupled Weight Decay
Regularization", Alg. 2 with the schedule multiplier folded into lr), step count t from 1:

    p  <- p - lr * wd * p
    m  <- beta1 * m + (1 - beta1) * g
    v  <- beta2 * v + (1 - beta2) * g * g
    p  <- p - lr * (m / (1 - beta1**t)) / (sqrt(v / (1 - beta2**t)) + eps)

All arithmetic in float64 whatever the storage type of the inputs; the caller rounds the
results to its storage type.
"""
import numpy as np


def adamw_step(p, m, v, g, t, lr, beta1, beta2, eps, weight_decay):
    p = np.asarray(p, np.float64)
    m = np.asarray(m, np.float64)
    v = np.asarray(v, np.float64)
    g = np.asarray(g, np.float64)
    lr, beta1, beta2, eps, weight_decay = map(float, (lr, beta1, beta2, eps, weight_decay))
    assert t >= 1
    p = p - lr * weight_decay * p
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * (g * g)
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    p = p - lr * m_hat / (np.sqrt(v_hat) + eps)
    return p, m, v
