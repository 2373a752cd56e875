"""Test infrastructure only (imported by tests/ and bench legs that time the CPU baseline): one AdamW step in
fp64 numpy, written out from the published update rule (Adam with bias-corrected moments and decoupled
weight decay), which is what a mixed-precision trainer with sharded optimizer state (Section 3 of the paper:
ZeRO-1 and mixed precision) runs on each rank's shard.

    g = grad * grad_scale
    m = beta1 m + (1 - beta1) g
    v = beta2 v + (1 - beta2) g^2
    w = w - lr * ( (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps) + weight_decay * w )
"""
import numpy as np


def adam_step(w, g, m, v, lr, beta1, beta2, eps, weight_decay, grad_scale, t):
    w, g, m, v = (np.asarray(a, dtype=np.float64) for a in (w, g, m, v))
    g = g * grad_scale
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    w = w - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * w)
    return w, m, v
