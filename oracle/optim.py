"""Optimizer updates applied once per step (Section 3.2, step 5).

The paper leaves the optimizer to the framework; the forms below are this
build's reading (parity unpinned by the paper, pinned by closed forms):
  SGD-momentum: v <- mu v + G ; theta <- theta - lr v          (v starts at 0)
  Adam:         m <- b1 m + (1-b1) G ; u <- b2 u + (1-b2) G^2
                theta <- theta - lr (m/(1-b1^t)) / (sqrt(u/(1-b2^t)) + eps), t from 1
"""
import numpy as np


def sgdm_update(theta, G, v, lr, momentum):
    theta = np.asarray(theta, dtype=np.float64)
    v_new = momentum * np.asarray(v, dtype=np.float64) + np.asarray(G, dtype=np.float64)
    return theta - lr * v_new, v_new


def adam_update(theta, G, m, u, t, lr, beta1, beta2, eps):
    """t is the 1-based index of this update."""
    theta = np.asarray(theta, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    m_new = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * G
    u_new = beta2 * np.asarray(u, dtype=np.float64) + (1.0 - beta2) * G * G
    m_hat = m_new / (1.0 - beta1 ** t)
    u_hat = u_new / (1.0 - beta2 ** t)
    return theta - lr * m_hat / (np.sqrt(u_hat) + eps), m_new, u_new
