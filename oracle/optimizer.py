"""fp64 reference for the parameter-server-side streaming operators that
follow the aggregation -- TEST INFRASTRUCTURE ONLY (same rule as the rest of
this package).

Sec. 4.1 (cost model, optimizer term) and Sec. 6 ("Optimizer step accounting
and pipelining"): non-GEMM operators and the optimizer update stay on the
parameter server; Adam runs per weight matrix right after that matrix's
gradient GEMM has been aggregated, at 26 bytes of memory traffic per parameter.

The paper names the optimizer (Adam) and its traffic, not its arithmetic; the
arithmetic below is the published algorithm (Kingma & Ba, Algorithm 1) with
optional decoupled weight decay (Loshchilov & Hutter), written out step by
step:
    m <- b1 m + (1 - b1) g
    v <- b2 v + (1 - b2) g^2
    mhat = m / (1 - b1^t),  vhat = v / (1 - b2^t)
    w <- w - lr (mhat / (sqrt(vhat) + eps) + wd w)
Reading of the 26 bytes: fp32 master weight read + written (8), fp32 m (8),
fp32 v (8), bf16 copy of the new weight written (2); the gradient is the
aggregated sum of the K-split partial blocks and is never stored.
"""
import numpy as np


def adam_step(w, m, v, g, lr, beta1, beta2, eps, weight_decay, step):
    """One Adam update in fp64.  w, m, v, g: arrays of one shape (any float
    dtype, widened exactly); step: 1-based update count.  Returns new (w, m, v)."""
    if step < 1:
        raise ValueError("step counts from 1")
    w = np.asarray(w, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m_new / (1.0 - beta1 ** step)
    v_hat = v_new / (1.0 - beta2 ** step)
    w_new = w - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * w)
    return w_new, m_new, v_new


def bf16_round(x):
    """fp32 -> bf16 round-to-nearest-even, returned as the fp32 value of the
    bf16 number (bit manipulation on the fp32 pattern; NaN not handled)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def add_residual(folded, residual):
    """C = aggregated sum + residual stream, in fp64."""
    return np.asarray(folded, dtype=np.float64) + np.asarray(residual, dtype=np.float64)
