"""Oracle for the optimizer step and the straggling-rate rule: TEST INFRASTRUCTURE, not a product path.

AdamW with decoupled weight decay on fp32 master weights, written from its definition in fp64 (the paper, Sec. 5.1,
only says the model states are sharded ZeRO-1 style; the rule itself is the usual one):
    m_t = b1 m + (1-b1) g;  v_t = b2 v + (1-b2) g^2;  w_t = w - lr ( m_t/(1-b1^t) / (sqrt(v_t/(1-b2^t)) + eps) + wd w )
and the profiler's rule of Sec. 3: rate = measured time per (layer x micro-batch) / reference; a shift is a relative
change of more than the threshold between two consecutive steps.
"""
import numpy as np


def adamw_step(w, m, v, g, t, lr, b1, b2, eps, wd):
    """One step (t = 1 for the first).  Returns (w, m, v) as new fp64 arrays."""
    g = np.asarray(g, dtype=np.float64)
    m = b1 * m + (1.0 - b1) * g
    v = b2 * v + (1.0 - b2) * g * g
    mhat = m / (1.0 - b1 ** t)
    vhat = v / (1.0 - b2 ** t)
    w = w - lr * (mhat / (np.sqrt(vhat) + eps) + wd * w)
    return w, m, v


def straggling_rates(elapsed_ms, units, tau_ref_ms, threshold):
    """elapsed_ms[i], units[i] = layers x micro-batches of step i.  Returns (rates, shifts)."""
    rates, shifts, prev = [], [], None
    for e, u in zip(elapsed_ms, units):
        x = (e / u) / tau_ref_ms
        shifts.append(prev is not None and abs(x - prev) / prev > threshold)
        rates.append(x)
        prev = x
    return rates, shifts
