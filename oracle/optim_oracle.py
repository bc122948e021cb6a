"""CPU oracle of the parameter update (test infrastructure only; numpy fp64).

The paper's workflow ends every mini-batch with "gradient computation and parameter update" (Section 2.3,
step 4) and names no optimiser.  This repository's reading: Adam (Kingma & Ba 2015, Algorithm 1) for the dense
weights, and for the learnable embedding tables the same update applied to the rows a mini-batch touched only
("lazy" / sparse Adam: the moments of untouched rows stay as they are, the bias correction uses the global
step count).  Only tests, the smoke check and the benchmark's CPU baseline may import this file.
"""
import numpy as np


def adam_step(theta, grad, m, v, step, lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8):
    """One update, `step` counted from 1.  Returns new (theta, m, v); inputs are not modified.
        m_t = b1 m + (1 - b1) g;  v_t = b2 v + (1 - b2) g^2
        theta_t = theta - lr * (m_t / (1 - b1^t)) / (sqrt(v_t / (1 - b2^t)) + eps)"""
    theta, grad = np.asarray(theta, np.float64), np.asarray(grad, np.float64)
    m = beta1 * np.asarray(m, np.float64) + (1.0 - beta1) * grad
    v = beta2 * np.asarray(v, np.float64) + (1.0 - beta2) * grad * grad
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    return theta - lr * mhat / (np.sqrt(vhat) + eps), m, v


def adam_rows_step(theta, ids, grad_rows, m, v, step, lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8):
    """The same update on the rows `ids` (distinct) of a table [V, F]; every other row, and its moments, keep
    their values."""
    ids = np.asarray(ids, np.int64)
    assert len(np.unique(ids)) == len(ids)
    theta, m, v = (np.array(a, dtype=np.float64, copy=True) for a in (theta, m, v))
    theta[ids], m[ids], v[ids] = adam_step(theta[ids], grad_rows, m[ids], v[ids], step, lr, beta1, beta2, eps)
    return theta, m, v
