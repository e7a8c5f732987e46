"""Float64 oracle of the optimiser step the paper trains its Transformers with (App. B, training
configuration table): Adam with bias correction and the inverse-square-root learning-rate schedule
with linear warm-up.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path imports this module; only tests/,
__graft_entry__.smoke() and bench.py's cpu_baseline leg may.  It shares no code with the HIP path.

The update is the plain definition of Adam (the algorithm the paper cites by name), written out:
    m_t = b1 m_{t-1} + (1 - b1) g          v_t = b2 v_{t-1} + (1 - b2) g^2
    mhat = m_t / (1 - b1^t)                vhat = v_t / (1 - b2^t)
    theta_t = theta_{t-1} - lr_t mhat / (sqrt(vhat) + eps)
Readings where the paper is silent: steps count from 1; eps is added to the root of the
bias-corrected second moment; no weight decay, no gradient clipping; in a bf16 run the weights are
kept in fp32 ("master") and the bf16 parameters are their round-to-nearest-even image.
"""
import numpy as np

BETA1, BETA2, EPS, WARMUP = 0.9, 0.98, 1e-9, 4000   # App. B


def lr_schedule(step, d_model=1024, warmup=WARMUP):
    """App. B: d_model^-0.5 * min(step^-0.5, step * warmup^-1.5), step >= 1."""
    if step < 1:
        raise ValueError("steps count from 1")
    return float(d_model) ** -0.5 * min(float(step) ** -0.5, float(step) * float(warmup) ** -1.5)


def adam_step(theta, g, m, v, step, lr, beta1=BETA1, beta2=BETA2, eps=EPS):
    """One Adam update in float64.  Returns (theta_new, m_new, v_new); inputs are not modified."""
    theta = np.asarray(theta, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m_new = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v_new = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    mhat = m_new / (1.0 - beta1 ** step)
    vhat = v_new / (1.0 - beta2 ** step)
    return theta - lr * mhat / (np.sqrt(vhat) + eps), m_new, v_new
