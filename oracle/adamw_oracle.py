"""CPU oracle for the AdamW parameter update.  TEST INFRASTRUCTURE ONLY.

Only tests and benchmarks' cpu legs may import it; the product path never does and shares no code with it.

What it computes: the optimiser the paper's experiments name (Experiments, both training set-ups: AdamW with a
peak learning rate), i.e. Adam with decoupled weight decay (Loshchilov & Hutter, the work cited there, Algorithm 2):
    m_t = beta1 m_{t-1} + (1 - beta1) g_t
    v_t = beta2 v_{t-1} + (1 - beta2) g_t^2
    mhat = m_t / (1 - beta1^t),  vhat = v_t / (1 - beta2^t)
    theta_t = theta_{t-1} - lr (mhat / (sqrt(vhat) + eps) + lambda theta_{t-1})
The paper gives the learning rates only.  Reading taken: the decay is multiplied by the learning rate (the schedule
multiplier of the cited algorithm times its step size is `lr`, as in the usual library form), epsilon is added to the
root of the corrected second moment, every parameter decays alike.  float64 throughout.

Pins (tests/test_oracle_adamw.py): closed forms (first step from a zero state; a constant gradient, for which
mhat = g and vhat = g^2 at every step; a zero gradient, which leaves pure geometric decay) and the library optimiser
torch.optim.AdamW on the CPU over several steps of random gradients.
"""
import numpy as np


def adamw_step(theta, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01):
    """One update at step t (t = 1 for the first).  Returns new (theta, m, v); inputs are not modified."""
    theta = np.asarray(theta, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    theta = theta - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * theta)
    return theta, m, v
