"""SGD with momentum and L2 weight decay on the full-precision weights (CPU oracle, test infrastructure only).

Alg. 1 step 10 updates the full-precision copy of the weights kept across iterations (Sec. 2.4) from the
gradient taken with respect to the ternary weights; Sec. 2.4 and Sec. 3 name the optimiser (SGD with momentum,
L2 weight decay) and Table 1 its constants (momentum 0.9, weight decay 1e-4).  The paper prints no update formula.
Reading taken here (the common one of the frameworks of its time): the decay enters the gradient, the velocity
accumulates gradients, the learning rate multiplies the velocity:

    g = dW + weight_decay * W
    V' = momentum * V + g
    W' = W - lr * V'

Everything is float64 here; the caller decides where state is rounded to float32.  With the updated weights
comes the sum of |W'| that the threshold rule of the next iteration needs (Delta = f * mean|W'|, end of
Sec. 2.3), so that a fused update + reduction can be checked against it.
"""

import math

import numpy as np


def sgd_step(w, v, dw, lr, momentum, weight_decay):
    """One update; returns (W', V') as float64 arrays of the shape of `w`."""
    w = np.asarray(w, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dw = np.asarray(dw, dtype=np.float64)
    g = dw + float(weight_decay) * w
    v_new = float(momentum) * v + g
    w_new = w - float(lr) * v_new
    return w_new, v_new


def abs_sum(w):
    """sum_i |W_i| in float64 (exactly rounded for small inputs)."""
    a = np.abs(np.asarray(w, dtype=np.float64).ravel())
    if a.size <= (1 << 20):
        return math.fsum(a.tolist())
    return float(np.sum(a, dtype=np.float64))
