"""Sign binarizer of the binary-weight comparison networks (CPU oracle, test infrastructure only).

Sec. 3 of the paper compares against binary precision weight networks (BPWNs) whose weights are binarized with
the sign function.  The scale that goes with the sign codes is not printed; the reading taken here is the one the
paper's own derivation gives when no weight is set to zero: with every index in I_Delta (Delta below every |W_i|),
Eq. 5 is alpha = (1/n) * sum |W_i|, which is also the minimiser of ||W - alpha*B||^2 over alpha >= 0, B in {-1,+1}^n
(Eq. 1 with the zero state removed).  sign(0) is taken as +1 (a code has to be chosen; it does not change the error).

Precision reading as for the ternarizer: the sum is float64, alpha is rounded once to float32.
"""

import math

import numpy as np


def binarize_group(w):
    """codes (int8 in {-1,+1}, shape of w) and alpha (float32) for one group of weights."""
    w = np.asarray(w, dtype=np.float32)
    codes = np.where(w < 0, np.int8(-1), np.int8(1)).astype(np.int8)
    a = np.abs(w.astype(np.float64).ravel())
    s = math.fsum(a.tolist()) if a.size <= (1 << 20) else float(np.sum(a, dtype=np.float64))
    return codes, np.float32(s / float(w.size))


def binarize(w, groups=1):
    """w [rows][C][R][S] (or [rows][K]); `groups` equal groups of consecutive filters.
    Returns codes (int8, shape of w) and alpha float32[groups]."""
    w = np.asarray(w, dtype=np.float32)
    rows = w.shape[0]
    assert rows % groups == 0
    per = rows // groups
    codes = np.empty(w.shape, dtype=np.int8)
    alpha = np.empty(groups, dtype=np.float32)
    for g in range(groups):
        codes[g * per:(g + 1) * per], alpha[g] = binarize_group(w[g * per:(g + 1) * per])
    return codes, alpha
