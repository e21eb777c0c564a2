"""Sort-based threshold ternarizer (CPU oracle, test infrastructure only).

Follows Sec. 2.3 of the paper: the threshold function (Eq. 3), the index set
I_Delta and the optimal scale for a given threshold (Eq. 5), the rule of thumb
Delta = f * mean|W| (end of Sec. 2.3; Alg. 1 step 4 with f printed as 0.75),
and the per-filter loop of Alg. 1 steps 3-7 (one "group" = one filter; a single
group = one layer).  Also holds the objectives the rule approximates (Eq. 1,
Eq. 4, Eq. 6) so that tests can brute-force them.

Precision reading (the paper fixes only "float32" weights): sums are
accumulated in float64, Delta and alpha are each rounded once to float32, and
every comparison |W_i| > Delta is a float32 comparison.
"""

import itertools
import math

import numpy as np


def _sum64(values):
    """Sum of float64 values: exactly rounded for small inputs, pairwise above."""
    v = np.asarray(values, dtype=np.float64)
    if v.size <= (1 << 20):
        return math.fsum(v.tolist())
    return float(np.sum(v, dtype=np.float64))


def threshold(w, delta_factor):
    """Delta = f * (1/n) * sum |W_i|  (rule of thumb, Sec. 2.3; Alg. 1 step 4).

    `delta_factor` is taken as a float32 and widened exactly; the quotient is
    rounded once to float32.  n is the number of weights in the group.
    """
    w = np.asarray(w, dtype=np.float32).ravel()
    f = float(np.float32(delta_factor))
    s1 = _sum64(np.abs(w))
    return np.float32((f * s1) / float(w.size))


def codes_from_threshold(w, delta):
    """Eq. 3: +1 if W_i > Delta, -1 if W_i < -Delta, 0 if |W_i| <= Delta."""
    w = np.asarray(w, dtype=np.float32)
    d = np.float32(delta)
    out = np.zeros(w.shape, dtype=np.int8)
    out[w > d] = 1
    out[w < -d] = -1
    return out


def ternarize_group(w, delta_factor):
    """Ternarize one group of weights.

    Returns (codes int8, delta float32, alpha float32, nnz int).
    Steps: sort |W| descending; Delta by the rule of thumb; |I_Delta| by binary
    search in the sorted magnitudes; alpha = mean of the |I_Delta| largest
    magnitudes (Eq. 5); codes by Eq. 3 straight from W.  The two routes to
    |I_Delta| (search in the sort, and counting non-zero codes) must agree.
    An all-zero group gives Delta = 0, no non-zero code, and alpha := 0.
    """
    w = np.asarray(w, dtype=np.float32).ravel()
    n = w.size
    if n == 0:
        raise ValueError("empty group")
    a = np.abs(w)
    order = np.argsort(-a, kind="stable")
    a_desc = a[order]
    delta = threshold(w, delta_factor)
    # a_desc is descending; count entries strictly greater than delta
    c = int(np.searchsorted(-a_desc, -delta, side="left"))
    codes = codes_from_threshold(w, delta)
    nnz = int(np.count_nonzero(codes))
    if nnz != c:
        raise AssertionError("sort route and code route disagree on |I_Delta|")
    if c > 0:
        s_i = _sum64(a_desc[:c])
        alpha = np.float32(s_i / float(c))
    else:
        alpha = np.float32(0.0)
    return codes, delta, alpha, c


def ternarize(w, delta_factor, groups=1):
    """Ternarize a weight tensor split into `groups` equal contiguous groups.

    groups=1 is per-layer; groups=number of filters is Alg. 1 as printed.
    Returns (codes int8 with w's shape, delta f32[groups], alpha f32[groups],
    nnz int64[groups]).
    """
    w = np.asarray(w, dtype=np.float32)
    flat = w.reshape(-1)
    if groups < 1 or flat.size % groups != 0:
        raise ValueError("groups must divide the number of weights")
    per = flat.size // groups
    codes = np.empty(flat.size, dtype=np.int8)
    delta = np.empty(groups, dtype=np.float32)
    alpha = np.empty(groups, dtype=np.float32)
    nnz = np.empty(groups, dtype=np.int64)
    for g in range(groups):
        seg = flat[g * per:(g + 1) * per]
        cg, dg, ag, ng = ternarize_group(seg, delta_factor)
        codes[g * per:(g + 1) * per] = cg
        delta[g], alpha[g], nnz[g] = dg, ag, ng
    return codes.reshape(w.shape), delta, alpha, nnz


def alpha_alg1(w, codes):
    """Alg. 1 step 6: alpha = (W . W~) / (W~ . W~), in float64."""
    w = np.asarray(w, dtype=np.float64).ravel()
    t = np.asarray(codes, dtype=np.float64).ravel()
    den = float(np.dot(t, t))
    if den == 0.0:
        return 0.0
    return _sum64(w * t) / den


def objective_j(w, alpha, codes):
    """Eq. 1: J(alpha, W~) = || W - alpha * W~ ||_2^2, in float64."""
    w = np.asarray(w, dtype=np.float64).ravel()
    t = np.asarray(codes, dtype=np.float64).ravel()
    r = w - float(alpha) * t
    return _sum64(r * r)


def cut_objective(w):
    """Eq. 6 for every cut of the sorted magnitudes.

    Returns (a_desc, g) with g[k-1] = (sum of the k largest |W_i|)^2 / k for
    k = 1..n.  The best threshold maximises g (the paper prints arg min; with
    alpha from Eq. 5 substituted, J = sum W_i^2 - g, so minimising J means
    maximising g).
    """
    a = np.sort(np.abs(np.asarray(w, dtype=np.float64).ravel()))[::-1]
    s = np.cumsum(a)
    k = np.arange(1, a.size + 1, dtype=np.float64)
    return a, (s * s) / k


def brute_force_eq1(w):
    """Global optimum of Eq. 1 by enumerating all 3^n ternary vectors (tiny n).

    For each W~ the best alpha >= 0 is max(0, (W . W~)/(W~ . W~)).
    Returns (J_min, alpha, codes).
    """
    w = np.asarray(w, dtype=np.float64).ravel()
    n = w.size
    if n > 13:
        raise ValueError("3^n enumeration is for tiny inputs only")
    best = (float(np.dot(w, w)), 0.0, np.zeros(n, dtype=np.int8))
    for t in itertools.product((-1, 0, 1), repeat=n):
        tv = np.array(t, dtype=np.float64)
        den = float(np.dot(tv, tv))
        if den == 0.0:
            continue
        al = max(0.0, float(np.dot(w, tv)) / den)
        r = w - al * tv
        j = float(np.dot(r, r))
        if j < best[0]:
            best = (j, al, np.array(t, dtype=np.int8))
    return best
