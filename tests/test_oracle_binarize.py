"""Pins of the sign binarizer oracle (the BPWN comparison of Sec. 3) and of its 1-bit packing."""

import itertools

import numpy as np
import pytest

from oracle import binarize as ob
from oracle import packing as op
from oracle import ternarize as ot


def test_hand_example():
    w = np.array([[0.5, -0.25, 0.0, -1.25]], dtype=np.float32)
    codes, alpha = ob.binarize(w)
    assert codes.tolist() == [[1, -1, 1, -1]]
    assert float(alpha[0]) == 0.5          # (0.5 + 0.25 + 0 + 1.25) / 4


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_is_the_least_squares_optimum_by_brute_force(seed):
    # Eq. 1 without the zero state: min over alpha >= 0 and B in {-1,+1}^n of ||W - alpha B||^2.
    # For fixed B the best alpha is max(0, <W,B>/n); enumerate every B.
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(9).astype(np.float32)
    best = (np.inf, None, None)
    for signs in itertools.product((-1.0, 1.0), repeat=9):
        b = np.array(signs)
        a = max(0.0, float(np.dot(w.astype(np.float64), b)) / 9)
        err = float(np.sum((w.astype(np.float64) - a * b) ** 2))
        if err < best[0]:
            best = (err, a, b)
    codes, alpha = ob.binarize(w.reshape(1, 9))
    assert np.array_equal(codes.ravel(), best[2].astype(np.int8))
    assert float(alpha[0]) == pytest.approx(best[1], rel=1e-6)


def test_equals_the_ternarizer_with_no_weight_zeroed():
    # Eq. 5 with every index in I_Delta (threshold below every |W_i|) is the mean of |W|; Eq. 3 is then the sign
    rng = np.random.default_rng(3)
    w = rng.standard_normal((4, 6, 3, 3)).astype(np.float32)
    w[np.abs(w) < 1e-3] = 0.5
    codes, alpha = ob.binarize(w)
    delta = np.float32(1e-6)
    t_codes = ot.codes_from_threshold(w, delta)
    assert np.array_equal(codes, np.asarray(t_codes, dtype=np.int8).reshape(w.shape))
    assert float(alpha[0]) == pytest.approx(float(ot.alpha_alg1(w, t_codes)), rel=1e-6)
    assert float(alpha[0]) == pytest.approx(float(np.mean(np.abs(w.astype(np.float64)))), rel=1e-7)


def test_per_filter_groups():
    rng = np.random.default_rng(4)
    w = rng.standard_normal((6, 5)).astype(np.float32)
    codes, alpha = ob.binarize(w, groups=3)
    for g in range(3):
        assert float(alpha[g]) == pytest.approx(float(np.mean(np.abs(w[2 * g:2 * g + 2]))), rel=1e-6)
    assert np.array_equal(codes, np.where(w < 0, -1, 1))


def test_pack1_hand_word_and_roundtrip():
    # k = 0 (+), 1 (-), 2 (-), 3 (+), 35 (-): bits 16 (k=1), 1 (k=2) of word 0; k=35 = 32 + 2*1 + 1 -> bit 17 of word 1
    codes = np.ones((1, 40), dtype=np.int8)
    codes[0, [1, 2, 35]] = -1
    p = op.pack_matrix1(codes)
    assert p.shape == (1, 4)
    assert int(p[0, 0]) == (1 << 16) | (1 << 1)
    assert int(p[0, 1]) == (1 << 17)
    assert int(p[0, 2]) == 0 and int(p[0, 3]) == 0
    rng = np.random.default_rng(8)
    for rows, k in ((3, 1), (5, 127), (2, 128), (7, 300)):
        c = np.where(rng.standard_normal((rows, k)) < 0, -1, 1).astype(np.int8)
        back, clean = op.unpack_matrix1(op.pack_matrix1(c), rows, k)
        assert clean and np.array_equal(back, c)
    assert op.words_per_row1(1) == 4 and op.words_per_row1(128) == 4 and op.words_per_row1(129) == 8
