"""Pins for the conv / inner-product / backward oracle and the packing oracle.

Forward: library routine (torch CPU conv2d in float64, numpy matmul), the
multiplication-free form of Eq. 2, closed forms (all-ones input, unit impulse),
hand-enumerated tiny case.  Backward (Alg. 1 steps 9-10): adjoint identities,
central finite differences, torch autograd.  Fused block tail: hand case with every term alone and
together, torch batch_norm + relu.  Bias gradient: hand case, torch autograd, adjoint of the bias term.
Packing: explicit bit patterns."""

import numpy as np
import pytest
import torch

from oracle import conv as oc
from oracle import packing as op
from paper_1605_04711_amd import workloads as wl

CASES = [
    # N H  W  C  O  R  S  stride pad dil
    (2, 7, 9, 3, 5, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 12, 11, 4, 6, 5, 5, (1, 1), (0, 0), (1, 1)),
    (2, 15, 14, 3, 4, 7, 7, (2, 2), (3, 3), (1, 1)),
    (1, 13, 13, 8, 3, 3, 3, (1, 1), (6, 6), (6, 6)),
    (2, 9, 8, 6, 7, 1, 1, (2, 2), (0, 0), (1, 1)),
    (1, 10, 9, 2, 3, 3, 2, (2, 1), (1, 0), (1, 2)),
]


def rand_case(case, seed):
    n, h, w, c, o, r, s, st, pd, dl = case
    g = np.random.default_rng(seed)
    x = wl.bf16_round(g.standard_normal((n, h, w, c)).astype(np.float32))
    codes = g.integers(-1, 2, size=(o, c, r, s)).astype(np.int8)
    alpha = float(np.float32(g.uniform(0.01, 0.2)))
    return x, codes, alpha, st, pd, dl


def torch_conv(x, wt, st, pd, dl):
    xt = torch.from_numpy(np.ascontiguousarray(x.transpose(0, 3, 1, 2))).double()
    y = torch.nn.functional.conv2d(xt, torch.from_numpy(wt).double(), stride=st, padding=pd, dilation=dl)
    return y.permute(0, 2, 3, 1).contiguous().numpy()


@pytest.mark.parametrize("ci", range(len(CASES)))
def test_forward_equals_library_conv_on_alpha_codes(ci, oracle_lib):
    x, codes, alpha, st, pd, dl = rand_case(CASES[ci], ci)
    y = oc.conv2d_fwd(x, codes, alpha, st, pd, dl)
    ref = torch_conv(x, alpha * codes.astype(np.float64), st, pd, dl)
    assert y.shape == ref.shape
    assert np.max(np.abs(y - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    # multiplication-free form (alpha X) (+) W~ of Eq. 2
    y2 = oc.conv2d_fwd(x, codes, alpha, st, pd, dl, addsub=True)
    assert np.max(np.abs(y - y2)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    # sampled evaluation agrees with the full tensor
    idx = np.random.default_rng(ci).integers(0, y.size, size=200)
    assert np.array_equal(oc.conv2d_fwd_at(x, codes, alpha, idx, st, pd, dl), y.ravel()[idx])


def test_forward_per_filter_alpha_and_bias(oracle_lib):
    x, codes, _, st, pd, dl = rand_case(CASES[0], 42)
    alpha = np.array([0.1, 0.2, 0.3, 0.4, 0.5])
    bias = np.array([1.0, -1.0, 0.5, 0.0, 2.0])
    y = oc.conv2d_fwd(x, codes, alpha, st, pd, dl, bias=bias)
    ref = torch_conv(x, alpha[:, None, None, None] * codes.astype(np.float64), st, pd, dl) + bias
    assert np.max(np.abs(y - ref)) <= 1e-12


def test_all_ones_counts_in_bounds_taps(oracle_lib):
    # X == 1 and every code +1: Z = alpha * C * (number of taps that fall inside the image)
    n, h, w, c, o, r, s = 1, 6, 5, 3, 2, 3, 3
    x = np.ones((n, h, w, c), dtype=np.float32)
    codes = np.ones((o, c, r, s), dtype=np.int8)
    y = oc.conv2d_fwd(x, codes, 0.5, (1, 1), (1, 1), (1, 1))
    rows = np.array([2] + [3] * (h - 2) + [2])
    cols = np.array([2] + [3] * (w - 2) + [2])
    expect = 0.5 * c * np.outer(rows, cols)
    assert np.array_equal(y[0, :, :, 0], expect) and np.array_equal(y[0, :, :, 1], expect)
    # dilation 2, pad 2: border rows see 2 taps, the rest 3 (h = 6)
    y = oc.conv2d_fwd(x, codes, 1.0, (1, 1), (2, 2), (2, 2))
    assert y.shape == (1, 6, 5, 2)
    assert y[0, 0, 0, 0] == c * 2 * 2 and y[0, 2, 2, 0] == c * 3 * 3


def test_unit_impulse_returns_unflipped_kernel(oracle_lib):
    # cross-correlation: an impulse at (2,2) of channel c0 puts W~[o,c0,r,s] at output (2-r+1, 2-s+1)
    h = w = 5
    c, o = 2, 3
    g = np.random.default_rng(3)
    codes = g.integers(-1, 2, size=(o, c, 3, 3)).astype(np.int8)
    x = np.zeros((1, h, w, c), dtype=np.float32)
    x[0, 2, 2, 1] = 1.0
    y = oc.conv2d_fwd(x, codes, 1.0, (1, 1), (1, 1), (1, 1))
    for r in range(3):
        for s in range(3):
            assert np.array_equal(y[0, 2 - r + 1, 2 - s + 1, :], codes[:, 1, r, s].astype(np.float64))


def test_tiny_case_enumerated_by_hand(oracle_lib):
    # 1x1x3x1 input [1,2,3], one 1x2 filter [+1,-1], no padding: outputs 1-2, 2-3
    x = np.array([1, 2, 3], dtype=np.float32).reshape(1, 1, 3, 1)
    codes = np.array([1, -1], dtype=np.int8).reshape(1, 1, 1, 2)
    y = oc.conv2d_fwd(x, codes, 2.0)
    assert y.ravel().tolist() == [-2.0, -2.0]
    dx = oc.conv2d_bwd_data(np.array([1, 10], dtype=np.float32).reshape(1, 1, 2, 1), codes, 2.0, (1, 1, 3, 1))
    assert dx.ravel().tolist() == [2.0, 18.0, -20.0]
    dw = oc.conv2d_bwd_weight(x, np.array([1, 10], dtype=np.float32).reshape(1, 1, 2, 1), (1, 1, 1, 2))
    assert dw.ravel().tolist() == [21.0, 32.0]


def test_gemm_is_matmul_and_1x1_conv(oracle_lib):
    g = np.random.default_rng(5)
    m, n, k = 37, 11, 70
    x = wl.bf16_round(g.standard_normal((m, k)).astype(np.float32))
    codes = g.integers(-1, 2, size=(n, k)).astype(np.int8)
    bias = g.standard_normal(n)
    y = oc.gemm_fwd(x, codes, 0.3, bias=bias)
    ref = 0.3 * (x.astype(np.float64) @ codes.astype(np.float64).T) + bias
    assert np.max(np.abs(y - ref)) <= 1e-12
    yc = oc.conv2d_fwd(x.reshape(m, 1, 1, k), codes.reshape(n, k, 1, 1), 0.3, bias=bias)
    assert np.array_equal(yc.reshape(m, n), y)
    idx = g.integers(0, m * n, size=50)
    assert np.array_equal(oc.gemm_fwd_at(x, codes, 0.3, idx, bias=bias), y.ravel()[idx])


@pytest.mark.parametrize("ci", range(len(CASES)))
def test_backward_adjoint_identities_and_autograd(ci, oracle_lib):
    x, codes, alpha, st, pd, dl = rand_case(CASES[ci], 100 + ci)
    g = np.random.default_rng(200 + ci)
    y = oc.conv2d_fwd(x, codes, alpha, st, pd, dl)
    dy = wl.bf16_round(g.standard_normal(y.shape).astype(np.float32))
    dx = oc.conv2d_bwd_data(dy, codes, alpha, x.shape, st, pd, dl)
    dw = oc.conv2d_bwd_weight(x, dy, codes.shape, st, pd, dl)
    t = alpha * codes.astype(np.float64)
    lhs = float(np.sum(y * dy))
    # <conv(X,T), G> = <X, bwd_data(G,T)> = <T, bwd_weight(X,G)>
    assert abs(lhs - float(np.sum(x.astype(np.float64) * dx))) <= 1e-10 * max(1.0, abs(lhs))
    assert abs(lhs - float(np.sum(t * dw))) <= 1e-10 * max(1.0, abs(lhs))
    # torch autograd on a float conv whose weight is T
    xt = torch.from_numpy(np.ascontiguousarray(x.transpose(0, 3, 1, 2))).double().requires_grad_(True)
    wt = torch.from_numpy(t).double().requires_grad_(True)
    out = torch.nn.functional.conv2d(xt, wt, stride=st, padding=pd, dilation=dl)
    out.backward(torch.from_numpy(np.ascontiguousarray(dy.transpose(0, 3, 1, 2))).double())
    assert np.max(np.abs(xt.grad.permute(0, 2, 3, 1).numpy() - dx)) <= 1e-11 * max(1.0, np.abs(dx).max())
    assert np.max(np.abs(wt.grad.numpy() - dw)) <= 1e-11 * max(1.0, np.abs(dw).max())
    # sampled variants
    i1 = g.integers(0, dx.size, size=100)
    assert np.array_equal(oc.conv2d_bwd_data_at(dy, codes, alpha, x.shape, i1, st, pd, dl), dx.ravel()[i1])
    i2 = g.integers(0, dw.size, size=40)
    assert np.array_equal(oc.conv2d_bwd_weight_at(x, dy, codes.shape, i2, st, pd, dl), dw.ravel()[i2])
    assert np.allclose(oc.bias_grad(dy), dy.astype(np.float64).sum(axis=(0, 1, 2)))


def test_finite_differences_of_the_forward(oracle_lib):
    x, codes, alpha, st, pd, dl = rand_case(CASES[2], 7)
    g = np.random.default_rng(8)
    y = oc.conv2d_fwd(x, codes, alpha, st, pd, dl)
    gmat = g.standard_normal(y.shape).astype(np.float32)
    dx = oc.conv2d_bwd_data(gmat, codes, alpha, x.shape, st, pd, dl)
    # L = <conv(X,T), G> is linear in X: a central difference is exact up to rounding
    for _ in range(10):
        pos = tuple(g.integers(0, d) for d in x.shape)
        e = np.zeros_like(x)
        e[pos] = 0.5
        lp = np.sum(oc.conv2d_fwd(x + e, codes, alpha, st, pd, dl) * gmat)
        lm = np.sum(oc.conv2d_fwd(x - e, codes, alpha, st, pd, dl) * gmat)
        assert abs((lp - lm) - dx[pos]) <= 1e-9 * max(1.0, abs(dx[pos]))


def test_packing_bit_patterns():
    # one row, K = 20: k=0 -> +1, k=1 -> -1, k=2 -> +1, k=15 -> -1, k=16 -> -1, k=19 -> +1
    codes = np.zeros((1, 20), dtype=np.int8)
    codes[0, [0, 2, 19]] = 1
    codes[0, [1, 15, 16]] = -1
    p = op.pack_matrix(codes)
    assert p.shape == (1, 8) and p.dtype == np.uint32
    # word 0: k=0 -> bits[0,1]=01; k=2 -> bits[2,3]=01; k=1 -> bits[16,17]=11; k=15 -> bits[30,31]=11
    assert int(p[0, 0]) == (0b01 | (0b01 << 2) | (0b11 << 16) | (0b11 << 30))
    # word 1: k=16 (even, i=0) -> bits[0,1]=11; k=19 (odd, i=1) -> bits[18,19]=01
    assert int(p[0, 1]) == (0b11 | (0b01 << 18))
    assert not p[0, 2:].any()
    back, bad, clean = op.unpack_matrix(p, 1, 20)
    assert np.array_equal(back, codes) and not bad and clean
    assert op.packed_bytes(3, 20) == 3 * 32 and op.packed_bytes(2, 129) == 2 * 64
    _, bad, _ = op.unpack_matrix(np.array([[2, 0, 0, 0, 0, 0, 0, 0]], dtype=np.uint32), 1, 20)
    assert bad
    _, _, clean = op.unpack_matrix(np.array([[0, 1 << 8, 0, 0, 0, 0, 0, 0]], dtype=np.uint32), 1, 20)
    assert not clean                      # k = 16+8 = 24 is padding and must be zero


def test_packing_round_trip_and_orders():
    g = np.random.default_rng(0)
    o, c, r, s = 5, 7, 3, 2
    codes = g.integers(-1, 2, size=(o, c, r, s)).astype(np.int8)
    m = op.to_matrix(codes)
    assert m[3, (1 * s + 1) * c + 4] == codes[3, 4, 1, 1]         # k = (r*S+s)*C + c
    mt = op.to_matrix_t(codes)
    assert mt[4, (2 * s + 0) * o + 3] == codes[3, 4, 2, 0]        # k_T = (r*S+s)*O + o
    back, bad, clean = op.unpack_weights(op.pack_weights(codes), o, c, r, s)
    assert np.array_equal(back, codes) and not bad and clean
    back, bad, clean = op.unpack_weights_t(op.pack_weights_t(codes), o, c, r, s)
    assert np.array_equal(back, codes) and not bad and clean
    # 16x smaller than float32 once K is a multiple of 128
    assert op.packed_bytes(64, 1152) * 16 == 64 * 1152 * 4


# --- fused block tail (X_next = g(Z) of Eq. 2 behind the folded batch-norm affine of Sec. 2.4) ----------

def test_epilogue_hand_case_each_term_alone_and_together():
    # Z of shape [1][1][2][2] (two pixels, two channels), channel index last
    z = np.array([[1.0, -2.0], [-3.0, 4.0]]).reshape(1, 1, 2, 2)
    scale = np.array([2.0, -1.0])
    shift = np.array([0.5, 1.0])
    res = np.array([[-4.0, 1.0], [10.0, -6.0]]).reshape(1, 1, 2, 2)
    flat = lambda a: a.reshape(2, 2).tolist()
    assert flat(oc.epilogue(z)) == [[1.0, -2.0], [-3.0, 4.0]]
    assert flat(oc.epilogue(z, scale=scale)) == [[2.0, 2.0], [-6.0, -4.0]]
    assert flat(oc.epilogue(z, shift=shift)) == [[1.5, -1.0], [-2.5, 5.0]]
    assert flat(oc.epilogue(z, residual=res)) == [[-3.0, -1.0], [7.0, -2.0]]
    assert flat(oc.epilogue(z, relu=True)) == [[1.0, 0.0], [0.0, 4.0]]
    # affine first (scale, then shift), residual after the affine, ReLU last:
    # pixel 0: (1*2+0.5-4, -2*-1+1+1) = (-1.5, 4); pixel 1: (-3*2+0.5+10, 4*-1+1-6) = (4.5, -9)
    assert flat(oc.epilogue(z, scale=scale, shift=shift, residual=res)) == [[-1.5, 4.0], [4.5, -9.0]]
    assert flat(oc.epilogue(z, scale=scale, shift=shift, residual=res, relu=True)) == [[0.0, 4.0], [4.5, 0.0]]
    # orders a mistake would produce give different numbers on this case
    wrong_shift_first = (z + shift) * scale + res
    wrong_res_first = (z + res) * scale + shift
    got = oc.epilogue(z, scale=scale, shift=shift, residual=res)
    assert not np.array_equal(got, wrong_shift_first) and not np.array_equal(got, wrong_res_first)
    # the input is not modified
    assert flat(z) == [[1.0, -2.0], [-3.0, 4.0]]


def test_epilogue_equals_library_batchnorm_block(oracle_lib):
    # relu(batch_norm(conv(X, T)) + residual) with the affine folded:
    # scale = gamma / sqrt(var + eps), shift = beta - mean * scale
    x, codes, alpha, st, pd, dl = rand_case(CASES[0], 77)
    g = np.random.default_rng(78)
    o = codes.shape[0]
    gamma, beta = g.uniform(0.5, 1.5, o), g.standard_normal(o)
    mean, var, eps = g.standard_normal(o), g.uniform(0.5, 2.0, o), 1e-5
    z = oc.conv2d_fwd(x, codes, alpha, st, pd, dl)
    res = g.standard_normal(z.shape)
    scale = gamma / np.sqrt(var + eps)
    shift = beta - mean * scale
    got = oc.epilogue(z, scale=scale, shift=shift, residual=res, relu=True)
    zt = torch.from_numpy(np.ascontiguousarray(torch_conv(x, alpha * codes.astype(np.float64), st, pd, dl)
                                               .transpose(0, 3, 1, 2)))
    bn = torch.nn.functional.batch_norm(zt, torch.from_numpy(mean), torch.from_numpy(var),
                                        torch.from_numpy(gamma), torch.from_numpy(beta), False, 0.0, eps)
    ref = torch.relu(bn + torch.from_numpy(np.ascontiguousarray(res.transpose(0, 3, 1, 2))))
    ref = ref.permute(0, 2, 3, 1).numpy()
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.abs(ref).max())
    assert (got == 0).any() and (got > 0).any()


# --- bias gradient (Alg. 1 step 9 applied to the additive term of the block) -----------------------------

def test_bias_grad_hand_case_and_autograd(oracle_lib):
    # two images of 1x2 pixels, three channels: db[o] adds the four pixels of channel o
    dy = np.array([[[[1, 10, 100], [2, 20, 200]]],
                   [[[3, 30, 300], [4, 40, 400]]]], dtype=np.float32)
    assert dy.shape == (2, 1, 2, 3)
    assert oc.bias_grad(dy).tolist() == [10.0, 100.0, 1000.0]
    # library cross-check: autograd of a convolution with a bias term
    x, codes, alpha, st, pd, dl = rand_case(CASES[2], 55)
    g = np.random.default_rng(56)
    t = alpha * codes.astype(np.float64)
    xt = torch.from_numpy(np.ascontiguousarray(x.transpose(0, 3, 1, 2))).double()
    b = torch.zeros(codes.shape[0], dtype=torch.float64, requires_grad=True)
    out = torch.nn.functional.conv2d(xt, torch.from_numpy(t), b, stride=st, padding=pd, dilation=dl)
    dyr = wl.bf16_round(g.standard_normal(tuple(out.permute(0, 2, 3, 1).shape)).astype(np.float32))
    out.backward(torch.from_numpy(np.ascontiguousarray(dyr.transpose(0, 3, 1, 2))).double())
    db = oc.bias_grad(dyr)
    assert db.shape == (codes.shape[0],)
    assert np.max(np.abs(db - b.grad.numpy())) <= 1e-12 * max(1.0, np.abs(db).max())
    # the forward's bias term and db are adjoint: <1, dY> per channel
    y0 = oc.conv2d_fwd(x, codes, alpha, st, pd, dl)
    y1 = oc.conv2d_fwd(x, codes, alpha, st, pd, dl, bias=np.arange(codes.shape[0], dtype=np.float64))
    lhs = float(np.sum((y1 - y0) * dyr))
    assert abs(lhs - float(np.dot(np.arange(codes.shape[0]), db))) <= 1e-10 * max(1.0, abs(lhs))
