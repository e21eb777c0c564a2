"""Seeded random shapes through the specialised forward kernels (first layers with three channels, 3x3 layers
over 64 channels, two convolutions over one input, the float32 path with K ranges) and random geometries through
forward, data gradient and weight gradient, against the direct-loop oracle (Eq. 2; Alg. 1 steps 8-10): the fixed
cases elsewhere pick shapes by hand, these do not."""

import numpy as np
import pytest
import torch

from oracle import conv as oc
from oracle import ternarize as ot
from paper_1605_04711_amd import api
from paper_1605_04711_amd import workloads as wl
from parity import BF16_TOL, FP32_TOL, rel_err, to_dev_bf16, to_dev_f32, to_host_f64

pytestmark = pytest.mark.gpu

F = 0.7


def _tail(rng, shape, o):
    relu, use_res = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    sc = rng.uniform(0.5, 1.5, o).astype(np.float32)
    sf = rng.standard_normal(o).astype(np.float32)
    res = wl.bf16_round(rng.standard_normal(shape).astype(np.float32)) if use_res else None
    return relu, sc, sf, res


@pytest.mark.parametrize("seed", range(16))
def test_random_3x3_layers_over_64_channels(seed):
    rng = np.random.default_rng(1000 + seed)
    n, h, w_ = int(rng.integers(1, 6)), int(rng.integers(3, 41)), int(rng.integers(3, 41))
    o = int(rng.choice([64, 128, 192]))
    pd = (int(rng.integers(0, 3)), int(rng.integers(0, 3)))
    if h + 2 * pd[0] < 3 or w_ + 2 * pd[1] < 3:
        pd = (1, 1)
    groups = int(rng.choice([1, o, 4]))
    x = wl.bf16_round(rng.standard_normal((n, h, w_, 64)).astype(np.float32))
    w = (rng.standard_normal((o, 64, 3, 3)) * 0.06).astype(np.float32)
    tw = api.twn_ternarize(to_dev_f32(w), F, groups=groups, transposed=True)
    codes, delta, alpha, nnz = ot.ternarize(w, F, groups=groups)
    ref0 = oc.conv2d_fwd(x, codes, alpha, (1, 1), pd, (1, 1))
    relu, sc, sf, res = _tail(rng, ref0.shape, o)
    y = api.twn_conv2d_fwd(to_dev_bf16(x), tw, (1, 1), pd, (1, 1), scale=to_dev_f32(sc), shift=to_dev_f32(sf),
                           residual=None if res is None else to_dev_bf16(res), relu=relu)
    assert rel_err(to_host_f64(y), oc.epilogue(ref0, sc, sf, res, relu=relu)) <= BF16_TOL
    if o == 64:
        dy = wl.bf16_round(rng.standard_normal(ref0.shape).astype(np.float32))
        dx, _, _ = api.twn_conv2d_bwd_ste(None, to_dev_bf16(dy), tw, (1, 1), pd, (1, 1), need_dx=True, need_dw=False,
                                          x_shape=(n, h, w_, 64))
        assert rel_err(to_host_f64(dx), oc.conv2d_bwd_data(dy, codes, alpha, (n, h, w_, 64), (1, 1), pd, (1, 1))) <= BF16_TOL


@pytest.mark.parametrize("seed", range(16))
def test_random_first_layers(seed):
    rng = np.random.default_rng(2000 + seed)
    n, h, w_ = int(rng.integers(1, 5)), int(rng.integers(7, 50)), 2 * int(rng.integers(4, 25))
    o = 8 * int(rng.integers(1, 20))
    r, s = int(rng.choice([1, 3, 5, 7])), int(rng.choice([1, 3, 5, 7]))
    st = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
    pd = (int(rng.integers(0, r // 2 + 2)), int(rng.integers(0, s // 2 + 2)))
    groups = int(rng.choice([1, o]))
    x = wl.bf16_round(rng.standard_normal((n, h, w_, 3)).astype(np.float32))
    w = (rng.standard_normal((o, 3, r, s)) * 0.2).astype(np.float32)
    tw = api.twn_ternarize(to_dev_f32(w), F, groups=groups)
    codes, delta, alpha, nnz = ot.ternarize(w, F, groups=groups)
    ref0 = oc.conv2d_fwd(x, codes, alpha, st, pd, (1, 1))
    relu, sc, sf, res = _tail(rng, ref0.shape, o)
    y = api.twn_conv2d_fwd(to_dev_bf16(x), tw, st, pd, (1, 1), scale=to_dev_f32(sc), shift=to_dev_f32(sf),
                           residual=None if res is None else to_dev_bf16(res), relu=relu)
    assert rel_err(to_host_f64(y), oc.epilogue(ref0, sc, sf, res, relu=relu)) <= BF16_TOL


@pytest.mark.parametrize("seed", range(10))
def test_random_block_heads(seed):
    rng = np.random.default_rng(3000 + seed)
    n, h, w_ = int(rng.integers(1, 4)), int(rng.integers(4, 30)), int(rng.integers(4, 30))
    c = 8 * int(rng.integers(1, 20))
    o0 = 8 * int(rng.integers(1, 24))
    o1 = o0 if rng.integers(0, 2) else 8 * int(rng.integers(1, 24))
    x = wl.bf16_round(rng.standard_normal((n, h, w_, c)).astype(np.float32))
    w0 = (rng.standard_normal((o0, c, 3, 3)) * 0.05).astype(np.float32)
    w1 = (rng.standard_normal((o1, c, 1, 1)) * 0.1).astype(np.float32)
    tw0, tw1 = api.twn_ternarize(to_dev_f32(w0), F), api.twn_ternarize(to_dev_f32(w1), F)
    c0, _, a0, _ = ot.ternarize(w0, F)
    c1, _, a1, _ = ot.ternarize(w1, F)
    geos = (((2, 2), (1, 1), (1, 1)), ((2, 2), (0, 0), (1, 1)))
    y0, y1 = api.twn_conv2d_fwd_pair(to_dev_bf16(x), (tw0, tw1), geos, relus=(True, False))
    assert rel_err(to_host_f64(y0), oc.epilogue(oc.conv2d_fwd(x, c0, a0, *geos[0]), relu=True)) <= BF16_TOL
    assert rel_err(to_host_f64(y1), oc.conv2d_fwd(x, c1, a1, *geos[1])) <= BF16_TOL


@pytest.mark.parametrize("seed", range(12))
def test_random_float32_products(seed):
    rng = np.random.default_rng(4000 + seed)
    m, n, k = int(rng.integers(1, 300)), int(rng.integers(1, 300)), int(rng.integers(1, 3000))
    x = rng.uniform(-1.0, 1.0, (m, k)).astype(np.float32)
    w = (rng.standard_normal((n, k)) * 0.05).astype(np.float32)
    tw = api.twn_ternarize(to_dev_f32(w), F)
    codes, delta, alpha, nnz = ot.ternarize(w.reshape(n, k, 1, 1), F)
    y = api.twn_gemm_fwd(to_dev_f32(x), tw, y_dtype=torch.float32)
    assert rel_err(to_host_f64(y), oc.gemm_fwd(x, codes.reshape(n, k), alpha)) <= FP32_TOL


@pytest.mark.parametrize("seed", range(20))
def test_random_geometries_forward_and_backward(seed):
    rng = np.random.default_rng(5000 + seed)
    n, h, w_ = int(rng.integers(1, 5)), int(rng.integers(3, 34)), int(rng.integers(3, 34))
    c = int(rng.choice([8, 16, 24, 32, 64, 72, 128, 192, 256]))
    o = int(rng.choice([8, 10, 16, 40, 64, 72, 128, 136, 256, 320]))
    r, s = int(rng.choice([1, 3, 5])), int(rng.choice([1, 3, 5]))
    st = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
    dl = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
    pd = (int(rng.integers(0, 3)), int(rng.integers(0, 3)))
    if h + 2 * pd[0] < dl[0] * (r - 1) + 1 or w_ + 2 * pd[1] < dl[1] * (s - 1) + 1:
        pd = (dl[0] * (r - 1), dl[1] * (s - 1))
    x = wl.bf16_round(rng.standard_normal((n, h, w_, c)).astype(np.float32))
    w = (rng.standard_normal((o, c, r, s)) * np.sqrt(2.0 / (c * r * s))).astype(np.float32)
    tw = api.twn_ternarize(to_dev_f32(w), F, transposed=True)
    codes, delta, alpha, nnz = ot.ternarize(w, F)
    ref0 = oc.conv2d_fwd(x, codes, alpha, st, pd, dl)
    relu = bool(rng.integers(0, 2))
    y = api.twn_conv2d_fwd(to_dev_bf16(x), tw, st, pd, dl, relu=relu)
    assert rel_err(to_host_f64(y), oc.epilogue(ref0, relu=relu)) <= BF16_TOL
    dy = wl.bf16_round(rng.standard_normal(ref0.shape).astype(np.float32))
    dx, dw, _ = api.twn_conv2d_bwd_ste(to_dev_bf16(x), to_dev_bf16(dy), tw, st, pd, dl)
    assert rel_err(to_host_f64(dx), oc.conv2d_bwd_data(dy, codes, alpha, x.shape, st, pd, dl)) <= BF16_TOL
    assert rel_err(to_host_f64(dw), oc.conv2d_bwd_weight(x, dy, codes.shape, st, pd, dl)) <= 1e-3
