"""GPU parity of the binary-weight comparison (Sec. 3): twn_binarize against the sign oracle (codes bit-exact, alpha
within 1e-6), and the forward contraction with 1-bit weights (TWN_VAR_BF16_SIGN1_POSTSCALE) against the forward
oracle fed the same sign codes and alpha, to the bf16-MFMA bar of the ternary paths."""

import numpy as np
import pytest
import torch

from oracle import binarize as ob
from oracle import conv as oc
from oracle import packing as op
from paper_1605_04711_amd import api
from paper_1605_04711_amd import workloads as wl
from parity import BF16_TOL, packed_to_host, rel_err, to_dev_bf16, to_dev_f32, to_host_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("groups", [1, "rows"])
@pytest.mark.parametrize("shape", [(64, 256), (33, 1152), (17, 24), (1, 1), (5, 3, 3, 3), (64, 32, 5, 5), (128, 128, 3, 3),
                                   (64, 3, 7, 7), (1000, 512)])
def test_binarize(shape, groups):
    g = shape[0] if groups == "rows" else 1
    w = wl.normal(13, shape[0] + shape[1], shape, std=0.05)
    w.ravel()[::7] = 0.0                                    # zeros take the code +1
    w.ravel()[3::11] = -0.0
    bw = api.twn_binarize(to_dev_f32(w), groups=g)
    torch.cuda.synchronize()
    w4 = w if w.ndim == 4 else w.reshape(w.shape[0], w.shape[1], 1, 1)
    codes, alpha = ob.binarize(w4, groups=g)
    assert np.array_equal(packed_to_host(bw.packed), op.pack_weights1(codes))
    assert np.all(np.abs(bw.alpha.cpu().numpy() - alpha) <= 1e-6 * np.abs(alpha))
    o, c, r, s = w4.shape
    back, clean = op.unpack_matrix1(packed_to_host(bw.packed), o, r * s * c)
    assert clean and np.array_equal(back, op.to_matrix(codes))


CONV = [  # N, H, W, C, O, R, S, stride, pad, dil
    (2, 12, 12, 64, 64, 3, 3, 1, 1, 1),
    (2, 9, 11, 32, 48, 3, 3, 2, 1, 1),
    (1, 14, 14, 3, 32, 5, 5, 1, 2, 1),        # K = 75: the padded sign bits meet zero activations
    (3, 7, 7, 128, 200, 1, 1, 1, 0, 1),
    (1, 10, 10, 16, 24, 3, 3, 1, 2, 2),
]


@pytest.mark.parametrize("case", range(len(CONV)))
def test_conv_forward_with_sign_codes(case):
    n, h, w_, c, o, r, s, st, pd, dl = CONV[case]
    w = wl.normal(13, 100 + case, (o, c, r, s), std=0.05)
    x = wl.bf16_round(wl.normal(13, 200 + case, (n, h, w_, c)))
    bw = api.twn_binarize(to_dev_f32(w))
    y = api.twn_conv2d_fwd(to_dev_bf16(x), bw, (st, st), (pd, pd), (dl, dl), variant=api.TWN_VAR_BF16_SIGN1_POSTSCALE)
    torch.cuda.synchronize()
    codes, alpha = ob.binarize(w)
    ref = oc.conv2d_fwd(x, codes, alpha, (st, st), (pd, pd), (dl, dl))
    assert rel_err(to_host_f64(y), ref) <= BF16_TOL
    # per-filter scales and the fused tail
    bwf = api.twn_binarize(to_dev_f32(w), groups=o)
    scale = wl.normal(13, 300 + case, (o,), std=0.2) + 1.0
    shift = wl.normal(13, 400 + case, (o,), std=0.5)
    y2 = api.twn_conv2d_fwd(to_dev_bf16(x), bwf, (st, st), (pd, pd), (dl, dl), variant=api.TWN_VAR_BF16_SIGN1_POSTSCALE,
                            scale=to_dev_f32(scale), shift=to_dev_f32(shift), relu=True)
    torch.cuda.synchronize()
    codes_f, alpha_f = ob.binarize(w, groups=o)
    ref2 = oc.epilogue(oc.conv2d_fwd(x, codes_f, alpha_f, (st, st), (pd, pd), (dl, dl)), scale=scale, shift=shift, relu=True)
    assert rel_err(to_host_f64(y2), ref2) <= BF16_TOL


@pytest.mark.parametrize("mnk", [(96, 64, 256), (300, 200, 1000), (64, 1000, 512), (1, 8, 24)])
def test_gemm_forward_with_sign_codes(mnk):
    m, n, k = mnk
    w = wl.normal(13, 500 + m, (n, k), std=0.05)
    x = wl.bf16_round(wl.normal(13, 600 + m, (m, k)))
    bw = api.twn_binarize(to_dev_f32(w))
    y = api.twn_gemm_fwd(to_dev_bf16(x), bw, variant=api.TWN_VAR_BF16_SIGN1_POSTSCALE)
    torch.cuda.synchronize()
    codes, alpha = ob.binarize(w.reshape(n, k, 1, 1))
    ref = oc.conv2d_fwd(x.reshape(m, 1, 1, k), codes, alpha).reshape(m, n)
    assert rel_err(to_host_f64(y), ref) <= BF16_TOL


def test_sign_codes_are_forward_only_and_need_their_variant():
    w = wl.normal(13, 700, (32, 16, 3, 3), std=0.05)
    bw = api.twn_binarize(to_dev_f32(w))
    x = to_dev_bf16(wl.bf16_round(wl.normal(13, 701, (1, 8, 8, 16))))
    with pytest.raises(ValueError):
        api.twn_conv2d_fwd(x, bw, (1, 1), (1, 1), (1, 1))      # the ternary variant does not read 1-bit codes
