"""GPU parity of twn_sgd_update against the oracle (Alg. 1 step 10; momentum and weight decay of Table 1), and of the
ternarization that reuses the pass-1 sums the update leaves behind (Sec. 2.3 rule of thumb on the updated weights).

Bar: W and V within 1e-6 of the float64 oracle relative to max(|value|, rms) (three float32 fused multiply-adds
against float64: under 4 ulp); Delta, alpha, |I_Delta| and the packed codes of twn_ternarize_presummed bit-identical
to twn_ternarize's on the updated tensor, and equal to the oracle's ternarization of it."""

import numpy as np
import pytest
import torch

from oracle import packing as op
from oracle import sgd as osgd
from oracle import ternarize as ot
from paper_1605_04711_amd import api
from paper_1605_04711_amd import workloads as wl
from parity import packed_to_host, to_dev_f32

pytestmark = pytest.mark.gpu

REL = 1e-6


def close(gpu, ref):
    ref = np.asarray(ref, dtype=np.float64)
    floor = max(float(np.sqrt(np.mean(ref * ref))), 1e-30)
    return np.all(np.abs(gpu.astype(np.float64) - ref) <= REL * np.maximum(np.abs(ref), floor))


def f32(x):
    return float(np.float32(x))


# tensors: whole chunks of 4096, ragged tails, fewer weights than one chunk, more chunks than blocks
@pytest.mark.parametrize("shape", [(64, 64), (33, 1152), (7, 5), (1, 1), (1000, 4224), (128, 128, 3, 3), (64, 3, 7, 7),
                                   (2048, 2048 + 16)])
def test_update_and_presummed_ternarize(shape):
    lr, mu, wd = 0.1, 0.9, 1e-4
    w = wl.normal(11, 1, shape, std=0.05)
    v = wl.normal(11, 2, shape, std=0.01)
    dw = wl.normal(11, 3, shape, std=0.02)
    W, V, dW = to_dev_f32(w), to_dev_f32(v), to_dev_f32(dw)
    rows, k = shape[0], int(np.prod(shape[1:]))
    ref_tw = api.twn_ternarize(W, 0.7, transposed=True)            # allocates outputs of the right shapes
    out = api.twn_ternarize(W, 0.7, transposed=True)
    ws = torch.empty(api.lib().twn_ternarize_workspace_bytes(
        api.ctypes.byref(api.WeightDesc(ref_tw.rows, ref_tw.C, ref_tw.R, ref_tw.S)), 1), dtype=torch.uint8, device=W.device)
    for step in range(2):
        w_ref, v_ref = osgd.sgd_step(W.cpu().numpy(), V.cpu().numpy(), dw, f32(lr), f32(mu), f32(wd))
        api.twn_sgd_update(W, V, dW, lr, mu, wd, tern_workspace=ws)
        api.twn_ternarize_presummed(W, out, ws, 0.7)
        torch.cuda.synchronize()
        assert close(W.cpu().numpy(), w_ref) and close(V.cpu().numpy(), v_ref)
        api.twn_ternarize(W, 0.7, out=ref_tw)
        torch.cuda.synchronize()
        for a, b in ((out.delta, ref_tw.delta), (out.alpha, ref_tw.alpha), (out.nnz, ref_tw.nnz),
                     (out.packed, ref_tw.packed), (out.packed_T, ref_tw.packed_T)):
            assert torch.equal(a, b)
        w_now = W.cpu().numpy()
        w4 = w_now.reshape(rows, -1, 1, 1) if w_now.ndim == 2 else w_now
        codes, delta, alpha, nnz = ot.ternarize(w4, 0.7)
        assert np.array_equal(out.nnz.cpu().numpy(), nnz)
        assert np.array_equal(packed_to_host(out.packed), op.pack_weights(codes))
        assert abs(float(out.delta.cpu()[0]) - float(delta[0])) <= REL * float(delta[0])
        # the sum behind Delta is the L1 norm of the updated weights
        assert float(out.delta.cpu()[0]) == pytest.approx(f32(0.7) * osgd.abs_sum(w_now) / w_now.size, rel=REL)


def test_special_cases_and_no_workspace():
    w = wl.normal(11, 5, (300, 77), std=0.05)
    dw = wl.normal(11, 6, (300, 77), std=0.02)
    # zero momentum and decay: plain gradient descent, velocity equals the gradient
    W, V, dW = to_dev_f32(w), torch.zeros(300, 77, device="cuda"), to_dev_f32(dw)
    api.twn_sgd_update(W, V, dW, 0.25, 0.0, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(V, dW)
    w_ref, _ = osgd.sgd_step(w, np.zeros_like(w), dw, 0.25, 0.0, 0.0)
    assert close(W.cpu().numpy(), w_ref)
    # zero learning rate: weights untouched, velocity still accumulates
    W2 = to_dev_f32(w)
    api.twn_sgd_update(W2, V, dW, 0.0, 0.9, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(W2, to_dev_f32(w))
    _, v_ref = osgd.sgd_step(w, dw, dw, 0.0, f32(0.9), 0.0)
    assert close(V.cpu().numpy(), v_ref)


def test_argument_errors():
    W = torch.zeros(64, device="cuda")
    with pytest.raises(TypeError):
        api.twn_sgd_update(W, W.double(), W, 0.1)
    L = api.lib()
    vp = api.ctypes.c_void_p
    st = api._stream(None)
    assert L.twn_sgd_update(None, vp(W.data_ptr()), vp(W.data_ptr()), 64, 0.1, 0.9, 0.0, None, 0, st) == -1
    assert L.twn_sgd_update(vp(W.data_ptr()), vp(W.data_ptr()), vp(W.data_ptr()), 0, 0.1, 0.9, 0.0, None, 0, st) != 0
    assert L.twn_sgd_update(vp(W.data_ptr() + 4), vp(W.data_ptr()), vp(W.data_ptr()), 8, 0.1, 0.9, 0.0, None, 0, st) != 0
    small = torch.zeros(64, dtype=torch.uint8, device="cuda")
    assert L.twn_sgd_update(vp(W.data_ptr()), vp(W.data_ptr()), vp(W.data_ptr()), 64, 0.1, 0.9, 0.0,
                            vp(small.data_ptr()), 64, st) != 0
