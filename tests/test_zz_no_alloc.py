"""The entry point that allocates nothing, twn_ternarize_static, against twn_ternarize (whose own parity with the
oracle is the subject of test_gpu_ternarize.py): bit-identical outputs on two calls in a row, the second with a
smaller input, so that whatever the first call left in the library's per-device array is seen to be harmless."""

import numpy as np
import pytest
import torch

from paper_1605_04711_amd import api

pytestmark = pytest.mark.gpu


def _pair(shape, seed, groups, transposed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    w = (torch.randn(shape, generator=g) * 0.05).cuda()
    ref = api.twn_ternarize(w, 0.7, groups=groups, transposed=transposed)
    rows, c, r, s = shape if len(shape) == 4 else (shape[0], shape[1], 1, 1)
    out = api._new_ternary_weights(rows, c, r, s, groups, transposed, w.device)
    for t in (out.packed, out.packed_T, out.delta, out.alpha, out.nnz):
        if t is not None:
            t.fill_(-1 if t.dtype != torch.float32 else float("nan"))
    before = torch.cuda.memory_allocated()
    api.twn_ternarize_static(w, out, 0.7)
    assert torch.cuda.memory_allocated() == before         # nothing came from torch's allocator either
    torch.cuda.synchronize()
    assert torch.equal(out.packed, ref.packed)
    if transposed:
        assert torch.equal(out.packed_T, ref.packed_T)
    assert torch.equal(out.delta, ref.delta) and torch.equal(out.alpha, ref.alpha) and torch.equal(out.nnz, ref.nnz)
    assert int(out.nnz.sum()) > 0


def test_static_scratch_matches_workspace_entry_point_twice():
    assert api.lib().twn_ternarize_static_scratch_bytes() == 98304
    # large first (4096 blocks' worth of partials are written), then smaller inputs that use fewer blocks
    _pair((2048, 4096), 1, 1, False)          # flat streaming kernels, 512 blocks
    _pair((300, 200), 2, 1, True)             # gather kernel, few blocks
    _pair((128, 64, 3, 3), 3, 1, True)        # tile kernel
    _pair((64, 3, 7, 7), 4, 64, False)        # per-filter groups (no partials at all)
    _pair((48, 40), 5, 1, False)              # smaller again
