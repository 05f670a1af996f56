"""bnn_conv2d_noalloc (the entry point that allocates nothing) against bnn_conv2d, through the C ABI:
two calls in a row on the same GPU, the second on a smaller input, so the second runs over the first
call's leftovers in the library's fixed scratch array."""
import numpy as np
import pytest
import torch

from paper_1911_04477_amd import binding as B
from paper_1911_04477_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pair(shape, seed, with_f32):
    d = inputs.conv_inputs(shape, seed=seed)
    x = torch.from_numpy(inputs.inject_specials(d["x"], seed, frac=1e-3)).to(DEV)
    wp = B.bnn_pack_conv_weight(torch.from_numpy(d["w"]).to(DEV))
    sc, bi = torch.from_numpy(d["scale"]).to(DEV), torch.from_numpy(d["bias"]).to(DEV)
    st, pd = (shape.sH, shape.sW), (shape.pH, shape.pW)
    want_i, want_f = B.bnn_conv2d(x, wp, shape.D, shape.kH, shape.kW, st, pd, sc if with_f32 else None,
                                  bi if with_f32 else None, want_int=True)
    got_i = torch.full_like(want_i, -12345)
    got_f = torch.full_like(want_f, float("nan")) if with_f32 else None
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.bnn_conv2d_noalloc(x, wp, shape.D, shape.kH, shape.kW, st, pd, got_i, got_f, sc if with_f32 else None,
                         bi if with_f32 else None)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(got_i, want_i)
    if with_f32:
        assert torch.equal(got_f, want_f)  # same kernels, same bits (the contract asks 1e-6 relative)
    return want_i


def test_noalloc_conv2d_matches_conv2d_twice_second_smaller():
    big = inputs.ConvShape(N=6, C=200, H=20, W=17, D=70, kH=3, kW=3, sH=1, sW=1, pH=1, pW=1)
    small = inputs.ConvShape(N=2, C=200, H=9, W=10, D=33, kH=3, kW=3, sH=1, sW=1, pH=1, pW=1)
    print("noalloc conv2d: first call", big, flush=True)
    _pair(big, 11, with_f32=True)
    print("noalloc conv2d: second call, smaller", small, flush=True)
    _pair(small, 12, with_f32=True)
    print("noalloc conv2d: third call, pointwise stride 2", flush=True)
    _pair(inputs.ConvShape(N=3, C=70, H=12, W=12, D=9, kH=1, kW=1, sH=2, sW=2, pH=0, pW=0), 13, with_f32=False)


def test_noalloc_conv2d_rejects_problems_over_the_limit():
    L = B.lib()
    limit = int(L.bnn_conv2d_noalloc_max_bytes())
    assert limit == 8 << 20
    # cfg 5a needs 6.4 MB: inside; twice its batch: outside, reported before anything is launched
    assert int(L.bnn_conv2d_workspace_bytes(64, 256, 56, 56, 3, 3, 1, 1, 1, 1)) <= limit
    assert int(L.bnn_conv2d_workspace_bytes(128, 256, 56, 56, 3, 3, 1, 1, 1, 1)) > limit
    x = torch.zeros(16, dtype=torch.float32, device=DEV)  # never read: the size check comes first
    st = L.bnn_conv2d_noalloc(x.data_ptr(), x.data_ptr(), 128, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1, x.data_ptr(), None,
                              None, None, None)
    assert st == 5  # BNN_ERR_WORKSPACE
