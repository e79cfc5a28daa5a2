"""The FC entry point that allocates nothing (partial sums in the library's fixed device
array), called through the C ABI: its output against bsp_fc_fused's, bit for bit, on two calls
in a row, the second smaller; a layer beyond the array's size is refused."""
import numpy as np
import pytest

import paper_2407_09453_amd as bsp
from synthetic import draw_layer

from gpu_util import make_layer, to_device

pytestmark = pytest.mark.gpu


def _layer(B, I, O, seed, d=0.5):
    c = draw_layer("fcs", B=B, L=1, J=1, I=I, O=O, H=1, K=1, stride=1, pad=0, bo=8, bi=8,
                   dtype="bf16", mask_kind="exact", density=d, seed=seed, b_std=0.5)
    return c, make_layer(c)


def _both(layer, X, B, O, residual, relu):
    import torch
    st = torch.cuda.current_stream().cuda_stream
    bias = None if layer.d_bias is None else layer.d_bias.data_ptr()
    res = None if residual is None else residual.data_ptr()
    Y0 = torch.full((B, O), float("nan"), dtype=torch.bfloat16, device="cuda")
    Y1 = torch.full((B, O), float("nan"), dtype=torch.bfloat16, device="cuda")
    bsp.bsp_fc_fused(layer.struct, X.data_ptr(), bias, res, relu, Y0.data_ptr(), B, st)
    bsp.bsp_fc_fused_static(layer.struct, X.data_ptr(), bias, res, relu, Y1.data_ptr(), B, st)
    torch.cuda.synchronize()
    return Y0, Y1


def test_static_scratch_matches_allocating_entry_point_twice():
    import torch
    # cut into eight channel ranges: 8 x 16 x 512 floats of partial sums
    c, layer = _layer(16, 12544, 512, 901)
    X = to_device(c).reshape(16, 12544)
    R = torch.randn(16, 512, device="cuda").to(torch.bfloat16)
    Y0, Y1 = _both(layer, X, 16, 512, R, True)
    assert not torch.isnan(Y0.float()).any() and torch.equal(Y0, Y1)
    # a smaller input next: fewer rows of the batch, then a smaller layer (whose partial sums
    # cover only the start of what the first call left in the array)
    Y0, Y1 = _both(layer, X[:5].contiguous(), 5, 512, None, False)
    assert not torch.isnan(Y0.float()).any() and torch.equal(Y0, Y1)
    c2, layer2 = _layer(3, 6000, 72, 902, d=0.3)
    X2 = to_device(c2).reshape(3, 6000)
    Y0, Y1 = _both(layer2, X2, 3, 72, None, True)
    assert not torch.isnan(Y0.float()).any() and torch.equal(Y0, Y1)
    # and a layer whose activations fit LDS (no partial sums at all)
    c3, layer3 = _layer(32, 2048, 1000, 903)
    X3 = to_device(c3).reshape(32, 2048)
    Y0, Y1 = _both(layer3, X3, 32, 1000, None, False)
    assert not torch.isnan(Y0.float()).any() and torch.equal(Y0, Y1)


def test_static_scratch_refuses_what_does_not_fit():
    import torch
    # 64 pixels: ranges of at most 1056 channels -> 16 ranges x 64 x 1032 floats = 4.2 MB > 4 MiB
    c, layer = _layer(64, 12544, 1032, 904, d=0.1)
    X = to_device(c).reshape(64, 12544)
    Y = torch.full((64, 1032), -7.0, dtype=torch.bfloat16, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    with pytest.raises(bsp.BspError) as e:
        bsp.bsp_fc_fused_static(layer.struct, X.data_ptr(), layer.d_bias.data_ptr(), None, False,
                                Y.data_ptr(), 64, st)
    assert e.value.code == -7
    torch.cuda.synchronize()
    assert bool((Y == -7.0).all())          # nothing was launched
    bsp.bsp_fc_fused(layer.struct, X.data_ptr(), layer.d_bias.data_ptr(), None, False,
                     Y.data_ptr(), 64, st)  # the allocating entry point takes it
    torch.cuda.synchronize()
    assert not bool((Y == -7.0).all())
