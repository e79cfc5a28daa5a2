"""The thin-input kernel on its own (bsp_conv2d_only with BSP_KERNEL_FIRST) against the oracle,
element by element: one to four input channels, 3x3 and 7x7 windows, strides 1 and 2, rows of
odd and even length, dropped block rows at every granularity, fused epilogue, the first layers
of the three networks at full width, and what it declines (needs a GPU)."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp
from synthetic import draw_layer

from gpu_util import assert_close, gpu_conv, make_layer, oracle_conv, to_device, to_host

pytestmark = pytest.mark.gpu

GRANS = [(8, 8), (4, 16), (16, 4)]


def _run_first(c, residual=None, relu=False):
    import torch
    layer = make_layer(c)
    Y = torch.full((c.B, c.M, c.N, c.O), float("nan"), dtype=layer.torch_dtype, device="cuda")
    layer.conv2d(to_device(c), c.stride, c.pad, out=Y, family=bsp.BSP_KERNEL_FIRST,
                 residual=residual, relu=relu)
    torch.cuda.synchronize()
    return to_host(Y)


# (B, L, J, I, O, H, K, stride, pad)
SHAPES = [
    (2, 20, 37, 3, 64, 3, 3, 1, 1),         # rows of odd length: copied two bytes at a time
    (2, 21, 40, 3, 64, 3, 3, 1, 1),         # even length: copied as dwords; a ragged last band
    (9, 30, 46, 3, 64, 7, 7, 2, 3),         # five steps, stride 2, more images than XCDs
    (2, 29, 31, 3, 32, 3, 3, 2, 0),         # no padding, two strips
    (1, 12, 18, 1, 32, 3, 3, 1, (1, 0)),    # one channel, padding of rows only
    (1, 12, 18, 2, 64, 3, 3, 1, (0, 1)),    # two channels, padding of columns only
    (1, 11, 16, 4, 64, 3, 3, 1, 1),         # four channels: two steps, an instance that is not compiled (declined)
    (1, 5, 5, 3, 64, 7, 7, 1, 3),           # an image smaller than the window's reach
    (3, 4, 70, 3, 32, 7, 7, 2, 3),          # one band, several lane tiles, O = 32 with five steps
    (1, 14, 19, 1, 32, 5, 5, 1, 2),         # 5x5 over one channel: 25 indices, one step
    (2, 20, 23, 3, 64, 3, 3, 3, 1),         # stride 3
    (1, 6, 300, 3, 64, 3, 3, 1, 1),         # rows longer than any image of the three networks
]


@pytest.mark.parametrize("bo,bi", GRANS)
def test_first_kernel_shapes(bo, bi):
    rng = np.random.default_rng(11)
    for n, (B, L, J, I, O, H, K, s, p) in enumerate(SHAPES):
        c = draw_layer("first", B=B, L=L, J=J, I=I, O=O, H=H, K=K, stride=s, pad=p, bo=bo, bi=bi,
                       dtype="bf16", seed=8700 + n, b_std=0.5)
        # a thin layer has one block column: its mask drops whole block rows
        c.gamma[:] = rng.integers(0, 2, size=c.gamma.shape)
        print("first case", n, (B, L, J, I, O, H, K, s, p, bo, bi), flush=True)
        steps = -(-H * K * I // 32)
        if steps not in (1, 5):
            with pytest.raises(bsp.BspError) as e:
                _run_first(c)
            assert e.value.code == -6
            continue
        assert_close(_run_first(c), oracle_conv(c), "bf16", f"first shape {n} {bo}x{bi}")


def test_first_kernel_mask_extremes():
    for kind in ("zeros", "ones"):
        c = draw_layer("first", B=2, L=14, J=14, I=3, O=64, H=3, K=3, stride=1, pad=1,
                       dtype="bf16", seed=8750, b_std=0.5)
        c.gamma[:] = 0 if kind == "zeros" else 1
        y = _run_first(c)
        if kind == "zeros":
            want = oracle.round_to_storage(c.bias.astype(np.float64), "bf16").astype(np.float64)
            assert (y == want).all(), "an all-zero mask gives cast(bias) exactly"
        assert_close(y, oracle_conv(c), "bf16", kind)


def test_first_kernel_fused_epilogue():
    import torch
    c = draw_layer("first", B=2, L=15, J=22, I=3, O=64, H=7, K=7, stride=2, pad=3,
                   dtype="bf16", seed=8760, b_std=0.5)
    rng = np.random.default_rng(1)
    R = oracle.round_to_storage(rng.standard_normal((c.B, c.M, c.N, c.O)), "bf16")
    Rd = torch.from_numpy(R).to(torch.bfloat16).cuda()
    for res, relu in ((Rd, True), (Rd, False), (None, True)):
        y = _run_first(c, residual=res, relu=relu)
        ref = oracle.conv2d_fused(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad,
                                  residual=None if res is None else R, relu=relu)
        assert_close(y, ref, "bf16", f"fused res={res is not None} relu={relu}")


@pytest.mark.parametrize("L,J,O,H,s,p", [(224, 224, 64, 3, 1, 1), (224, 224, 64, 7, 2, 3),
                                         (299, 299, 32, 3, 2, 0)])
def test_first_layers_of_the_networks_full_width(L, J, O, H, s, p):
    """Full image size, one image (the oracle's time); the dispatcher must pick this kernel."""
    c = draw_layer("first", B=1, L=L, J=J, I=3, O=O, H=H, K=H, stride=s, pad=p, dtype="bf16",
                   seed=8770 + H + s)
    ref = oracle_conv(c)
    assert_close(_run_first(c), ref, "bf16", "first layer, kernel alone")
    assert (gpu_conv(c) == _run_first(c)).all(), "bsp_conv2d takes the same kernel"


def test_first_kernel_declines_what_it_cannot_do():
    for kw in (dict(I=8, O=64, H=3, K=3), dict(I=3, O=48, H=3, K=3), dict(I=3, O=64, H=5, K=5),
               dict(I=3, O=256, H=3, K=3)):
        c = draw_layer("first", B=1, L=9, J=9, stride=1, pad=1, dtype="bf16", seed=1, **kw)
        with pytest.raises(bsp.BspError) as e:
            _run_first(c)
        assert e.value.code == -6
