"""The pointwise kernel on its own (bsp_conv2d_only with BSP_KERNEL_PW) against the oracle,
element by element: shallow and deep 1x1 layers, strides 1 and 2, all granularities, pixel
counts with ragged tile tails, channel counts that are no power of two, empty strips, fused
epilogue (needs a GPU)."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp
from synthetic import draw_layer

from gpu_util import assert_close, make_layer, oracle_conv, to_device, to_host

pytestmark = pytest.mark.gpu

GRANS = [(8, 8), (4, 16), (16, 4)]


def _run_pw(c, layer=None, residual=None, relu=False):
    import torch
    layer = layer or make_layer(c)
    Y = torch.full((c.B, c.M, c.N, c.O), float("nan"), dtype=layer.torch_dtype, device="cuda")
    layer.conv2d(to_device(c), c.stride, c.pad, out=Y, family=bsp.BSP_KERNEL_PW,
                 residual=residual, relu=relu)
    torch.cuda.synchronize()
    return to_host(Y)


# (B, L, J, I, O, stride)
SHAPES = [
    (4, 14, 14, 256, 128, 1),
    (16, 7, 7, 520, 64, 1),       # channels no multiple of 128, pixel count with a ragged tail
    (2, 28, 28, 64, 256, 2),      # strided (downsample)
    (3, 14, 14, 1024, 64, 1),     # deep: a staged pixel is two KiB
    (5, 7, 7, 2048, 48, 1),       # deepest single slab at 8-channel units
    (2, 14, 14, 1024, 96, 2),
    (1, 56, 56, 64, 64, 1),
    (3, 9, 11, 24, 40, 1),        # fewer channels than one staged piece group
    (1, 13, 5, 72, 8, 1),         # one block row, 65 pixels
    (2, 28, 28, 128, 512, 1),
]


@pytest.mark.parametrize("bo,bi", GRANS)
def test_pw_kernel_shapes(bo, bi):
    for n, (B, L, J, I, O, s) in enumerate(SHAPES):
        if bi == 4 and I > 1024:
            continue  # 4-channel units: more than 256 of them need a second slab (declined)
        c = draw_layer("pw", B=B, L=L, J=J, I=I, O=O, H=1, K=1, stride=s, pad=0, bo=bo, bi=bi,
                       dtype="bf16", mask_kind="bernoulli", density=0.5, seed=8600 + n, b_std=0.5)
        print("pw case", n, (B, L, J, I, O, s, bo, bi), flush=True)
        assert_close(_run_pw(c), oracle_conv(c), "bf16", f"pw shape {n} {bo}x{bi}")


@pytest.mark.parametrize("kind,density", [("zeros", 0.0), ("ones", 1.0), ("exact", 0.1),
                                          ("row_balanced", 0.5)])
def test_pw_kernel_mask_extremes(kind, density):
    c = draw_layer("pw", B=2, L=14, J=14, I=256, O=96, H=1, K=1, stride=1, pad=0,
                   dtype="bf16", mask_kind=kind, density=density, seed=8700, b_std=0.5)
    y = _run_pw(c)
    if kind == "zeros":
        want = oracle.round_to_storage(c.bias.astype(np.float64), "bf16").astype(np.float64)
        assert (y == want).all(), "an all-zero mask gives cast(bias) exactly"
    assert_close(y, oracle_conv(c), "bf16", kind)


def test_pw_kernel_empty_block_rows():
    c = draw_layer("pw", B=2, L=14, J=14, I=512, O=64, H=1, K=1, stride=1, pad=0,
                   dtype="bf16", mask_kind="bernoulli", density=0.5, seed=8750, b_std=0.5)
    c.gamma[1, :] = 0
    c.gamma[4:6, :] = 0
    assert_close(_run_pw(c), oracle_conv(c), "bf16", "empty block rows")


@pytest.mark.parametrize("bo,bi", GRANS)
def test_pw_kernel_fused_epilogue(bo, bi):
    import torch
    c = draw_layer("pw", B=2, L=14, J=14, I=256, O=64, H=1, K=1, stride=1, pad=0, bo=bo, bi=bi,
                   dtype="bf16", seed=8800, b_std=0.5)
    rng = np.random.default_rng(1)
    R = oracle.round_to_storage(rng.standard_normal((c.B, c.M, c.N, c.O)), "bf16")
    Rd = torch.from_numpy(R).to(torch.bfloat16).cuda()
    for res, relu in ((Rd, True), (Rd, False), (None, True)):
        y = _run_pw(c, residual=res, relu=relu)
        ref = oracle.conv2d_fused(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad,
                                  residual=None if res is None else R, relu=relu)
        assert_close(y, ref, "bf16", f"fused {bo}x{bi} res={res is not None} relu={relu}")


def test_pw_kernel_declines_what_it_cannot_do():
    c = draw_layer("pw", B=1, L=9, J=9, I=64, O=64, H=3, K=3, stride=1, pad=1, dtype="bf16", seed=1)
    with pytest.raises(bsp.BspError) as e:
        _run_pw(c)
    assert e.value.code == -6
    c = draw_layer("pw", B=1, L=9, J=9, I=64, O=64, H=1, K=1, stride=1, pad=1, dtype="bf16", seed=1)
    with pytest.raises(bsp.BspError) as e:
        _run_pw(c)
    assert e.value.code == -6
