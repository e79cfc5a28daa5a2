"""The row-band kernel on its own (bsp_conv2d_only with BSP_KERNEL_ROWS) against the oracle,
element by element: 7xK, 3xK and 1xK windows (1xK with K > 1), strides 1 and 2, all granularities, ragged image
sizes and tile tails, empty strips, fused epilogue (needs a GPU)."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp
from synthetic import draw_layer

from gpu_util import assert_close, make_layer, oracle_conv, to_device, to_host

pytestmark = pytest.mark.gpu

GRANS = [(8, 8), (4, 16), (16, 4)]


def _run_rows(c, layer=None, residual=None, relu=False):
    import torch
    layer = layer or make_layer(c)
    Y = torch.full((c.B, c.M, c.N, c.O), float("nan"), dtype=layer.torch_dtype, device="cuda")
    layer.conv2d(to_device(c), c.stride, c.pad, out=Y, family=bsp.BSP_KERNEL_ROWS,
                 residual=residual, relu=relu)
    torch.cuda.synchronize()
    return to_host(Y)


# (B, L, J, I, O, H, K, stride, pad)
SHAPES = [
    (2, 14, 14, 64, 64, 3, 3, 1, 1),       # two bands of seven rows
    (3, 7, 7, 128, 32, 3, 3, 1, 1),        # images smaller than a lane tile
    (2, 28, 28, 64, 32, 3, 3, 1, 1),
    (1, 56, 56, 64, 64, 3, 3, 1, 1),       # rows wider than a workgroup's columns
    (2, 17, 13, 72, 48, 3, 3, 1, 1),       # ragged rows and columns, channels not a power of two
    (2, 15, 15, 64, 64, 3, 3, 2, 1),       # stride 2
    (1, 28, 28, 136, 16, 3, 3, 2, 1),      # two slabs, the second with one chunk
    (2, 9, 20, 264, 24, 3, 3, 1, 0),       # no padding, three slabs
    (2, 12, 12, 32, 16, 1, 3, 1, (0, 1)),  # 1x3
    (2, 12, 12, 32, 16, 3, 1, 1, (1, 0)),  # 3x1
    (1, 17, 17, 128, 64, 1, 7, 1, (0, 3)),  # 1x7
    (2, 17, 17, 160, 48, 7, 1, 1, (3, 0)),  # 7x1, two slabs
    (1, 9, 20, 64, 32, 7, 3, 1, (3, 1)),    # 7x3, no full band
    (2, 12, 12, 264, 40, 1, 3, 1, (0, 1)),  # 1x3 over three slabs, few steps in the last
]


@pytest.mark.parametrize("bo,bi", GRANS)
def test_rows_kernel_shapes(bo, bi):
    for n, (B, L, J, I, O, H, K, s, p) in enumerate(SHAPES):
        c = draw_layer("rows", B=B, L=L, J=J, I=I, O=O, H=H, K=K, stride=s, pad=p, bo=bo, bi=bi,
                       dtype="bf16", mask_kind="bernoulli", density=0.5, seed=8100 + n, b_std=0.5)
        print("rows case", n, (B, L, J, I, O, H, K, s, p, bo, bi), flush=True)
        assert_close(_run_rows(c), oracle_conv(c), "bf16", f"rows shape {n} {bo}x{bi}")


@pytest.mark.parametrize("kind,density", [("zeros", 0.0), ("ones", 1.0), ("exact", 0.1),
                                          ("row_balanced", 0.5)])
def test_rows_kernel_mask_extremes(kind, density):
    c = draw_layer("rows", B=2, L=14, J=14, I=128, O=96, H=3, K=3, stride=1, pad=1,
                   dtype="bf16", mask_kind=kind, density=density, seed=8200, b_std=0.5)
    y = _run_rows(c)
    ref = oracle_conv(c)
    if kind == "zeros":
        want = oracle.round_to_storage(c.bias.astype(np.float64), "bf16").astype(np.float64)
        assert (y == want).all(), "an all-zero mask gives cast(bias) exactly"
    assert_close(y, ref, "bf16", kind)


def test_rows_kernel_empty_block_rows():
    c = draw_layer("rows", B=2, L=14, J=14, I=64, O=64, H=3, K=3, stride=1, pad=1,
                   dtype="bf16", mask_kind="bernoulli", density=0.5, seed=8300, b_std=0.5)
    c.gamma[1, :] = 0
    c.gamma[4:6, :] = 0
    assert_close(_run_rows(c), oracle_conv(c), "bf16", "empty block rows")


@pytest.mark.parametrize("H,K,p", [(3, 3, 1), (1, 7, (0, 3)), (7, 1, (3, 0))])
def test_rows_kernel_empty_slabs(H, K, p):
    """Strips with no step in a whole slab of input channels (the middle one, the last one, all
    but one), block rows with nothing at all: the flat step sequence has to find each step's
    slab and pass every slab's barrier all the same."""
    c = draw_layer("rows", B=3, L=9, J=17, I=392, O=80, H=H, K=K, stride=1, pad=p,
                   dtype="bf16", mask_kind="bernoulli", density=0.6, seed=8350 + H, b_std=0.5)
    nbc = c.gamma.shape[1]            # 49 block columns: slabs of 16, 16, 16 and 1
    c.gamma[0:4, 16:32] = 0           # no step in the second slab
    c.gamma[4:6, 32:] = 0             # none in the last two
    c.gamma[6, :] = 0
    c.gamma[6, nbc - 1] = 1           # only the last slab's single block
    c.gamma[7, :] = 0                 # an empty block row
    c.gamma[8:10, 0:48] = 0           # only the last block column
    assert_close(_run_rows(c), oracle_conv(c), "bf16", f"empty slabs {H}x{K}")


def test_rows_kernel_fused_epilogue():
    import torch
    for (H, K, p) in ((3, 3, 1), (1, 3, (0, 1))):
        c = draw_layer("rows", B=2, L=14, J=14, I=64, O=64, H=H, K=K, stride=1, pad=p,
                       dtype="bf16", seed=8400 + H, b_std=0.5)
        rng = np.random.default_rng(1)
        R = oracle.round_to_storage(rng.standard_normal((c.B, c.M, c.N, c.O)), "bf16")
        Rd = torch.from_numpy(R).to(torch.bfloat16).cuda()
        for res, relu in ((Rd, True), (Rd, False), (None, True)):
            y = _run_rows(c, residual=res, relu=relu)
            ref = oracle.conv2d_fused(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad,
                                      residual=None if res is None else R, relu=relu)
            assert_close(y, ref, "bf16", f"fused {H}x{K} res={res is not None} relu={relu}")


def test_rows_kernel_config1_full_size():
    from synthetic import config_cases
    c = next(config_cases(1))
    assert_close(_run_rows(c), oracle_conv(c), "bf16", "config 1")


def test_rows_kernel_declines_what_it_cannot_do():
    c = draw_layer("rows", B=1, L=9, J=9, I=64, O=64, H=5, K=5, stride=1, pad=2, dtype="bf16",
                   seed=1)
    with pytest.raises(bsp.BspError) as e:
        _run_rows(c)
    assert e.value.code == -6
    # one-row windows at stride 2 are not compiled (they were once run through the stride-1
    # instance: wrong rows of the patch)
    c = draw_layer("rows", B=2, L=8, J=19, I=264, O=256, H=1, K=3, stride=2, pad=(0, 1), dtype="bf16", seed=1)
    with pytest.raises(bsp.BspError) as e:
        _run_rows(c)
    assert e.value.code == -6
    # pointwise layers belong to the pointwise kernel
    c = draw_layer("rows", B=2, L=14, J=14, I=64, O=64, H=1, K=1, stride=1, pad=0, dtype="bf16", seed=1)
    with pytest.raises(bsp.BspError) as e:
        _run_rows(c)
    assert e.value.code == -6
