"""The band kernel on its own (bsp_conv2d_only with BSP_KERNEL_BAND) against the oracle, element
by element: 3x3 stride-1 layers with at most 128 input channels; ragged rows, rows cut into
column chunks, bands with a short tail, images smaller than a band, all mask extremes, fused
epilogue, config 1 at full size (needs a GPU)."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp
from synthetic import draw_layer

from gpu_util import assert_close, make_layer, oracle_conv, to_device, to_host

pytestmark = pytest.mark.gpu


def _run_band(c, residual=None, relu=False):
    import torch
    layer = make_layer(c)
    Y = torch.full((c.B, c.M, c.N, c.O), float("nan"), dtype=layer.torch_dtype, device="cuda")
    layer.conv2d(to_device(c), c.stride, c.pad, out=Y, family=bsp.BSP_KERNEL_BAND,
                 residual=residual, relu=relu)
    torch.cuda.synchronize()
    return to_host(Y)


# (B, L, J, I, O)
SHAPES = [
    (2, 14, 14, 64, 64),
    (40, 7, 7, 64, 32),        # images smaller than a band; four rows per band
    (1, 56, 56, 64, 64),       # four column tiles, the last half full
    (2, 28, 28, 128, 128),     # 256-byte pixels, eight strips x two column tiles
    (3, 17, 13, 72, 48),       # ragged rows and columns, channels no power of two
    (2, 9, 64, 64, 64),        # four chunks of sixteen columns
    (2, 20, 100, 64, 64),      # two column chunks: 64 + 36 columns
    (1, 11, 70, 128, 128),     # 256-byte pixels, eight strips: chunks of 32, 32 and 6 columns
    (1, 9, 224, 64, 64),       # 64 + 64 + 64 + 32
    (3, 10, 33, 64, 96),       # six strips: chunks of 16, 16 and one column
    (2, 30, 50, 8, 16),        # one 16-byte piece per pixel
    (33, 15, 20, 24, 8),       # one block row of eight channels
]


@pytest.mark.parametrize("bo,bi", [(8, 8), (4, 16)])
def test_band_kernel_shapes(bo, bi):
    for n, (B, L, J, I, O) in enumerate(SHAPES):
        if bi == 16 and I % 16:
            continue
        c = draw_layer("band", B=B, L=L, J=J, I=I, O=O, H=3, K=3, stride=1, pad=1, bo=bo, bi=bi,
                       dtype="bf16", mask_kind="bernoulli", density=0.5, seed=8900 + n, b_std=0.5)
        print("band case", n, (B, L, J, I, O, bo, bi), flush=True)
        assert_close(_run_band(c), oracle_conv(c), "bf16", f"band shape {n} {bo}x{bi}")


@pytest.mark.parametrize("B,L,J,I,O", [(2, 14, 14, 64, 64), (3, 20, 37, 80, 192), (40, 30, 21, 64, 64),
                                       (1, 5, 3, 16, 16)])
def test_band_kernel_without_padding(B, L, J, I, O):
    """Windows that stay inside the image (padding 0): the output is two rows and columns smaller."""
    c = draw_layer("band0", B=B, L=L, J=J, I=I, O=O, H=3, K=3, stride=1, pad=0, dtype="bf16",
                   mask_kind="bernoulli", density=0.5, seed=9000 + L, b_std=0.5)
    assert (c.M, c.N) == (L - 2, J - 2)
    assert_close(_run_band(c), oracle_conv(c), "bf16", f"band pad 0 {(B, L, J, I, O)}")


@pytest.mark.parametrize("kind,density", [("zeros", 0.0), ("ones", 1.0), ("exact", 0.1),
                                          ("row_balanced", 0.5)])
def test_band_kernel_mask_extremes(kind, density):
    c = draw_layer("band", B=2, L=14, J=14, I=128, O=96, H=3, K=3, stride=1, pad=1,
                   dtype="bf16", mask_kind=kind, density=density, seed=8950, b_std=0.5)
    y = _run_band(c)
    if kind == "zeros":
        want = oracle.round_to_storage(c.bias.astype(np.float64), "bf16").astype(np.float64)
        assert (y == want).all(), "an all-zero mask gives cast(bias) exactly"
    assert_close(y, oracle_conv(c), "bf16", kind)


def test_band_kernel_fused_epilogue():
    import torch
    c = draw_layer("band", B=2, L=14, J=14, I=64, O=64, H=3, K=3, stride=1, pad=1,
                   dtype="bf16", seed=8960, b_std=0.5)
    rng = np.random.default_rng(1)
    R = oracle.round_to_storage(rng.standard_normal((c.B, c.M, c.N, c.O)), "bf16")
    Rd = torch.from_numpy(R).to(torch.bfloat16).cuda()
    for res, relu in ((Rd, True), (Rd, False), (None, True)):
        y = _run_band(c, residual=res, relu=relu)
        ref = oracle.conv2d_fused(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad,
                                  residual=None if res is None else R, relu=relu)
        assert_close(y, ref, "bf16", f"fused res={res is not None} relu={relu}")


# Enough images for bands of seven rows (the small shapes above get four-row bands):
# (B, L, J, I, O)
SEVEN_ROW_SHAPES = [
    (34, 41, 50, 72, 64),      # last band six rows; four chunks, the last one two columns; four strips
    (29, 50, 28, 128, 128),    # 256-byte pixels; eight strips, one pair of column tiles; last band one row
    (67, 17, 13, 72, 48),      # last band three rows; one column tile
    (50, 25, 20, 64, 64),      # last band four rows
    (40, 33, 64, 16, 16),      # last band five rows
    (8, 60, 150, 64, 64),      # column chunks on seven-row bands: 64 + 64 + 22
]


@pytest.mark.parametrize("bo,bi", [(8, 8), (4, 16)])
def test_band_kernel_seven_row_shapes(bo, bi):
    for n, (B, L, J, I, O) in enumerate(SEVEN_ROW_SHAPES):
        if bi == 16 and I % 16:
            continue
        c = draw_layer("bandp", B=B, L=L, J=J, I=I, O=O, H=3, K=3, stride=1, pad=1, bo=bo, bi=bi,
                       dtype="bf16", mask_kind="bernoulli", density=0.5, seed=8970 + n, b_std=0.5)
        print("seven-row band case", n, (B, L, J, I, O, bo, bi), flush=True)
        assert_close(_run_band(c), oracle_conv(c), "bf16", f"seven-row band shape {n} {bo}x{bi}")


@pytest.mark.parametrize("kind,density", [("zeros", 0.0), ("ones", 1.0), ("exact", 0.1)])
def test_band_kernel_seven_row_mask_extremes_and_epilogue(kind, density):
    import torch
    c = draw_layer("bandp", B=50, L=25, J=20, I=64, O=64, H=3, K=3, stride=1, pad=1,
                   dtype="bf16", mask_kind=kind, density=density, seed=8990, b_std=0.5)
    y = _run_band(c)
    if kind == "zeros":
        want = oracle.round_to_storage(c.bias.astype(np.float64), "bf16").astype(np.float64)
        assert (y == want).all(), "an all-zero mask gives cast(bias) exactly"
    assert_close(y, oracle_conv(c), "bf16", kind)
    rng = np.random.default_rng(2)
    R = oracle.round_to_storage(rng.standard_normal((c.B, c.M, c.N, c.O)), "bf16")
    Rd = torch.from_numpy(R).to(torch.bfloat16).cuda()
    # the fused epilogue is the unfused result plus residual, ReLU, one more rounding: exactly
    yf = _run_band(c, residual=Rd, relu=True)
    want = oracle.round_to_storage(np.maximum(y.astype(np.float32) + R.astype(np.float32), np.float32(0)), "bf16")
    assert (yf == want).all(), f"seven-row fused {kind}"


def test_band_kernel_config1_full_size():
    from synthetic import config_cases
    c = next(config_cases(1))
    assert_close(_run_band(c), oracle_conv(c), "bf16", "config 1")


def test_band_kernel_declines_what_it_cannot_do():
    for kw in (dict(I=256, O=64, J=14, stride=1), dict(I=64, O=64, J=14, stride=2),
               dict(I=64, O=512, J=14, stride=1),
               dict(I=32, O=64, J=40, stride=1),     # several chunks of thin pixels
               dict(I=64, O=32, J=70, stride=1)):    # several chunks, two strips
        c = draw_layer("band", B=1, L=14, J=kw["J"], I=kw["I"], O=kw["O"], H=3, K=3,
                       stride=kw["stride"], pad=1, dtype="bf16", seed=1)
        with pytest.raises(bsp.BspError) as e:
            _run_band(c)
        assert e.value.code == -6, kw
    c = draw_layer("band", B=1, L=14, J=14, I=64, O=64, H=3, K=3, stride=1, pad=1, bo=16, bi=4,
                   dtype="bf16", seed=1)
    with pytest.raises(bsp.BspError) as e:     # 4-channel contraction units are left to the other kernels
        _run_band(c)
    assert e.value.code == -6
