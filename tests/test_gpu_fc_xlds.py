"""FC layers (8x8 blocks) through the kernel that keeps the activations in LDS and streams the
compressed block rows past them, against the CPU oracle element by element: whole X in LDS
(waves sharing rows or owning them), X cut into channel ranges with partial sums in scratch
memory, every batch-tile count, ragged channel counts, empty rows, fused epilogue."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp
from synthetic import draw_layer

from gpu_util import assert_close, make_layer, to_device, to_host

pytestmark = pytest.mark.gpu


CASES = [
    # B, I, O, density
    (16, 512, 1024, 0.5),      # two rows per workgroup, four waves a row
    (1, 64, 1024, 0.5),        # one step per row at most
    (32, 2048, 1000, 0.5),     # ResNet50's classifier: eight waves a row, two batch tiles
    (33, 264, 1032, 0.3),      # three batch tiles (run as four), O not a multiple of 16
    (64, 128, 2048, 0.55),     # four batch tiles
    (5, 1024, 1030, 0.1),      # O % 8 = 6: the last block row hangs over
    (16, 4096, 4096, 0.5),     # VGG16 fc7
    (16, 12544, 256, 0.5),     # X does not fit: eight channel ranges, waves share rows
    (16, 25088, 512, 0.5),     # VGG16 fc6's X with fewer outputs: ranges x sixteen-row groups
    (48, 2512, 72, 0.7),       # four batch tiles force ranges on a short layer; ragged last range
    (7, 5000, 2096, 1.0),      # all blocks kept, two ranges rounded to eight
    (3, 6000, 40, 0.0),        # no block kept: bias only, through the partial sums
]


@pytest.mark.parametrize("B,I,O,d", CASES)
def test_fc_xlds_vs_oracle(B, I, O, d):
    import torch
    c = draw_layer("fcx", B=B, L=1, J=1, I=I, O=O, H=1, K=1, stride=1, pad=0, bo=8, bi=8,
                   dtype="bf16", mask_kind="exact", density=d, seed=B * 11 + O + I, b_std=0.5)
    c.gamma = c.gamma.copy()
    if c.gamma.shape[0] > 3:
        c.gamma[3, :] = 0                               # an empty block row: bias only
    if c.gamma.shape[0] > 1 and d > 0:
        c.gamma[1, :] = 1                               # a full one
    layer = make_layer(c)
    X = to_device(c).reshape(B, I)
    Y = torch.full((B, O), float("nan"), dtype=torch.bfloat16, device="cuda")
    X4 = X.view(B, 1, 1, I)
    layer.conv2d(X4, out=Y.view(B, 1, 1, O), family=bsp.BSP_KERNEL_FC)
    torch.cuda.synchronize()
    ref = oracle.fc(c.X.reshape(B, I), c.W.reshape(O, I), c.bias, c.gamma, 8, 8)
    assert_close(to_host(Y), ref, "bf16", f"fc xlds {B}x{I}->{O} d={d}")
    R = torch.randn(B, O, device="cuda").to(torch.bfloat16)
    Yf = layer.conv2d(X4, residual=R.view(B, 1, 1, O), relu=True, family=bsp.BSP_KERNEL_FC).view(B, O)
    torch.cuda.synchronize()
    assert torch.equal(Yf, torch.relu(Y.float() + R.float()).to(torch.bfloat16))
    # a second call gives the same bits (the partial sums are added in a fixed order)
    Y2 = layer.conv2d(X4, family=bsp.BSP_KERNEL_FC).view(B, O)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)
