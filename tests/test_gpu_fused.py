"""Fused residual / ReLU epilogue: every kernel of the dispatcher against the oracle, and
against the unfused HIP layer followed by torch's element-wise ops (needs a GPU)."""
import numpy as np
import pytest

import oracle
from synthetic import draw_layer

from gpu_util import assert_close, make_layer, to_device, to_host

pytestmark = pytest.mark.gpu

SHAPES = [
    # B, L, J, I, O, H, K, stride, pad                       (kernel the dispatcher picks)
    (2, 20, 20, 64, 64, 3, 3, (1, 1), (1, 1)),       # LDS-resident, one slab
    (1, 14, 14, 192, 128, 3, 3, (1, 1), (1, 1)),     # LDS-resident, three slabs
    (3, 13, 13, 128, 96, 1, 1, (1, 1), (0, 0)),      # LDS-resident, pointwise
    (1, 12, 12, 16, 16, 5, 5, (1, 1), (2, 2)),       # ring-tile kernel (5x5 window)
    (8, 1, 1, 512, 48, 1, 1, (1, 1), (0, 0)),        # weight-streaming FC
    (1, 3, 3, 20, 12, 3, 3, (1, 1), (1, 1)),         # general kernel, ragged O and I
    (2, 15, 13, 3, 64, 7, 7, (2, 2), (3, 3)),        # first layer (narrow input)
]


def _case(shape, seed, dtype):
    B, L, J, I, O, H, K, s, p = shape
    c = draw_layer("f", B=B, L=L, J=J, I=I, O=O, H=H, K=K, stride=s, pad=p, bo=8, bi=8,
                   dtype=dtype, mask_kind="bernoulli", density=0.5, seed=seed, b_std=0.5)
    rng = np.random.default_rng(seed + 1)
    R = oracle.round_to_storage(rng.standard_normal((c.B, c.M, c.N, c.O)) * 2.0, dtype)
    return c, R.astype(np.float32)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("residual,relu", [(True, True), (True, False), (False, True)])
def test_fused_epilogue_vs_oracle(dtype, residual, relu):
    import torch
    for n, shape in enumerate(SHAPES):
        c, R = _case(shape, 700 + n, dtype)
        layer = make_layer(c)
        Rd = to_device(c, R) if residual else None
        print("case", n, shape, dtype, residual, relu, flush=True)
        Y = layer.conv2d(to_device(c), c.stride, c.pad, residual=Rd, relu=relu)
        torch.cuda.synchronize()
        ref = oracle.conv2d_fused(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad,
                                  residual=R if residual else None, relu=relu, dtype=dtype)
        y = to_host(Y)
        if relu:
            assert (y >= 0).all()
        # the intermediate rounding may fall on the other side of a tie than the fp64 oracle's:
        # compare on the scale of the pre-activation values
        pre = oracle.conv2d(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad)
        scale = np.maximum(np.abs(pre) + (np.abs(R) if residual else 0), np.sqrt(np.mean(pre * pre)))
        tol = {"bf16": 2e-2, "f32": 1e-5}[dtype]
        assert (np.abs(y - ref) <= tol * scale).all(), (shape, float((np.abs(y - ref) / scale).max()))


def test_fused_equals_unfused_layer_plus_torch_ops():
    """Bit for bit: the fused call against bsp_conv2d followed by torch's add and relu in bf16
    (each rounding once), which is the arithmetic the header promises."""
    import torch
    for n, shape in enumerate(SHAPES):
        c, R = _case(shape, 800 + n, "bf16")
        layer = make_layer(c)
        X, Rd = to_device(c), to_device(c, R)
        Yf = layer.conv2d(X, c.stride, c.pad, residual=Rd, relu=True)
        Y0 = layer.conv2d(X, c.stride, c.pad)
        want = torch.relu((Y0.float() + Rd.float())).to(torch.bfloat16)
        torch.cuda.synchronize()
        assert torch.equal(Yf, want), shape
        Yr = layer.conv2d(X, c.stride, c.pad, relu=True)
        assert torch.equal(Yr, torch.relu(Y0)), shape


def test_fc_fused():
    import torch
    c, R = _case((16, 1, 1, 1024, 200, 1, 1, (1, 1), (0, 0)), 900, "bf16")
    layer = make_layer(c)
    X = to_device(c).reshape(c.B, c.I)
    Rd = to_device(c, R).reshape(c.B, c.O)
    Y = layer.fc(X, residual=Rd, relu=True)
    Y0 = layer.fc(X)
    torch.cuda.synchronize()
    assert torch.equal(Y, torch.relu(Y0.float() + Rd.float()).to(torch.bfloat16))
