"""Per-layer parity at the full sizes of the network-shaped configurations
(ResNet50 at batch 32; VGG16 and InceptionV3 at batch 16): every layer runs
through the dispatcher on the GPU with its own seeded N(0,1) input, into an
output buffer pre-filled with NaN, and is compared with the oracle element by
element (a sampled comparison, corners included, runs first as a quick
pre-check that names the position).  Layers are independent here on purpose:
parity is per layer, never through a chain of bf16 layers."""
import numpy as np
import pytest

import oracle
from synthetic import config_cases

from gpu_util import TIGHT, TOL, assert_close, make_layer, to_device, to_host

pytestmark = pytest.mark.gpu


def _positions(c, rng, count=1500):
    B, M, N, O = c.B, c.M, c.N, c.O
    pos = np.stack([rng.integers(0, B, count), rng.integers(0, M, count),
                    rng.integers(0, N, count), rng.integers(0, O, count)], axis=1)
    edge = [(0, 0, 0, 0), (B - 1, M - 1, N - 1, O - 1), (0, M - 1, 0, O - 1), (B - 1, 0, N - 1, 0),
            (B // 2, M - 1, N // 2, O // 2), (B // 2, M // 2, N - 1, O - 1)]
    return np.concatenate([pos, np.array(edge, dtype=np.int64)], axis=0)


def _check_layer(c, rng):
    import torch
    layer = make_layer(c)
    Y = torch.full((c.B, c.M, c.N, c.O), float("nan"), dtype=layer.torch_dtype, device="cuda")
    if c.L == 1 and c.J == 1 and c.H == 1 and c.K == 1:
        layer.fc(to_device(c).reshape(c.B, c.I), out=Y.view(c.B, c.O))
    else:
        layer.conv2d(to_device(c), c.stride, c.pad, out=Y)
    torch.cuda.synchronize()
    y = to_host(Y)
    del Y
    assert y.shape == (c.B, c.M, c.N, c.O)
    assert np.isfinite(y).all(), f"{c.name}: an output was never written (or is not finite)"
    pos = _positions(c, rng)
    ref = oracle.conv2d_at(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, pos, c.stride, c.pad)
    got = y[tuple(pos.T)]
    rms = float(np.sqrt(np.mean(ref * ref)))
    scale = np.maximum(np.abs(ref), rms)
    err = np.abs(got - ref) / scale
    assert err.max() <= TOL[c.dtype], f"{c.name}: worst {err.max():.3e} at {pos[np.argmax(err)]}"
    # every element against the full oracle result
    full = oracle.conv2d(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad)
    assert_close(y, full, c.dtype, c.name)
    rms = float(np.sqrt(np.mean(full * full)))
    return float((np.abs(y - full) / np.maximum(np.abs(full), rms)).max())


@pytest.mark.parametrize("cfg,net", [(3, "resnet50"), (4, "vgg16"), (4, "inception_v3")])
def test_network_layers(cfg, net):
    rng = np.random.default_rng(cfg)
    worst = 0.0
    n = 0
    for c in config_cases(cfg):
        if c.meta.get("net") != net:
            continue
        print(net, c.name, (c.B, c.L, c.J, c.I), "->", c.O, f"{c.H}x{c.K}", c.stride, c.pad,
              "nnzb", c.nnzb, flush=True)
        worst = max(worst, _check_layer(c, rng))
        n += 1
    print(net, "layers", n, "worst rel err", worst, flush=True)
    assert n == {"resnet50": 54, "vgg16": 16, "inception_v3": 95}[net]
