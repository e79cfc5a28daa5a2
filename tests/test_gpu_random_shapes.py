"""Seeded random layer shapes through the dispatcher against the oracles: bf16, fp32 and int8,
all granularities, windows up to 7x7, strides, paddings, ragged channel counts (needs a GPU)."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp
from synthetic import draw_layer

from gpu_util import assert_close, gpu_conv, oracle_conv

pytestmark = pytest.mark.gpu

GRANS = [(8, 8), (4, 16), (16, 4)]
CH_IN = [3, 8, 16, 24, 40, 64, 72, 128, 200, 264, 512]
CH_OUT = [8, 16, 24, 48, 64, 100, 136, 256]


def _random_shapes(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        H, K = int(rng.choice([1, 1, 2, 3, 3, 5, 7])), int(rng.choice([1, 1, 2, 3, 3, 5, 7]))
        ph, pw = int(rng.integers(0, H)), int(rng.integers(0, K))
        sh, sw = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        L, J = int(rng.integers(max(1, H - 2 * ph), 26)), int(rng.integers(max(1, K - 2 * pw), 26))
        if L + 2 * ph < H or J + 2 * pw < K:
            continue
        B = int(rng.integers(1, 4))
        I, O = int(rng.choice(CH_IN)), int(rng.choice(CH_OUT))
        if B * L * J * I * H * K * O > 3e9:       # keep the oracle quick
            continue
        if I * H * K > 4608:                      # the contraction length the derived bounds assume
            continue
        bo, bi = GRANS[int(rng.integers(0, 3))]
        out.append((B, L, J, I, O, H, K, (sh, sw), (ph, pw), bo, bi))
    return out


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_random_shapes_float(dtype):
    for n, (B, L, J, I, O, H, K, s, p, bo, bi) in enumerate(_random_shapes(77, 40)):
        c = draw_layer("r", B=B, L=L, J=J, I=I, O=O, H=H, K=K, stride=s, pad=p, bo=bo, bi=bi,
                       dtype=dtype, mask_kind="bernoulli", density=0.5, seed=6000 + n, b_std=0.5)
        print("case", n, (B, L, J, I, O, H, K, s, p, bo, bi), dtype, flush=True)
        assert_close(gpu_conv(c), oracle_conv(c), dtype, f"random shape {n}")


# (B, L, J, I, O, H, K, stride, pad, bo, bi): shapes that a wider random search once caught the
# dispatcher on (one-row windows at stride 2 with at least 128 input and output channels)
REGRESSIONS = [
    (2, 8, 19, 264, 256, 1, 3, (2, 2), (0, 1), 16, 4),
    (1, 6, 17, 512, 136, 1, 3, (2, 2), (0, 0), 8, 8),
    (2, 6, 18, 128, 256, 1, 3, (2, 2), (0, 2), 16, 4),
    (3, 23, 1, 264, 136, 1, 3, (2, 2), (0, 1), 8, 8),
    (2, 9, 21, 256, 128, 1, 7, (2, 1), (0, 3), 8, 8),
    (2, 21, 9, 256, 128, 7, 1, (1, 2), (3, 0), 8, 8),
]


def test_regression_shapes():
    for n, (B, L, J, I, O, H, K, s, p, bo, bi) in enumerate(REGRESSIONS):
        c = draw_layer("r", B=B, L=L, J=J, I=I, O=O, H=H, K=K, stride=s, pad=p, bo=bo, bi=bi,
                       dtype="bf16", mask_kind="bernoulli", density=0.5, seed=6500 + n, b_std=0.5)
        print("regression case", n, (B, L, J, I, O, H, K, s, p, bo, bi), flush=True)
        assert_close(gpu_conv(c), oracle_conv(c), "bf16", f"regression shape {n}")


def test_random_shapes_int8():
    import torch
    rng = np.random.default_rng(5)
    for n, (B, L, J, I, O, H, K, s, p, bo, bi) in enumerate(_random_shapes(78, 40)):
        X = rng.integers(-128, 128, (B, L, J, I), dtype=np.int8)
        W = rng.integers(-128, 128, (O, H, K, I), dtype=np.int8)
        bias = rng.integers(-2 ** 16, 2 ** 16, O).astype(np.int32)
        gamma = (rng.random((-(-O // bo), -(-I // bi))) < 0.5).astype(np.uint8)
        print("case", n, (B, L, J, I, O, H, K, s, p, bo, bi), flush=True)
        layer = bsp.BspLayerI8(W, gamma, bo, bi, bias=bias)
        Xd = torch.from_numpy(X).cuda()
        shift = int(rng.integers(0, 14))
        Y8 = layer.conv2d(Xd, s, p, shift=shift)
        Y32 = layer.conv2d(Xd, s, p)
        torch.cuda.synchronize()
        want = oracle.conv2d_i8(X, W, bias, gamma, bo, bi, s, p)
        assert (Y32.cpu().numpy().astype(np.int64) == want).all(), n
        assert (Y8.cpu().numpy() == oracle.requant_shift(want, shift)).all(), (n, shift)


def _tiled_shapes(seed, count):
    """Shapes with whole 16-channel chunks and more pixels: these land in the LDS-resident
    kernels (bf16 and int8), with several tiles, slabs and strip groups."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        H, K = [(1, 1), (3, 3), (3, 3), (1, 7), (7, 1), (3, 1)][int(rng.integers(0, 6))]
        s = int(rng.integers(1, 3))
        p = (H // 2, K // 2) if rng.random() < 0.7 else (0, 0)
        L, J = int(rng.integers(max(8, H), 44)), int(rng.integers(max(8, K), 44))
        B = int(rng.integers(1, 4))
        I = int(rng.choice([16, 32, 64, 128, 192, 256]))
        O = int(rng.choice([16, 32, 64, 128, 192]))
        if B * L * J * I * H * K * O > 1.5e9 or I * H * K > 4608:
            continue
        bo, bi = GRANS[int(rng.integers(0, 3))]
        out.append((B, L, J, I, O, H, K, (s, s), p, bo, bi))
    return out


def test_random_tiled_shapes_bf16_and_int8():
    import torch
    rng = np.random.default_rng(6)
    for n, (B, L, J, I, O, H, K, s, p, bo, bi) in enumerate(_tiled_shapes(79, 24)):
        print("case", n, (B, L, J, I, O, H, K, s, p, bo, bi), flush=True)
        c = draw_layer("t", B=B, L=L, J=J, I=I, O=O, H=H, K=K, stride=s, pad=p, bo=bo, bi=bi,
                       dtype="bf16", mask_kind="exact", density=0.5, seed=7000 + n, b_std=0.5)
        assert_close(gpu_conv(c), oracle_conv(c), "bf16", f"tiled shape {n}")
        X = rng.integers(-128, 128, (B, L, J, I), dtype=np.int8)
        W = rng.integers(-128, 128, (O, H, K, I), dtype=np.int8)
        bias = rng.integers(-2 ** 16, 2 ** 16, O).astype(np.int32)
        layer = bsp.BspLayerI8(W, c.gamma, bo, bi, bias=bias)
        shift = int(rng.integers(4, 14))
        Y8 = layer.conv2d(torch.from_numpy(X).cuda(), s, p, shift=shift)
        torch.cuda.synchronize()
        want = oracle.conv2d_i8(X, W, bias, c.gamma, bo, bi, s, p, shift=shift)
        assert (Y8.cpu().numpy() == want).all(), (n, shift)
