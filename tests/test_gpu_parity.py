"""HIP path vs CPU oracle, element by element, through the C ABI (needs a GPU)."""
import numpy as np
import pytest

import oracle
from synthetic import config_cases, draw_layer

from gpu_util import assert_close, gpu_conv, make_layer, oracle_conv, to_device, to_host

pytestmark = pytest.mark.gpu

GRANS = [(8, 8), (4, 16), (16, 4)]

SHAPES = [
    # B, L, J, I, O, H, K, stride, pad
    (2, 7, 9, 16, 32, 3, 3, (1, 1), (1, 1)),
    (1, 9, 8, 32, 16, 3, 3, (2, 2), (1, 1)),
    (2, 6, 11, 16, 48, 1, 7, (1, 1), (0, 3)),
    (2, 11, 6, 48, 16, 7, 1, (1, 1), (3, 0)),
    (1, 12, 12, 16, 16, 5, 5, (1, 1), (2, 2)),
    (1, 15, 13, 3, 16, 7, 7, (2, 2), (3, 3)),       # fewer channels than a block: dense
    (3, 5, 4, 24, 40, 1, 1, (1, 1), (0, 0)),        # ragged for 16-wide blocks
    (1, 8, 10, 16, 16, 3, 3, (2, 1), (0, 2)),
    (1, 9, 9, 64, 80, 1, 1, (2, 2), (0, 0)),
    (5, 17, 17, 160, 192, 1, 1, (1, 1), (0, 0)),    # several tiles + ragged pixel tail
    (2, 14, 14, 72, 1000 // 8 * 8, 3, 3, (1, 1), (1, 1)),
    (1, 3, 3, 20, 12, 3, 3, (1, 1), (1, 1)),        # ragged O and I
    (2, 14, 14, 272, 48, 3, 3, (1, 1), (1, 1)),     # three channel slabs
    (1, 28, 28, 320, 64, 1, 1, (1, 1), (0, 0)),     # two slabs, pointwise
    (2, 15, 15, 136, 32, 3, 3, (2, 2), (1, 1)),     # two slabs, strided
    (1, 9, 9, 512, 32, 1, 1, (2, 2), (0, 0)),       # strided pointwise, two slabs
    (1, 20, 33, 64, 64, 3, 3, (1, 1), (1, 1)),      # tiles hang over both image edges
    (1, 8, 8, 16, 16, 1, 1, (1, 1), (1, 1)),        # padded pointwise
    (16, 1, 1, 1024, 200, 1, 1, (1, 1), (0, 0)),    # FC, one batch tile, ragged strip count
    (33, 1, 1, 520, 64, 1, 1, (1, 1), (0, 0)),      # FC, batch over three tiles
    (2, 5, 5, 256, 48, 1, 1, (1, 1), (0, 0)),       # 50 pixels: weight-streaming path
    (64, 1, 1, 4096, 32, 1, 1, (1, 1), (0, 0)),     # FC, long strips split over waves
]


def _draw(shape, seed, bo, bi, dtype, kind="bernoulli", d=0.5):
    B, L, J, I, O, H, K, s, p = shape
    return draw_layer("t", B=B, L=L, J=J, I=I, O=O, H=H, K=K, stride=s, pad=p, bo=bo, bi=bi,
                      dtype=dtype, mask_kind=kind, density=d, seed=seed, b_std=0.5)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("bo,bi", GRANS)
@pytest.mark.parametrize("general", [True, False], ids=["general", "dispatch"])
def test_shapes(dtype, bo, bi, general):
    for n, shape in enumerate(SHAPES):
        c = _draw(shape, 1000 + n, bo, bi, dtype)
        print("case", n, shape, dtype, bo, bi, "general" if general else "dispatch", flush=True)
        y = gpu_conv(c, general=general)
        assert_close(y, oracle_conv(c), dtype, f"shape {n} {shape}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("bo,bi", GRANS)
def test_empty_mask_is_exactly_bias(dtype, bo, bi):
    c = _draw(SHAPES[0], 7, bo, bi, dtype, kind="zeros")
    y = gpu_conv(c)
    want = oracle.round_to_storage(c.bias.astype(np.float64), dtype).astype(np.float64)
    assert (y == want).all()
    y0 = gpu_conv(c, bias=False)
    assert (y0 == 0).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_zeroed_block_contents_are_never_read_into_the_result(dtype):
    c = _draw(SHAPES[4], 8, 8, 8, dtype)
    y = gpu_conv(c)
    keep = oracle.expand_mask(c.gamma, c.O, c.I, 8, 8)[:, None, None, :]
    c.W = np.where(keep, c.W, np.float32(3e38))
    y2 = gpu_conv(c)
    assert (y == y2).all()


def test_config0_fc_fp32():
    c = next(config_cases(0))
    layer = make_layer(c)
    import torch
    X = torch.from_numpy(c.X.reshape(c.B, c.I)).cuda()
    Y = layer.fc(X)
    torch.cuda.synchronize()
    ref = oracle.fc(c.X.reshape(c.B, c.I), c.W.reshape(c.O, c.I), c.bias, c.gamma, 8, 8)
    assert_close(to_host(Y), ref, "f32", "config 0")


def test_eq4_closed_form_on_gpu():
    """Eq. (3)-(4): anti-diagonal 2x2 block operand; only A1*B2 etc. survive."""
    import torch
    rng = np.random.default_rng(4)
    b = 8
    X = rng.standard_normal((2 * b, 2 * b)).astype(np.float32)
    Wb = rng.standard_normal((2 * b, 2 * b)).astype(np.float32)
    g = np.array([[0, 1], [1, 0]], dtype=np.uint8)
    import paper_2407_09453_amd as bsp
    layer = bsp.BspLayer(Wb.reshape(2 * b, 1, 1, 2 * b), g, 8, 8, "f32")
    Y = to_host(layer.fc(torch.from_numpy(X).cuda()))
    Xd, Wd = X.astype(np.float64), Wb.astype(np.float64)
    np.testing.assert_allclose(Y[:, :b], Xd[:, b:] @ Wd[:b, b:].T, rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose(Y[:, b:], Xd[:, :b] @ Wd[b:, :b].T, rtol=1e-5, atol=1e-5)


def test_conv1x1_equals_fc_on_gpu():
    import torch
    c = _draw((2, 5, 7, 64, 48, 1, 1, (1, 1), (0, 0)), 11, 8, 8, "bf16")
    layer = make_layer(c)
    X = to_device(c)
    Yc = layer.conv2d(X)
    Yf = layer.fc(X.reshape(-1, c.I))
    torch.cuda.synchronize()
    assert torch.equal(Yc.reshape(-1, c.O), Yf)


def test_one_mask_three_granularities_on_gpu():
    rng = np.random.default_rng(12)
    c = _draw((1, 6, 6, 64, 48, 3, 3, (1, 1), (1, 1)), 13, 8, 8, "bf16", kind="ones")
    sup = (rng.random((c.O // 16, c.I // 16)) < 0.5).astype(np.uint8)
    ref = None
    for bo, bi in GRANS:
        c.bo, c.bi = bo, bi
        c.gamma = np.kron(sup, np.ones((16 // bo, 16 // bi), dtype=np.uint8))
        y = gpu_conv(c)
        r = oracle_conv(c)
        assert_close(y, r, "bf16", f"{bo}x{bi}")
        if ref is None:
            ref = r
        assert (r == ref).all()


def test_config1_full_size():
    c = next(config_cases(1))
    for general in (True, False):
        y = gpu_conv(c, general=general)
        assert_close(y, oracle_conv(c), "bf16", f"config 1 general={general}")


def test_config2_granularity_sweep():
    for c in config_cases(2):
        print(c.name, flush=True)
        y = gpu_conv(c)
        assert_close(y, oracle_conv(c), "bf16", c.name)


EDGE_SHAPES = [
    (2, 20, 20, 64, 64, 3, 3, (1, 1), (1, 1)),      # LDS-resident kernel, one slab
    (1, 14, 14, 192, 128, 3, 3, (1, 1), (1, 1)),    # three slabs, two strip groups
    (3, 13, 13, 128, 96, 1, 1, (1, 1), (0, 0)),     # pointwise, ragged strip group
    (8, 1, 1, 512, 48, 1, 1, (1, 1), (0, 0)),       # weight-streaming FC
]


@pytest.mark.parametrize("kind,d", [("bernoulli", 0.1), ("bernoulli", 0.9), ("row_balanced", 0.5),
                                    ("exact", 0.25)])
def test_mask_extremes(kind, d):
    """Very sparse masks leave whole block rows and whole strips without any kept block
    (their outputs must be the bias alone); very dense ones fill every step."""
    for n, shape in enumerate(EDGE_SHAPES):
        c = _draw(shape, 2000 + n, 8, 8, "bf16", kind=kind, d=d)
        if kind == "bernoulli" and d < 0.5:
            c.gamma = c.gamma.copy()
            c.gamma.reshape(-(-c.O // 8), -1)[1::3, :] = 0      # empty block rows
            c.gamma.reshape(-(-c.O // 8), -1)[4:6, :] = 0       # one empty strip
        print("case", n, shape, kind, d, "nnzb", int(c.gamma.sum()), flush=True)
        assert_close(gpu_conv(c), oracle_conv(c), "bf16", f"{kind} {d} shape {n}")


def test_nothing_is_written_outside_y():
    """Y sits in the middle of a larger buffer filled with a sentinel; every kernel of
    the dispatcher must leave the guard zones untouched."""
    import torch
    for n, shape in enumerate(SHAPES + EDGE_SHAPES):
        c = _draw(shape, 3000 + n, 8, 8, "bf16")
        layer = make_layer(c)
        oshape = layer.out_shape(c.B, c.L, c.J, c.stride, c.pad)
        numel = int(np.prod(oshape))
        guard = 4096
        buf = torch.full((numel + 2 * guard,), -7.0, dtype=torch.bfloat16, device="cuda")
        Y = buf[guard:guard + numel].view(oshape)
        layer.conv2d(to_device(c), c.stride, c.pad, out=Y)
        torch.cuda.synchronize()
        assert bool((buf[:guard] == -7.0).all()) and bool((buf[guard + numel:] == -7.0).all()), shape
        assert_close(to_host(Y), oracle_conv(c), "bf16", f"guarded shape {n}")


def test_repeated_launches_give_identical_bits():
    import torch
    for shape in EDGE_SHAPES:
        c = _draw(shape, 4000, 8, 8, "bf16")
        layer = make_layer(c)
        X = to_device(c)
        Y1 = layer.conv2d(X, c.stride, c.pad).clone()
        Y2 = layer.conv2d(X, c.stride, c.pad)
        torch.cuda.synchronize()
        assert torch.equal(Y1, Y2)


def test_empty_batch_is_a_no_op():
    import torch
    c = _draw(EDGE_SHAPES[0], 5000, 8, 8, "bf16")
    layer = make_layer(c)
    X = torch.zeros((1, c.L, c.J, c.I), dtype=torch.bfloat16, device="cuda")[:0]
    Yb = torch.full(layer.out_shape(1, c.L, c.J, c.stride, c.pad), -7.0, dtype=torch.bfloat16,
                    device="cuda")
    Y = layer.conv2d(X, c.stride, c.pad, out=Yb[:0])
    torch.cuda.synchronize()
    assert Y.shape[0] == 0 and bool((Yb == -7.0).all())


@pytest.mark.parametrize("B,I,O,d", [(16, 512, 1024, 0.5), (33, 264, 1032, 0.3), (64, 128, 2048, 0.55),
                                     (5, 1024, 1030, 0.1), (1, 64, 1024, 0.5)])
def test_fc_block_row_streaming_kernel(B, I, O, d):
    """Sparse FC layers with many block rows take the kernel that streams the compressed
    block rows; fused epilogue included."""
    import torch
    c = draw_layer("fcrows", B=B, L=1, J=1, I=I, O=O, H=1, K=1, stride=1, pad=0, bo=8, bi=8,
                   dtype="bf16", mask_kind="exact", density=d, seed=B * 7 + O, b_std=0.5)
    c.gamma = c.gamma.copy()
    c.gamma[3, :] = 0                                   # an empty block row: bias only
    layer = make_layer(c)
    X = to_device(c).reshape(B, I)
    Y = layer.fc(X)
    torch.cuda.synchronize()
    ref = oracle.fc(c.X.reshape(B, I), c.W.reshape(O, I), c.bias, c.gamma, 8, 8)
    assert_close(to_host(Y), ref, "bf16", f"fc rows {B}x{I}->{O}")
    R = torch.randn(B, O, device="cuda").to(torch.bfloat16)
    Yf = layer.fc(X, residual=R, relu=True)
    torch.cuda.synchronize()
    assert torch.equal(Yf, torch.relu(Y.float() + R.float()).to(torch.bfloat16))
