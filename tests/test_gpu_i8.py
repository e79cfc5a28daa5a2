"""8-bit integer layers: HIP path vs the integer oracle, bit for bit (needs a GPU)."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp

pytestmark = pytest.mark.gpu

GRANS = [(8, 8), (4, 16), (16, 4)]

SHAPES = [
    # B, L, J, I, O, H, K, stride, pad
    (2, 7, 9, 16, 32, 3, 3, (1, 1), (1, 1)),
    (1, 9, 8, 32, 16, 3, 3, (2, 2), (1, 1)),
    (2, 6, 11, 16, 48, 1, 7, (1, 1), (0, 3)),
    (1, 12, 12, 16, 16, 5, 5, (1, 1), (2, 2)),
    (1, 15, 13, 3, 16, 7, 7, (2, 2), (3, 3)),       # fewer channels than a block: dense
    (3, 5, 4, 24, 40, 1, 1, (1, 1), (0, 0)),        # ragged for 16-wide blocks
    (1, 3, 3, 20, 12, 3, 3, (1, 1), (1, 1)),        # ragged O and I
    (5, 17, 17, 160, 192, 1, 1, (1, 1), (0, 0)),    # several tiles + ragged pixel tail
    (2, 14, 14, 72, 120, 3, 3, (1, 1), (1, 1)),
    (33, 1, 1, 520, 64, 1, 1, (1, 1), (0, 0)),      # FC
    (4, 30, 30, 64, 64, 3, 3, (1, 1), (1, 1)),      # enough work for four pixel tiles a wave
]


def _draw(shape, seed, bo, bi, extreme=False):
    B, L, J, I, O, H, K, s, p = shape
    rng = np.random.default_rng(seed)
    if extreme:
        X = rng.choice(np.array([-128, 127], dtype=np.int8), (B, L, J, I))
        W = rng.choice(np.array([-128, 127], dtype=np.int8), (O, H, K, I))
    else:
        X = rng.integers(-128, 128, (B, L, J, I), dtype=np.int8)
        W = rng.integers(-128, 128, (O, H, K, I), dtype=np.int8)
    bias = rng.integers(-2 ** 18, 2 ** 18, O).astype(np.int32)
    nbr, nbc = -(-O // bo), -(-I // bi)
    gamma = (rng.random((nbr, nbc)) < 0.5).astype(np.uint8)
    if I < bi:
        gamma[:] = 1
    return X, W, bias, gamma, s, p


@pytest.mark.parametrize("bo,bi", GRANS)
def test_int32_sums_bit_exact(bo, bi):
    import torch
    for n, shape in enumerate(SHAPES):
        X, W, bias, gamma, s, p = _draw(shape, 100 + n, bo, bi, extreme=(n % 3 == 0))
        print("case", n, shape, bo, bi, flush=True)
        layer = bsp.BspLayerI8(W, gamma, bo, bi, bias=bias)
        Y = layer.conv2d(torch.from_numpy(X).cuda(), s, p)
        torch.cuda.synchronize()
        want = oracle.conv2d_i8(X, W, bias, gamma, bo, bi, s, p)
        assert Y.dtype == torch.int32
        assert (Y.cpu().numpy().astype(np.int64) == want).all(), (shape, bo, bi)


@pytest.mark.parametrize("shift", [0, 1, 7, 12, 31])
def test_shifted_int8_output_bit_exact(shift):
    import torch
    for n, shape in enumerate(SHAPES[:8]):
        X, W, bias, gamma, s, p = _draw(shape, 200 + n, 8, 8)
        layer = bsp.BspLayerI8(W, gamma, 8, 8, bias=bias)
        Y = layer.conv2d(torch.from_numpy(X).cuda(), s, p, shift=shift)
        torch.cuda.synchronize()
        want = oracle.conv2d_i8(X, W, bias, gamma, 8, 8, s, p, shift=shift)
        assert Y.dtype == torch.int8 and (Y.cpu().numpy() == want).all(), (shape, shift)


LDS_SHAPES = [
    # channel counts in whole 16-code chunks: these take the LDS-resident int8 kernel
    (2, 20, 20, 64, 64, 3, 3, (1, 1), (1, 1)),       # one slab
    (1, 14, 14, 192, 128, 3, 3, (1, 1), (1, 1)),     # two slabs, two strip groups
    (3, 13, 13, 128, 96, 1, 1, (1, 1), (0, 0)),      # pointwise, ragged strip group
    (2, 15, 15, 144, 32, 3, 3, (2, 2), (1, 1)),      # two slabs, strided
    (1, 9, 9, 512, 48, 1, 1, (2, 2), (0, 0)),        # strided pointwise
    (1, 20, 33, 64, 64, 3, 3, (1, 1), (1, 1)),       # tiles hang over both image edges
    (2, 6, 11, 16, 48, 1, 7, (1, 1), (0, 3)),
    (2, 11, 6, 48, 16, 7, 1, (1, 1), (3, 0)),
    (2, 40, 40, 32, 16, 3, 3, (1, 1), (1, 1)),       # several tiles per workgroup
]


@pytest.mark.parametrize("bo,bi", GRANS)
def test_lds_int8_kernel_bit_exact(bo, bi):
    import torch
    for n, shape in enumerate(LDS_SHAPES):
        X, W, bias, gamma, s, p = _draw(shape, 300 + n, bo, bi, extreme=(n % 4 == 0))
        print("case", n, shape, bo, bi, flush=True)
        layer = bsp.BspLayerI8(W, gamma, bo, bi, bias=bias)
        Xd = torch.from_numpy(X).cuda()
        for shift in (0, 6, 11):
            Y = layer.conv2d(Xd, s, p, shift=shift)
            torch.cuda.synchronize()
            want = oracle.conv2d_i8(X, W, bias, gamma, bo, bi, s, p, shift=shift)
            assert (Y.cpu().numpy() == want).all(), (shape, bo, bi, shift)
        # the int32 sums (general kernel) shifted on the host give the same bytes
        Y32 = layer.conv2d(Xd, s, p).cpu().numpy().astype(np.int64)
        assert (oracle.requant_shift(Y32, 6) == oracle.conv2d_i8(X, W, bias, gamma, bo, bi, s, p, shift=6)).all()


def test_int8_config1_full_size():
    import torch
    from synthetic import config_cases
    c = next(config_cases(1))
    Wq, _ = bsp.bsp_quantize(c.W)
    Xq = np.clip(np.rint(c.X * 32.0), -128, 127).astype(np.int8)
    bias = np.arange(c.O, dtype=np.int32) * 37 - 1000
    layer = bsp.BspLayerI8(Wq, c.gamma, c.bo, c.bi, bias=bias)
    Y = layer.conv2d(torch.from_numpy(Xq).cuda(), c.stride, c.pad, shift=9)
    torch.cuda.synchronize()
    want = oracle.conv2d_i8(Xq, Wq, bias, c.gamma, c.bo, c.bi, c.stride, c.pad, shift=9)
    assert (Y.cpu().numpy() == want).all()
    assert np.abs(want).max() > 20 and (want == 127).sum() < want.size // 100   # a live, unsaturated layer


def test_rounding_ties_and_saturation_on_gpu():
    """One kept block of ones against chosen inputs puts exact ties and both saturation ends
    into the sums."""
    import torch
    W = np.ones((8, 1, 1, 8), dtype=np.int8)
    gamma = np.ones((1, 1), dtype=np.uint8)
    sums = np.array([8, -8, 24, -24, 7, -9, 2040, 2047, -2056, -2064, 100000, -100000], dtype=np.int64)
    X = np.zeros((len(sums), 1, 1, 8), dtype=np.int8)
    bias = np.zeros(8, dtype=np.int32)
    # sum = x0 + bias; use the bias for the large magnitudes
    for i, v in enumerate(sums):
        X[i, 0, 0, 0] = np.clip(v, -128, 127)
    layer = bsp.BspLayerI8(W, gamma, 8, 8, bias=bias)
    Y32 = layer.conv2d(torch.from_numpy(X).cuda())
    torch.cuda.synchronize()
    got32 = Y32.cpu().numpy().astype(np.int64)[:, 0, 0, 0]
    assert (got32 == np.clip(sums, -128, 127)).all()
    # the large sums through the bias path, one layer per value
    for v in sums:
        layer = bsp.BspLayerI8(W, gamma, 8, 8, bias=np.full(8, v, dtype=np.int32))
        Y = layer.fc(torch.zeros((1, 8), dtype=torch.int8, device="cuda"), shift=4)
        torch.cuda.synchronize()
        want = max(-128, min(127, (int(v) + 8) // 16))
        assert int(Y[0, 0]) == want, (v, int(Y[0, 0]), want)


def test_quantized_layer_end_to_end_tracks_the_float_layer():
    """Eq. (8) codes through the integer layer, rescaled by Delta, stay within the
    quantization error bound of the masked float layer (a sanity check of scales, not a
    parity bar: I * Delta / 2 * max|x| per output)."""
    import torch
    rng = np.random.default_rng(77)
    B, L, J, I, O = 2, 9, 9, 64, 32
    W = (rng.standard_normal((O, 3, 3, I)) * 0.05).astype(np.float32)
    gamma = (rng.random((O // 8, I // 8)) < 0.5).astype(np.uint8)
    Xq = rng.integers(-128, 128, (B, L, J, I), dtype=np.int8)
    Wq, delta = bsp.bsp_quantize(W)
    layer = bsp.BspLayerI8(Wq, gamma, 8, 8)
    acc = layer.conv2d(torch.from_numpy(Xq).cuda(), (1, 1), (1, 1)).cpu().numpy().astype(np.float64)
    ref = oracle.conv2d(Xq.astype(np.float32), W, None, gamma, 8, 8, (1, 1), (1, 1))
    bound = 9 * I * (delta / 2) * 128 + delta * 128      # all taps kept, plus the clamped maximum
    assert np.abs(acc * delta - ref).max() <= bound


def test_i8_error_codes():
    import torch
    X, W, bias, gamma, s, p = _draw(SHAPES[0], 1, 8, 8)
    layer = bsp.BspLayerI8(W, gamma, 8, 8, bias=bias)
    Xd = torch.from_numpy(X).cuda()
    with pytest.raises(bsp.BspError) as e:
        layer.conv2d(Xd, s, p, shift=32)
    assert e.value.code == -2
    fl = bsp.BspLayer(W.astype(np.float32), gamma, 8, 8, "bf16")
    Y = torch.empty(layer.out_shape(2, 7, 9, s, p), dtype=torch.int32, device="cuda")
    with pytest.raises(bsp.BspError) as e:       # float weights through the integer entry point
        bsp.bsp_conv2d_i8(fl.struct, Xd.data_ptr(), None, Y.data_ptr(), bsp.BSP_I32, 0, 2, 7, 9, s, p, 0)
    assert e.value.code == -5
    with pytest.raises(bsp.BspError) as e:       # integer weights through the float entry point
        bsp.bsp_conv2d(layer.struct, Xd.data_ptr(), None, Y.data_ptr(), 2, 7, 9, s, p, 0)
    assert e.value.code == -5
