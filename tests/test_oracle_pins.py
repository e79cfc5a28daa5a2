"""Pins for the CPU oracle: it is checked against things other than itself.

  * the index example printed with Eq. (1)              (tests/golden)
  * the closed form of Eq. (3)-(4)                      (tests/golden)
  * a library dense convolution / matmul for Gamma = 1  (torch, numpy)
  * a scatter-form brute force on tiny shapes
  * invariants: empty mask -> bias only; linear over blocks; zeroed blocks'
    contents are irrelevant; one mask at three granularities; 1x1 == FC
  * planted mistakes (flip, transpose, wrong padding, ...) in a copy of the
    definition must each trip at least one pin
"""
import os

import numpy as np
import pytest
import torch

import oracle
from synthetic import draw_layer

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [[int(t) for t in ln.split()] for ln in f
                if ln.strip() and not ln.startswith("#")]


def oracle_conv(X, W, bias, gamma, bo, bi, stride, pad):
    return oracle.conv2d(X, W, bias, gamma, bo, bi, stride, pad)


# --------------------------------------------------------------- Eq. (1) example
def test_eq1_worked_example_indices():
    (bo, bi, l, c, o0, o1, i0, i1), = _rows("eq1_worked_example.txt")
    O, I, H, K = 16, 64, 3, 2
    W = np.ones((O, H, K, I), dtype=np.float32)
    gamma = np.ones((O // bo, I // bi), dtype=np.uint8)
    gamma[l, c] = 0
    Wm = oracle.apply_mask(W, gamma, bo, bi)
    zero = (Wm == 0)
    expect = np.zeros((O, H, K, I), dtype=bool)
    expect[o0:o1 + 1, :, :, i0:i1 + 1] = True
    assert (zero == expect).all()
    keep = oracle.expand_mask(gamma, O, I, bo, bi)
    assert (~keep).sum() == (o1 - o0 + 1) * (i1 - i0 + 1) == bo * bi


# ------------------------------------------------------------ Eq. (3)-(4) example
@pytest.mark.parametrize("b", [4, 8])
def test_eq4_closed_form(b):
    rng = np.random.default_rng(4)
    A = [rng.standard_normal((b, b)) for _ in range(4)]
    Bm = [None, rng.standard_normal((b, b)), rng.standard_normal((b, b)), None]
    # dense right operand with junk in the two blocks the mask removes
    junk = [rng.standard_normal((b, b)) * 1e3 for _ in range(2)]
    Bfull = np.block([[junk[0], Bm[1]], [Bm[2], junk[1]]])
    X = np.block([[A[0], A[1]], [A[2], A[3]]])
    Wbar = Bfull.T.copy()                     # Y = X . Wbar^T  <=>  C = A . B
    gamma_B = np.array([[0, 1], [1, 0]], dtype=np.uint8)
    gamma_W = gamma_B.T.copy()                # anti-diagonal either way
    if b == 8:
        Y = oracle.fc(X, Wbar, None, gamma_W, 8, 8)
    else:
        # 4x16 / 16x4 do not tile a 2x2 arrangement of 4x4 blocks: use the
        # general masked layer through an explicit select instead
        keep = np.kron(gamma_W, np.ones((b, b))) != 0
        Y = oracle.fc(X, np.where(keep, Wbar, 0.0), None,
                      np.ones((1, 1), dtype=np.uint8), 8, 8)
    C = [Y[:b, :b], Y[:b, b:], Y[b:, :b], Y[b:, b:]]
    for ci, ai, bj in _rows("eq4_block_product.txt"):
        np.testing.assert_allclose(C[ci], A[ai] @ Bm[bj], rtol=1e-12, atol=1e-12)


# ----------------------------------------------- pins usable on any `conv` callable
CONV_SHAPES = [
    # B, L, J, I, O, H, K, stride, pad
    (2, 7, 9, 16, 24, 3, 3, (1, 1), (1, 1)),
    (1, 9, 8, 8, 16, 3, 3, (2, 2), (1, 1)),
    (2, 6, 11, 16, 8, 1, 7, (1, 1), (0, 3)),
    (2, 11, 6, 16, 8, 7, 1, (1, 1), (3, 0)),
    (1, 12, 12, 8, 8, 5, 5, (1, 1), (2, 2)),
    (1, 15, 13, 3, 16, 7, 7, (2, 2), (3, 3)),
    (3, 5, 4, 24, 40, 1, 1, (1, 1), (0, 0)),
    (1, 8, 10, 16, 16, 3, 3, (2, 1), (0, 2)),
    (1, 9, 9, 16, 16, 1, 1, (2, 2), (0, 0)),
]


def _draw(shape, seed, bo=8, bi=8, kind="bernoulli", d=0.5):
    B, L, J, I, O, H, K, s, p = shape
    return draw_layer("t", B=B, L=L, J=J, I=I, O=O, H=H, K=K, stride=s, pad=p,
                      bo=bo, bi=bi, dtype="f32", mask_kind=kind, density=d,
                      seed=seed, w_std=0.3, b_std=0.5)


def check_library_dense(conv):
    """Gamma = 1 equals torch's dense conv2d in fp64 (cross-correlation, zero
    padding, floor output size)."""
    for n, shape in enumerate(CONV_SHAPES):
        c = _draw(shape, 100 + n, kind="ones")
        Y = conv(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad)
        Xt = torch.from_numpy(c.X.astype(np.float64)).permute(0, 3, 1, 2)
        Wt = torch.from_numpy(c.W.astype(np.float64)).permute(0, 3, 1, 2)
        ref = torch.nn.functional.conv2d(
            Xt, Wt, torch.from_numpy(c.bias.astype(np.float64)),
            stride=c.stride, padding=c.pad).permute(0, 2, 3, 1).numpy()
        assert Y.shape == ref.shape, shape
        np.testing.assert_allclose(Y, ref, rtol=1e-11, atol=1e-11, err_msg=str(shape))


def scatter_brute_force(X, W, bias, gamma, bo, bi, stride, pad):
    """Every (input pixel, tap, kept weight) pushes its product to the one
    output it feeds: the same sum as the definition, organised the other way
    round, in pure Python."""
    B, L, J, I = X.shape
    O, H, K, _ = W.shape
    M = (L + 2 * pad[0] - H) // stride[0] + 1
    N = (J + 2 * pad[1] - K) // stride[1] + 1
    Y = np.zeros((B, M, N, O))
    Y += np.asarray(bias, dtype=np.float64)
    for o in range(O):
        for i in range(I):
            if not gamma[o // bo][i // bi]:
                continue
            for h in range(H):
                for k in range(K):
                    w = float(W[o, h, k, i])
                    for y in range(L):
                        t = y + pad[0] - h
                        if t < 0 or t % stride[0] or t // stride[0] >= M:
                            continue
                        for x in range(J):
                            u = x + pad[1] - k
                            if u < 0 or u % stride[1] or u // stride[1] >= N:
                                continue
                            Y[:, t // stride[0], u // stride[1], o] += \
                                w * X[:, y, x, i].astype(np.float64)
    return Y


TINY = [
    ((1, 5, 5, 16, 16, 3, 3, (1, 1), (1, 1)), 8, 8),
    ((1, 5, 6, 16, 16, 3, 3, (2, 2), (1, 1)), 4, 16),
    ((1, 6, 5, 16, 16, 1, 7, (1, 1), (0, 3)), 16, 4),
    ((1, 5, 5, 16, 16, 5, 5, (1, 2), (2, 0)), 8, 8),
    ((2, 4, 4, 12, 20, 1, 1, (1, 1), (0, 0)), 8, 8),      # ragged O and I
    ((1, 7, 7, 16, 16, 7, 7, (2, 2), (3, 3)), 16, 4),
]


def check_brute_force(conv):
    for n, (shape, bo, bi) in enumerate(TINY):
        c = _draw(shape, 200 + n, bo=bo, bi=bi)
        Y = conv(c.X, c.W, c.bias, c.gamma, bo, bi, c.stride, c.pad)
        ref = scatter_brute_force(c.X, c.W, c.bias, c.gamma, bo, bi, c.stride, c.pad)
        np.testing.assert_allclose(Y, ref, rtol=1e-11, atol=1e-11, err_msg=str(shape))


def check_zero_mask(conv):
    c = _draw(CONV_SHAPES[0], 300, kind="zeros")
    Y = conv(c.X, c.W, c.bias, c.gamma, c.bo, c.bi, c.stride, c.pad)
    assert (Y == c.bias.astype(np.float64)).all()


def check_linearity(conv):
    """Y(Gamma) - b = sum over kept blocks n of (Y(e_n) - b)."""
    c = _draw((1, 6, 6, 24, 16, 3, 3, (1, 1), (1, 1)), 301)
    b64 = c.bias.astype(np.float64)
    Y = conv(c.X, c.W, c.bias, c.gamma, 8, 8, c.stride, c.pad)
    total = np.zeros_like(Y)
    for l, col in zip(*np.nonzero(c.gamma)):
        e = np.zeros_like(c.gamma)
        e[l, col] = 1
        total += conv(c.X, c.W, c.bias, e, 8, 8, c.stride, c.pad) - b64
    np.testing.assert_allclose(Y - b64, total, rtol=1e-10, atol=1e-10)


def check_masked_content_ignored(conv):
    c = _draw(CONV_SHAPES[1], 302)
    Y = conv(c.X, c.W, c.bias, c.gamma, 8, 8, c.stride, c.pad)
    keep = oracle.expand_mask(c.gamma, c.O, c.I, 8, 8)[:, None, None, :]
    W2 = np.where(keep, c.W, np.float32(1e30))
    Y2 = conv(c.X, W2, c.bias, c.gamma, 8, 8, c.stride, c.pad)
    assert (Y == Y2).all()


ALL_CHECKS = [check_library_dense, check_brute_force, check_zero_mask,
              check_linearity, check_masked_content_ignored]


@pytest.mark.parametrize("check", ALL_CHECKS, ids=lambda f: f.__name__)
def test_oracle_pin(check):
    check(oracle_conv)


# -------------------------------------------------- the pins do catch mistakes
def _definition_copy(bug):
    """The definition again in numpy, with one planted mistake."""
    def conv(X, W, bias, gamma, bo, bi, stride, pad):
        X = X.astype(np.float64)
        W = W.astype(np.float64)
        B, L, J, I = X.shape
        O, H, K, _ = W.shape
        g = np.asarray(gamma)
        if bug == "mask_transposed_granularity":
            bo_, bi_ = bi, bo
            nbr, nbc = -(-O // bo_), -(-I // bi_)
            gg = np.resize(g, (nbr, nbc))
            keep = gg[np.ix_(np.arange(O) // bo_, np.arange(I) // bi_)] != 0
        elif bug == "mask_inverted":
            keep = ~oracle.expand_mask(g, O, I, bo, bi)
        else:
            keep = oracle.expand_mask(g, O, I, bo, bi)
        Wm = np.where(keep[:, None, None, :], W, 0.0)
        if bug == "flip":
            Wm = Wm[:, ::-1, ::-1, :]
        if bug == "swap_hk" and H == K:
            Wm = Wm.transpose(0, 2, 1, 3)
        ph, pw = pad
        if bug == "pad_swapped":
            ph, pw = pw, ph
        sh, sw = stride
        if bug == "stride_swapped":
            sh, sw = sw, sh
        M = (L + 2 * pad[0] - H) // stride[0] + 1
        N = (J + 2 * pad[1] - K) // stride[1] + 1
        Xp = np.zeros((B, L + 2 * ph + 8, J + 2 * pw + 8, I))
        Xp[:, ph:ph + L, pw:pw + J, :] = X
        Y = np.zeros((B, M, N, O))
        for h in range(H):
            for k in range(K):
                sl = Xp[:, h:h + sh * M:sh, k:k + sw * N:sw, :][:, :M, :N, :]
                Y += np.einsum("bmni,oi->bmno", sl, Wm[:, h, k, :])
        if bug != "no_bias":
            Y += np.asarray(bias, dtype=np.float64)
        if bug == "dropped_tap" and H * K > 1:
            Y -= np.einsum("bmni,oi->bmno",
                           Xp[:, H - 1:H - 1 + sh * M:sh, K - 1:K - 1 + sw * N:sw, :][:, :M, :N, :],
                           Wm[:, H - 1, K - 1, :])
        return Y
    return conv


def test_unplanted_copy_passes_all_pins():
    for check in ALL_CHECKS:
        check(_definition_copy(None))


@pytest.mark.parametrize("bug", ["flip", "swap_hk", "pad_swapped", "stride_swapped",
                                 "no_bias", "dropped_tap", "mask_inverted",
                                 "mask_transposed_granularity"])
def test_planted_mistake_is_caught(bug):
    caught = 0
    for check in ALL_CHECKS:
        try:
            check(_definition_copy(bug))
        except (AssertionError, ValueError):
            caught += 1
    assert caught >= 1, bug


# ------------------------------------------------------------ further invariants
def test_fc_ones_mask_is_matmul():
    rng = np.random.default_rng(7)
    X = rng.standard_normal((5, 40)).astype(np.float32)
    Wb = rng.standard_normal((24, 40)).astype(np.float32)
    b = rng.standard_normal(24).astype(np.float32)
    Y = oracle.fc(X, Wb, b, np.ones((3, 5), dtype=np.uint8), 8, 8)
    ref = X.astype(np.float64) @ Wb.astype(np.float64).T + b.astype(np.float64)
    np.testing.assert_allclose(Y, ref, rtol=1e-12, atol=1e-12)


def test_conv1x1_equals_fc_on_flattened_pixels():
    c = _draw((2, 5, 7, 32, 16, 1, 1, (1, 1), (0, 0)), 11)
    Yc = oracle.conv2d(c.X, c.W, c.bias, c.gamma, 8, 8)
    Yf = oracle.fc(c.X.reshape(-1, c.I), c.W.reshape(c.O, c.I), c.bias, c.gamma, 8, 8)
    assert (Yc.reshape(-1, c.O) == Yf).all()


def test_one_mask_three_granularities():
    """A mask constant on 16x16 super-blocks can be written at 8x8, 4x16 and
    16x4; the layer output must not depend on which."""
    rng = np.random.default_rng(12)
    c = _draw((1, 6, 6, 64, 48, 3, 3, (1, 1), (1, 1)), 13, kind="ones")
    sup = (rng.random((c.O // 16, c.I // 16)) < 0.5).astype(np.uint8)
    outs = []
    for bo, bi in ((8, 8), (4, 16), (16, 4)):
        g = np.kron(sup, np.ones((16 // bo, 16 // bi), dtype=np.uint8))
        outs.append(oracle.conv2d(c.X, c.W, c.bias, g, bo, bi, c.stride, c.pad))
    assert (outs[0] == outs[1]).all() and (outs[0] == outs[2]).all()


def test_conv2d_at_matches_full():
    c = _draw(CONV_SHAPES[7], 14)
    Y = oracle.conv2d(c.X, c.W, c.bias, c.gamma, 8, 8, c.stride, c.pad)
    rng = np.random.default_rng(1)
    pos = np.stack([rng.integers(0, s, 50) for s in Y.shape], axis=1)
    got = oracle.conv2d_at(c.X, c.W, c.bias, c.gamma, 8, 8, pos, c.stride, c.pad)
    assert (got == Y[tuple(pos.T)]).all()


def test_flop_count_follows_blocks():
    # exactly half the blocks -> exactly half the dense count (Section I, item 3)
    c = _draw((2, 6, 6, 64, 64, 3, 3, (1, 1), (1, 1)), 15, kind="exact", d=0.5)
    dense = 2 * c.P * c.O * c.I * c.H * c.K
    assert oracle.flops_nonzero(c.P, c.nnzb, 8, 8, 3, 3) * 2 == dense
    # and it equals 2 x (number of kept scalar weights) x pixels
    kept = oracle.expand_mask(c.gamma, c.O, c.I, 8, 8).sum() * c.H * c.K
    assert oracle.flops_nonzero(c.P, c.nnzb, 8, 8, 3, 3) == 2 * c.P * kept


def test_eq2_row_sparsity_and_row_ptr():
    c = _draw((1, 1, 1, 128, 64, 1, 1, (1, 1), (0, 0)), 16, kind="row_balanced", d=0.25)
    S = oracle.row_sparsity(c.gamma)
    assert np.allclose(S, 0.75)
    row_ptr, col_idx, payload = oracle.pack_reference(c.W, c.gamma, 8, 8)
    nbc = c.gamma.shape[1]
    assert (np.diff(row_ptr) == np.round(nbc * (1 - S))).all()
    c2 = _draw((1, 1, 1, 128, 64, 1, 1, (1, 1), (0, 0)), 17)
    S2 = oracle.row_sparsity(c2.gamma)
    rp2, ci2, _ = oracle.pack_reference(c2.W, c2.gamma, 8, 8)
    assert (np.diff(rp2) == nbc - np.round(S2 * nbc)).all()
    for l in range(len(rp2) - 1):
        cols = ci2[rp2[l]:rp2[l + 1]]
        assert (np.diff(cols) > 0).all()
        assert (np.flatnonzero(c2.gamma[l]) == cols).all()


@pytest.mark.parametrize("bo,bi", [(8, 8), (4, 16), (16, 4)])
@pytest.mark.parametrize("O,I", [(32, 48), (20, 12), (1000 // 8, 3)])
def test_pack_reference_roundtrip(bo, bi, O, I):
    c = draw_layer("t", B=1, L=3, J=3, I=I, O=O, H=3, K=2, bo=bo, bi=bi, dtype="f32",
                   mask_kind="bernoulli", density=0.6, seed=18)
    for pd in ("f32", "bf16"):
        rp, ci, pl = oracle.pack_reference(c.W, c.gamma, bo, bi, pd)
        assert pl.shape == (c.nnzb, bo, 3, 2, bi)
        Wd = oracle.unpack_reference(rp, ci, pl, O, 3, 2, I, bo, bi)
        Wm = oracle.apply_mask(c.W, c.gamma, bo, bi)
        if pd == "bf16":
            Wm = oracle.round_to_storage(Wm.astype(np.float64), "bf16")
        assert (Wd.view(np.uint32) == Wm.view(np.uint32)).all()


def test_bf16_rounding_bit_patterns():
    # hand-worked cases: exact, below half, tie to even (down), tie to even (up), above half
    f = np.array([0x3F800000, 0x3F807FFF, 0x3F808000, 0x3F818000, 0x3F808001,
                  0xBF808000, 0xBF818000, 0x00000000, 0x80000000],
                 dtype=np.uint32).view(np.float32)
    want = np.array([0x3F80, 0x3F80, 0x3F80, 0x3F82, 0x3F81,
                     0xBF80, 0xBF82, 0x0000, 0x8000], dtype=np.uint16)
    assert (oracle.bf16_bits_rne(f) == want).all()


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(19)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (oracle.bf16_bits_rne(x) == lib).all()


def test_fused_epilogue_against_library_ops():
    """conv -> store in bf16 -> + residual -> relu, each step by torch (fp64 conv, bf16 cast)."""
    import torch
    rng = np.random.default_rng(21)
    B, L, J, I, O = 2, 6, 7, 16, 24
    X = oracle.round_to_storage(rng.standard_normal((B, L, J, I)), "bf16")
    W = oracle.round_to_storage(rng.standard_normal((O, 3, 3, I)) * 0.1, "bf16")
    bias = rng.standard_normal(O).astype(np.float32)
    gamma = (rng.random((O // 8, I // 8)) < 0.6).astype(np.uint8)
    R = oracle.round_to_storage(rng.standard_normal((B, L, J, O)), "bf16")
    Wm = oracle.apply_mask(W, gamma, 8, 8)
    y = torch.nn.functional.conv2d(torch.from_numpy(X.astype(np.float64)).permute(0, 3, 1, 2),
                                   torch.from_numpy(Wm.astype(np.float64)).permute(0, 3, 1, 2),
                                   torch.from_numpy(bias.astype(np.float64)), padding=1)
    y = y.permute(0, 2, 3, 1).to(torch.float32).to(torch.bfloat16).to(torch.float64)
    want = torch.relu(y + torch.from_numpy(R.astype(np.float64))).numpy()
    got = oracle.conv2d_fused(X, W, bias, gamma, 8, 8, (1, 1), (1, 1), residual=R, relu=True)
    # the fp32 hop of the torch cast can move a value sitting on a bf16 tie: allow one bf16 ulp there
    assert np.abs(got - want).max() <= 2.0 ** -7 * np.abs(want).max()
    assert (np.abs(got - want) > 0).mean() < 0.01
    plain = oracle.conv2d_fused(X, W, bias, gamma, 8, 8, (1, 1), (1, 1))
    assert (plain == oracle.conv2d(X, W, bias, gamma, 8, 8, (1, 1), (1, 1))).all()
    only_relu = oracle.conv2d_fused(X, W, bias, gamma, 8, 8, (1, 1), (1, 1), relu=True)
    assert (only_relu >= 0).all() and (only_relu[plain > 0.01] > 0).all()


def _chain_case(rng, B, L, J, I, C, O, density=0.6):
    def layer(o, h, i, std):
        W = oracle.round_to_storage(rng.standard_normal((o, h, h, i)) * std, "bf16")
        b = rng.standard_normal(o).astype(np.float32) * 0.5
        g = (rng.random((o // 8, i // 8)) < density).astype(np.uint8)
        return W, b, g
    X = oracle.round_to_storage(rng.standard_normal((B, L, J, I)), "bf16")
    return X, [layer(C, 1, I, 0.2), layer(C, 3, C, 0.1), layer(O, 1, C, 0.2)]


def test_bottleneck_chain_against_library_ops():
    """1x1 -> relu -> 3x3 -> relu -> 1x1 -> + residual -> relu, every layer by torch's fp64
    convolution and every hand-over by torch's bf16 cast."""
    import torch
    rng = np.random.default_rng(33)
    B, L, J, I, C, O = 2, 7, 9, 32, 16, 32
    X, layers = _chain_case(rng, B, L, J, I, C, O)
    R = oracle.round_to_storage(rng.standard_normal((B, L, J, O)), "bf16")

    def tconv(x, W, b, g, pad):
        Wm = oracle.apply_mask(W, g, 8, 8)
        y = torch.nn.functional.conv2d(x.permute(0, 3, 1, 2),
                                       torch.from_numpy(Wm.astype(np.float64)).permute(0, 3, 1, 2),
                                       torch.from_numpy(b.astype(np.float64)), padding=pad)
        return y.permute(0, 2, 3, 1).to(torch.float32).to(torch.bfloat16).to(torch.float64)

    t = torch.from_numpy(X.astype(np.float64))
    t = torch.relu(tconv(t, *layers[0], 0))
    t = torch.relu(tconv(t, *layers[1], 1))
    want = torch.relu(tconv(t, *layers[2], 0) + torch.from_numpy(R.astype(np.float64))).numpy()
    got = oracle.bottleneck(X, layers, 8, 8, residual=R)
    # a bf16 tie moved by the cast's fp32 hop in an early layer can move a later value by a
    # few ulp: nearly all values agree exactly, the rest within a loose bound
    assert (np.abs(got - want) > 0).mean() < 0.02
    assert np.abs(got - want).max() <= 2.0 ** -5 * max(1.0, np.abs(want).max())


def test_bottleneck_chain_identity_weights_by_hand():
    """Identity 1x1 layers and a 3x3 whose only tap is the centre (identity) make the chain
    relu(relu(x) + r); a 3x3 whose only tap is (0, 0) shifts the image by one pixel down and
    right, with zeros entering at the top and left edge (padding 1)."""
    rng = np.random.default_rng(34)
    B, L, J, C = 1, 5, 6, 8
    X = oracle.round_to_storage(rng.standard_normal((B, L, J, C)), "bf16")
    R = oracle.round_to_storage(rng.standard_normal((B, L, J, C)), "bf16")
    eye = np.eye(C, dtype=np.float32).reshape(C, 1, 1, C)
    zero = np.zeros(C, dtype=np.float32)
    ones = np.ones((1, 1), dtype=np.uint8)
    centre = np.zeros((C, 3, 3, C), dtype=np.float32)
    centre[:, 1, 1, :] = np.eye(C)
    got = oracle.bottleneck(X, [(eye, zero, ones), (centre, zero, ones), (eye, zero, ones)], 8, 8, residual=R)
    assert (got == np.maximum(np.maximum(X, 0) + R, 0)).all()
    corner = np.zeros((C, 3, 3, C), dtype=np.float32)
    corner[:, 0, 0, :] = np.eye(C)
    got = oracle.bottleneck(X, [(eye, zero, ones), (corner, zero, ones), (eye, zero, ones)], 8, 8)
    want = np.zeros_like(X, dtype=np.float64)
    want[:, 1:, 1:, :] = np.maximum(X, 0)[:, :-1, :-1, :]
    assert (got == want).all()
    # a zero mask on the middle layer leaves only biases: relu(b3 + W3 relu(b2))
    b2 = np.arange(C, dtype=np.float32) - 3
    b3 = np.full(C, 0.25, dtype=np.float32)
    got = oracle.bottleneck(X, [(eye, zero, ones), (centre, b2, np.zeros((1, 1), np.uint8)), (eye, b3, ones)], 8, 8)
    assert (got == np.broadcast_to(np.maximum(np.maximum(b2, 0) + b3, 0).astype(np.float64), got.shape)).all()
