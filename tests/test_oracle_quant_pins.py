"""Pins for the integer oracle (oracle/quant.py): each test fixes it to something it does
not compute itself — a hand-worked case of Eq. (8), Python's exact integers, numpy's int64
einsum — and the planted-mistake tests show that a plausible slip fails one of them."""
import itertools

import numpy as np
import pytest

import oracle


def test_eq8_hand_example():
    # Eq. (8) with N = 8: Delta = max|W| / 128.  W chosen so every quotient is known.
    W = np.array([0.64, -0.64, 0.005, 0.0125, -0.0125, 0.32, 0.0], dtype=np.float64)
    q, delta = oracle.quantize_eq8(W, 8)
    assert delta == pytest.approx(0.64 / 128.0, rel=0, abs=1e-18)        # 0.005
    # 0.64/0.005 = 128 -> does not fit int8, stored as 127; -128 fits
    # 0.0125/0.005 = 2.5 -> tie, to even -> 2; -2.5 -> -2; 0.32 -> 64
    assert q.tolist() == [127, -128, 1, 2, -2, 64, 0]
    assert q.dtype == np.int8


def test_eq8_error_bound_and_grid():
    rng = np.random.default_rng(5)
    W = rng.standard_normal((37, 3, 3, 29)) * 0.05
    q, delta = oracle.quantize_eq8(W)
    assert delta == np.abs(W).max() / 128.0
    err = np.abs(W - q.astype(np.float64) * delta)
    clipped = (W / delta) > 127.5
    assert (err[~clipped] <= delta / 2 * (1 + 1e-12)).all()
    assert clipped.sum() <= 1 and (err[clipped] <= delta * (1 + 1e-12)).all()
    # exact multiples of Delta map to themselves
    k = np.arange(-128, 128)
    q2, d2 = oracle.quantize_eq8(np.concatenate([k * 0.25, [32.0]]))   # max = 32 -> Delta .25
    assert d2 == 0.25 and q2[:-1].tolist() == k.tolist() and q2[-1] == 127
    # other widths use the same formula
    q4, d4 = oracle.quantize_eq8(np.array([1.0, -1.0, 0.3]), bits=4)
    assert d4 == 0.125 and q4.tolist() == [7, -8, 2]
    qz, dz = oracle.quantize_eq8(np.zeros(5))
    assert dz == 0.0 and not qz.any()


def test_requant_shift_against_python_integers():
    vals = [0, 1, -1, 7, 8, 9, -7, -8, -9, 24, -24, 2047, 2048, -2048, -2049, 2 ** 31 - 1,
            -2 ** 31, 1016, 1015, -1032, -1033, 12345, -12345]
    for shift in (0, 1, 4, 7, 15):
        want = []
        for v in vals:
            # round to nearest, ties upward == floor((v + half) / 2^shift), then saturate
            y = (v + (1 << (shift - 1))) // (1 << shift) if shift else v
            want.append(max(-128, min(127, y)))
        got = oracle.requant_shift(np.array(vals, dtype=np.int64), shift)
        assert got.tolist() == want, shift
    # ties: 8 >> 4 with rounding = 1 (0.5 rounds up), -8 -> 0 (-0.5 rounds up), -24 -> -1
    assert oracle.requant_shift(np.array([8, -8, 24, -24]), 4).tolist() == [1, 0, 2, -1]


def _brute(Xq, Wq, bias, gamma, bo, bi, stride, pad):
    B, L, J, I = Xq.shape
    O, H, K, _ = Wq.shape
    M = (L + 2 * pad[0] - H) // stride[0] + 1
    N = (J + 2 * pad[1] - K) // stride[1] + 1
    Y = np.zeros((B, M, N, O), dtype=object)
    for n, m, q, o in itertools.product(range(B), range(M), range(N), range(O)):
        s = int(bias[o]) if bias is not None else 0
        for h, k, i in itertools.product(range(H), range(K), range(I)):
            if not gamma[o // bo, i // bi]:
                continue
            y, x = m * stride[0] + h - pad[0], q * stride[1] + k - pad[1]
            if 0 <= y < L and 0 <= x < J:
                s += int(Wq[o, h, k, i]) * int(Xq[n, y, x, i])
        Y[n, m, q, o] = s
    return Y.astype(np.int64)


@pytest.mark.parametrize("H,K,stride,pad", [(1, 1, (1, 1), (0, 0)), (3, 3, (1, 1), (1, 1)),
                                            (3, 2, (2, 1), (1, 0)), (1, 5, (1, 2), (0, 2))])
def test_integer_conv_against_python_int_loop(H, K, stride, pad):
    rng = np.random.default_rng(H * 10 + K)
    B, L, J, I, O = 2, 5, 6, 16, 16
    Xq = rng.integers(-128, 128, (B, L, J, I), dtype=np.int8)
    Wq = rng.integers(-128, 128, (O, H, K, I), dtype=np.int8)
    bias = rng.integers(-2 ** 20, 2 ** 20, O).astype(np.int32)
    for bo, bi in ((8, 8), (4, 16), (16, 4)):
        gamma = (rng.random((O // bo, I // bi)) < 0.5).astype(np.uint8)
        want = _brute(Xq, Wq, bias, gamma, bo, bi, stride, pad)
        got = oracle.conv2d_i8(Xq, Wq, bias, gamma, bo, bi, stride, pad)
        assert got.dtype == np.int64 and (got == want).all()
        assert (oracle.conv2d_i8(Xq, Wq, bias, gamma, bo, bi, stride, pad, shift=9)
                == oracle.requant_shift(want, 9)).all()


def test_integer_fc_against_int64_einsum_with_extreme_codes():
    rng = np.random.default_rng(3)
    B, I, O = 7, 512, 64
    Xq = rng.choice(np.array([-128, 127], dtype=np.int8), (B, I))       # worst-case magnitudes
    Wq = rng.choice(np.array([-128, 127], dtype=np.int8), (O, I))
    gamma = np.ones((O // 8, I // 8), dtype=np.uint8)
    gamma[::2, 1::3] = 0
    Wm = Wq.astype(np.int64) * np.kron(gamma, np.ones((8, 8), dtype=np.int64))
    bias = np.full(O, -2 ** 24, dtype=np.int32)
    want = np.einsum("bi,oi->bo", Xq.astype(np.int64), Wm) + bias.astype(np.int64)
    assert (oracle.fc_i8(Xq, Wq, bias, gamma, 8, 8) == want).all()
    # all-zero mask: the bias alone
    z = oracle.fc_i8(Xq, Wq, bias, np.zeros_like(gamma), 8, 8)
    assert (z == bias.astype(np.int64)[None, :]).all()


def _quantizer_with(bug):
    """Eq. (8) again with one planted mistake (None: the definition itself)."""
    def quantize(W, bits=8):
        W = np.asarray(W, dtype=np.float64)
        top = float(np.max(np.abs(W))) if W.size else 0.0
        if top == 0.0:
            return np.zeros(W.shape, dtype=np.int8), 0.0
        levels = 2 ** bits if bug == "delta_2N" else 2 ** (bits - 1)
        delta = top / float(levels)
        r = W / delta
        if bug == "ties_away":
            q = np.sign(r) * np.floor(np.abs(r) + 0.5)
        elif bug == "truncate":
            q = np.trunc(r)
        else:
            q = np.rint(r)
        if bug == "no_clip":
            q = ((q + 128) % 256) - 128                    # what a bare narrowing cast does
        elif bug == "symmetric_clip":
            q = np.clip(q, -(2 ** (bits - 1)) + 1, 2 ** (bits - 1) - 1)
        else:
            q = np.clip(q, -(2 ** (bits - 1)), 2 ** (bits - 1) - 1)
        return q.astype(np.int8), delta
    return quantize


def _shift_with(bug):
    def requant(acc, shift):
        acc = np.asarray(acc, dtype=np.int64)
        if shift == 0:
            y = acc
        elif bug == "shift_truncates":
            y = acc >> shift
        elif bug == "shift_ties_away":
            y = np.sign(acc) * ((np.abs(acc) + (1 << (shift - 1))) >> shift)
        else:
            y = (acc + (1 << (shift - 1))) >> shift
        if bug == "shift_no_saturation":
            return (((y + 128) % 256) - 128).astype(np.int8)
        return np.clip(y, -128, 127).astype(np.int8)
    return requant


def _run_pins(quantize, requant, monkeypatch):
    """The pins above, run against the given functions; returns how many fail."""
    failed = 0
    with monkeypatch.context() as m:
        m.setattr(oracle, "quantize_eq8", quantize)
        m.setattr(oracle, "requant_shift", requant)
        for pin in (test_eq8_hand_example, test_eq8_error_bound_and_grid,
                    test_requant_shift_against_python_integers):
            try:
                pin()
            except AssertionError:
                failed += 1
    return failed


def test_unplanted_copies_pass_the_pins(monkeypatch):
    assert _run_pins(_quantizer_with(None), _shift_with(None), monkeypatch) == 0


@pytest.mark.parametrize("bug", ["ties_away", "truncate", "no_clip", "symmetric_clip", "delta_2N",
                                 "shift_truncates", "shift_ties_away", "shift_no_saturation"])
def test_planted_mistakes_are_caught(bug, monkeypatch):
    """A tie rule, a clip, a scale or a rounding offset changed by one step fails a pin."""
    assert _run_pins(_quantizer_with(bug), _shift_with(bug), monkeypatch) >= 1, bug


def test_pack_reference_i8_structure():
    rng = np.random.default_rng(9)
    Wq = rng.integers(-128, 128, (20, 3, 1, 12), dtype=np.int8)          # ragged for 8x8
    gamma = np.array([[1, 0], [0, 1], [1, 1]], dtype=np.uint8)
    rp, ci, pl = oracle.pack_reference_i8(Wq, gamma, 8, 8)
    assert rp.tolist() == [0, 1, 2, 4] and ci.tolist() == [0, 1, 0, 1]
    assert pl.dtype == np.int8 and pl.shape == (4, 8, 3, 1, 8)
    assert (pl[1][:, :, :, :4] == Wq[8:16, :, :, 8:12]).all() and not pl[1][:, :, :, 4:].any()
    assert (pl[2][:4] == Wq[16:20, :, :, 0:8]).all() and not pl[2][4:].any()
