"""CPU oracle for the 8-bit integer path: the round-to-nearest quantizer of the
paper's Eq. (8) and integer convolution / FC layers on masked int8 weights.

TEST INFRASTRUCTURE ONLY (see oracle.py): nothing on the product path imports it.

Quantizer, Section V, Eq. (8):  W_q = Delta * Round(W / Delta),
Delta = max|W| / 2^(N-1).  The integer code q = Round(W / Delta) lies in
[-2^(N-1), 2^(N-1)]; the single value +2^(N-1) (reached only where W = +max|W|)
does not fit N signed bits and is stored as 2^(N-1) - 1.  "Round" is round to
nearest with ties to even (the paper does not name the tie rule; IEEE default).

Layer, Section V ("a convolution has one quantized input INT8 with ... (power of
two scale) ... weight 8 bits and bias 32", Section III for the bias widths):
  acc[n,m,q,o] = bias[o] + sum_{h,k,i} Wm[o,h,k,i] * X[n, m*s+h-p, q*s+k-p, i]
in exact integer arithmetic (int8 x int8 products, 32-bit bias, a sum that fits 32
bits), Wm the mask-applied codes as in oracle.py.  The output is either that
32-bit sum or, for a power-of-two output scale, the sum shifted right by `shift`
bits with rounding to nearest (ties upward: add 2^(shift-1), arithmetic shift) and
saturated to [-128, 127].

Pins (tests/test_oracle_quant_pins.py): Delta and the codes of a hand example;
|W - W_q| <= Delta/2 away from the clipped maximum; codes of exact multiples of
Delta; ties; the integer sums against a brute-force Python-int loop and against
numpy int64 einsum; the shift against Python's integer floor division, including
ties, negative sums and both saturation ends.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

from . import oracle as _o


def quantize_eq8(W: np.ndarray, bits: int = 8) -> Tuple[np.ndarray, float]:
    """Eq. (8): integer codes (int8 for bits <= 8) and Delta.  All-zero W gives Delta 0
    and all-zero codes."""
    W = np.asarray(W, dtype=np.float64)
    top = float(np.max(np.abs(W))) if W.size else 0.0
    if top == 0.0:
        return np.zeros(W.shape, dtype=np.int8), 0.0
    delta = top / float(2 ** (bits - 1))
    q = np.rint(W / delta)                       # ties to even
    q = np.clip(q, -(2 ** (bits - 1)), 2 ** (bits - 1) - 1)
    return q.astype(np.int8), delta


def requant_shift(acc: np.ndarray, shift: int) -> np.ndarray:
    """Power-of-two rescale of 32-bit sums to int8: round to nearest (ties upward),
    saturate."""
    acc = np.asarray(acc, dtype=np.int64)
    if shift < 0:
        raise ValueError("shift")
    y = (acc + (1 << (shift - 1))) >> shift if shift > 0 else acc
    return np.clip(y, -128, 127).astype(np.int8)


def conv2d_i8(Xq: np.ndarray, Wq: np.ndarray, bias: Optional[np.ndarray], gamma: np.ndarray,
              bo: int, bi: int, stride=(1, 1), pad=(0, 0), shift: Optional[int] = None
              ) -> np.ndarray:
    """Integer layer.  Xq int8 [B][L][J][I], Wq int8 [O][H][K][I], bias int32 [O] or None.
    Returns the exact sums (int64 array holding 32-bit values) or, with `shift`, int8.

    The sum is taken by the fp64 direct convolution of oracle.py: every product is below
    2^14 and every partial sum far below 2^53, so fp64 holds them exactly."""
    Xq = np.asarray(Xq)
    Wq = np.asarray(Wq)
    assert Xq.dtype == np.int8 and Wq.dtype == np.int8
    b = None if bias is None else np.asarray(bias, dtype=np.int64).astype(np.float64)
    y = _o.conv2d(Xq.astype(np.float32), Wq.astype(np.float32), b, gamma, bo, bi, stride, pad)
    acc = np.rint(y).astype(np.int64)
    assert np.all(acc == y), "a sum was not an integer: fp64 lost exactness"
    assert np.all(np.abs(acc) < 2 ** 31), "sum does not fit 32 bits"
    return acc if shift is None else requant_shift(acc, shift)


def fc_i8(Xq, Wq, bias, gamma, bo, bi, shift=None):
    """Y[B][O] on Xq[B][I], Wq[O][I]: the 1x1 case."""
    Xq = np.asarray(Xq)
    Wq = np.asarray(Wq)
    y = conv2d_i8(Xq.reshape(Xq.shape[0], 1, 1, -1), Wq.reshape(Wq.shape[0], 1, 1, -1), bias,
                  gamma, bo, bi, shift=shift)
    return y.reshape(Xq.shape[0], -1)


def pack_reference_i8(Wq: np.ndarray, gamma: np.ndarray, bo: int, bi: int):
    """Compressed-block-row form of int8 codes (same structure as oracle.pack_reference)."""
    rp, ci, pl = _o.pack_reference(np.asarray(Wq).astype(np.float32), gamma, bo, bi, "f32")
    return rp, ci, pl.astype(np.int8)
