"""CPU oracle: block-sparse conv / FC inference by its plain definition.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path imports this module;
it shares no code, table or helper with the HIP library.

The method reaches, faster, exactly the result of an ordinary dense layer
whose weights had whole blocks zeroed, so the oracle is that definition
written out:

  1. mask:   Wm[o,h,k,i] = W[o,h,k,i] if Gamma[o div b_o, i div b_i] else +0
             (paper Eq. (1): a zero entry of Gamma zeroes W[i,*,*,j] for the
             b_o output channels and b_i input channels of that block; the
             mask is applied, i.e. the layer uses Gamma*W, Section IV-A)
  2. layer:  Y = Wm * X + b as a dense cross-correlation in fp64
             (paper Section I for the shapes; the C routine states the sum)

A fully-connected layer is the 1x1 case (Section III).  Inputs arrive already
rounded to their storage type and are widened to fp64 here.

Also here, as independent checks of the host packer: a pure-numpy block
compaction (row pointers / column indices / per-block payload, Section III:
compressed block row storage) and bf16 round-to-nearest-even by bit
arithmetic.

Pins (tests/test_oracle_pins.py): the paper's worked index example for
Eq. (1); the closed form of Eq. (4); a dense library convolution and matmul
for the all-ones mask; a scatter-form brute force on tiny shapes; linearity
over blocks; bias-only for the empty mask; the three-layer chain against the
same chain built from a library convolution with explicit bf16 casts, and
against a hand case with identity weights.  The stride / padding / output-size
conventions are not fixed by the paper: for those the oracle is pinned only
to the usual deep-learning-framework convention (parity unpinned by the
paper itself).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bsp_oracle.c")
_LIB = os.path.join(_HERE, "libbsp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C part of the oracle with gcc (OpenMP)."""
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared",
                               "-std=c11", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, dp = ctypes.c_int64, ctypes.POINTER(ctypes.c_double)
        lib.oracle_conv2d.restype = ctypes.c_int
        lib.oracle_conv2d.argtypes = [dp, dp, dp, dp] + [i64] * 11 + [ctypes.c_int]
        lib.oracle_conv2d_at.restype = ctypes.c_int
        lib.oracle_conv2d_at.argtypes = [dp, dp, dp, ctypes.POINTER(i64), i64, dp] + [i64] * 11
        _lib = lib
    return _lib


def _dptr(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.POINTER(ctypes.c_double)()
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


# ----------------------------------------------------------------- step 1: mask
def expand_mask(gamma: np.ndarray, O: int, I: int, bo: int, bi: int) -> np.ndarray:
    """Gamma (block rows x block columns) -> boolean O x I map over W-bar.

    Entry (l, iota) of Gamma governs output channels l*b_o .. (l+1)*b_o - 1 and
    input channels iota*b_i .. (iota+1)*b_i - 1 (Eq. (1)); blocks that overhang
    O or I are clipped.
    """
    gamma = np.asarray(gamma)
    nbr, nbc = -(-O // bo), -(-I // bi)
    if gamma.shape != (nbr, nbc):
        raise ValueError(f"Gamma must be {nbr}x{nbc}, got {gamma.shape}")
    if not np.isin(gamma, (0, 1)).all():
        raise ValueError("Gamma must be binary")
    o = np.arange(O) // bo
    i = np.arange(I) // bi
    return gamma[np.ix_(o, i)] != 0


def apply_mask(W: np.ndarray, gamma: np.ndarray, bo: int, bi: int) -> np.ndarray:
    """Wm = Gamma applied to W (O x H x K x I): a select, not a multiply."""
    O, H, K, I = W.shape
    keep = expand_mask(gamma, O, I, bo, bi)
    return np.where(keep[:, None, None, :], W, np.zeros((), dtype=W.dtype))


# ---------------------------------------------------------------- step 2: layer
def out_size(L: int, J: int, H: int, K: int, stride, pad) -> Tuple[int, int]:
    return ((L + 2 * pad[0] - H) // stride[0] + 1,
            (J + 2 * pad[1] - K) // stride[1] + 1)


def conv2d(X: np.ndarray, W: np.ndarray, bias: Optional[np.ndarray],
           gamma: np.ndarray, bo: int, bi: int, stride=(1, 1), pad=(0, 0),
           threads: int = 0, return_threads: bool = False):
    """Y[B,M,N,O] (fp64) for NHWC X[B,L,J,I], OHWI W, mask Gamma."""
    B, L, J, I = X.shape
    O, H, K, I2 = W.shape
    if I2 != I:
        raise ValueError("channel mismatch")
    M, N = out_size(L, J, H, K, stride, pad)
    if M < 1 or N < 1:
        raise ValueError("empty output")
    Wm = np.ascontiguousarray(apply_mask(W, gamma, bo, bi), dtype=np.float64)
    Xd = np.ascontiguousarray(X, dtype=np.float64)
    bd = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    Y = np.empty((B, M, N, O), dtype=np.float64)
    used = _load().oracle_conv2d(_dptr(Xd), _dptr(Wm), _dptr(bd), _dptr(Y),
                                 B, L, J, I, O, H, K, stride[0], stride[1],
                                 pad[0], pad[1], threads)
    if used < 0:
        raise RuntimeError("oracle_conv2d failed")
    return (Y, used) if return_threads else Y


def conv2d_fused(X, W, bias, gamma, bo, bi, stride=(1, 1), pad=(0, 0), residual=None,
                 relu: bool = False, dtype: str = "bf16") -> np.ndarray:
    """The layer followed by an element-wise residual add and activation in the storage
    type: act(round(conv + bias) + residual) in fp64, the caller's comparison supplying the
    last rounding.  (Paper Section VI fuses a layer with what follows it; the arithmetic is
    that of the separate operations: the convolution's result is first stored in `dtype`.)"""
    y = conv2d(X, W, bias, gamma, bo, bi, stride, pad)
    if residual is None and not relu:
        return y
    y = round_to_storage(y, dtype).astype(np.float64)
    if residual is not None:
        y = y + np.asarray(residual, dtype=np.float64)
    if relu:
        y = np.maximum(y, 0.0)
    return y


def bottleneck(X, layers, bo, bi, residual=None, dtype: str = "bf16") -> np.ndarray:
    """A chain of three layers kept on chip between them (paper Section VI, depth-wise
    tiling of consecutive layers): 1x1 -> 3x3 (padding 1) -> 1x1, a ReLU after each, the
    residual added before the last one.  `layers` is [(W, bias, gamma)] * 3.  Tiling does
    not change the arithmetic: this is the three layers one after the other, each result
    rounded to the storage type before the next layer reads it (as it would be if it went
    through memory); returns fp64, the caller's comparison supplying the last rounding."""
    (W1, b1, g1), (W2, b2, g2), (W3, b3, g3) = layers
    t1 = round_to_storage(conv2d_fused(X, W1, b1, g1, bo, bi, (1, 1), (0, 0), relu=True, dtype=dtype), dtype)
    t2 = round_to_storage(conv2d_fused(t1, W2, b2, g2, bo, bi, (1, 1), (1, 1), relu=True, dtype=dtype), dtype)
    return conv2d_fused(t2, W3, b3, g3, bo, bi, (1, 1), (0, 0), residual=residual, relu=True, dtype=dtype)


def conv2d_at(X, W, bias, gamma, bo, bi, positions: np.ndarray,
              stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """The outputs Y[n,m,q,o] at the listed (n,m,q,o) rows only (fp64)."""
    B, L, J, I = X.shape
    O, H, K, _ = W.shape
    Wm = np.ascontiguousarray(apply_mask(W, gamma, bo, bi), dtype=np.float64)
    Xd = np.ascontiguousarray(X, dtype=np.float64)
    bd = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    pos = np.ascontiguousarray(positions, dtype=np.int64).reshape(-1, 4)
    out = np.empty(pos.shape[0], dtype=np.float64)
    rc = _load().oracle_conv2d_at(
        _dptr(Xd), _dptr(Wm), _dptr(bd),
        pos.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), pos.shape[0],
        _dptr(out), B, L, J, I, O, H, K, stride[0], stride[1], pad[0], pad[1])
    if rc != 0:
        raise RuntimeError(f"oracle_conv2d_at failed ({rc})")
    return out


def fc(X: np.ndarray, Wbar: np.ndarray, bias, gamma, bo: int, bi: int,
       threads: int = 0) -> np.ndarray:
    """Y[B,O] = X[B,I] . (Gamma applied to W-bar[O,I])^T + b: the 1x1 layer."""
    B, I = X.shape
    O = Wbar.shape[0]
    Y = conv2d(X.reshape(B, 1, 1, I), Wbar.reshape(O, 1, 1, I), bias, gamma,
               bo, bi, threads=threads)
    return Y.reshape(B, O)


# ------------------------------------------------------------ operation counts
def flops_nonzero(P: int, nnzb: int, bo: int, bi: int, H: int, K: int) -> int:
    """Multiply-adds x2 done for nonzero blocks only: each kept block costs
    b_o*b_i*H*K MACs per output pixel (advantages 3 and 4 of Section I: the
    count per row and per block is known, and halving the blocks halves it)."""
    return 2 * P * nnzb * bo * bi * H * K


def row_sparsity(gamma: np.ndarray) -> np.ndarray:
    """Eq. (2) for every block row: (N - sum_i Gamma[o,i]) / N."""
    g = np.asarray(gamma, dtype=np.int64)
    n = g.shape[1]
    return (n - g.sum(axis=1)) / n


# ------------------------------------------------ storage-type rounding (bf16)
def bf16_bits_rne(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even.
    Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = (u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


def round_to_storage(y: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 result -> the value a dtype-typed output buffer would hold."""
    if dtype == "f32":
        return y.astype(np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(bf16_bits_rne(y.astype(np.float32)))
    raise ValueError(dtype)


# ------------------------------------------------- independent block compaction
def pack_reference(W: np.ndarray, gamma: np.ndarray, bo: int, bi: int,
                   payload_dtype: str = "f32"):
    """Compressed-block-row form of (Gamma, W), built with plain loops.

    row_ptr[l+1] - row_ptr[l] = number of kept blocks in block row l
    (= N(1 - S_l) by Eq. (2)); col_idx lists the kept block columns of each
    row in ascending order; payload[n] is the b_o x H x K x b_i sub-tensor of W
    for kept block n (input channel innermost), with +0 where a block
    overhangs O or I.  Returns (row_ptr int32, col_idx int32, payload) where
    payload is float32 or, for "bf16", uint16 bit patterns.
    """
    W = np.asarray(W, dtype=np.float32)
    O, H, K, I = W.shape
    nbr, nbc = -(-O // bo), -(-I // bi)
    gamma = np.asarray(gamma)
    if gamma.shape != (nbr, nbc):
        raise ValueError("Gamma shape")
    row_ptr = [0]
    col_idx = []
    blocks = []
    for l in range(nbr):
        for c in range(nbc):
            if gamma[l, c]:
                col_idx.append(c)
                blk = np.zeros((bo, H, K, bi), dtype=np.float32)
                o0, i0 = l * bo, c * bi
                no, ni = min(bo, O - o0), min(bi, I - i0)
                blk[:no, :, :, :ni] = W[o0:o0 + no, :, :, i0:i0 + ni]
                blocks.append(blk)
        row_ptr.append(len(col_idx))
    payload = (np.stack(blocks) if blocks
               else np.zeros((0, bo, H, K, bi), dtype=np.float32))
    if payload_dtype == "bf16":
        payload = bf16_bits_rne(payload).reshape(payload.shape)
    elif payload_dtype != "f32":
        raise ValueError(payload_dtype)
    return (np.asarray(row_ptr, dtype=np.int32),
            np.asarray(col_idx, dtype=np.int32), payload)


def unpack_reference(row_ptr, col_idx, payload, O, H, K, I, bo, bi) -> np.ndarray:
    """Inverse of pack_reference onto a dense fp32 O x H x K x I tensor."""
    if payload.dtype == np.uint16:
        payload = bf16_bits_to_f32(payload).reshape(payload.shape)
    W = np.zeros((O, H, K, I), dtype=np.float32)
    for l in range(len(row_ptr) - 1):
        for n in range(row_ptr[l], row_ptr[l + 1]):
            c = int(col_idx[n])
            o0, i0 = l * bo, c * bi
            no, ni = min(bo, O - o0), min(bi, I - i0)
            W[o0:o0 + no, :, :, i0:i0 + ni] = payload[n][:no, :, :, :ni]
    return W
