"""Seeded random tensors and block masks for conv / FC layers.

Draw order for one layer is fixed: X, W, bias, then the mask, all from one
``numpy.random.Generator(PCG64(seed))``.  Values meant for a bf16 layer are
snapped onto the bf16 grid here (low 16 bits of the fp32 pattern cleared), so
both consumers receive bit-identical stored values and neither has to round an
input.  Nothing in this file multiplies, masks or packs weights.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 240709453


def seed_for(config: int, layer: int = 0) -> int:
    """Seed of layer ``layer`` of benchmark configuration ``config``."""
    return BASE_SEED + 1000 * int(config) + int(layer)


def bf16_grid(a: np.ndarray) -> np.ndarray:
    """Snap fp32 values onto the bf16 grid by clearing the low 16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)


def n_blocks(O: int, I: int, bo: int, bi: int) -> Tuple[int, int]:
    return (O + bo - 1) // bo, (I + bi - 1) // bi


def draw_mask(rng: np.random.Generator, nbr: int, nbc: int, kind: str,
              density: float) -> np.ndarray:
    """A uint8 block mask of shape (nbr, nbc); 1 = block kept, 0 = zeroed.

    kind:
      "bernoulli"    each block kept independently with probability ``density``
      "exact"        exactly round(density*nbr*nbc) blocks kept, uniformly at
                     random over the layer (rows end up unbalanced)
      "row_balanced" every block row keeps exactly round(density*nbc) blocks
      "ones"/"zeros" constant masks
    """
    if kind == "ones":
        return np.ones((nbr, nbc), dtype=np.uint8)
    if kind == "zeros":
        return np.zeros((nbr, nbc), dtype=np.uint8)
    if kind == "bernoulli":
        return (rng.random((nbr, nbc)) < density).astype(np.uint8)
    if kind == "exact":
        total = nbr * nbc
        keep = int(round(density * total))
        g = np.zeros(total, dtype=np.uint8)
        g[rng.permutation(total)[:keep]] = 1
        return g.reshape(nbr, nbc)
    if kind == "row_balanced":
        keep = int(round(density * nbc))
        g = np.zeros((nbr, nbc), dtype=np.uint8)
        for r in range(nbr):
            g[r, rng.permutation(nbc)[:keep]] = 1
        return g
    raise ValueError(f"unknown mask kind {kind!r}")


@dataclass
class LayerCase:
    """One synthetic layer: shapes, stored-precision tensors, mask."""
    name: str
    B: int
    L: int
    J: int
    I: int
    O: int
    H: int
    K: int
    stride: Tuple[int, int]
    pad: Tuple[int, int]
    bo: int
    bi: int
    dtype: str                      # "f32" or "bf16": storage type of X, W, Y
    X: np.ndarray                   # float32 [B, L, J, I], on the dtype's grid
    W: np.ndarray                   # float32 [O, H, K, I], on the dtype's grid
    bias: np.ndarray                # float32 [O]
    gamma: np.ndarray               # uint8 [ceil(O/bo), ceil(I/bi)]
    mask_kind: str = "exact"
    density: float = 0.5
    seed: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def M(self) -> int:
        return (self.L + 2 * self.pad[0] - self.H) // self.stride[0] + 1

    @property
    def N(self) -> int:
        return (self.J + 2 * self.pad[1] - self.K) // self.stride[1] + 1

    @property
    def P(self) -> int:
        return self.B * self.M * self.N

    @property
    def nnzb(self) -> int:
        return int(self.gamma.sum())


def draw_layer(name: str, *, B: int, L: int, J: int, I: int, O: int,
               H: int = 1, K: int = 1, stride=(1, 1), pad=(0, 0),
               bo: int = 8, bi: int = 8, dtype: str = "bf16",
               mask_kind: str = "exact", density: float = 0.5,
               seed: int = 0, x_std: float = 1.0,
               w_std: Optional[float] = None, b_std: float = 0.01,
               draw_x: bool = True) -> LayerCase:
    """Draw X ~ N(0, x_std), W ~ N(0, w_std), bias ~ N(0, b_std) and a mask.

    ``w_std=None`` uses sqrt(2/(I*H*K)) so a chain of layers keeps O(1)
    activations.  ``draw_x=False`` draws X's values all the same, in pieces
    that are thrown away, so that W, bias and the mask are exactly those of
    ``draw_x=True`` for the same seed; it returns an empty X, and callers
    supply their own activations.
    """
    if dtype not in ("f32", "bf16"):
        raise ValueError(dtype)
    rng = np.random.Generator(np.random.PCG64(seed))
    if isinstance(stride, int):
        stride = (stride, stride)
    if isinstance(pad, int):
        pad = (pad, pad)
    if w_std is None:
        w_std = float(np.sqrt(2.0 / (I * H * K)))
    if draw_x:
        X = rng.standard_normal((B, L, J, I), dtype=np.float32) * np.float32(x_std)
    else:
        left = B * L * J * I        # the generator fills element by element: pieces = whole
        while left > 0:
            n = min(left, 1 << 22)
            rng.standard_normal(n, dtype=np.float32)
            left -= n
        X = np.zeros((0, L, J, I), dtype=np.float32)
    W = rng.standard_normal((O, H, K, I), dtype=np.float32) * np.float32(w_std)
    bias = rng.standard_normal((O,), dtype=np.float32) * np.float32(b_std)
    nbr, nbc = n_blocks(O, I, bo, bi)
    if I < bi:
        # fewer input channels than one block is wide: the layer stays dense
        mask_kind_eff = "ones"
    else:
        mask_kind_eff = mask_kind
    gamma = draw_mask(rng, nbr, nbc, mask_kind_eff, density)
    if dtype == "bf16":
        X = bf16_grid(X)
        W = bf16_grid(W)
    return LayerCase(name=name, B=B, L=L, J=J, I=I, O=O, H=H, K=K,
                     stride=tuple(stride), pad=tuple(pad), bo=bo, bi=bi,
                     dtype=dtype, X=X, W=W, bias=bias, gamma=gamma,
                     mask_kind=mask_kind_eff, density=density, seed=seed)
