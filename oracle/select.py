"""CPU oracle for choosing the mask from the weights (paper Section IV, "Predetermined
Sparsity ratio and Full Training Ahead", and the step of "Sparsity Ratio as Incremental").

TEST INFRASTRUCTURE ONLY (see oracle.py): nothing on the product path imports it.

Each mask entry gamma_i stands for one block W_i (b_o x H x K x b_i weights).  Its
importance is one of
    L2(W_i) = sqrt(sum_k w_k^2),   L1(W_i) = sum_k |w_k|,
    Var(W_i) = (1/n) sum_k (w_k - mu)^2 with mu = (1/n) sum_k w_k,
n the number of entries of the block as it is stored (a block that overhangs O or I counts
its missing entries as zeros, like the packer).  Blocks are sorted by ascending importance
and the first ones are zeroed: half of them in the paper, here round((1 - density) * n).
The paper does this "for the entire network or for one convolution at a time"; per layer
here, or per block row (the row-balanced variant of its Fig. 2).  Ties (equal importance)
are broken by block position, lower index zeroed first: the paper names no rule.

Incremental step: with k entries of the mask not yet zeroed beyond the target, zero the
max(ceil(5% of k), 1) least important of the kept blocks ("at each iteration at least one
block will be set to zero"; the printed min(., 1) would never zero more than one).
"""
from __future__ import annotations

import math

import numpy as np

L2, L1, VAR = 0, 1, 2


def block_importance(W: np.ndarray, bo: int, bi: int, measure: int) -> np.ndarray:
    """fp64 importance of every block, [ceil(O/bo)][ceil(I/bi)], by explicit loops."""
    W = np.asarray(W, dtype=np.float64)
    O, H, K, I = W.shape
    nbr, nbc = -(-O // bo), -(-I // bi)
    out = np.zeros((nbr, nbc), dtype=np.float64)
    n = bo * H * K * bi
    for l in range(nbr):
        for c in range(nbc):
            blk = np.zeros((bo, H, K, bi), dtype=np.float64)
            sub = W[l * bo:(l + 1) * bo, :, :, c * bi:(c + 1) * bi]
            blk[:sub.shape[0], :, :, :sub.shape[3]] = sub
            v = blk.reshape(-1)
            if measure == L2:
                out[l, c] = math.sqrt(math.fsum(x * x for x in v))
            elif measure == L1:
                out[l, c] = math.fsum(abs(x) for x in v)
            elif measure == VAR:
                mu = math.fsum(v) / n
                out[l, c] = math.fsum((x - mu) * (x - mu) for x in v) / n
            else:
                raise ValueError(measure)
    return out


def _zero_lowest(score: np.ndarray, gamma: np.ndarray, count: int) -> None:
    """Zero `count` kept entries of the flat gamma with the lowest score, ties by index."""
    kept = [i for i in range(score.size) if gamma[i]]
    kept.sort(key=lambda i: (score[i], i))
    for i in kept[:count]:
        gamma[i] = 0


def select_mask(W: np.ndarray, bo: int, bi: int, measure: int = L2, density: float = 0.5,
                per_row: bool = False) -> np.ndarray:
    score = block_importance(W, bo, bi, measure)
    gamma = np.ones(score.shape, dtype=np.uint8)
    if per_row:
        for l in range(score.shape[0]):
            row = gamma[l]
            _zero_lowest(score[l], row, row.size - int(round(density * row.size)))
    else:
        flat = gamma.reshape(-1)
        _zero_lowest(score.reshape(-1), flat, flat.size - int(round(density * flat.size)))
    return gamma


def incremental_step(W: np.ndarray, gamma: np.ndarray, bo: int, bi: int, measure: int = L2,
                     target_density: float = 0.5) -> np.ndarray:
    """One step of the incremental schedule on a copy of gamma."""
    score = block_importance(W, bo, bi, measure)
    g = np.array(gamma, dtype=np.uint8).reshape(score.shape).copy()
    flat = g.reshape(-1)
    keep_target = int(round(target_density * flat.size))
    k = int(flat.sum()) - keep_target                 # still to be zeroed
    if k <= 0:
        return g
    _zero_lowest(score.reshape(-1), flat, min(k, max(int(math.ceil(0.05 * k)), 1)))
    return g
