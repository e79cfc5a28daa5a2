"""CPU oracle for the block-sparse x block-sparse product of the paper's Section III-A,
    C = (Gamma A) (Omega B)^t,
A and B cut into k x k blocks, Gamma / Omega one entry per block:
    C_ij = sum_c gamma_ic A_ic (omega_jc B_jc)^t        (blocks; i, j block rows, c block column)
"There will be a meaningful product to compute if and only if" both blocks are kept.

TEST INFRASTRUCTURE ONLY (see oracle.py): nothing on the product path imports it.

The method reaches exactly the dense product of the two masked matrices, so the oracle is that
definition: mask both operands, multiply in fp64 with the library matmul.  Pins
(tests/test_oracle_spgemm_pins.py): the block formula above written as explicit loops over
matching index pairs of the two sorted column lists; a hand-sized case; the count of
meaningful block products.
"""
from __future__ import annotations

import numpy as np


def mask_blocks(A: np.ndarray, gamma: np.ndarray, k: int) -> np.ndarray:
    """Zero the k x k blocks of A whose gamma entry is 0 (a select, not a multiply)."""
    A = np.asarray(A, dtype=np.float64)
    g = np.kron(np.asarray(gamma, dtype=bool), np.ones((k, k), dtype=bool))
    return np.where(g[:A.shape[0], :A.shape[1]], A, 0.0)


def spgemm_nt(A: np.ndarray, gamma: np.ndarray, B: np.ndarray, omega: np.ndarray, k: int) -> np.ndarray:
    """C = (Gamma A)(Omega B)^t in fp64.  A: [Ra*k][N*k], B: [Rb*k][N*k]."""
    return mask_blocks(A, gamma, k) @ mask_blocks(B, omega, k).T


def matching_block_products(gamma: np.ndarray, omega: np.ndarray) -> int:
    """How many k x k block products are meaningful: pairs (i, j, c) with both blocks kept."""
    return int((np.asarray(gamma, dtype=np.int64) @ np.asarray(omega, dtype=np.int64).T).sum())
