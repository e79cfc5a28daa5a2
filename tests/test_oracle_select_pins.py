"""Pins for the mask-selection oracle (oracle/select.py): hand-worked blocks for each
importance measure (Section IV), library norms, and the ordering rules."""
import numpy as np
import pytest

import oracle
from oracle import select as sel


def _w_from_blocks(vals, bo=8, bi=8):
    """One 8x8 block per entry of vals (2-D list), every weight of the block = that value,
    except the first weight which is doubled (so the variance is not zero)."""
    rows, cols = len(vals), len(vals[0])
    W = np.zeros((rows * bo, 1, 1, cols * bi))
    for l in range(rows):
        for c in range(cols):
            W[l * bo:(l + 1) * bo, 0, 0, c * bi:(c + 1) * bi] = vals[l][c]
            W[l * bo, 0, 0, c * bi] = 2 * vals[l][c]
    return W


def test_measures_by_hand():
    # one block: 63 weights of a and one of 2a, n = 64
    a = 0.5
    W = _w_from_blocks([[a]])
    l2 = oracle.block_importance(W, 8, 8, sel.L2)[0, 0]
    l1 = oracle.block_importance(W, 8, 8, sel.L1)[0, 0]
    var = oracle.block_importance(W, 8, 8, sel.VAR)[0, 0]
    assert l2 == pytest.approx(np.sqrt(63 * a * a + 4 * a * a), rel=1e-15)
    assert l1 == pytest.approx(65 * a, rel=1e-15)
    mu = 65 * a / 64
    assert var == pytest.approx((63 * (a - mu) ** 2 + (2 * a - mu) ** 2) / 64, rel=1e-13)


def test_measures_against_numpy_with_window_and_ragged_edges():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((20, 3, 2, 12))              # ragged for 8x8 and 16x4
    for bo, bi in ((8, 8), (4, 16), (16, 4)):
        nbr, nbc = -(-20 // bo), -(-12 // bi)
        Wp = np.zeros((nbr * bo, 3, 2, nbc * bi))
        Wp[:20, :, :, :12] = W
        blocks = Wp.reshape(nbr, bo, 3, 2, nbc, bi).transpose(0, 4, 1, 2, 3, 5).reshape(nbr, nbc, -1)
        np.testing.assert_allclose(oracle.block_importance(W, bo, bi, sel.L2),
                                   np.linalg.norm(blocks, axis=2), rtol=1e-13)
        np.testing.assert_allclose(oracle.block_importance(W, bo, bi, sel.L1),
                                   np.abs(blocks).sum(axis=2), rtol=1e-13)
        np.testing.assert_allclose(oracle.block_importance(W, bo, bi, sel.VAR),
                                   blocks.var(axis=2), rtol=1e-12)


def test_first_half_by_ascending_importance_and_ties():
    # importances 3 1 2 / 1 4 1 (L1-like ordering by magnitude); ties among the 1s
    W = _w_from_blocks([[3.0, 1.0, 2.0], [1.0, 4.0, 1.0]])
    g = oracle.select_mask(W, 8, 8, sel.L1, 0.5)
    # three of six zeroed: the three blocks of value 1, lowest indices first -> all of them
    assert g.tolist() == [[1, 0, 1], [0, 1, 0]]
    g2 = oracle.select_mask(W, 8, 8, sel.L1, 4 / 6)      # two zeroed: the first two 1s
    assert g2.tolist() == [[1, 0, 1], [0, 1, 1]]
    gr = oracle.select_mask(W, 8, 8, sel.L2, 1 / 3, per_row=True)   # keep one per row
    assert gr.tolist() == [[1, 0, 0], [0, 1, 0]]
    assert oracle.select_mask(W, 8, 8, sel.L2, 1.0).all()
    assert not oracle.select_mask(W, 8, 8, sel.L2, 0.0).any()


def test_incremental_step_counts():
    rng = np.random.default_rng(2)
    W = rng.standard_normal((64, 1, 1, 320))             # 8 x 40 = 320 blocks
    g = np.ones((8, 40), dtype=np.uint8)
    zeroed = []
    for _ in range(200):
        g2 = oracle.incremental_step(W, g, 8, 8, sel.L2, 0.5)
        z = int(g.sum() - g2.sum())
        if z == 0:
            break
        zeroed.append(z)
        assert (g2 <= g).all()
        g = g2
    assert g.sum() == 160
    # first step: k = 160 to go -> ceil(8) = 8; near the end single blocks
    assert zeroed[0] == 8 and zeroed[-1] == 1 and min(zeroed) == 1
    # the path ends at the one-shot choice only if importance does not change: same W here
    assert (g == oracle.select_mask(W, 8, 8, sel.L2, 0.5)).all()
