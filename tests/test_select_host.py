"""Mask selection in libbsp (host) against the selection oracle: scores to rounding, masks
bit for bit (no GPU needed)."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp

GRANS = [(8, 8), (4, 16), (16, 4)]


@pytest.mark.parametrize("bo,bi", GRANS)
@pytest.mark.parametrize("measure", [0, 1, 2])
def test_scores_and_masks_match_oracle(bo, bi, measure):
    rng = np.random.default_rng(bo * 10 + measure)
    for O, H, K, I in ((64, 3, 3, 64), (20, 2, 1, 12), (48, 1, 1, 80)):
        W = (rng.standard_normal((O, H, K, I)) * 0.05).astype(np.float32)
        s = bsp.bsp_block_importance(W, bo, bi, measure)
        s0 = oracle.block_importance(W, bo, bi, measure)
        np.testing.assert_allclose(s, s0, rtol=1e-13, atol=1e-300)
        for density in (0.5, 0.25, 0.8):
            for per_row in (False, True):
                g = bsp.bsp_select_mask(W, bo, bi, measure, density, per_row)
                g0 = oracle.select_mask(W, bo, bi, measure, density, per_row)
                assert g.dtype == np.uint8 and (g == g0).all(), (O, density, per_row)
                n = g.shape[1] if per_row else g.size
                want = int(round(density * n)) * (g.shape[0] if per_row else 1)
                assert int(g.sum()) == want


def test_ties_go_by_block_index():
    W = np.zeros((16, 1, 1, 24), dtype=np.float32)           # 2 x 3 blocks of 8x8
    vals = [[3.0, 1.0, 2.0], [1.0, 4.0, 1.0]]
    for l in range(2):
        for c in range(3):
            W[l * 8:(l + 1) * 8, 0, 0, c * 8:(c + 1) * 8] = vals[l][c]
    assert bsp.bsp_select_mask(W, 8, 8, 1, 4 / 6).tolist() == [[1, 0, 1], [0, 1, 1]]
    assert bsp.bsp_select_mask(W, 8, 8, 0, 1 / 3, True).tolist() == [[1, 0, 0], [0, 1, 0]]


def test_incremental_schedule_follows_oracle_to_the_target():
    rng = np.random.default_rng(4)
    W = rng.standard_normal((64, 1, 1, 320)).astype(np.float32)
    g = np.ones((8, 40), dtype=np.uint8)
    g0 = g.copy()
    steps = 0
    while True:
        g, z = bsp.bsp_mask_step(W, g, 8, 8, 0, 0.5)
        g0n = oracle.incremental_step(W, g0, 8, 8, 0, 0.5)
        assert (g == g0n).all() and z == int(g0.sum() - g0n.sum())
        g0 = g0n
        if z == 0:
            break
        steps += 1
    assert g.sum() == 160 and steps > 20
    assert (g == bsp.bsp_select_mask(W, 8, 8, 0, 0.5)).all()


def test_selection_errors():
    W = np.zeros((8, 1, 1, 8), dtype=np.float32)
    with pytest.raises(bsp.BspError) as e:
        bsp.bsp_select_mask(W, 8, 8, 0, 1.5)
    assert e.value.code == -2
    with pytest.raises(bsp.BspError) as e:
        bsp.bsp_block_importance(W, 8, 8, 7)
    assert e.value.code == -2
    with pytest.raises(bsp.BspError) as e:
        bsp.bsp_select_mask(W, 5, 8, 0, 0.5)
    assert e.value.code == -6
    with pytest.raises(bsp.BspError) as e:
        bsp.bsp_mask_step(W, np.full((1, 1), 2, np.uint8), 8, 8)
    assert e.value.code == -3
