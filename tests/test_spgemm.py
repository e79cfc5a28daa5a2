"""Block-sparse x block-sparse product: host segment pointers (CPU) and the HIP kernel against
the oracle (GPU)."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp


def _draw(Ra, Rb, N, seed, da=0.5, db=0.5):
    rng = np.random.default_rng(seed)
    A = oracle.round_to_storage(rng.standard_normal((Ra * 8, N * 8)), "bf16").astype(np.float32)
    B = oracle.round_to_storage(rng.standard_normal((Rb * 8, N * 8)), "bf16").astype(np.float32)
    gamma = (rng.random((Ra, N)) < da).astype(np.uint8)
    omega = (rng.random((Rb, N)) < db).astype(np.uint8)
    return A, gamma, B, omega


def test_segment_pointers_host():
    """seg_ptr[r][s] is where row r's kept blocks with column >= 16 s start: checked against a
    search of the mask itself, on a shape with a ragged last sixteen."""
    A, gamma, _, _ = _draw(5, 3, 37, 1)
    rp, ci, pl = bsp.bsp_pack(A.reshape(40, 1, 1, 37 * 8), gamma, 8, 8, bsp.BSP_BF16)
    seg = bsp.bsp_bcsr_segments(rp, ci, 5, 37)
    assert seg.shape == (5, 4)
    for r in range(5):
        for s in range(4):
            assert seg[r, s] == rp[r] + int(gamma[r, :16 * s].sum())
        assert seg[r, 0] == rp[r] and seg[r, 3] == rp[r + 1]
        for s in range(3):
            cols = ci[seg[r, s]:seg[r, s + 1]]
            assert ((cols >= 16 * s) & (cols < 16 * s + 16)).all()
            assert cols.tolist() == [c for c in range(16 * s, min(16 * s + 16, 37)) if gamma[r, c]]
            for n, c in zip(range(seg[r, s], seg[r, s + 1]), cols):
                blk = oracle.bf16_bits_to_f32(pl[n].reshape(8, 8))
                assert (blk == A[r * 8:(r + 1) * 8, c * 8:(c + 1) * 8]).all()
    with pytest.raises(bsp.BspError) as e:
        bsp.bsp_bcsr_segments(np.array([0, 2, 1], np.int32), ci, 2, 37)
    assert e.value.code == -4


@pytest.mark.gpu
@pytest.mark.parametrize("Ra,Rb,N", [(2, 2, 4), (5, 3, 7), (16, 16, 16), (33, 17, 21), (64, 64, 128), (40, 150, 200)])
def test_spgemm_vs_oracle(Ra, Rb, N):
    import torch
    for da, db in ((0.5, 0.5), (0.1, 0.9), (1.0, 1.0), (0.0, 0.5)):
        A, gamma, B, omega = _draw(Ra, Rb, N, Ra * 100 + N, da, db)
        Am, Bm = bsp.BspMatrix(A, gamma), bsp.BspMatrix(B, omega)
        C = Am.matmul_nt(Bm)
        torch.cuda.synchronize()
        want = oracle.spgemm_nt(A, gamma, B, omega, 8)
        got = C.cpu().numpy().astype(np.float64)
        assert got.shape == want.shape
        scale = np.maximum(np.abs(want), np.sqrt(np.mean(want * want)) + 1e-30)
        # exact bf16 products, fp32 accumulation of at most 8 N terms
        assert (np.abs(got - want) <= 1e-5 * scale + 1e-30).all(), (da, db)
        if da == 0.0:
            assert not got.any()


@pytest.mark.gpu
def test_spgemm_ignores_masked_contents_and_writes_every_element():
    import torch
    A, gamma, B, omega = _draw(9, 7, 11, 5)
    C0 = bsp.BspMatrix(A, gamma).matmul_nt(bsp.BspMatrix(B, omega))
    A2 = np.where(np.kron(gamma, np.ones((8, 8))) > 0, A, np.float32(3e38))
    out = torch.full((72, 56), float("nan"), device="cuda")
    C1 = bsp.BspMatrix(A2, gamma).matmul_nt(bsp.BspMatrix(B, omega), out=out)
    torch.cuda.synchronize()
    assert torch.equal(C0, C1) and not torch.isnan(C1).any()
