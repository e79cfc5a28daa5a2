"""Host side of the 8-bit path: the C quantizer against the oracle's Eq. (8), the packer on
int8 codes against the oracle's independent packer, error codes (no GPU needed)."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp

GRANS = [(8, 8), (4, 16), (16, 4)]


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_quantizer_matches_oracle_bit_for_bit(bits):
    rng = np.random.default_rng(bits)
    W = (rng.standard_normal((64, 3, 3, 24)) * 0.05).astype(np.float32)
    W.reshape(-1)[:6] = np.float32([0.0, W.max(), -np.abs(W).max(), 1e-9, -1e-9, np.abs(W).max()])
    q, d = bsp.bsp_quantize(W, bits)
    q0, d0 = oracle.quantize_eq8(W, bits)
    assert d == d0 and q.dtype == np.int8 and (q == q0).all()


def test_quantizer_hand_example_and_ties():
    W = np.float32([0.5, -0.5, 0.009765625, 0.005859375, -0.005859375, 0.25])   # Delta = 2^-8
    q, d = bsp.bsp_quantize(W)
    assert d == 0.5 / 128
    # 128 -> 127 (clamped); 2.5 -> 2 and 1.5 -> 2 (ties to even); -1.5 -> -2
    assert q.tolist() == [127, -128, 2, 2, -2, 64]
    z, dz = bsp.bsp_quantize(np.zeros(7, np.float32))
    assert dz == 0.0 and not z.any()
    with pytest.raises(bsp.BspError) as e:
        bsp.bsp_quantize(W, 9)
    assert e.value.code == -2


@pytest.mark.parametrize("bo,bi", GRANS)
@pytest.mark.parametrize("O,I,H,K", [(64, 64, 3, 3), (20, 12, 2, 3), (48, 80, 1, 7), (16, 3, 7, 7)])
def test_pack_int8_codes_bit_exact_and_roundtrip(bo, bi, O, I, H, K):
    rng = np.random.default_rng(O + I + H)
    Wq = rng.integers(-128, 128, (O, H, K, I), dtype=np.int8)
    gamma = (rng.random((-(-O // bo), -(-I // bi))) < 0.5).astype(np.uint8)
    rp0, ci0, pl0 = oracle.pack_reference_i8(Wq, gamma, bo, bi)
    rp, ci, pl = bsp.bsp_pack(Wq, gamma, bo, bi, bsp.BSP_I8)
    assert pl.dtype == np.int8
    assert (rp == rp0).all() and (ci == ci0).all() and pl.tobytes() == pl0.tobytes()
    back = bsp.bsp_unpack(rp, ci, pl, O, H, K, I, bo, bi)
    keep = oracle.expand_mask(gamma, O, I, bo, bi)[:, None, None, :]
    assert back.dtype == np.int8 and (back == np.where(keep, Wq, 0)).all()
    plan = bsp.bsp_plan_build(rp, ci, pl, O, H, K, I, bo, bi)
    assert plan[15] == bsp.BSP_I8
    _check_i8_steps(plan, np.where(keep, Wq, 0), O, H, K, I)


def _check_i8_steps(plan, Wm, O, H, K, I):
    """Decode the int8 step section (16-channel chunks, four (chunk, tap) pairs a step, sixteen
    codes per lane) and rebuild the masked weights from it: every nonzero code must appear
    exactly where the descriptors say, and nothing else."""
    nstrips, slab, nslabs, nsteps = plan[8], plan[16], plan[17], plan[18]
    off_slab, off_xdesc, off_wfrag = plan[19], plan[20], plan[21]
    slab_chunks = slab // 16
    assert nslabs == -(-(-(-I // 16)) // slab_chunks) and (nsteps > 0 or not Wm.any())
    sp = plan[off_slab:off_slab + nstrips * (nslabs + 1)].reshape(nstrips, nslabs + 1)
    xd = plan[off_xdesc:off_xdesc + nsteps * 4].reshape(nsteps, 4)
    wf = plan[off_wfrag:off_wfrag + nsteps * 64 * 4].view(np.int8).reshape(nsteps, 4, 16, 16)
    Ip = -(-I // 16) * 16
    got = np.zeros((nstrips * 16, H, K, Ip), dtype=np.int64)
    seen = np.zeros((nstrips * 16, H, K, Ip), dtype=np.int64)
    for t in range(nstrips):
        for sl in range(nslabs):
            for st in range(sp[t, sl], sp[t, sl + 1]):
                for g in range(4):
                    d = int(xd[st, g])
                    c, r, k = (d & 0xFFFF) + sl * slab_chunks, (d >> 16) & 0xFF, (d >> 24) & 0xFF
                    frag = wf[st, g].astype(np.int64)               # [row j][16 codes]
                    if not frag.any():
                        continue                                     # padding pair or all-zero
                    got[t * 16:(t + 1) * 16, r, k, c * 16:(c + 1) * 16] += frag
                    seen[t * 16:(t + 1) * 16, r, k, c * 16:(c + 1) * 16] += 1
    assert seen.max() <= 1                                           # no pair listed twice
    want = np.zeros_like(got)
    want[:O, :, :, :I] = Wm
    assert (got == want).all()


def test_mixed_int8_and_float_types_are_refused():
    Wq = np.zeros((8, 1, 1, 8), dtype=np.int8)
    g = np.ones((1, 1), dtype=np.uint8)
    with pytest.raises(bsp.BspError) as e:
        bsp.bsp_pack(Wq, g, 8, 8, bsp.BSP_BF16)
    assert e.value.code == -5
    with pytest.raises(bsp.BspError) as e:
        bsp.bsp_pack(Wq.astype(np.float32), g, 8, 8, bsp.BSP_I8)
    assert e.value.code == -5
