"""The row-band section of the launch plan, decoded on the host: strips are groups of block
rows, column steps list (unit, dx) items, rfrag holds the weights in operand order.  Rebuilt
from the section alone, the weights must equal the masked bf16 weights bit for bit, each
kept element exactly once; the 16x4 granularity must carry no zero-filled unit."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp
from synthetic import draw_layer

GRANS = [(8, 8), (4, 16), (16, 4)]


def _rows_section(plan):
    off = int(plan[24])
    assert off > 0 and off % 4 == 0
    return plan[off:], off


def _decode_rows(plan, O, H, K, I, bo, bi):
    rs, _ = _rows_section(plan)
    nstrips, slab, nslabs, ncs = (int(v) for v in rs[0:4])
    o_strip, o_slab, o_desc, o_frag, cw = (int(v) for v in rs[5:10])
    assert cw == (4 if bi == 4 else 8) and o_frag % 4 == 0
    ips = 32 // cw
    rstrip = rs[o_strip:o_strip + nstrips * 4].reshape(nstrips, 4)
    rslab = rs[o_slab:o_slab + nstrips * (nslabs + 1)].reshape(nstrips, nslabs + 1)
    rdesc = rs[o_desc:o_desc + ncs * 4].reshape(ncs, 4)
    rfrag = rs[o_frag:o_frag + ncs * H * 256].view(np.uint16).reshape(ncs, H, 64, 8)
    assert rslab[0, 0] == 0 and rslab[-1, -1] == ncs
    assert (np.diff(rslab.reshape(-1)) >= 0).all()
    W = np.zeros((O, H, K, I), dtype=np.uint16)
    seen = np.zeros((O, H, K, I), dtype=np.int32)
    chans_seen = []
    items = 0
    for t in range(nstrips):
        for q in range(4):
            if rstrip[t, q] >= 0:
                chans_seen.extend(range(rstrip[t, q], rstrip[t, q] + 4))
        for sl in range(nslabs):
            for cs in range(rslab[t, sl], rslab[t, sl + 1]):
                for q in range(4):
                    d = int(rdesc[cs, q]) & 0xFFFFFFFF
                    for h in range(ips // 4):
                        code = (d >> (16 * h)) & 0xFFFF
                        assert cw == 4 or d >> 16 == 0
                        dx, in_slab = code >> 8, code & 0xFF
                        unit = in_slab + sl * (slab // cw)
                        assert dx < K and in_slab < slab // cw
                        vals = rfrag[cs, :, q * 16:(q + 1) * 16, h * cw:(h + 1) * cw]   # [H][16][cw]
                        if code == 0 and not vals.any():
                            continue        # padding item (or an all-zero first item)
                        items += 1
                        for j in range(16):
                            ch = rstrip[t, j // 4]
                            if ch < 0:
                                assert not vals[:, j].any()
                                continue
                            o = ch + j % 4
                            W[o, :, dx, unit * cw:(unit + 1) * cw] = vals[:, j]
                            seen[o, :, dx, unit * cw:(unit + 1) * cw] += 1
    assert sorted(chans_seen) == list(range(O)), "every output channel belongs to one strip row"
    assert seen.max() <= 1
    return W, items, rs


@pytest.mark.parametrize("bo,bi", GRANS)
@pytest.mark.parametrize("O,I,H,K", [(64, 64, 3, 3), (40, 24, 1, 1), (48, 320, 1, 1),
                                     (32, 272, 3, 3), (1000, 40, 1, 1), (24, 16, 3, 1),
                                     (16, 136, 1, 7)])
def test_rows_section_holds_exactly_the_kept_weights(bo, bi, O, I, H, K):
    c = draw_layer("t", B=1, L=4, J=4, I=I, O=O, H=H, K=K, bo=bo, bi=bi, dtype="bf16",
                   seed=O + I + bo + 5, draw_x=False)
    rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, bo, bi, bsp.BSP_BF16)
    plan = bsp.bsp_plan_build(rp, ci, pl, O, H, K, I, bo, bi)
    assert plan.nbytes == bsp.bsp_plan_size(rp, ci, O, H, K, I, bo, bi, bsp.BSP_BF16)
    Wd, items, rs = _decode_rows(plan, O, H, K, I, bo, bi)
    Wm = oracle.bf16_bits_rne(oracle.apply_mask(c.W, c.gamma, bo, bi)).reshape(c.W.shape)
    assert (Wd == Wm).all()
    kept_units, union_units = int(rs[12]), int(rs[13])
    cw = 4 if bi == 4 else 8
    nunits = -(-I // cw)
    assert kept_units == sum(min(nunits, (int(cj) + 1) * bi // cw) - int(cj) * bi // cw for cj in ci)
    if bo == 16:
        assert union_units == kept_units, "16x4 blocks: a strip is one block row, nothing is filled"
    else:
        assert kept_units // (16 // bo) <= union_units <= kept_units


def test_grouping_puts_rows_with_equal_columns_together():
    # block rows 0..7: rows r and r+4 keep the same columns, so the best strips pair them and the
    # strips run no zero-filled unit at all
    O, I = 64, 128
    rng = np.random.default_rng(3)
    half = (rng.random((4, I // 8)) < 0.5).astype(np.uint8)
    gamma = np.concatenate([half, half], axis=0)
    W = rng.standard_normal((O, 1, 1, I)).astype(np.float32)
    rp, ci, pl = bsp.bsp_pack(W, gamma, 8, 8, bsp.BSP_BF16)
    plan = bsp.bsp_plan_build(rp, ci, pl, O, 1, 1, I, 8, 8)
    rs, _ = _rows_section(plan)
    assert int(rs[13]) * 2 == int(rs[12]) == int(gamma.sum())
    rstrip = rs[int(rs[5]):int(rs[5]) + int(rs[0]) * 4].reshape(-1, 4)
    for row in rstrip:
        assert abs(int(row[2]) - int(row[0])) == 32      # rows r and r+4: channels 32 apart


def test_no_rows_section_where_it_cannot_serve():
    for (O, I, dt) in [(64, 20, "bf16"), (20, 64, "bf16"), (64, 64, "f32")]:
        c = draw_layer("t", B=1, L=1, J=1, I=I, O=O, dtype=dt, seed=1, draw_x=False)
        code = bsp.BSP_BF16 if dt == "bf16" else bsp.BSP_F32
        rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, 8, 8, code)
        plan = bsp.bsp_plan_build(rp, ci, pl, O, 1, 1, I, 8, 8)
        assert plan[24] == 0


@pytest.mark.parametrize("bo,bi", GRANS)
def test_pointwise_layers_keep_one_slab_and_windows_of_64_channels(bo, bi):
    """A 1x1 layer's section has all input channels in one slab (up to 256 units) and its
    strips in window order: strip s produces channels of [64 * (s // 4), 64 * (s // 4) + 64)
    only, so four consecutive strips cover whole 128-byte lines of the output."""
    O, I = 200, 1024 if bi == 4 else 2048
    c = draw_layer("t", B=1, L=2, J=2, I=I, O=O, H=1, K=1, bo=bo, bi=bi, dtype="bf16", seed=77,
                   draw_x=False)
    rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, bo, bi, bsp.BSP_BF16)
    plan = bsp.bsp_plan_build(rp, ci, pl, O, 1, 1, I, bo, bi)
    rs, _ = _rows_section(plan)
    nstrips, slab, nslabs = (int(v) for v in rs[0:3])
    assert slab == I and nslabs == 1 and int(rs[14]) == 4
    assert nstrips == -(-O // 16)
    rstrip = rs[int(rs[5]):int(rs[5]) + nstrips * 4].reshape(nstrips, 4)
    for s in range(nstrips):
        ch = rstrip[s][rstrip[s] >= 0]
        assert len(ch) and (ch // 64 == s // 4).all(), (s, rstrip[s])
    Wd, _, _ = _decode_rows(plan, O, 1, 1, I, bo, bi)
    Wm = oracle.bf16_bits_rne(oracle.apply_mask(c.W, c.gamma, bo, bi)).reshape(c.W.shape)
    assert (Wd == Wm).all()
    # wider layers than one descriptor can address get a second slab (served by other kernels)
    c = draw_layer("t", B=1, L=2, J=2, I=2 * I, O=16, H=1, K=1, bo=bo, bi=bi, dtype="bf16", seed=78,
                   draw_x=False)
    rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, bo, bi, bsp.BSP_BF16)
    rs, _ = _rows_section(bsp.bsp_plan_build(rp, ci, pl, 16, 1, 1, 2 * I, bo, bi))
    assert int(rs[1]) == I and int(rs[2]) == 2
    # windows do not apply to layers with a window of taps
    c = draw_layer("t", B=1, L=4, J=4, I=64, O=128, H=3, K=3, bo=bo, bi=bi, dtype="bf16", seed=79,
                   draw_x=False)
    rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, bo, bi, bsp.BSP_BF16)
    rs, _ = _rows_section(bsp.bsp_plan_build(rp, ci, pl, 128, 3, 3, 64, bo, bi))
    assert int(rs[14]) == 0
