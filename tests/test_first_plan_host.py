"""Host: the plan's thin-input section (layers with at most four input channels) holds the
masked weights in the operand order the kernel expects; checked against the dense W directly."""
import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp
from synthetic import draw_layer


def _section(c, bo, bi):
    row_ptr, col_idx, payload = bsp.bsp_pack(c.W, c.gamma, bo, bi, bsp.BSP_BF16)
    plan = bsp.bsp_plan_build(row_ptr, col_idx, payload, c.O, c.H, c.K, c.I, bo, bi)
    off = int(plan[25])
    return plan, off


@pytest.mark.parametrize("bo,bi", [(8, 8), (4, 16), (16, 4)])
@pytest.mark.parametrize("I,O,H,K", [(3, 64, 3, 3), (3, 64, 7, 7), (3, 32, 3, 3), (1, 32, 5, 3), (4, 64, 3, 3)])
def test_first_section_holds_masked_weights(bo, bi, I, O, H, K):
    c = draw_layer("first", B=1, L=8, J=8, I=I, O=O, H=H, K=K, stride=1, pad=1, bo=bo, bi=bi,
                   dtype="bf16", seed=4100 + I + O + H)
    rng = np.random.default_rng(7)
    c.gamma[:] = rng.integers(0, 2, size=c.gamma.shape)      # whole block rows dropped
    c.gamma[0, 0] = 1
    plan, off = _section(c, bo, bi)
    assert off > 0 and off % 4 == 0
    NS, steps, Kt, off_frag = (int(v) for v in plan[off:off + 4])
    assert (NS, steps, Kt) == (O // 16, -(-H * K * I // 32), H * K * I)
    frag = plan[off + off_frag:off + off_frag + steps * NS * 64 * 4].view(np.uint16).reshape(steps, NS, 64, 8)
    Wb = oracle.round_to_storage(c.W.astype(np.float64), "bf16").astype(np.float32)
    Wbits = (Wb.view(np.uint32) >> 16).astype(np.uint16)      # bf16 patterns of the rounded weights
    flat = Wbits.reshape(O, H * K * I)
    for t in range(steps):
        for s in range(NS):
            for lane in range(64):
                g, j = lane >> 4, lane & 15
                ch = (j >> 2) * 4 * NS + 4 * s + (j & 3)
                kept = c.gamma[ch // bo, 0] != 0
                for e in range(8):
                    k = 32 * t + 8 * g + e
                    want = flat[ch, k] if (kept and k < Kt) else 0
                    assert frag[t, s, lane, e] == want, (t, s, lane, e)


def test_first_section_absent_for_wide_inputs():
    c = draw_layer("first", B=1, L=8, J=8, I=8, O=64, H=3, K=3, stride=1, pad=1, dtype="bf16", seed=1)
    plan, off = _section(c, 8, 8)
    assert off == 0
    c = draw_layer("first", B=1, L=8, J=8, I=3, O=24, H=3, K=3, stride=1, pad=1, dtype="bf16", seed=1)
    plan, off = _section(c, 8, 8)
    assert off == 0    # output channels that do not fill 16-row tiles
