"""Host side of libbsp (no GPU): the packer is bit-exact against the oracle's
independent numpy packer, its error paths return codes, the launch plan
addresses exactly the kept weights, and the library exports what the header
declares."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2407_09453_amd as bsp
from synthetic import draw_layer

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GRANS = [(8, 8), (4, 16), (16, 4)]


def _case(O, I, H, K, bo, bi, seed, kind="bernoulli", d=0.5):
    return draw_layer("t", B=1, L=max(H, 2), J=max(K, 2), I=I, O=O, H=H, K=K, bo=bo, bi=bi,
                      dtype="f32", mask_kind=kind, density=d, seed=seed)


def test_header_symbols_exported():
    import glob
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert [os.path.basename(h) for h in headers] == ["bsp.h", "bsp_bench.h"]
    text = "".join(open(h).read() for h in headers)
    names = set(re.findall(r"\b(bsp_[a-z0-9_]+)\s*\(", text))
    names -= {"bsp_weights"}
    assert {"bsp_pack", "bsp_fc", "bsp_conv2d"} <= names
    lib = ctypes.CDLL(bsp.lib_path())
    for n in sorted(names):
        assert hasattr(lib, n), n
    assert bsp.bsp_version() == 1
    assert set(bsp.binding.EXPORTS) == names


@pytest.mark.parametrize("bo,bi", GRANS)
@pytest.mark.parametrize("O,I,H,K", [(64, 64, 3, 3), (32, 48, 1, 1), (20, 12, 2, 3),
                                     (1000, 40, 1, 1), (16, 3, 7, 7), (48, 80, 1, 7)])
@pytest.mark.parametrize("pd", ["f32", "bf16"])
def test_pack_bit_exact_vs_oracle_packer(bo, bi, O, I, H, K, pd):
    c = _case(O, I, H, K, bo, bi, seed=O * 7 + I + H)
    rp0, ci0, pl0 = oracle.pack_reference(c.W, c.gamma, bo, bi, pd)
    rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, bo, bi, bsp.BSP_F32 if pd == "f32" else bsp.BSP_BF16)
    assert rp.dtype == np.int32 and ci.dtype == np.int32
    assert (rp == rp0).all() and (ci == ci0).all()
    assert pl.shape == pl0.shape
    a = pl.view(np.uint32) if pd == "f32" else pl
    b = pl0.view(np.uint32) if pd == "f32" else pl0
    assert (a == b).all()
    assert bsp.bsp_pack_count(c.gamma, O, I, bo, bi) == c.nnzb == rp[-1]
    assert bsp.bsp_validate(rp, ci, O, I, bo, bi) == 0


@pytest.mark.parametrize("bo,bi", GRANS)
def test_unpack_roundtrip_is_masked_weights(bo, bi):
    c = _case(40, 56, 3, 1, bo, bi, seed=3)
    for code, pd in ((bsp.BSP_F32, "f32"), (bsp.BSP_BF16, "bf16")):
        rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, bo, bi, code)
        Wd = bsp.bsp_unpack(rp, ci, pl, 40, 3, 1, 56, bo, bi)
        Wm = oracle.apply_mask(c.W, c.gamma, bo, bi)
        if pd == "bf16":
            assert (Wd == oracle.bf16_bits_rne(Wm).reshape(Wm.shape)).all()
        else:
            assert (Wd.view(np.uint32) == Wm.view(np.uint32)).all()


def test_pack_bf16_input_widens_exactly():
    c = _case(16, 16, 1, 1, 8, 8, seed=5, kind="ones")
    Wb = oracle.bf16_bits_rne(c.W).reshape(c.W.shape)
    rp, ci, pl = bsp.bsp_pack(Wb, c.gamma, 8, 8, bsp.BSP_F32)
    ref = oracle.pack_reference(oracle.bf16_bits_to_f32(Wb).reshape(c.W.shape), c.gamma, 8, 8)[2]
    assert (pl.view(np.uint32) == ref.view(np.uint32)).all()


def test_structure_follows_mask_not_values():
    c = _case(16, 16, 1, 1, 8, 8, seed=6, kind="ones")
    W = c.W.copy()
    W[:8, :, :, :8] = 0.0                       # a kept block of zeros is stored
    g = np.array([[1, 0], [1, 1]], dtype=np.uint8)   # a zeroed block with values is dropped
    rp, ci, pl = bsp.bsp_pack(W, g, 8, 8)
    assert list(rp) == [0, 1, 3] and list(ci) == [0, 0, 1]
    assert (pl[0] == 0).all()


def test_error_codes():
    lib = bsp.load_library()
    g = np.ones((2, 2), dtype=np.uint8)
    n = ctypes.c_int64()
    assert lib.bsp_pack_count(None, 16, 16, 8, 8, ctypes.byref(n)) == -1
    assert lib.bsp_pack_count(g.ctypes.data, 16, 16, 8, 4, ctypes.byref(n)) == -6
    assert lib.bsp_pack_count(g.ctypes.data, 0, 16, 8, 8, ctypes.byref(n)) == -2
    g2 = g.copy()
    g2[1, 1] = 2
    assert lib.bsp_pack_count(g2.ctypes.data, 16, 16, 8, 8, ctypes.byref(n)) == -3
    W = np.zeros((16, 1, 1, 16), dtype=np.float32)
    rp = np.zeros(3, dtype=np.int32)
    ci = np.zeros(4, dtype=np.int32)
    pl = np.zeros(4 * 64, dtype=np.float32)
    args = lambda **kw: [W.ctypes.data, kw.get("wd", 0), g.ctypes.data, 16, 1, 1, 16, 8, 8,
                         kw.get("pd", 0), rp.ctypes.data, ci.ctypes.data, kw.get("cc", 4),
                         pl.ctypes.data, kw.get("pc", pl.nbytes)]
    assert lib.bsp_pack(*args()) == 0
    assert lib.bsp_pack(*args(pc=pl.nbytes - 1)) == -7
    assert lib.bsp_pack(*args(cc=3)) == -7
    assert lib.bsp_pack(*args(pd=7)) == -5
    assert lib.bsp_pack(*args(wd=2)) == -5
    # malformed index arrays
    assert bsp.bsp_validate([0, 2, 4], [0, 1, 0, 1], 16, 16, 8, 8) == 0
    assert bsp.bsp_validate([1, 2, 4], [0, 1, 0, 1], 16, 16, 8, 8) == -4
    assert bsp.bsp_validate([0, 3, 2], [0, 1, 0, 1], 16, 16, 8, 8) == -4
    assert bsp.bsp_validate([0, 2, 4], [1, 0, 0, 1], 16, 16, 8, 8) == -4
    assert bsp.bsp_validate([0, 2, 4], [0, 2, 0, 1], 16, 16, 8, 8) == -4
    assert bsp.bsp_validate([0, 2, 4], [0, 0, 0, 1], 16, 16, 8, 8) == -4
    assert "granularity" in bsp.bsp_strerror(-6)
    with pytest.raises(bsp.BspError):
        bsp.bsp_plan_build([0, 3, 2], [0, 1, 0, 1], np.zeros(4 * 64, np.float32), 16, 1, 1, 16, 8, 8)
    # device entry points validate before touching the GPU
    w = bsp.bsp_weights()
    assert lib.bsp_fc(None, 16, None, 16, 1, None) == -1
    assert lib.bsp_fc(ctypes.byref(w), None, None, 16, 1, None) == -1
    w.O, w.I, w.H, w.K, w.bo, w.bi, w.dtype = 16, 16, 1, 1, 8, 8, 0
    w.plan, w.plan_bytes, w.payload, w.nnzb = 4096, 1024, 4096, 1
    assert lib.bsp_fc(ctypes.byref(w), 4096, None, 8192, 1, None) == -1    # no host copy of the plan
    w.plan_host = 4096
    assert lib.bsp_fc(ctypes.byref(w), 4096, None, 8192, -1, None) == -2
    assert lib.bsp_fc(ctypes.byref(w), 4100, None, 8192, 1, None) == -9
    w.bo = 2
    assert lib.bsp_fc(ctypes.byref(w), 4096, None, 8192, 1, None) == -6
    w.bo, w.dtype = 8, 9
    assert lib.bsp_fc(ctypes.byref(w), 4096, None, 8192, 1, None) == -5
    w.dtype, w.H = 0, 3
    assert lib.bsp_fc(ctypes.byref(w), 4096, None, 8192, 1, None) == -2
    assert lib.bsp_conv2d(ctypes.byref(w), 4096, None, 8192, 1, 2, 2, 1, 1, 0, 0, None) == -2
    assert lib.bsp_conv2d(ctypes.byref(w), 4096, None, 8192, 1, 8, 8, 0, 1, 0, 0, None) == -2


# --------------------------------------------------------------------------- plan
def _decode_plan(plan, payload, O, H, K, I, bo, bi):
    """Rebuild dense weights from the plan's offsets alone (test-side reading
    of the plan format: strips of 16 output channels, chunks of 8 input
    channels, up to four sources per cell)."""
    hdr = plan[:32]
    assert hdr[0] == 0x42535032
    nstrips, nchunks = hdr[8], hdr[9]
    sp = plan[hdr[10]:hdr[10] + nstrips + 1]
    xc = plan[hdr[11]:hdr[11] + nchunks]
    src = plan[hdr[12]:hdr[12] + 4 * nchunks].reshape(-1, 4)
    flat = payload.reshape(-1)
    HK = H * K
    W = np.zeros((16 * nstrips, HK, 8 * (-(-I // 8))), dtype=payload.dtype)
    visited = 0
    for t in range(nstrips):
        assert sp[t] <= sp[t + 1]
        cols = xc[sp[t]:sp[t + 1]]
        assert (np.diff(cols) > 0).all()
        for e in range(sp[t], sp[t + 1]):
            assert (src[e] >= 0).any()
            for jn in range(16):
                for tap in range(HK):
                    if bi >= 8:
                        s, r = jn // bo, jn % bo
                        if src[e, s] >= 0:
                            o = src[e, s] + (r * HK + tap) * bi
                            W[t * 16 + jn, tap, xc[e] * 8:xc[e] * 8 + 8] = flat[o:o + 8]
                            visited += 8
                    else:
                        for s in range(2):
                            if src[e, s] >= 0:
                                o = src[e, s] + (jn * HK + tap) * 4
                                W[t * 16 + jn, tap, xc[e] * 8 + 4 * s:xc[e] * 8 + 4 * s + 4] = flat[o:o + 4]
                                visited += 4
    return W[:O, :, :I].reshape(O, H, K, I), visited


@pytest.mark.parametrize("bo,bi", GRANS)
@pytest.mark.parametrize("O,I,H,K", [(64, 64, 3, 3), (40, 24, 1, 1), (20, 12, 2, 1), (1000, 40, 1, 1)])
def test_plan_addresses_exactly_the_kept_weights(bo, bi, O, I, H, K):
    c = _case(O, I, H, K, bo, bi, seed=O + I + bo)
    rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, bo, bi)
    plan = bsp.bsp_plan_build(rp, ci, pl, O, H, K, I, bo, bi)
    assert plan.nbytes == bsp.bsp_plan_size(rp, ci, O, H, K, I, bo, bi, bsp.BSP_F32)
    assert plan[18] == 0                      # fp32: no step section
    Wd, visited = _decode_plan(plan, pl, O, H, K, I, bo, bi)
    Wm = oracle.apply_mask(c.W, c.gamma, bo, bi)
    assert (Wd.view(np.uint32) == Wm.view(np.uint32)).all()
    # every stored element is reached exactly once, except those of chunks that lie wholly past I
    nxc = -(-I // 8)
    stored = sum(min(bi, 8 * nxc - int(cj) * bi) for cj in ci) * bo * H * K
    assert visited == stored


def test_plan_of_empty_and_full_masks():
    for kind in ("zeros", "ones"):
        c = _case(32, 32, 1, 1, 8, 8, seed=1, kind=kind)
        rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, 8, 8)
        plan = bsp.bsp_plan_build(rp, ci, pl, 32, 1, 1, 32, 8, 8)
        assert plan[9] == (0 if kind == "zeros" else 2 * 4)


def _decode_steps(plan, O, H, K, I):
    """Rebuild dense bf16 weights from the step section alone: slab_ptr gives
    each (strip, slab) its steps, xdesc says which (chunk, tap) each 16-lane
    group of a step multiplies, wfrag holds the 16 x 8 weights for it."""
    hdr = plan[:32]
    nstrips, slab, nslabs, nsteps = hdr[8], hdr[16], hdr[17], hdr[18]
    sp = plan[hdr[19]:hdr[19] + nstrips * (nslabs + 1)].reshape(nstrips, nslabs + 1)
    xd = plan[hdr[20]:hdr[20] + 4 * nsteps].reshape(nsteps, 4)
    wf = plan[hdr[21]:hdr[21] + nsteps * 256].view(np.uint16).reshape(nsteps, 4, 16, 8)
    W = np.zeros((16 * nstrips, H, K, 8 * (-(-I // 8))), dtype=np.uint16)
    seen = np.zeros((16 * nstrips, H, K, W.shape[3] // 8), dtype=np.int32)
    assert sp[0, 0] == 0 and sp[-1, -1] == nsteps
    assert (np.diff(sp.reshape(-1)) >= 0).all()
    nonnull = 0
    for t in range(nstrips):
        for sl in range(nslabs):
            for st in range(sp[t, sl], sp[t, sl + 1]):
                for g in range(4):
                    frag = wf[st, g]
                    d = int(xd[st, g])
                    xc, th, tw = (d & 0xFFFF) + sl * (slab // 8), (d >> 16) & 0xFF, (d >> 24) & 0xFF
                    if not frag.any() and d == 0:
                        continue            # padding pair (or a genuinely all-zero chunk 0, tap 0)
                    assert (d & 0xFFFF) < slab // 8 and th < H and tw < K
                    W[16 * t:16 * t + 16, th, tw, 8 * xc:8 * xc + 8] = frag
                    seen[16 * t:16 * t + 16, th, tw, xc] += 1
                    nonnull += 1
    assert seen.max() <= 1
    return W[:O, :, :, :I], nonnull


@pytest.mark.parametrize("bo,bi", GRANS)
@pytest.mark.parametrize("O,I,H,K", [(64, 64, 3, 3), (40, 24, 1, 1), (48, 320, 1, 1),
                                     (32, 272, 3, 3), (1000, 40, 1, 1), (20, 16, 2, 1)])
def test_step_section_holds_exactly_the_kept_weights(bo, bi, O, I, H, K):
    c = _case(O, I, H, K, bo, bi, seed=O + I + bo + 1)
    rp, ci, pl = bsp.bsp_pack(c.W, c.gamma, bo, bi, bsp.BSP_BF16)
    plan = bsp.bsp_plan_build(rp, ci, pl, O, H, K, I, bo, bi)
    assert plan.nbytes == bsp.bsp_plan_size(rp, ci, O, H, K, I, bo, bi, bsp.BSP_BF16)
    hdr = plan[:32]
    assert hdr[16] == min(-(-I // 8) * 8, 64 if H * K > 1 else 256)
    assert hdr[17] == -(-(-(-I // 8)) // (hdr[16] // 8))
    Wd, nonnull = _decode_steps(plan, O, H, K, I)
    Wm = oracle.bf16_bits_rne(oracle.apply_mask(c.W, c.gamma, bo, bi)).reshape(c.W.shape)
    assert (Wd == Wm).all()
    # steps are the pairs of each (strip, slab) rounded up to fours, nothing more
    nstrips, nslabs = hdr[8], hdr[17]
    sp = plan[hdr[10]:hdr[10] + nstrips + 1]
    xc = plan[hdr[11]:hdr[11] + hdr[9]]
    want = worst = 0
    for t in range(nstrips):
        cols = xc[sp[t]:sp[t + 1]] // (hdr[16] // 8)
        for sl in range(nslabs):
            st = -(-int((cols == sl).sum()) * H * K // 4)
            want += st
            worst = max(worst, st)
    assert hdr[18] == want
    assert hdr[23] == worst
