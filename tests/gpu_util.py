"""Helpers for the GPU parity tests: run a synthetic layer through libbsp and
compare with the CPU oracle."""
import numpy as np

import oracle

# Stated targets: fp32 1e-5, bf16 (fp32 accumulate) 2e-2, both relative.  An
# element-wise relative error is ill-posed where the exact value cancels to
# ~0, so the reference magnitude is max(|y|, rms(y)).
TOL = {"f32": 1e-5, "bf16": 2e-2}
# What the arithmetic should really achieve: one bf16 rounding of the result
# (2^-9) plus fp32 accumulation noise; used as a second, tighter gate.
TIGHT = {"f32": 4e-6, "bf16": 6e-3}


def to_device(c, X=None):
    import torch
    X = c.X if X is None else X
    t = torch.from_numpy(np.ascontiguousarray(X))
    if c.dtype == "bf16":
        t = t.to(torch.bfloat16)          # exact: values lie on the bf16 grid
    return t.cuda()


def to_host(Y):
    import torch
    return Y.to(torch.float32).cpu().numpy().astype(np.float64)


def make_layer(c, bias=True):
    import paper_2407_09453_amd as bsp
    return bsp.BspLayer(c.W, c.gamma, c.bo, c.bi, c.dtype, bias=c.bias if bias else None)


def gpu_conv(c, general=False, bias=True, layer=None):
    import torch
    layer = layer or make_layer(c, bias)
    Y = layer.conv2d(to_device(c), c.stride, c.pad, general=general)
    torch.cuda.synchronize()
    return to_host(Y)


def oracle_conv(c, bias=True):
    return oracle.conv2d(c.X, c.W, c.bias if bias else None, c.gamma, c.bo, c.bi, c.stride, c.pad)


def assert_close(y, ref, dtype, what=""):
    assert y.shape == ref.shape, (y.shape, ref.shape)
    assert np.isfinite(y).all(), what
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    scale = np.maximum(np.abs(ref), rms)
    err = np.abs(y - ref)
    bad = err > TOL[dtype] * scale
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} beyond {TOL[dtype]}; worst " \
        f"{(err / np.maximum(scale, 1e-300)).max():.3e} at {np.unravel_index(np.argmax(err), err.shape)}"
    tight = err > TIGHT[dtype] * scale + 1e-30
    assert not tight.any(), f"{what}: within the stated tolerance but {tight.sum()} elements " \
        f"beyond the derived bound {TIGHT[dtype]}; worst {(err / np.maximum(scale, 1e-300)).max():.3e}"
