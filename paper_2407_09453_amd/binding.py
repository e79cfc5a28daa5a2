"""ctypes binding of libbsp.so: same names as the C ABI, marshalling only.

Host functions take and return numpy arrays.  Device functions take raw
device addresses (ints) plus a ``bsp_weights`` struct; ``BspLayer`` is a small
convenience holder that packs a layer on the host, uploads the arrays with
torch (used for device memory and streams only) and fills the struct.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

BSP_F32 = 0
BSP_BF16 = 1
BSP_I8 = 2
BSP_I32 = 3
BSP_KERNEL_ROWS, BSP_KERNEL_LDS, BSP_KERNEL_TILE, BSP_KERNEL_FC, BSP_KERNEL_PW = 1, 2, 4, 8, 16
BSP_KERNEL_CHAIN = 32
BSP_KERNEL_BAND = 64
BSP_KERNEL_FIRST = 128

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libbsp.so")
_lib = None

EXPORTS = ("bsp_strerror", "bsp_version", "bsp_pack_count", "bsp_pack", "bsp_unpack",
           "bsp_validate", "bsp_plan_size", "bsp_plan_build", "bsp_fc", "bsp_conv2d",
           "bsp_conv2d_general", "bsp_quantize", "bsp_conv2d_i8", "bsp_fc_i8",
           "bsp_block_importance", "bsp_select_mask", "bsp_mask_step", "bsp_conv2d_fused",
           "bsp_fc_fused", "bsp_fc_fused_static", "bsp_bcsr_segments", "bsp_spgemm_nt",
           "bsp_conv2d_only", "bsp_bottleneck", "bsp_bench_copy", "bsp_bench_mfma_bf16", "bsp_bench_lds_read")


class BspError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {bsp_strerror(code)} ({code})")


class bsp_weights(ctypes.Structure):
    _fields_ = [("O", ctypes.c_int32), ("I", ctypes.c_int32), ("H", ctypes.c_int32),
                ("K", ctypes.c_int32), ("bo", ctypes.c_int32), ("bi", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("kernels", ctypes.c_int32),
                ("nnzb", ctypes.c_int64), ("row_ptr", ctypes.c_void_p),
                ("col_idx", ctypes.c_void_p), ("payload", ctypes.c_void_p),
                ("plan", ctypes.c_void_p), ("plan_bytes", ctypes.c_int64),
                ("plan_host", ctypes.c_void_p)]


class bsp_bcsr(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int32), ("cols", ctypes.c_int32), ("k", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("nnzb", ctypes.c_int64), ("row_ptr", ctypes.c_void_p),
                ("col_idx", ctypes.c_void_p), ("payload", ctypes.c_void_p),
                ("seg_ptr", ctypes.c_void_p)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libbsp.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("BSP_LIBRARY", _LIB_PATH)   # override: a differently built libbsp.so
    # libbsp launches on streams and memory that torch owns, so both must talk to the same
    # copy of the HIP runtime: torch ships its own, and whichever is loaded first serves the
    # whole process.  Loading libbsp first would bring in the system copy and leave torch's
    # handles meaningless to it (launches then fail).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it with "
            "`python -m paper_2407_09453_amd.build` (hipcc, gfx950)")
    lib = ctypes.CDLL(path)
    i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
    lib.bsp_strerror.restype = ctypes.c_char_p
    lib.bsp_strerror.argtypes = [ctypes.c_int]
    lib.bsp_version.restype = ctypes.c_int
    lib.bsp_version.argtypes = []
    lib.bsp_pack_count.restype = ctypes.c_int
    lib.bsp_pack_count.argtypes = [vp, i32, i32, i32, i32, ctypes.POINTER(i64)]
    lib.bsp_pack.restype = ctypes.c_int
    lib.bsp_pack.argtypes = [vp, i32, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, i64, vp, i64]
    lib.bsp_unpack.restype = ctypes.c_int
    lib.bsp_unpack.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp]
    lib.bsp_validate.restype = ctypes.c_int
    lib.bsp_validate.argtypes = [vp, vp, i32, i32, i32, i32]
    lib.bsp_plan_size.restype = ctypes.c_int
    lib.bsp_plan_size.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, ctypes.POINTER(i64)]
    lib.bsp_plan_build.restype = ctypes.c_int
    lib.bsp_plan_build.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, i64]
    wp = ctypes.POINTER(bsp_weights)
    lib.bsp_fc.restype = ctypes.c_int
    lib.bsp_fc.argtypes = [wp, vp, vp, vp, i32, vp]
    for name in ("bsp_conv2d", "bsp_conv2d_general"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [wp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp]
    f64 = ctypes.c_double
    lib.bsp_bcsr_segments.restype = ctypes.c_int
    lib.bsp_bcsr_segments.argtypes = [vp, vp, i32, i32, vp]
    lib.bsp_spgemm_nt.restype = ctypes.c_int
    lib.bsp_spgemm_nt.argtypes = [ctypes.POINTER(bsp_bcsr), ctypes.POINTER(bsp_bcsr), vp, vp]
    lib.bsp_conv2d_fused.restype = ctypes.c_int
    lib.bsp_conv2d_fused.argtypes = [wp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i32, i32, i32, vp]
    lib.bsp_conv2d_only.restype = ctypes.c_int
    lib.bsp_conv2d_only.argtypes = [wp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i32, i32, i32,
                                    i32, vp]
    lib.bsp_bottleneck.restype = ctypes.c_int
    lib.bsp_bottleneck.argtypes = [wp, wp, wp, vp, vp, vp, vp, vp, i32, vp, i32, i32, i32, vp]
    lib.bsp_fc_fused.restype = ctypes.c_int
    lib.bsp_fc_fused.argtypes = [wp, vp, vp, vp, i32, vp, i32, vp]
    lib.bsp_fc_fused_static.restype = ctypes.c_int
    lib.bsp_fc_fused_static.argtypes = [wp, vp, vp, vp, i32, vp, i32, vp]
    lib.bsp_block_importance.restype = ctypes.c_int
    lib.bsp_block_importance.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp]
    lib.bsp_select_mask.restype = ctypes.c_int
    lib.bsp_select_mask.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, f64, i32, vp]
    lib.bsp_mask_step.restype = ctypes.c_int
    lib.bsp_mask_step.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, f64, vp,
                                  ctypes.POINTER(i32)]
    lib.bsp_quantize.restype = ctypes.c_int
    lib.bsp_quantize.argtypes = [vp, i64, i32, vp, ctypes.POINTER(ctypes.c_double)]
    lib.bsp_conv2d_i8.restype = ctypes.c_int
    lib.bsp_conv2d_i8.argtypes = [wp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, vp]
    lib.bsp_fc_i8.restype = ctypes.c_int
    lib.bsp_fc_i8.argtypes = [wp, vp, vp, vp, i32, i32, i32, vp]
    lib.bsp_bench_copy.restype = ctypes.c_int
    lib.bsp_bench_copy.argtypes = [vp, vp, i64, vp]
    lib.bsp_bench_mfma_bf16.restype = ctypes.c_int
    lib.bsp_bench_mfma_bf16.argtypes = [vp, i32, i32, vp, vp]
    lib.bsp_bench_lds_read.restype = ctypes.c_int
    lib.bsp_bench_lds_read.argtypes = [vp, i32, i32, vp]
    _lib = lib
    return lib


def _check(rc: int, where: str):
    if rc != 0:
        raise BspError(rc, where)


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _np_dtype(code: int):
    if code == BSP_F32:
        return np.float32
    if code == BSP_BF16:
        return np.uint16
    if code == BSP_I8:
        return np.int8
    raise BspError(-5, "dtype")


# ------------------------------------------------------------------- host side
def bsp_strerror(code: int) -> str:
    return load_library().bsp_strerror(int(code)).decode()


def bsp_version() -> int:
    return load_library().bsp_version()


def bsp_pack_count(gamma: np.ndarray, O: int, I: int, bo: int, bi: int) -> int:
    g = np.ascontiguousarray(gamma, dtype=np.uint8)
    n = ctypes.c_int64(0)
    _check(load_library().bsp_pack_count(_np_ptr(g), O, I, bo, bi, ctypes.byref(n)),
           "bsp_pack_count")
    return n.value


def bsp_pack(W: np.ndarray, gamma: np.ndarray, bo: int, bi: int,
             payload_dtype: int = BSP_F32, w_dtype: Optional[int] = None
             ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(row_ptr, col_idx, payload[nnzb][bo][H][K][bi]).  ``W`` is float32, or
    uint16 holding bf16 bit patterns."""
    if w_dtype is None:
        w_dtype = BSP_BF16 if W.dtype == np.uint16 else BSP_I8 if W.dtype == np.int8 else BSP_F32
    W = np.ascontiguousarray(W, dtype=_np_dtype(w_dtype))
    O, H, K, I = W.shape
    g = np.ascontiguousarray(gamma, dtype=np.uint8)
    nbr, nbc = -(-O // bo), -(-I // bi)
    if g.size != nbr * nbc:
        raise BspError(-2, "bsp_pack (mask size)")
    nnzb = bsp_pack_count(g, O, I, bo, bi)
    row_ptr = np.zeros(nbr + 1, dtype=np.int32)
    col_idx = np.zeros(nnzb, dtype=np.int32)
    payload = np.zeros((nnzb, bo, H, K, bi), dtype=_np_dtype(payload_dtype))
    _check(load_library().bsp_pack(_np_ptr(W), w_dtype, _np_ptr(g), O, H, K, I, bo, bi,
                                   payload_dtype, _np_ptr(row_ptr), _np_ptr(col_idx),
                                   col_idx.size, _np_ptr(payload), payload.nbytes),
           "bsp_pack")
    return row_ptr, col_idx, payload


def bsp_unpack(row_ptr, col_idx, payload, O, H, K, I, bo, bi) -> np.ndarray:
    code = _payload_code(payload)
    W = np.empty((O, H, K, I), dtype=payload.dtype)
    _check(load_library().bsp_unpack(_np_ptr(np.ascontiguousarray(row_ptr, dtype=np.int32)),
                                     _np_ptr(np.ascontiguousarray(col_idx, dtype=np.int32)),
                                     _np_ptr(np.ascontiguousarray(payload)), code,
                                     O, H, K, I, bo, bi, _np_ptr(W)), "bsp_unpack")
    return W


def bsp_validate(row_ptr, col_idx, O, I, bo, bi) -> int:
    """Returns the status code (0 = well formed); does not raise."""
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    return load_library().bsp_validate(_np_ptr(rp), _np_ptr(ci), O, I, bo, bi)


def _payload_code(payload: np.ndarray) -> int:
    return BSP_BF16 if payload.dtype == np.uint16 else BSP_I8 if payload.dtype == np.int8 \
        else BSP_F32


BSP_IMPORTANCE_L2, BSP_IMPORTANCE_L1, BSP_IMPORTANCE_VAR = 0, 1, 2


def bsp_block_importance(W: np.ndarray, bo: int, bi: int, measure: int = 0) -> np.ndarray:
    Wf = np.ascontiguousarray(W, dtype=np.float32)
    O, H, K, I = Wf.shape
    score = np.zeros((-(-O // bo), -(-I // bi)), dtype=np.float64)
    _check(load_library().bsp_block_importance(_np_ptr(Wf), O, H, K, I, bo, bi, measure,
                                               _np_ptr(score)), "bsp_block_importance")
    return score


def bsp_select_mask(W: np.ndarray, bo: int, bi: int, measure: int = 0, density: float = 0.5,
                    per_row: bool = False) -> np.ndarray:
    """Gamma keeping the round(density * n) most important blocks."""
    Wf = np.ascontiguousarray(W, dtype=np.float32)
    O, H, K, I = Wf.shape
    gamma = np.zeros((-(-O // bo), -(-I // bi)), dtype=np.uint8)
    _check(load_library().bsp_select_mask(_np_ptr(Wf), O, H, K, I, bo, bi, measure, float(density),
                                          int(per_row), _np_ptr(gamma)), "bsp_select_mask")
    return gamma


def bsp_mask_step(W: np.ndarray, gamma: np.ndarray, bo: int, bi: int, measure: int = 0,
                  target_density: float = 0.5) -> Tuple[np.ndarray, int]:
    """(new Gamma, blocks zeroed) after one step of the incremental schedule."""
    Wf = np.ascontiguousarray(W, dtype=np.float32)
    O, H, K, I = Wf.shape
    g = np.array(gamma, dtype=np.uint8).reshape(-(-O // bo), -(-I // bi)).copy()
    z = ctypes.c_int32(0)
    _check(load_library().bsp_mask_step(_np_ptr(Wf), O, H, K, I, bo, bi, measure,
                                        float(target_density), _np_ptr(g), ctypes.byref(z)),
           "bsp_mask_step")
    return g, z.value


def bsp_quantize(W: np.ndarray, bits: int = 8) -> Tuple[np.ndarray, float]:
    """(int8 codes of the same shape, Delta) by the round-to-nearest quantizer."""
    Wf = np.ascontiguousarray(W, dtype=np.float32)
    codes = np.zeros(Wf.shape, dtype=np.int8)
    delta = ctypes.c_double(0.0)
    _check(load_library().bsp_quantize(_np_ptr(Wf), Wf.size, bits, _np_ptr(codes),
                                       ctypes.byref(delta)), "bsp_quantize")
    return codes, delta.value


def bsp_plan_size(row_ptr, col_idx, O, H, K, I, bo, bi, payload_dtype: int) -> int:
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    n = ctypes.c_int64(0)
    _check(load_library().bsp_plan_size(_np_ptr(rp), _np_ptr(ci), O, H, K, I, bo, bi,
                                        payload_dtype, ctypes.byref(n)), "bsp_plan_size")
    return n.value


def bsp_plan_build(row_ptr, col_idx, payload, O, H, K, I, bo, bi) -> np.ndarray:
    """The launch plan as an int32 array (copy it to the device as is)."""
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    pl = np.ascontiguousarray(payload)
    code = _payload_code(pl)
    nbytes = bsp_plan_size(rp, ci, O, H, K, I, bo, bi, code)
    plan = np.zeros(nbytes // 4, dtype=np.int32)
    _check(load_library().bsp_plan_build(_np_ptr(rp), _np_ptr(ci), _np_ptr(pl), code,
                                         O, H, K, I, bo, bi, _np_ptr(plan), plan.nbytes),
           "bsp_plan_build")
    return plan


# ----------------------------------------------------------------- device side
def bsp_fc(w: bsp_weights, X: int, bias: Optional[int], Y: int, B: int, stream: int = 0) -> None:
    _check(load_library().bsp_fc(ctypes.byref(w), X, bias, Y, B, stream), "bsp_fc")


def bsp_conv2d(w: bsp_weights, X: int, bias: Optional[int], Y: int, B: int, L: int, J: int,
               stride=(1, 1), pad=(0, 0), stream: int = 0) -> None:
    _check(load_library().bsp_conv2d(ctypes.byref(w), X, bias, Y, B, L, J, stride[0], stride[1],
                                     pad[0], pad[1], stream), "bsp_conv2d")


def bsp_conv2d_fused(w: bsp_weights, X: int, bias: Optional[int], residual: Optional[int],
                     relu: bool, Y: int, B: int, L: int, J: int, stride=(1, 1), pad=(0, 0),
                     stream: int = 0) -> None:
    _check(load_library().bsp_conv2d_fused(ctypes.byref(w), X, bias, residual, int(relu), Y, B, L,
                                           J, stride[0], stride[1], pad[0], pad[1], stream),
           "bsp_conv2d_fused")


def bsp_fc_fused(w: bsp_weights, X: int, bias: Optional[int], residual: Optional[int],
                 relu: bool, Y: int, B: int, stream: int = 0) -> None:
    _check(load_library().bsp_fc_fused(ctypes.byref(w), X, bias, residual, int(relu), Y, B,
                                       stream), "bsp_fc_fused")


def bsp_fc_fused_static(w: bsp_weights, X: int, bias: Optional[int], residual: Optional[int],
                        relu: bool, Y: int, B: int, stream: int = 0) -> None:
    """bsp_fc_fused without any allocation: partial sums go to the library's fixed array."""
    _check(load_library().bsp_fc_fused_static(ctypes.byref(w), X, bias, residual, int(relu), Y,
                                              B, stream), "bsp_fc_fused_static")


def bsp_conv2d_only(w: bsp_weights, X: int, bias: Optional[int], residual: Optional[int],
                    relu: bool, Y: int, B: int, L: int, J: int, stride=(1, 1), pad=(0, 0),
                    family: int = 0, stream: int = 0) -> None:
    _check(load_library().bsp_conv2d_only(ctypes.byref(w), X, bias, residual, int(relu), Y, B, L,
                                          J, stride[0], stride[1], pad[0], pad[1], family, stream),
           "bsp_conv2d_only")


def bsp_bottleneck(w1: bsp_weights, w2: bsp_weights, w3: bsp_weights, X: int,
                   bias1: Optional[int], bias2: Optional[int], bias3: Optional[int],
                   residual: Optional[int], relu: bool, Y: int, B: int, L: int, J: int,
                   stream: int = 0) -> None:
    _check(load_library().bsp_bottleneck(ctypes.byref(w1), ctypes.byref(w2), ctypes.byref(w3), X,
                                         bias1, bias2, bias3, residual, int(relu), Y, B, L, J,
                                         stream), "bsp_bottleneck")


def bottleneck(l1: "BspLayer", l2: "BspLayer", l3: "BspLayer", X, residual=None, relu=True,
               out=None, stream=None, force=False):
    """Marshals three BspLayers (1x1, 3x3, 1x1) and torch tensors into bsp_bottleneck.
    ``force`` sets BSP_KERNEL_CHAIN for the call."""
    import torch
    assert X.is_contiguous() and X.dtype == torch.bfloat16 and X.shape[-1] == l1.I
    B, L, J, _ = X.shape
    if out is None:
        out = torch.empty((B, L, J, l3.O), dtype=torch.bfloat16, device=X.device)
    if residual is not None:
        assert residual.is_contiguous() and residual.dtype == out.dtype and residual.shape == out.shape
    st = torch.cuda.current_stream(X.device).cuda_stream if stream is None else stream

    def bp(l):
        return None if l.d_bias is None else l.d_bias.data_ptr()
    saved = l1.struct.kernels
    if force:
        l1.struct.kernels = saved | BSP_KERNEL_CHAIN
    try:
        bsp_bottleneck(l1.struct, l2.struct, l3.struct, X.data_ptr(), bp(l1), bp(l2), bp(l3),
                       None if residual is None else residual.data_ptr(), relu, out.data_ptr(), B, L, J, st)
    finally:
        l1.struct.kernels = saved
    return out


def bsp_conv2d_general(w: bsp_weights, X: int, bias: Optional[int], Y: int, B: int, L: int,
                       J: int, stride=(1, 1), pad=(0, 0), stream: int = 0) -> None:
    _check(load_library().bsp_conv2d_general(ctypes.byref(w), X, bias, Y, B, L, J, stride[0],
                                             stride[1], pad[0], pad[1], stream),
           "bsp_conv2d_general")


def bsp_conv2d_i8(w: bsp_weights, X: int, bias: Optional[int], Y: int, y_dtype: int, shift: int,
                  B: int, L: int, J: int, stride=(1, 1), pad=(0, 0), stream: int = 0) -> None:
    _check(load_library().bsp_conv2d_i8(ctypes.byref(w), X, bias, Y, y_dtype, shift, B, L, J,
                                        stride[0], stride[1], pad[0], pad[1], stream),
           "bsp_conv2d_i8")


def bsp_fc_i8(w: bsp_weights, X: int, bias: Optional[int], Y: int, y_dtype: int, shift: int,
              B: int, stream: int = 0) -> None:
    _check(load_library().bsp_fc_i8(ctypes.byref(w), X, bias, Y, y_dtype, shift, B, stream),
           "bsp_fc_i8")


class BspLayer:
    """Pack one layer on the host and keep its arrays resident on a GPU.

    W is float32 [O][H][K][I] (values already representable in ``dtype``),
    gamma the block mask.  ``dtype`` is "f32" or "bf16" and is the element type
    of payload, X and Y.
    """

    def __init__(self, W: np.ndarray, gamma: np.ndarray, bo: int, bi: int,
                 dtype: str = "bf16", bias: Optional[np.ndarray] = None,
                 device: str = "cuda:0"):
        import torch
        load_library()
        self.code = {"f32": BSP_F32, "bf16": BSP_BF16}[dtype]
        self.dtype = dtype
        self.torch_dtype = torch.float32 if dtype == "f32" else torch.bfloat16
        O, H, K, I = W.shape
        self.O, self.H, self.K, self.I, self.bo, self.bi = O, H, K, I, bo, bi
        self.row_ptr, self.col_idx, self.payload = bsp_pack(
            np.ascontiguousarray(W, dtype=np.float32), gamma, bo, bi, self.code)
        self.plan = bsp_plan_build(self.row_ptr, self.col_idx, self.payload, O, H, K, I, bo, bi)
        self.nnzb = int(self.col_idx.size)
        self.device = torch.device(device)
        pl = self.payload.view(np.int16) if dtype == "bf16" else self.payload
        # one spare element so an empty payload still has a valid address
        self.d_payload = torch.zeros(max(pl.size, 8), dtype=torch.int16 if dtype == "bf16"
                                     else torch.float32, device=self.device)
        if pl.size:
            self.d_payload[:pl.size].copy_(torch.from_numpy(pl.reshape(-1)))
        self.d_row_ptr = torch.from_numpy(self.row_ptr).to(self.device)
        self.d_col_idx = torch.from_numpy(np.resize(self.col_idx, max(self.nnzb, 1))
                                          if self.nnzb else np.zeros(1, np.int32)).to(self.device)
        self.d_plan = torch.from_numpy(self.plan).to(self.device)
        self.d_bias = None if bias is None else \
            torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).to(self.device)
        self.struct = bsp_weights(O, I, H, K, bo, bi, self.code, 0, self.nnzb,
                                  self.d_row_ptr.data_ptr(), self.d_col_idx.data_ptr(),
                                  self.d_payload.data_ptr(), self.d_plan.data_ptr(),
                                  self.plan.nbytes, self.plan.ctypes.data)

    def out_shape(self, B, L, J, stride, pad):
        M = (L + 2 * pad[0] - self.H) // stride[0] + 1
        N = (J + 2 * pad[1] - self.K) // stride[1] + 1
        return (B, M, N, self.O)

    def conv2d(self, X, stride=(1, 1), pad=(0, 0), out=None, general=False, stream=None,
               residual=None, relu=False, family=None):
        """X: torch tensor [B][L][J][I] on the layer's device, contiguous.  ``residual`` (a
        tensor shaped like the output) and ``relu`` select the fused epilogue.  ``family``
        (a BSP_KERNEL_* bit, or 0) runs that kernel family only and raises BspError(-6) when
        the layer lies outside it."""
        import torch
        assert X.is_contiguous() and X.dtype == self.torch_dtype and X.shape[-1] == self.I
        B, L, J, _ = X.shape
        if out is None:
            out = torch.empty(self.out_shape(B, L, J, stride, pad), dtype=self.torch_dtype,
                              device=X.device)
        st = torch.cuda.current_stream(X.device).cuda_stream if stream is None else stream
        bias = None if self.d_bias is None else self.d_bias.data_ptr()
        if family is not None:
            bsp_conv2d_only(self.struct, X.data_ptr(), bias,
                            None if residual is None else residual.data_ptr(), relu,
                            out.data_ptr(), B, L, J, stride, pad, family, st)
            return out
        if residual is not None or relu:
            assert not general
            if residual is not None:
                assert residual.is_contiguous() and residual.dtype == self.torch_dtype \
                    and residual.shape == out.shape
            bsp_conv2d_fused(self.struct, X.data_ptr(), bias,
                             None if residual is None else residual.data_ptr(), relu,
                             out.data_ptr(), B, L, J, stride, pad, st)
            return out
        fn = bsp_conv2d_general if general else bsp_conv2d
        fn(self.struct, X.data_ptr(), bias, out.data_ptr(), B, L, J, stride, pad, st)
        return out

    def fc(self, X, out=None, stream=None, residual=None, relu=False):
        """X: torch tensor [B][I]."""
        import torch
        assert X.is_contiguous() and X.dtype == self.torch_dtype and X.shape[-1] == self.I
        B = X.shape[0]
        if out is None:
            out = torch.empty((B, self.O), dtype=self.torch_dtype, device=X.device)
        st = torch.cuda.current_stream(X.device).cuda_stream if stream is None else stream
        bias = None if self.d_bias is None else self.d_bias.data_ptr()
        if residual is not None or relu:
            bsp_fc_fused(self.struct, X.data_ptr(), bias,
                         None if residual is None else residual.data_ptr(), relu, out.data_ptr(),
                         B, st)
        else:
            bsp_fc(self.struct, X.data_ptr(), bias, out.data_ptr(), B, st)
        return out


def bsp_bcsr_segments(row_ptr, col_idx, rows: int, cols: int) -> np.ndarray:
    """[rows][ceil(cols/16) + 1]: where, in a block row's run of kept blocks, every sixteenth
    block column starts."""
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    seg = np.zeros((rows, (cols + 15) // 16 + 1), dtype=np.int32)
    _check(load_library().bsp_bcsr_segments(_np_ptr(rp), _np_ptr(ci), rows, cols, _np_ptr(seg)),
           "bsp_bcsr_segments")
    return seg


def bsp_spgemm_nt(A: bsp_bcsr, B: bsp_bcsr, C: int, stream: int = 0) -> None:
    _check(load_library().bsp_spgemm_nt(ctypes.byref(A), ctypes.byref(B), C, stream),
           "bsp_spgemm_nt")


# ---------------------------------------------------------- measurement helpers
def bsp_bench_copy(dst: int, src: int, nbytes: int, stream: int = 0) -> None:
    _check(load_library().bsp_bench_copy(dst, src, nbytes, stream), "bsp_bench_copy")


def bsp_bench_mfma_bf16(sink: int, waves: int, iters: int, clocks: Optional[int] = None,
                        stream: int = 0) -> None:
    _check(load_library().bsp_bench_mfma_bf16(sink, waves, iters, clocks, stream),
           "bsp_bench_mfma_bf16")


def bsp_bench_lds_read(sink: int, waves: int, iters: int, stream: int = 0) -> None:
    _check(load_library().bsp_bench_lds_read(sink, waves, iters, stream), "bsp_bench_lds_read")


class BspMatrix:
    """A block-sparse matrix (8x8 blocks, bf16) resident on a GPU, as an operand of the
    sparse x sparse product: M float32 [rows*8][cols*8] (values on the bf16 grid), gamma
    [rows][cols]."""

    def __init__(self, M: np.ndarray, gamma: np.ndarray, device: str = "cuda:0"):
        import torch
        load_library()
        M = np.ascontiguousarray(M, dtype=np.float32)
        R, Cc = M.shape[0] // 8, M.shape[1] // 8
        assert M.shape == (R * 8, Cc * 8)
        self.rows, self.cols = R, Cc
        self.row_ptr, self.col_idx, self.payload = bsp_pack(M.reshape(R * 8, 1, 1, Cc * 8), gamma,
                                                            8, 8, BSP_BF16)
        self.seg_ptr = bsp_bcsr_segments(self.row_ptr, self.col_idx, R, Cc)
        self.nnzb = int(self.col_idx.size)
        dev = torch.device(device)
        pl = self.payload.view(np.int16)
        self.d_payload = torch.zeros(max(pl.size, 8), dtype=torch.int16, device=dev)
        if pl.size:
            self.d_payload[:pl.size].copy_(torch.from_numpy(pl.reshape(-1)))
        self.d_row_ptr = torch.from_numpy(self.row_ptr).to(dev)
        self.d_col_idx = torch.from_numpy(self.col_idx if self.nnzb else np.zeros(1, np.int32)).to(dev)
        self.d_seg_ptr = torch.from_numpy(self.seg_ptr).to(dev)
        self.struct = bsp_bcsr(R, Cc, 8, BSP_BF16, self.nnzb, self.d_row_ptr.data_ptr(),
                               self.d_col_idx.data_ptr(), self.d_payload.data_ptr(),
                               self.d_seg_ptr.data_ptr())

    def matmul_nt(self, other: "BspMatrix", out=None, stream=None):
        """C = self . other^t, float32 [self.rows*8][other.rows*8]."""
        import torch
        if out is None:
            out = torch.empty((self.rows * 8, other.rows * 8), dtype=torch.float32,
                              device=self.d_payload.device)
        st = torch.cuda.current_stream(out.device).cuda_stream if stream is None else stream
        bsp_spgemm_nt(self.struct, other.struct, out.data_ptr(), st)
        return out


class BspLayerI8:
    """An 8-bit integer layer resident on a GPU: int8 weight codes [O][H][K][I] (e.g. from
    ``bsp_quantize``), block mask, optional int32 bias.  X is int8; Y is int8 after a rounding
    right shift, or the exact int32 sums when ``shift`` is None."""

    def __init__(self, Wq: np.ndarray, gamma: np.ndarray, bo: int, bi: int,
                 bias: Optional[np.ndarray] = None, device: str = "cuda:0"):
        import torch
        load_library()
        Wq = np.ascontiguousarray(Wq, dtype=np.int8)
        O, H, K, I = Wq.shape
        self.O, self.H, self.K, self.I, self.bo, self.bi = O, H, K, I, bo, bi
        self.row_ptr, self.col_idx, self.payload = bsp_pack(Wq, gamma, bo, bi, BSP_I8)
        self.plan = bsp_plan_build(self.row_ptr, self.col_idx, self.payload, O, H, K, I, bo, bi)
        self.nnzb = int(self.col_idx.size)
        self.device = torch.device(device)
        self.d_payload = torch.zeros(max(self.payload.size, 16), dtype=torch.int8,
                                     device=self.device)
        if self.payload.size:
            self.d_payload[:self.payload.size].copy_(torch.from_numpy(self.payload.reshape(-1)))
        self.d_row_ptr = torch.from_numpy(self.row_ptr).to(self.device)
        self.d_col_idx = torch.from_numpy(self.col_idx if self.nnzb
                                          else np.zeros(1, np.int32)).to(self.device)
        self.d_plan = torch.from_numpy(self.plan).to(self.device)
        self.d_bias = None if bias is None else \
            torch.from_numpy(np.ascontiguousarray(bias, dtype=np.int32)).to(self.device)
        self.struct = bsp_weights(O, I, H, K, bo, bi, BSP_I8, 0, self.nnzb,
                                  self.d_row_ptr.data_ptr(), self.d_col_idx.data_ptr(),
                                  self.d_payload.data_ptr(), self.d_plan.data_ptr(),
                                  self.plan.nbytes, self.plan.ctypes.data)

    def out_shape(self, B, L, J, stride, pad):
        M = (L + 2 * pad[0] - self.H) // stride[0] + 1
        N = (J + 2 * pad[1] - self.K) // stride[1] + 1
        return (B, M, N, self.O)

    def conv2d(self, X, stride=(1, 1), pad=(0, 0), shift: Optional[int] = None, out=None,
               stream=None):
        """X: int8 torch tensor [B][L][J][I] on the layer's device, contiguous."""
        import torch
        assert X.is_contiguous() and X.dtype == torch.int8 and X.shape[-1] == self.I
        B, L, J, _ = X.shape
        ydt = torch.int32 if shift is None else torch.int8
        if out is None:
            out = torch.empty(self.out_shape(B, L, J, stride, pad), dtype=ydt, device=X.device)
        assert out.dtype == ydt
        st = torch.cuda.current_stream(X.device).cuda_stream if stream is None else stream
        bsp_conv2d_i8(self.struct, X.data_ptr(),
                      None if self.d_bias is None else self.d_bias.data_ptr(), out.data_ptr(),
                      BSP_I32 if shift is None else BSP_I8, 0 if shift is None else shift,
                      B, L, J, stride, pad, st)
        return out

    def fc(self, X, shift: Optional[int] = None, out=None, stream=None):
        """X: int8 torch tensor [B][I]."""
        import torch
        assert X.is_contiguous() and X.dtype == torch.int8 and X.shape[-1] == self.I
        B = X.shape[0]
        ydt = torch.int32 if shift is None else torch.int8
        if out is None:
            out = torch.empty((B, self.O), dtype=ydt, device=X.device)
        st = torch.cuda.current_stream(X.device).cuda_stream if stream is None else stream
        bsp_fc_i8(self.struct, X.data_ptr(),
                  None if self.d_bias is None else self.d_bias.data_ptr(), out.data_ptr(),
                  BSP_I32 if shift is None else BSP_I8, 0 if shift is None else shift, B, st)
        return out
