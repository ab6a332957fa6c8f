"""ctypes binding of libpme.so.  Same names as the C entry points (minus the pme_ prefix)."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpme.so")

PATH_AUTO, PATH_GENERIC, PATH_MFMA = 0, 1, 2
F32, BF16 = 0, 1

# Every symbol include/pme.h declares.
EXPORTS = ("pme_hadamard_expand_quant", "pme_expand_quantize_weights", "pme_hadamard_expand_quant_mxfp4",
           "pme_mxfp4_gemm", "pme_expanded_linear_mxfp4", "pme_hadamard_expand_quant_asym", "pme_w4a4_gemm", "pme_w4a4_gemm_asym",
           "pme_weight_rowsum", "pme_expanded_linear", "pme_expanded_linear_static", "pme_expanded_linear_asym", "pme_workspace_bytes", "pme_hadamard_expand_f32",
           "pme_w4a4_gemm_i32", "pme_factor_order", "pme_base_block", "pme_pack_int4", "pme_gemm_plan", "pme_probe_copy", "pme_probe_read", "pme_probe_launch", "pme_probe_mfma",
           "pme_set_path", "pme_set_gemm_tile",
           "pme_get_path", "pme_status_string", "pme_version")


class PmeError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({lib().pme_status_string(status).decode()})")


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python paper_2503_17513_amd/csrc/build.py` "
                           "(or __graft_entry__.build()); there is no fallback implementation")
    L = C.CDLL(_LIB_PATH)
    i64, vp, sz, i32 = C.c_int64, C.c_void_p, C.c_size_t, C.c_int
    L.pme_hadamard_expand_quant.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, vp]
    L.pme_expand_quantize_weights.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, vp]
    L.pme_hadamard_expand_quant_mxfp4.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, vp]
    L.pme_mxfp4_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, i64, vp]
    L.pme_expanded_linear_mxfp4.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, i64, vp, i64, vp, sz, vp]
    L.pme_hadamard_expand_quant_asym.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, vp, vp]
    L.pme_hadamard_expand_f32.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp]
    L.pme_w4a4_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i64, vp, i64, vp]
    L.pme_w4a4_gemm_asym.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, i64, vp]
    L.pme_w4a4_gemm_i32.argtypes = [vp, vp, i64, i64, i64, vp, vp]
    L.pme_weight_rowsum.argtypes = [vp, i64, i64, vp, vp]
    L.pme_expanded_linear.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, i64, vp, i64, vp, sz, vp]
    L.pme_expanded_linear_static.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, i64, vp, i64, vp]
    L.pme_expanded_linear_asym.argtypes = [vp, i32, i64, i64, i64, i64, vp, vp, vp, i64, vp, i64, vp, sz, vp]
    L.pme_workspace_bytes.argtypes = [i64, i64, i64, i64]
    L.pme_workspace_bytes.restype = sz
    L.pme_factor_order.argtypes = [i64, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.pme_base_block.argtypes = [i64, vp]
    L.pme_pack_int4.argtypes = [vp, i64, i64, vp, vp]
    L.pme_gemm_plan.argtypes = [i32, i64, i64, i64, C.c_char_p, sz]
    L.pme_probe_copy.argtypes = [vp, vp, sz, vp]
    L.pme_probe_read.argtypes = [vp, sz, vp, sz, vp]
    L.pme_probe_launch.argtypes = [vp]
    L.pme_probe_mfma.argtypes = [i32, vp, sz, i32, C.POINTER(C.c_double), vp]
    L.pme_set_path.argtypes = [i32]
    L.pme_set_gemm_tile.argtypes = [i32]
    L.pme_set_gemm_tile.restype = None
    L.pme_set_path.restype = None
    L.pme_get_path.restype = i32
    L.pme_status_string.argtypes = [i32]
    L.pme_status_string.restype = C.c_char_p
    L.pme_version.restype = i32
    for name in EXPORTS:
        fn = getattr(L, name)
        if fn.restype is C.c_int and name not in ("pme_get_path", "pme_version"):
            fn.restype = C.c_int
    _lib = L
    return L


def _check(status: int, what: str):
    if status != 0:
        raise PmeError(status, what)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(x: torch.Tensor) -> int:
    if x.dtype == torch.float32:
        return F32
    if x.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"activations must be float32 or bfloat16, got {x.dtype}")


def _dev(t: torch.Tensor, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    return t.data_ptr()


def version() -> int:
    return lib().pme_version()


def set_path(p: int) -> None:
    lib().pme_set_path(int(p))


def set_gemm_tile(tile_id: int) -> None:
    lib().pme_set_gemm_tile(int(tile_id))


def get_path() -> int:
    return lib().pme_get_path()


def factor_order(d_e: int) -> tuple[int, int]:
    b, k = C.c_int32(), C.c_int32()
    _check(lib().pme_factor_order(d_e, C.byref(b), C.byref(k)), "pme_factor_order")
    return b.value, k.value


def base_block(b: int) -> np.ndarray:
    out = np.zeros((b, b), dtype=np.int8)
    _check(lib().pme_base_block(b, out.ctypes.data), "pme_base_block")
    return out


def workspace_bytes(T: int, d: int, d_e: int, N: int) -> int:
    return lib().pme_workspace_bytes(T, d, d_e, N)


def _rows(x: torch.Tensor):
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be [T, d] with unit stride along d")
    return x.shape[0], x.shape[1], x.stride(0) if x.shape[0] > 1 else max(x.stride(0), x.shape[1])


def hadamard_expand_quant(x: torch.Tensor, d_e: int, qx: torch.Tensor | None = None, sx: torch.Tensor | None = None):
    T, d, ldx = _rows(x)
    if qx is None:
        qx = torch.empty((T, d_e // 2), dtype=torch.uint8, device=x.device)
    if sx is None:
        sx = torch.empty((T,), dtype=torch.float32, device=x.device)
    _check(lib().pme_hadamard_expand_quant(_dev(x, "x"), _dtype_code(x), T, d, ldx, d_e, _dev(qx, "qx"),
                                           _dev(sx, "sx"), _stream()), "pme_hadamard_expand_quant")
    return qx, sx


def expand_quantize_weights(wt: torch.Tensor, d_e: int):
    """wt: [N, d] (torch Linear layout, W^T of the paper's d x N matrix) -> (qw [N, d_e/2], sw [N])."""
    N, d, ldw = _rows(wt)
    qw = torch.empty((N, d_e // 2), dtype=torch.uint8, device=wt.device)
    sw = torch.empty((N,), dtype=torch.float32, device=wt.device)
    _check(lib().pme_expand_quantize_weights(_dev(wt, "wt"), _dtype_code(wt), N, d, ldw, d_e, qw.data_ptr(),
                                             sw.data_ptr(), _stream()), "pme_expand_quantize_weights")
    return qw, sw


def hadamard_expand_quant_mxfp4(x: torch.Tensor, d_e: int, qx: torch.Tensor | None = None, ex: torch.Tensor | None = None):
    """-> (packed E2M1 codes [T, d_e/2] uint8, E8M0 scale bytes [T, d_e/32] uint8); into qx, ex when given."""
    T, d, ldx = _rows(x)
    if qx is None:
        qx = torch.empty((T, d_e // 2), dtype=torch.uint8, device=x.device)
    if ex is None:
        ex = torch.empty((T, d_e // 32), dtype=torch.uint8, device=x.device)
    if (qx.dtype != torch.uint8 or ex.dtype != torch.uint8 or tuple(qx.shape) != (T, d_e // 2) or tuple(ex.shape) != (T, d_e // 32)
            or not qx.is_contiguous() or not ex.is_contiguous()):
        raise ValueError("qx must be a contiguous uint8 [T, d_e/2] tensor and ex a contiguous uint8 [T, d_e/32] tensor")
    _check(lib().pme_hadamard_expand_quant_mxfp4(_dev(x, "x"), _dtype_code(x), T, d, ldx, d_e, _dev(qx, "qx"),
                                                 _dev(ex, "ex"), _stream()), "pme_hadamard_expand_quant_mxfp4")
    return qx, ex


def mxfp4_gemm(qx, ex, qw, ew, y: torch.Tensor | None = None) -> torch.Tensor:
    T, d_e, N = _gemm_shapes(qx, qw)
    if y is None:
        y = torch.empty((T, N), dtype=torch.bfloat16, device=qx.device)
    _check(lib().pme_mxfp4_gemm(_dev(qx, "qx"), _dev(ex, "ex"), _dev(qw, "qw"), _dev(ew, "ew"), T, d_e, N,
                                _dev(y, "y"), y.stride(0) if T > 1 else max(y.stride(0), N), _stream()),
           "pme_mxfp4_gemm")
    return y


def expanded_linear_mxfp4(x, d_e: int, qw, ew, y: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    T, d, ldx = _rows(x)
    N = qw.shape[0]
    need = workspace_bytes(T, d, d_e, N)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    if y is None:
        y = torch.empty((T, N), dtype=torch.bfloat16, device=x.device)
    _check(lib().pme_expanded_linear_mxfp4(_dev(x, "x"), _dtype_code(x), T, d, ldx, d_e, _dev(qw, "qw"),
                                           _dev(ew, "ew"), N, _dev(y, "y"),
                                           y.stride(0) if T > 1 else max(y.stride(0), N), _dev(workspace, "workspace"),
                                           workspace.numel() * workspace.element_size(), _stream()),
           "pme_expanded_linear_mxfp4")
    return y


def hadamard_expand_quant_asym(x: torch.Tensor, d_e: int, qx: torch.Tensor | None = None,
                               sx: torch.Tensor | None = None, zx: torch.Tensor | None = None):
    T, d, ldx = _rows(x)
    if qx is None:
        qx = torch.empty((T, d_e // 2), dtype=torch.uint8, device=x.device)
    if sx is None:
        sx = torch.empty((T,), dtype=torch.float32, device=x.device)
    if zx is None:
        zx = torch.empty((T,), dtype=torch.int32, device=x.device)
    _check(lib().pme_hadamard_expand_quant_asym(_dev(x, "x"), _dtype_code(x), T, d, ldx, d_e, _dev(qx, "qx"),
                                                _dev(sx, "sx"), _dev(zx, "zx"), _stream()),
           "pme_hadamard_expand_quant_asym")
    return qx, sx, zx


def hadamard_expand_f32(x: torch.Tensor, d_e: int) -> torch.Tensor:
    T, d, ldx = _rows(x)
    xhat = torch.empty((T, d_e), dtype=torch.float32, device=x.device)
    _check(lib().pme_hadamard_expand_f32(_dev(x, "x"), _dtype_code(x), T, d, ldx, d_e, xhat.data_ptr(), _stream()),
           "pme_hadamard_expand_f32")
    return xhat


def _gemm_shapes(qx, qw):
    if qx.dtype != torch.uint8 or qw.dtype != torch.uint8 or not qx.is_contiguous() or not qw.is_contiguous():
        raise ValueError("qx and qw must be contiguous uint8 tensors of packed codes")
    if qx.shape[1] != qw.shape[1]:
        raise ValueError("qx and qw disagree on d_e")
    return qx.shape[0], qx.shape[1] * 2, qw.shape[0]


def w4a4_gemm(qx, sx, qw, sw, y: torch.Tensor | None = None) -> torch.Tensor:
    T, d_e, N = _gemm_shapes(qx, qw)
    if y is None:
        y = torch.empty((T, N), dtype=torch.bfloat16, device=qx.device)
    _check(lib().pme_w4a4_gemm(_dev(qx, "qx"), _dev(sx, "sx"), _dev(qw, "qw"), _dev(sw, "sw"), T, d_e, N,
                               _dev(y, "y"), y.stride(0) if T > 1 else max(y.stride(0), N), _stream()),
           "pme_w4a4_gemm")
    return y


def w4a4_gemm_asym(qx, sx, zx, qw, sw, wsum, y: torch.Tensor | None = None) -> torch.Tensor:
    T, d_e, N = _gemm_shapes(qx, qw)
    if y is None:
        y = torch.empty((T, N), dtype=torch.bfloat16, device=qx.device)
    _check(lib().pme_w4a4_gemm_asym(_dev(qx, "qx"), _dev(sx, "sx"), _dev(zx, "zx"), _dev(qw, "qw"), _dev(sw, "sw"),
                                    _dev(wsum, "wsum"), T, d_e, N, _dev(y, "y"),
                                    y.stride(0) if T > 1 else max(y.stride(0), N), _stream()), "pme_w4a4_gemm_asym")
    return y


def expanded_linear_asym(x, d_e: int, qw, sw, wsum, y: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None):
    """The layer with per-token asymmetric int4 activations (the paper's W4A4 setting)."""
    T, d, ldx = _rows(x)
    N = qw.shape[0]
    if qw.shape[1] * 2 != d_e:
        raise ValueError("qw must be [N, d_e / 2]")
    need = workspace_bytes(T, d, d_e, N)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    if y is None:
        y = torch.empty((T, N), dtype=torch.bfloat16, device=x.device)
    _check(lib().pme_expanded_linear_asym(_dev(x, "x"), _dtype_code(x), T, d, ldx, d_e, _dev(qw, "qw"), _dev(sw, "sw"),
                                          _dev(wsum, "wsum"), N, _dev(y, "y"),
                                          y.stride(0) if T > 1 else max(y.stride(0), N), _dev(workspace, "workspace"),
                                          workspace.numel() * workspace.element_size(), _stream()),
           "pme_expanded_linear_asym")
    return y


def w4a4_gemm_i32(qx, qw) -> torch.Tensor:
    T, d_e, N = _gemm_shapes(qx, qw)
    acc = torch.empty((T, N), dtype=torch.int32, device=qx.device)
    _check(lib().pme_w4a4_gemm_i32(_dev(qx, "qx"), _dev(qw, "qw"), T, d_e, N, acc.data_ptr(), _stream()),
           "pme_w4a4_gemm_i32")
    return acc


def weight_rowsum(qw: torch.Tensor) -> torch.Tensor:
    N, kb = qw.shape
    wsum = torch.empty((N,), dtype=torch.int32, device=qw.device)
    _check(lib().pme_weight_rowsum(_dev(qw, "qw"), N, kb * 2, wsum.data_ptr(), _stream()), "pme_weight_rowsum")
    return wsum


def expanded_linear(x, d_e: int, qw, sw, y: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    T, d, ldx = _rows(x)
    N = qw.shape[0]
    if qw.shape[1] * 2 != d_e:
        raise ValueError("qw must be [N, d_e / 2]")
    need = workspace_bytes(T, d, d_e, N)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    if y is None:
        y = torch.empty((T, N), dtype=torch.bfloat16, device=x.device)
    _check(lib().pme_expanded_linear(_dev(x, "x"), _dtype_code(x), T, d, ldx, d_e, _dev(qw, "qw"), _dev(sw, "sw"), N,
                                     _dev(y, "y"), y.stride(0) if T > 1 else max(y.stride(0), N),
                                     _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                     _stream()), "pme_expanded_linear")
    return y


STATIC_SCRATCH_BYTES = 16 << 20


def expanded_linear_static(x, d_e: int, qw, sw, y: torch.Tensor):
    """pme_expanded_linear_static: the layer with the library's static scratch in place of a workspace; y is the
    caller's (the call itself allocates nothing)."""
    T, d, ldx = _rows(x)
    N = qw.shape[0]
    if qw.shape[1] * 2 != d_e:
        raise ValueError("qw must be [N, d_e / 2]")
    _check(lib().pme_expanded_linear_static(_dev(x, "x"), _dtype_code(x), T, d, ldx, d_e, _dev(qw, "qw"), _dev(sw, "sw"), N,
                                            _dev(y, "y"), y.stride(0) if T > 1 else max(y.stride(0), N), _stream()),
           "pme_expanded_linear_static")
    return y


def probe_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    _check(lib().pme_probe_copy(_dev(src, "src"), _dev(dst, "dst"), nbytes, _stream()), "pme_probe_copy")


def probe_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    _check(lib().pme_probe_read(_dev(src, "src"), nbytes, _dev(sink, "sink"), sink.numel(), _stream()), "pme_probe_read")


def probe_launch() -> None:
    _check(lib().pme_probe_launch(_stream()), "pme_probe_launch")


def probe_mfma(kind: int, out: torch.Tensor, iters: int) -> float:
    """Launch the matrix-core probe (kind 0 int8, 1 FP4; 2, 3 the same on pseudo-random codes) and return the
    operation count of the launch."""
    ops = C.c_double(0.0)
    _check(lib().pme_probe_mfma(int(kind), _dev(out, "out"), out.numel(), int(iters), C.byref(ops), _stream()),
           "pme_probe_mfma")
    return ops.value


def pack_int4(codes: torch.Tensor) -> torch.Tensor:
    """int8 codes [rows, K] in [-8, 7] -> packed uint8 [rows, K/2] on the device (even index in the low nibble).
    A host tensor is copied to the current device first."""
    if codes.dtype != torch.int8 or codes.dim() != 2:
        raise TypeError("codes must be an int8 [rows, K] tensor")
    codes = codes.cuda().contiguous()
    rows, K = codes.shape
    packed = torch.empty((rows, K // 2), dtype=torch.uint8, device=codes.device)
    _check(lib().pme_pack_int4(_dev(codes, "codes"), rows, K, packed.data_ptr(), _stream()), "pme_pack_int4")
    return packed


def gemm_plan(T: int, d_e: int, N: int, variant: int = 0) -> str:
    """Name of the kernel instantiation the GEMM of this shape would run (variant 0 symmetric int4, 1 asymmetric,
    2 MXFP4), as a profiler prints it."""
    buf = C.create_string_buffer(128)
    _check(lib().pme_gemm_plan(int(variant), T, d_e, N, buf, len(buf)), "pme_gemm_plan")
    return buf.value.decode()
