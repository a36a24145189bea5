"""ctypes binding of libchebykan.so: argument marshalling only.

Every step of the layer runs inside the HIP library; PyTorch appears here only
as the owner of device memory and streams.  There is no CPU fallback: if the
library is missing or no gfx950 device is current, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

from . import build as _build

CHEBYKAN_OK = 0
CHEBYKAN_ERR_NULL = -1
CHEBYKAN_ERR_SHAPE = -2
CHEBYKAN_ERR_WORKSPACE = -3
CHEBYKAN_ERR_DEVICE = -4
CHEBYKAN_ERR_LAUNCH = -5
CHEBYKAN_PASS_FORWARD = 0
CHEBYKAN_PASS_BACKWARD = 1
CHEBYKAN_MAX_DEGREE = 32

EXPORTS = (
    "chebykan_workspace_bytes", "chebykan_forward", "chebykan_backward",
    "chebykan_status_string", "chebykan_set_kernel_family", "chebykan_version",
    "chebykan_calibrate_mfma", "chebykan_calibrate_copy",
    "chebykan_lut_build", "chebykan_forward_lut", "chebykan_backward_lut",
    "chebykan_lut_build_derivative", "chebykan_backward_lut2",
    "chebykan_forward_basis", "chebykan_backward_basis",
    "chebykan_stack_workspace_bytes", "chebykan_stack_forward", "chebykan_stack_backward",
    "chebykan_init", "chebykan_backward_noalloc",
    "chebykan_trace_begin", "chebykan_trace_end", "chebykan_trace_get", "chebykan_trace_free",
)

_lib: Optional[ctypes.CDLL] = None


class ChebykanError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s failed: %s (status %d)" % (where, chebykan_status_string(status), status))


def library_path() -> str:
    return _build.LIB_PATH


def load() -> ctypes.CDLL:
    """Load the built library; build it first only if no built library exists."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB_PATH):
            _build.build_library()
        lib = ctypes.CDLL(_build.LIB_PATH)
        vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
        lib.chebykan_workspace_bytes.argtypes = [i64, ci, ci, ci, ci]
        lib.chebykan_workspace_bytes.restype = sz
        lib.chebykan_forward.argtypes = [vp, vp, vp, i64, ci, ci, ci, vp, sz, vp]
        lib.chebykan_forward.restype = ci
        lib.chebykan_backward.argtypes = [vp, vp, vp, vp, vp, i64, ci, ci, ci, vp, sz, vp]
        lib.chebykan_backward.restype = ci
        lib.chebykan_status_string.argtypes = [ci]
        lib.chebykan_status_string.restype = ctypes.c_char_p
        lib.chebykan_set_kernel_family.argtypes = [ci]
        lib.chebykan_set_kernel_family.restype = ci
        lib.chebykan_version.argtypes = []
        lib.chebykan_version.restype = ci
        ip = ctypes.POINTER(ctypes.c_int)
        pp = ctypes.POINTER(ctypes.c_void_p)
        lib.chebykan_stack_workspace_bytes.argtypes = [i64, ci, ip, ci]
        lib.chebykan_stack_workspace_bytes.restype = sz
        lib.chebykan_stack_forward.argtypes = [ci, ip, ci, i64, pp, pp, vp, sz, vp]
        lib.chebykan_stack_forward.restype = ci
        lib.chebykan_stack_backward.argtypes = [ci, ip, ci, i64, pp, pp, pp, pp, vp, sz, vp]
        lib.chebykan_stack_backward.restype = ci
        lib.chebykan_forward_basis.argtypes = [ci, vp, vp, vp, i64, ci, ci, ci, vp, sz, vp]
        lib.chebykan_forward_basis.restype = ci
        lib.chebykan_backward_basis.argtypes = [ci, vp, vp, vp, vp, vp, i64, ci, ci, ci, vp, sz, vp]
        lib.chebykan_backward_basis.restype = ci
        lib.chebykan_lut_build.argtypes = [vp, ci, ci]
        lib.chebykan_lut_build.restype = ci
        lib.chebykan_forward_lut.argtypes = [vp, vp, vp, ci, vp, i64, ci, ci, ci, vp, sz, vp]
        lib.chebykan_forward_lut.restype = ci
        lib.chebykan_backward_lut.argtypes = [vp, vp, vp, vp, ci, vp, vp, i64, ci, ci, ci, vp, sz, vp]
        lib.chebykan_backward_lut.restype = ci
        lib.chebykan_lut_build_derivative.argtypes = [vp, ci, ci]
        lib.chebykan_lut_build_derivative.restype = ci
        lib.chebykan_backward_lut2.argtypes = [vp, vp, vp, vp, vp, ci, vp, vp, i64, ci, ci, ci, vp, sz, vp]
        lib.chebykan_backward_lut2.restype = ci
        lib.chebykan_calibrate_mfma.argtypes = [vp, ci, ci, ctypes.POINTER(ctypes.c_double), vp]
        lib.chebykan_calibrate_mfma.restype = ci
        lib.chebykan_calibrate_copy.argtypes = [vp, vp, i64, vp]
        lib.chebykan_calibrate_copy.restype = ci
        lib.chebykan_backward_noalloc.argtypes = [vp, vp, vp, vp, vp, i64, ci, ci, ci, vp]
        lib.chebykan_backward_noalloc.restype = ci
        lib.chebykan_init.argtypes = []
        lib.chebykan_init.restype = ci
        lib.chebykan_trace_begin.argtypes = [ci]
        lib.chebykan_trace_begin.restype = ci
        lib.chebykan_trace_end.argtypes = [ctypes.POINTER(ci)]
        lib.chebykan_trace_end.restype = ci
        lib.chebykan_trace_get.argtypes = [ci, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_uint * 3),
                                           ctypes.POINTER(ctypes.c_uint), ctypes.POINTER(ci), ctypes.POINTER(ci),
                                           ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ci), ctypes.POINTER(ci),
                                           ctypes.POINTER(ctypes.c_float)]
        lib.chebykan_trace_get.restype = ci
        lib.chebykan_trace_free.argtypes = []
        lib.chebykan_trace_free.restype = None
        _lib = lib
    return _lib


# ---------------------------------------------------------------- raw calls
# Pointers are plain integers (device addresses) or None; status is returned.

def raw_forward(x_ptr, C_ptr, y_ptr, batch, n_in, n_out, degree, ws_ptr=None, ws_bytes=0, stream=None) -> int:
    return int(load().chebykan_forward(x_ptr, C_ptr, y_ptr, batch, n_in, n_out, degree, ws_ptr, ws_bytes, stream))


def raw_backward(x_ptr, C_ptr, dy_ptr, dx_ptr, dC_ptr, batch, n_in, n_out, degree, ws_ptr=None, ws_bytes=0,
                 stream=None) -> int:
    return int(load().chebykan_backward(x_ptr, C_ptr, dy_ptr, dx_ptr, dC_ptr, batch, n_in, n_out, degree,
                                        ws_ptr, ws_bytes, stream))


def chebykan_status_string(status: int) -> str:
    return load().chebykan_status_string(int(status)).decode()


def chebykan_workspace_bytes(batch: int, n_in: int, n_out: int, degree: int, which_pass: int) -> int:
    return int(load().chebykan_workspace_bytes(batch, n_in, n_out, degree, which_pass))


def chebykan_set_kernel_family(family: int) -> int:
    return int(load().chebykan_set_kernel_family(int(family)))


def chebykan_version() -> int:
    return int(load().chebykan_version())


def chebykan_init() -> None:
    """Prepare the current device (optional; needed before capturing the library's launches into a graph)."""
    st = int(load().chebykan_init())
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_init")


def chebykan_trace_begin(max_kernels: int) -> None:
    """Start timing every kernel the library launches from this thread (two event records per launch)."""
    st = int(load().chebykan_trace_begin(int(max_kernels)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_trace_begin")


def chebykan_trace_end():
    """Stop timing; returns (timed launches, launches dropped beyond the capacity)."""
    dropped = ctypes.c_int(0)
    n = int(load().chebykan_trace_end(ctypes.byref(dropped)))
    return n, int(dropped.value)


def chebykan_trace_records(count: int):
    """(kernel name, grid (x, y, z), block threads, layer, OP_* bits, share of that work, second layer, second
    OP_* bits, microseconds) per timed launch, in launch order.  The streams the launches went to must have been
    synchronised."""
    lib = load()
    out = []
    name, grid, block, us = ctypes.c_char_p(), (ctypes.c_uint * 3)(), ctypes.c_uint(0), ctypes.c_float(0.0)
    layer, ops, share = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_float(1.0)
    layer2, ops2 = ctypes.c_int(0), ctypes.c_int(0)
    for i in range(count):
        st = int(lib.chebykan_trace_get(i, ctypes.byref(name), ctypes.byref(grid), ctypes.byref(block),
                                        ctypes.byref(layer), ctypes.byref(ops), ctypes.byref(share), ctypes.byref(layer2),
                                        ctypes.byref(ops2), ctypes.byref(us)))
        if st != CHEBYKAN_OK:
            raise ChebykanError(st, "chebykan_trace_get")
        out.append((name.value.decode(), (int(grid[0]), int(grid[1]), int(grid[2])), int(block.value),
                    int(layer.value), int(ops.value), float(share.value), int(layer2.value), int(ops2.value),
                    float(us.value)))
    return out


OP_FORWARD, OP_DX, OP_DC, OP_SUM = 1, 2, 4, 8


def chebykan_trace_free() -> None:
    load().chebykan_trace_free()


def chebykan_calibrate_mfma(sink, workgroups: int, iterations: int, stream=None) -> float:
    """Enqueue the register-only MFMA loop; returns the flop count of the launch."""
    _check(sink, "sink")
    if sink.numel() < workgroups * 256:
        raise ValueError("sink needs workgroups*256 floats")
    flops = ctypes.c_double(0.0)
    st = int(load().chebykan_calibrate_mfma(sink.data_ptr(), workgroups, iterations, ctypes.byref(flops),
                                            _stream_ptr(stream)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_calibrate_mfma")
    return flops.value


def chebykan_calibrate_copy(dst, src, stream=None) -> int:
    """Enqueue dst = src as a plain streaming copy; returns the bytes moved each way."""
    _check(src, "src")
    _check(dst, "dst", src.shape)
    st = int(load().chebykan_calibrate_copy(dst.data_ptr(), src.data_ptr(), src.numel(), _stream_ptr(stream)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_calibrate_copy")
    return src.numel() * 4


# ------------------------------------------------------------ tensor calls

def _check(t, name, shape=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError("%s must be a contiguous fp32 tensor on the GPU" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ws(workspace, need):
    if need == 0:
        return None, 0
    if workspace is None:
        raise ValueError("this call needs a workspace of %d bytes" % need)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous GPU tensor")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def chebykan_forward(x, C, y, workspace=None, stream=None) -> None:
    """Enqueue y = layer(x; C) on the stream (torch's current stream by default)."""
    _check(x, "x")
    B, I = x.shape
    _check(C, "C")
    if C.dim() != 3 or C.shape[0] != I:
        raise ValueError("C must be [in, out, degree+1]")
    O, K = int(C.shape[1]), int(C.shape[2])
    _check(y, "y", (B, O))
    need = chebykan_workspace_bytes(B, I, O, K - 1, CHEBYKAN_PASS_FORWARD)
    ws_ptr, ws_bytes = _ws(workspace, need)
    st = raw_forward(x.data_ptr(), C.data_ptr(), y.data_ptr(), B, I, O, K - 1, ws_ptr, ws_bytes,
                     _stream_ptr(stream))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_forward")


def chebykan_backward(x, C, dy, dx, dC, workspace=None, stream=None) -> None:
    """Enqueue dx and/or dC (pass None to skip one) on the stream."""
    _check(x, "x")
    B, I = x.shape
    _check(C, "C")
    if C.dim() != 3 or C.shape[0] != I:
        raise ValueError("C must be [in, out, degree+1]")
    O, K = int(C.shape[1]), int(C.shape[2])
    _check(dy, "dy", (B, O))
    if dx is not None:
        _check(dx, "dx", (B, I))
    if dC is not None:
        _check(dC, "dC", (I, O, K))
    need = chebykan_workspace_bytes(B, I, O, K - 1, CHEBYKAN_PASS_BACKWARD)
    ws_ptr, ws_bytes = _ws(workspace, need)
    st = raw_backward(x.data_ptr(), C.data_ptr(), dy.data_ptr(),
                      None if dx is None else dx.data_ptr(), None if dC is None else dC.data_ptr(),
                      B, I, O, K - 1, ws_ptr, ws_bytes, _stream_ptr(stream))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_backward")


CHEBYKAN_NOALLOC_SCRATCH_BYTES = 32 << 20


def raw_backward_noalloc(x_ptr, C_ptr, dy_ptr, dx_ptr, dC_ptr, batch, n_in, n_out, degree, stream=None) -> int:
    return int(load().chebykan_backward_noalloc(x_ptr, C_ptr, dy_ptr, dx_ptr, dC_ptr, batch, n_in, n_out, degree, stream))


def chebykan_backward_noalloc(x, C, dy, dx, dC, stream=None) -> None:
    """chebykan_backward on the library's own static scratch: no workspace argument, no allocation."""
    _check(x, "x")
    B, I = x.shape
    _check(C, "C")
    if C.dim() != 3 or C.shape[0] != I:
        raise ValueError("C must be [in, out, degree+1]")
    O, K = int(C.shape[1]), int(C.shape[2])
    _check(dy, "dy", (B, O))
    if dx is not None:
        _check(dx, "dx", (B, I))
    if dC is not None:
        _check(dC, "dC", (I, O, K))
    st = raw_backward_noalloc(x.data_ptr(), C.data_ptr(), dy.data_ptr(),
                              None if dx is None else dx.data_ptr(), None if dC is None else dC.data_ptr(),
                              B, I, O, K - 1, _stream_ptr(stream))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_backward_noalloc")


def chebykan_lut_build(degree: int, lut_size: int):
    """The table of T_0..T_degree on lut_size uniform samples of [-1, 1] as a CPU fp32 tensor [degree+1, lut_size]."""
    import torch
    lut = torch.empty((degree + 1, lut_size), dtype=torch.float32)
    st = int(load().chebykan_lut_build(lut.data_ptr(), int(degree), int(lut_size)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_lut_build")
    return lut


def _check_lut(lut, K):
    _check(lut, "lut")
    if lut.dim() != 2 or lut.shape[0] != K:
        raise ValueError("lut must be [degree+1, lut_size]")
    return int(lut.shape[1])


def chebykan_forward_lut(x, C, lut, y, workspace=None, stream=None) -> None:
    """Table-interpolated forward: y = layer(x; C) with the basis read from lut ([degree+1, lut_size], GPU)."""
    _check(x, "x")
    B, I = x.shape
    _check(C, "C")
    if C.dim() != 3 or C.shape[0] != I:
        raise ValueError("C must be [in, out, degree+1]")
    O, K = int(C.shape[1]), int(C.shape[2])
    n = _check_lut(lut, K)
    _check(y, "y", (B, O))
    need = chebykan_workspace_bytes(B, I, O, K - 1, CHEBYKAN_PASS_FORWARD)
    ws_ptr, ws_bytes = _ws(workspace, need)
    st = int(load().chebykan_forward_lut(x.data_ptr(), C.data_ptr(), lut.data_ptr(), n, y.data_ptr(), B, I, O, K - 1,
                                         ws_ptr, ws_bytes, _stream_ptr(stream)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_forward_lut")


def chebykan_backward_lut(x, C, dy, lut, dx, dC, workspace=None, stream=None) -> None:
    """Table-interpolated backward: dx and/or dC (pass None to skip one)."""
    _check(x, "x")
    B, I = x.shape
    _check(C, "C")
    if C.dim() != 3 or C.shape[0] != I:
        raise ValueError("C must be [in, out, degree+1]")
    O, K = int(C.shape[1]), int(C.shape[2])
    n = _check_lut(lut, K)
    _check(dy, "dy", (B, O))
    if dx is not None:
        _check(dx, "dx", (B, I))
    if dC is not None:
        _check(dC, "dC", (I, O, K))
    need = chebykan_workspace_bytes(B, I, O, K - 1, CHEBYKAN_PASS_BACKWARD)
    ws_ptr, ws_bytes = _ws(workspace, need)
    st = int(load().chebykan_backward_lut(x.data_ptr(), C.data_ptr(), dy.data_ptr(), lut.data_ptr(), n,
                                          None if dx is None else dx.data_ptr(),
                                          None if dC is None else dC.data_ptr(),
                                          B, I, O, K - 1, ws_ptr, ws_bytes, _stream_ptr(stream)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_backward_lut")


def chebykan_lut_build_derivative(degree: int, lut_size: int):
    """The auxiliary table of T_0'..T_degree' on the same grid as chebykan_lut_build, CPU fp32 [degree+1, lut_size]."""
    import torch
    dlut = torch.empty((degree + 1, lut_size), dtype=torch.float32)
    st = int(load().chebykan_lut_build_derivative(dlut.data_ptr(), int(degree), int(lut_size)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_lut_build_derivative")
    return dlut


def chebykan_backward_lut2(x, C, dy, lut, dlut, dx, dC, workspace=None, stream=None) -> None:
    """Table-interpolated backward with the derivative taken from the auxiliary table dlut."""
    _check(x, "x")
    B, I = x.shape
    _check(C, "C")
    if C.dim() != 3 or C.shape[0] != I:
        raise ValueError("C must be [in, out, degree+1]")
    O, K = int(C.shape[1]), int(C.shape[2])
    n = _check_lut(lut, K)
    if _check_lut(dlut, K) != n:
        raise ValueError("lut and dlut must have the same number of samples")
    _check(dy, "dy", (B, O))
    if dx is not None:
        _check(dx, "dx", (B, I))
    if dC is not None:
        _check(dC, "dC", (I, O, K))
    need = chebykan_workspace_bytes(B, I, O, K - 1, CHEBYKAN_PASS_BACKWARD)
    ws_ptr, ws_bytes = _ws(workspace, need)
    st = int(load().chebykan_backward_lut2(x.data_ptr(), C.data_ptr(), dy.data_ptr(), lut.data_ptr(), dlut.data_ptr(), n,
                                           None if dx is None else dx.data_ptr(),
                                           None if dC is None else dC.data_ptr(),
                                           B, I, O, K - 1, ws_ptr, ws_bytes, _stream_ptr(stream)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_backward_lut2")


BASIS_CHEBYSHEV, BASIS_LEGENDRE, BASIS_HERMITE, BASIS_FOURIER = 0, 1, 2, 3


def chebykan_forward_basis(basis: int, x, C, y, workspace=None, stream=None) -> None:
    """Forward of the layer on another basis family (BASIS_* constants)."""
    _check(x, "x")
    B, I = x.shape
    _check(C, "C")
    if C.dim() != 3 or C.shape[0] != I:
        raise ValueError("C must be [in, out, degree+1]")
    O, K = int(C.shape[1]), int(C.shape[2])
    _check(y, "y", (B, O))
    need = chebykan_workspace_bytes(B, I, O, K - 1, CHEBYKAN_PASS_FORWARD)
    ws_ptr, ws_bytes = _ws(workspace, need)
    st = int(load().chebykan_forward_basis(int(basis), x.data_ptr(), C.data_ptr(), y.data_ptr(), B, I, O, K - 1,
                                           ws_ptr, ws_bytes, _stream_ptr(stream)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_forward_basis")


def chebykan_backward_basis(basis: int, x, C, dy, dx, dC, workspace=None, stream=None) -> None:
    """dx and/or dC of the layer on another basis family (pass None to skip one)."""
    _check(x, "x")
    B, I = x.shape
    _check(C, "C")
    if C.dim() != 3 or C.shape[0] != I:
        raise ValueError("C must be [in, out, degree+1]")
    O, K = int(C.shape[1]), int(C.shape[2])
    _check(dy, "dy", (B, O))
    if dx is not None:
        _check(dx, "dx", (B, I))
    if dC is not None:
        _check(dC, "dC", (I, O, K))
    need = chebykan_workspace_bytes(B, I, O, K - 1, CHEBYKAN_PASS_BACKWARD)
    ws_ptr, ws_bytes = _ws(workspace, need)
    st = int(load().chebykan_backward_basis(int(basis), x.data_ptr(), C.data_ptr(), dy.data_ptr(),
                                            None if dx is None else dx.data_ptr(),
                                            None if dC is None else dC.data_ptr(),
                                            B, I, O, K - 1, ws_ptr, ws_bytes, _stream_ptr(stream)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_backward_basis")


def _int_array(values):
    return (ctypes.c_int * len(values))(*[int(v) for v in values])


def _ptr_array(tensors):
    return (ctypes.c_void_p * len(tensors))(*[None if t is None else t.data_ptr() for t in tensors])


def chebykan_stack_workspace_bytes(batch: int, widths, degree: int) -> int:
    return int(load().chebykan_stack_workspace_bytes(int(batch), len(widths) - 1, _int_array(widths), int(degree)))


def _stack_shapes(Cs, acts):
    widths = [int(Cs[0].shape[0])] + [int(c.shape[1]) for c in Cs]
    K = int(Cs[0].shape[2])
    B = int(acts[0].shape[0])
    for l, c in enumerate(Cs):
        _check(c, "C[%d]" % l, (widths[l], widths[l + 1], K))
    return widths, K - 1, B


def chebykan_stack_forward(Cs, acts, workspace=None, stream=None) -> None:
    """Forward through a stack: acts[0] is the input, acts[l+1] receives the output of layer l."""
    widths, degree, B = _stack_shapes(Cs, acts)
    if len(acts) != len(Cs) + 1:
        raise ValueError("acts needs one more entry than Cs")
    for l, a in enumerate(acts):
        _check(a, "act[%d]" % l, (B, widths[l]))
    need = chebykan_stack_workspace_bytes(B, widths, degree)
    ws_ptr, ws_bytes = _ws(workspace, need)
    st = int(load().chebykan_stack_forward(len(Cs), _int_array(widths), degree, B, _ptr_array(Cs), _ptr_array(acts),
                                           ws_ptr, ws_bytes, _stream_ptr(stream)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_stack_forward")


def chebykan_stack_backward(Cs, acts, grads, dCs, workspace=None, stream=None) -> None:
    """Backward through a stack: grads[-1] is the incoming dy; grads[l] (l < n) and dCs[l] are written.

    acts holds the inputs of every layer (n entries, or n+1 with the unused last output);
    grads[0] and any dCs[l] may be None (skipped)."""
    widths, degree, B = _stack_shapes(Cs, acts)
    n = len(Cs)
    if len(grads) != n + 1 or len(dCs) != n or len(acts) < n:
        raise ValueError("grads needs n+1 entries, dCs n, acts at least n")
    for l in range(n):
        _check(acts[l], "act[%d]" % l, (B, widths[l]))
        if dCs[l] is not None:
            _check(dCs[l], "dC[%d]" % l, tuple(Cs[l].shape))
    for l, g in enumerate(grads):
        if g is not None:
            _check(g, "grad[%d]" % l, (B, widths[l]))
    need = chebykan_stack_workspace_bytes(B, widths, degree)
    ws_ptr, ws_bytes = _ws(workspace, need)
    st = int(load().chebykan_stack_backward(n, _int_array(widths), degree, B, _ptr_array(Cs),
                                            _ptr_array(list(acts[:n])), _ptr_array(grads), _ptr_array(dCs),
                                            ws_ptr, ws_bytes, _stream_ptr(stream)))
    if st != CHEBYKAN_OK:
        raise ChebykanError(st, "chebykan_stack_backward")


def alloc_stack_workspace(batch: int, widths, degree: int, device="cuda"):
    import torch
    need = chebykan_stack_workspace_bytes(batch, widths, degree)
    return torch.empty(need, dtype=torch.uint8, device=device) if need else None


def alloc_workspace(batch: int, n_in: int, n_out: int, degree: int, device="cuda"):
    """A torch byte tensor large enough for both passes of one layer (None if none is needed)."""
    import torch
    need = max(chebykan_workspace_bytes(batch, n_in, n_out, degree, CHEBYKAN_PASS_FORWARD),
               chebykan_workspace_bytes(batch, n_in, n_out, degree, CHEBYKAN_PASS_BACKWARD))
    if need == 0:
        return None
    return torch.empty(need, dtype=torch.uint8, device=device)
