"""Thin binding over the C ABI of ``libac_mi355x.so`` (see ``include/ac.h``).

Argument marshalling only: every function takes device tensors (PyTorch-ROCm is
used for device memory and streams, nothing else), passes their addresses,
leading dimensions and sizes to the entry point of the same name, and raises
``AcError`` on a non-zero status.  There is no CPU fallback: if the HIP library
has not been built, loading fails with an ImportError.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libac_mi355x.so")

AC_OK = 0
AC_ERR_NULL, AC_ERR_SHAPE, AC_ERR_STRIDE, AC_ERR_SHIFT = -1, -2, -3, -4
AC_ERR_ACT, AC_ERR_ALIAS, AC_ERR_WORKSPACE, AC_ERR_LAUNCH = -5, -6, -7, -8
AC_ERR_PLAN = -9
AC_ACT_NONE, AC_ACT_RELU = 0, 1

# every symbol include/ac.h declares
EXPORTS = ("ac_gemm_i8", "ac_gemm_i8_workspace_bytes", "ac_conv2d_i8", "ac_gemm_bf16", "ac_batched_gemm_f32",
           "ac_tinympc_forward_f32", "ac_gemm_i8_acc32", "ac_gemm_i8_static",
           "ac_gemm_i8_t", "ac_gemm_i8_planned", "ac_conv2d_i8_planned", "ac_gemm_i8_planned_workspace_bytes", "ac_gemm_bf16_planned",
           "ac_gemm_bf16_planned_workspace_bytes", "ac_gemm_bf16_ws", "ac_gemm_bf16_workspace_bytes",
           "ac_gemm_i8_auto_plan", "ac_gemm_bf16_auto_plan",
           "ac_status_string", "ac_version")

_lib = None


class AcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({status_string(status)})")


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library, with argument types declared."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2505_18574_amd.build` "
                "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, sz, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t, ctypes.c_float
        L.ac_gemm_i8.restype = i32
        L.ac_gemm_i8.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, i32, vp, sz, vp]
        L.ac_gemm_i8_static.restype = i32
        L.ac_gemm_i8_static.argtypes = L.ac_gemm_i8.argtypes[:-3] + [vp]
        L.ac_gemm_i8_workspace_bytes.restype = sz
        L.ac_gemm_i8_workspace_bytes.argtypes = [i32, i32, i32]
        L.ac_conv2d_i8.restype = i32
        L.ac_conv2d_i8.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, i32, i32, vp, sz, vp]
        L.ac_conv2d_i8_planned.restype = i32
        L.ac_conv2d_i8_planned.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, i32, i32, vp, sz, i32, i32, vp]
        L.ac_gemm_bf16.restype = i32
        L.ac_gemm_bf16.argtypes = [vp, i64, vp, i64, vp, i64, i32, i32, i32, f32, f32, vp]
        L.ac_batched_gemm_f32.restype = i32
        L.ac_batched_gemm_f32.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, vp]
        L.ac_gemm_i8_acc32.restype = i32
        L.ac_gemm_i8_acc32.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, i32, i32, i32, vp]
        L.ac_tinympc_forward_f32.restype = i32
        L.ac_tinympc_forward_f32.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i64, vp]
        L.ac_gemm_i8_t.restype = i32
        L.ac_gemm_i8_t.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, i32, i32, i32, vp]
        L.ac_gemm_i8_planned.restype = i32
        L.ac_gemm_i8_planned.argtypes = L.ac_gemm_i8.argtypes[:-1] + [i32, i32, vp]
        L.ac_gemm_i8_planned_workspace_bytes.restype = sz
        L.ac_gemm_i8_planned_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.ac_gemm_bf16_ws.restype = i32
        L.ac_gemm_bf16_ws.argtypes = L.ac_gemm_bf16.argtypes[:-1] + [vp, sz, vp]
        L.ac_gemm_bf16_workspace_bytes.restype = sz
        L.ac_gemm_bf16_workspace_bytes.argtypes = [i32, i32, i32]
        L.ac_gemm_bf16_planned.restype = i32
        L.ac_gemm_bf16_planned.argtypes = L.ac_gemm_bf16.argtypes[:-1] + [vp, sz, i32, i32, vp]
        L.ac_gemm_bf16_planned_workspace_bytes.restype = sz
        L.ac_gemm_bf16_planned_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
        pi32 = ctypes.POINTER(i32)
        L.ac_gemm_i8_auto_plan.restype = None
        L.ac_gemm_i8_auto_plan.argtypes = [i32, i32, i32, i32, pi32, pi32]
        L.ac_gemm_bf16_auto_plan.restype = None
        L.ac_gemm_bf16_auto_plan.argtypes = [i32, i32, i32, pi32, pi32]
        L.ac_status_string.restype = ctypes.c_char_p
        L.ac_status_string.argtypes = [i32]
        L.ac_version.restype = i32
        L.ac_version.argtypes = []
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().ac_status_string(int(status)).decode()


ac_status_string = status_string


def ac_version() -> int:
    return int(lib().ac_version())


def ac_gemm_i8_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().ac_gemm_i8_workspace_bytes(M, N, K))


def ac_gemm_i8_planned_workspace_bytes(M: int, N: int, K: int, tile: int, splits: int) -> int:
    return int(lib().ac_gemm_i8_planned_workspace_bytes(M, N, K, tile, splits))


def ac_gemm_bf16_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().ac_gemm_bf16_workspace_bytes(M, N, K))


def ac_gemm_bf16_planned_workspace_bytes(M: int, N: int, K: int, tile: int, splits: int) -> int:
    return int(lib().ac_gemm_bf16_planned_workspace_bytes(M, N, K, tile, splits))


def ac_gemm_i8_auto_plan(M: int, N: int, K: int, have_workspace: bool = True):
    """(tile, splits) that ac_gemm_i8 chooses for this shape."""
    tile, splits = ctypes.c_int32(0), ctypes.c_int32(0)
    lib().ac_gemm_i8_auto_plan(M, N, K, int(bool(have_workspace)), ctypes.byref(tile), ctypes.byref(splits))
    return tile.value, splits.value


def ac_gemm_bf16_auto_plan(M: int, N: int, K: int):
    """(tile, splits) that ac_gemm_bf16 chooses for this shape."""
    tile, splits = ctypes.c_int32(0), ctypes.c_int32(0)
    lib().ac_gemm_bf16_auto_plan(M, N, K, ctypes.byref(tile), ctypes.byref(splits))
    return tile.value, splits.value


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check2d(t, dtype, name):
    if t.dtype != dtype or t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1) or not t.is_cuda:
        raise ValueError(f"{name}: expected a 2-D row-major device tensor of {dtype}")


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _ptr(workspace), workspace.numel() * workspace.element_size()


def _gemm_i8_args(A, B, bias, C):
    _check2d(A, torch.int8, "A")
    _check2d(B, torch.int8, "B")
    _check2d(C, torch.int8, "C")
    M, K = A.shape
    N = B.shape[1]
    if B.shape[0] != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    bias_ld = 0
    if bias is not None:
        if bias.dtype != torch.int32 or not bias.is_cuda:
            raise ValueError("bias: expected int32 device tensor")
        if bias.dim() == 2:
            if tuple(bias.shape) != (M, N) or bias.stride(1) != 1:
                raise ValueError("bias matrix must be M x N row-major")
            bias_ld = bias.stride(0)
        elif tuple(bias.shape) != (N,) or (N > 1 and bias.stride(0) != 1):
            raise ValueError("bias vector must have N contiguous entries")
    return [_ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(bias), bias_ld, _ptr(C), C.stride(0), M, N, K]


def ac_gemm_i8(A, B, bias, C, shift: int, act: int = AC_ACT_NONE, workspace=None, stream=None):
    """C[M,N] int8 = stage(A[M,K] . B[K,N] + bias); bias is None, (N,) or (M,N) int32.  Returns C."""
    wp, wb = _ws(workspace)
    st = lib().ac_gemm_i8(*_gemm_i8_args(A, B, bias, C), shift, act, wp, wb, _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_gemm_i8")
    return C


AC_STATIC_SCRATCH_BYTES = 16 << 20


def ac_gemm_i8_static(A, B, bias, C, shift: int, act: int = AC_ACT_NONE, stream=None):
    """ac_gemm_i8 whose K-slice partial sums go through the buffer inside the library (no workspace, no allocation).  Returns C."""
    st = lib().ac_gemm_i8_static(*_gemm_i8_args(A, B, bias, C), shift, act, _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_gemm_i8_static")
    return C


def ac_gemm_i8_t(A, B, bias, C, shift: int, act: int = AC_ACT_NONE, trans_a: bool = False, trans_b: bool = False, stream=None):
    """ac_gemm_i8 with A given as A^T (K x M) when trans_a and B as B^T (N x K) when trans_b.  Returns C."""
    _check2d(A, torch.int8, "A")
    _check2d(B, torch.int8, "B")
    _check2d(C, torch.int8, "C")
    K, M = (A.shape if trans_a else A.shape[::-1])
    N, K2 = (B.shape if trans_b else B.shape[::-1])
    if K2 != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    bias_ld = 0
    if bias is not None:
        if bias.dtype != torch.int32 or not bias.is_cuda:
            raise ValueError("bias: expected int32 device tensor")
        if bias.dim() == 2:
            if tuple(bias.shape) != (M, N) or bias.stride(1) != 1:
                raise ValueError("bias matrix must be M x N row-major")
            bias_ld = bias.stride(0)
        elif tuple(bias.shape) != (N,) or (N > 1 and bias.stride(0) != 1):
            raise ValueError("bias vector must have N contiguous entries")
    st = lib().ac_gemm_i8_t(_ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(bias), bias_ld, _ptr(C), C.stride(0),
                            M, N, K, shift, act, int(bool(trans_a)), int(bool(trans_b)), _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_gemm_i8_t")
    return C


def ac_gemm_i8_planned(A, B, bias, C, shift: int, act: int, tile: int, splits: int, workspace=None, stream=None):
    """ac_gemm_i8 with the block tile code (64, 128, 192, 256; 320 / 160 = weight-stationary) and the K split named by the caller.  Returns C."""
    wp, wb = _ws(workspace)
    st = lib().ac_gemm_i8_planned(*_gemm_i8_args(A, B, bias, C), shift, act, wp, wb, tile, splits, _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_gemm_i8_planned")
    return C


def ac_conv2d_i8(x, w, bias, out, stride: int, pad: int, shift: int, act: int = AC_ACT_NONE, workspace=None, stream=None,
                 plan=None):
    """out[Nb,OH,OW,Cout] int8 = stage(conv(x[Nb,H,W,Cin], w[KH,KW,Cin,Cout]) + bias[Cout]).  Returns out.

    plan = (tile, splits) goes through ac_conv2d_i8_planned."""
    for t, name in ((x, "x"), (w, "w"), (out, "out")):
        if t.dtype != torch.int8 or t.dim() != 4 or not t.is_contiguous() or not t.is_cuda:
            raise ValueError(f"{name}: expected a dense 4-D int8 device tensor")
    Nb, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    if bias is not None and (bias.dtype != torch.int32 or tuple(bias.shape) != (Cout,) or not bias.is_contiguous()):
        raise ValueError("bias: expected (Cout,) int32")
    OH = (H + 2 * pad - KH) // stride + 1
    OW = (W + 2 * pad - KW) // stride + 1
    if tuple(out.shape) != (Nb, OH, OW, Cout):
        raise ValueError(f"out: expected shape {(Nb, OH, OW, Cout)}")
    wp, wb = _ws(workspace)
    if plan is not None:
        st = lib().ac_conv2d_i8_planned(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), Nb, H, W, Cin, Cout, KH, KW, stride, pad,
                                        shift, act, wp, wb, int(plan[0]), int(plan[1]), _stream(stream))
        if st != AC_OK:
            raise AcError(st, "ac_conv2d_i8_planned")
        return out
    st = lib().ac_conv2d_i8(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), Nb, H, W, Cin, Cout, KH, KW, stride, pad,
                            shift, act, wp, wb, _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_conv2d_i8")
    return out


def _gemm_bf16_args(A, B, C):
    ok = (torch.bfloat16, torch.int16, torch.uint16)
    for t, name in ((A, "A"), (B, "B")):
        if t.dtype not in ok or t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1) or not t.is_cuda:
            raise ValueError(f"{name}: expected a 2-D row-major bf16 device tensor")
    _check2d(C, torch.float32, "C")
    M, K = A.shape
    N = B.shape[1]
    if B.shape[0] != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    return [_ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(C), C.stride(0), M, N, K]


def ac_gemm_bf16(A, B, C, alpha: float = 1.0, beta: float = 0.0, stream=None):
    """C[M,N] fp32 = alpha * A[M,K] . B[K,N] + beta * C; A, B are bf16 (torch.bfloat16, or int16/uint16 bit patterns)."""
    st = lib().ac_gemm_bf16(*_gemm_bf16_args(A, B, C), float(alpha), float(beta), _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_gemm_bf16")
    return C


def ac_gemm_bf16_ws(A, B, C, alpha: float = 1.0, beta: float = 0.0, workspace=None, stream=None):
    """ac_gemm_bf16 that sums the slices of a cut K range through `workspace` (in a fixed order) when one is given.  Returns C."""
    wp, wb = _ws(workspace)
    st = lib().ac_gemm_bf16_ws(*_gemm_bf16_args(A, B, C), float(alpha), float(beta), wp, wb, _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_gemm_bf16_ws")
    return C


def ac_gemm_bf16_planned(A, B, C, alpha: float, beta: float, tile: int, splits: int, workspace=None, stream=None):
    """ac_gemm_bf16 with the block tile code (64, 128, 192, 256) and the K split named by the caller; a split sums through
    `workspace` when one is given, else with atomic adds into C.  Returns C."""
    wp, wb = _ws(workspace)
    st = lib().ac_gemm_bf16_planned(*_gemm_bf16_args(A, B, C), float(alpha), float(beta), wp, wb, tile, splits, _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_gemm_bf16_planned")
    return C


def ac_batched_gemm_f32(A, B, C=None, x=None, d=None, y=None, stream=None):
    """Per item: C = A . B (n x n), y = C . x + d.  A, B, C: [batch,n,n]; x, d, y: [batch,n]; fp32 dense."""
    for t, name in ((A, "A"), (B, "B"), (C, "C"), (x, "x"), (d, "d"), (y, "y")):
        if t is not None and (t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda):
            raise ValueError(f"{name}: expected a dense fp32 device tensor")
    batch, n, n2 = A.shape
    if n != n2 or tuple(B.shape) != (batch, n, n):
        raise ValueError("A, B must be [batch, n, n]")
    if C is not None and tuple(C.shape) != (batch, n, n):
        raise ValueError("C must be [batch, n, n]")
    for t, name in ((x, "x"), (d, "d"), (y, "y")):
        if t is not None and tuple(t.shape) != (batch, n):
            raise ValueError(f"{name} must be [batch, n]")
    st = lib().ac_batched_gemm_f32(_ptr(A), _ptr(B), _ptr(C), _ptr(x), _ptr(d), _ptr(y), n, batch, _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_batched_gemm_f32")
    return C, y


def ac_tinympc_forward_f32(Adyn, Bdyn, Kinf, x0, d, u, x_out=None, stream=None):
    """Batched TinyMPC forward pass: u[b,i] = -Kinf x[b,i] - d[b,i]; x[b,i+1] = Adyn x[b,i] + Bdyn u[b,i].

    Adyn [nx,nx], Bdyn [nx,nu], Kinf [nu,nx], x0 [batch,nx], d and u [batch,horizon,nu], x_out [batch,horizon+1,nx] or None."""
    for t, name in ((Adyn, "Adyn"), (Bdyn, "Bdyn"), (Kinf, "Kinf"), (x0, "x0"), (d, "d"), (u, "u"), (x_out, "x_out")):
        if t is not None and (t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda):
            raise ValueError(f"{name}: expected a dense fp32 device tensor")
    nx, nu = Bdyn.shape
    batch, horizon, nu2 = d.shape
    if tuple(Adyn.shape) != (nx, nx) or tuple(Kinf.shape) != (nu, nx) or nu2 != nu or tuple(x0.shape) != (batch, nx):
        raise ValueError("shape mismatch")
    if tuple(u.shape) != (batch, horizon, nu) or (x_out is not None and tuple(x_out.shape) != (batch, horizon + 1, nx)):
        raise ValueError("output shape mismatch")
    st = lib().ac_tinympc_forward_f32(_ptr(Adyn), _ptr(Bdyn), _ptr(Kinf), _ptr(x0), _ptr(d), _ptr(u), _ptr(x_out),
                                      nx, nu, horizon, batch, _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_tinympc_forward_f32")
    return u, x_out


def ac_gemm_i8_acc32(A, B, bias, C, stream=None):
    """C[M,N] int32 = A[M,K] . B[K,N] + bias (raw accumulator: no scaling, no activation).  Returns C."""
    _check2d(A, torch.int8, "A")
    _check2d(B, torch.int8, "B")
    _check2d(C, torch.int32, "C")
    M, K = A.shape
    N = B.shape[1]
    if B.shape[0] != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    bias_ld = 0
    if bias is not None:
        if bias.dtype != torch.int32 or not bias.is_cuda:
            raise ValueError("bias: expected int32 device tensor")
        if bias.dim() == 2:
            bias_ld = bias.stride(0)
    st = lib().ac_gemm_i8_acc32(_ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(bias), bias_ld, _ptr(C), C.stride(0),
                                M, N, K, _stream(stream))
    if st != AC_OK:
        raise AcError(st, "ac_gemm_i8_acc32")
    return C
