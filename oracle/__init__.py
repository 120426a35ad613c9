"""CPU oracle (test infrastructure only).

Thin ctypes loader around ``oracle.c``: the plain, slow definition of the dense
tensor operations of arxiv 2505.18574 that the GPU library is checked against.
Nothing in the product path may import this package; it exists for the tests,
the smoke check and the CPU-baseline leg of the benchmark.  It imports nothing
from the GPU package and shares no code with it.

``build()`` compiles ``oracle.c`` with gcc; ``lib()`` loads the result (building
it first only if no built library is present).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")
_LIB = None

ACT_NONE = 0
ACT_RELU = 1


def build() -> str:
    """Compile oracle.c -> liboracle.so (gcc -O2, OpenMP over independent rows)."""
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, _SRC]
    subprocess.run(cmd, check=True)
    global _LIB
    _LIB = None
    return _SO


def lib() -> ctypes.CDLL:
    global _LIB
    if _LIB is None:
        if not os.path.exists(_SO):
            build()
        L = ctypes.CDLL(_SO)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        dbl = ctypes.c_double
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_rne_rshift.restype = i64
        L.oracle_rne_rshift.argtypes = [i64, i32]
        L.oracle_requantise.restype = ctypes.c_int8
        L.oracle_requantise.argtypes = [i64, i32, i32]
        L.oracle_rne_rshift_vec.restype = None
        L.oracle_rne_rshift_vec.argtypes = [vp, i32, vp, i64]
        L.oracle_requantise_vec.restype = None
        L.oracle_requantise_vec.argtypes = [vp, i32, i32, vp, i64]
        L.oracle_gemm_i8.restype = i64
        L.oracle_gemm_i8.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, i64, i64, i64, i32, i32, vp]
        L.oracle_conv2d_i8.restype = i64
        L.oracle_conv2d_i8.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, i64, i64, i32, i32]
        L.oracle_im2col_i8.restype = None
        L.oracle_im2col_i8.argtypes = [vp, vp, i64, i64, i64, i64, i64, i64, i64, i64]
        L.oracle_bf16_to_double.restype = dbl
        L.oracle_bf16_to_double.argtypes = [ctypes.c_uint16]
        L.oracle_gemm_bf16.restype = None
        L.oracle_gemm_bf16.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, i64, i64, dbl, dbl]
        L.oracle_gemm_bf16_at.restype = None
        L.oracle_gemm_bf16_at.argtypes = [vp, i64, vp, i64, vp, i64, i64, dbl, dbl, vp, vp, i64, vp, vp]
        L.oracle_gemm_i8_at.restype = None
        L.oracle_gemm_i8_at.argtypes = [vp, i64, vp, i64, vp, i64, i64, i32, i32, vp, vp, i64, vp]
        L.oracle_batched_gemm_f32.restype = None
        L.oracle_batched_gemm_f32.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64]
        L.oracle_tinympc_forward.restype = None
        L.oracle_tinympc_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64]
        _LIB = L
    return _LIB


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def rne_rshift(v: int, s: int) -> int:
    return int(lib().oracle_rne_rshift(int(v), int(s)))


def requantise(acc: int, shift: int, act: int) -> int:
    return int(lib().oracle_requantise(int(acc), int(shift), int(act)))


def rne_rshift_vec(v, s: int):
    v = _c(v, np.int64)
    out = np.empty_like(v)
    lib().oracle_rne_rshift_vec(_p(v), int(s), _p(out), v.size)
    return out


def requantise_vec(acc, shift: int, act: int):
    acc = _c(acc, np.int64)
    out = np.empty(acc.shape, dtype=np.int8)
    lib().oracle_requantise_vec(_p(acc), int(shift), int(act), _p(out), acc.size)
    return out


def gemm_i8(A, B, bias=None, shift=0, act=ACT_NONE, return_acc=False):
    """A: (M,K) int8, B: (K,N) int8, bias: None | (N,) | (M,N) int32 -> (M,N) int8.

    Raises if an exact sum does not fit int32 (the accelerator's accumulator type)."""
    A = _c(A, np.int8)
    B = _c(B, np.int8)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    bias_ld = 0
    if bias is not None:
        bias = _c(bias, np.int32)
        if bias.ndim == 2:
            assert bias.shape == (M, N)
            bias_ld = N
        else:
            assert bias.shape == (N,)
    C = np.empty((M, N), dtype=np.int8)
    acc = np.empty((M, N), dtype=np.int64) if return_acc else None
    ovf = lib().oracle_gemm_i8(_p(A), max(K, 1), _p(B), max(N, 1), _p(bias), bias_ld, _p(C), max(N, 1),
                               M, N, K, shift, act, _p(acc))
    if ovf:
        raise OverflowError(f"{ovf} sums do not fit int32")
    return (C, acc) if return_acc else C


def gemm_i8_at(A, B, bias, shift, act, rows, cols):
    A = _c(A, np.int8)
    B = _c(B, np.int8)
    K = A.shape[1]
    N = B.shape[1]
    bias_ld = 0
    if bias is not None:
        bias = _c(bias, np.int32)
        bias_ld = N if bias.ndim == 2 else 0
    rows = _c(rows, np.int64)
    cols = _c(cols, np.int64)
    out = np.empty(rows.shape[0], dtype=np.int8)
    lib().oracle_gemm_i8_at(_p(A), K, _p(B), N, _p(bias), bias_ld, K, shift, act, _p(rows), _p(cols), rows.shape[0], _p(out))
    return out


def conv_out_size(H, KH, stride, pad):
    return (H + 2 * pad - KH) // stride + 1


def conv2d_i8(x, w, bias=None, stride=1, pad=0, shift=0, act=ACT_NONE):
    """x: (Nb,H,W,Cin) int8, w: (KH,KW,Cin,Cout) int8, bias: (Cout,) int32 -> (Nb,OH,OW,Cout) int8."""
    x = _c(x, np.int8)
    w = _c(w, np.int8)
    Nb, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    assert Cin == Cin2
    if bias is not None:
        bias = _c(bias, np.int32)
        assert bias.shape == (Cout,)
    OH, OW = conv_out_size(H, KH, stride, pad), conv_out_size(W, KW, stride, pad)
    out = np.empty((Nb, max(OH, 0), max(OW, 0), Cout), dtype=np.int8)
    ovf = lib().oracle_conv2d_i8(_p(x), _p(w), _p(bias), _p(out), Nb, H, W, Cin, Cout, KH, KW, stride, pad, shift, act)
    if ovf:
        raise OverflowError(f"{ovf} sums do not fit int32")
    return out


def im2col_i8(x, KH, KW, stride, pad):
    x = _c(x, np.int8)
    Nb, H, W, Cin = x.shape
    OH, OW = conv_out_size(H, KH, stride, pad), conv_out_size(W, KW, stride, pad)
    col = np.empty((Nb * OH * OW, KH * KW * Cin), dtype=np.int8)
    lib().oracle_im2col_i8(_p(x), _p(col), Nb, H, W, Cin, KH, KW, stride, pad)
    return col


def bf16_to_double(bits):
    bits = np.asarray(bits, dtype=np.uint16)
    f = lib().oracle_bf16_to_double
    return np.array([f(int(b)) for b in bits.ravel()], dtype=np.float64).reshape(bits.shape)


def gemm_bf16(A_bits, B_bits, alpha=1.0, beta=0.0, C_in=None):
    """A_bits: (M,K) uint16 bf16 patterns, B_bits: (K,N); returns fp64 (M,N)."""
    A = _c(A_bits, np.uint16)
    B = _c(B_bits, np.uint16)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    if C_in is not None:
        C_in = _c(C_in, np.float32)
        assert C_in.shape == (M, N)
    elif beta != 0.0:
        raise ValueError("beta != 0 needs C_in")
    out = np.empty((M, N), dtype=np.float64)
    lib().oracle_gemm_bf16(_p(A), max(K, 1), _p(B), max(N, 1), _p(C_in), max(N, 1), _p(out), M, N, K, float(alpha), float(beta))
    return out


def gemm_bf16_at(A_bits, B_bits, rows, cols, alpha=1.0, beta=0.0, C_in=None):
    """Spot values of gemm_bf16 at (rows[s], cols[s]); returns (values, sum_k |a*b|)."""
    A = _c(A_bits, np.uint16)
    B = _c(B_bits, np.uint16)
    K = A.shape[1]
    N = B.shape[1]
    if C_in is not None:
        C_in = _c(C_in, np.float32)
    rows = _c(rows, np.int64)
    cols = _c(cols, np.int64)
    out = np.empty(rows.shape[0], dtype=np.float64)
    mag = np.empty(rows.shape[0], dtype=np.float64)
    lib().oracle_gemm_bf16_at(_p(A), K, _p(B), N, _p(C_in), N, K, float(alpha), float(beta), _p(rows), _p(cols),
                              rows.shape[0], _p(out), _p(mag))
    return out, mag


def batched_gemm_f32(A, B, x=None, d=None):
    """A, B: (batch,n,n) fp32; x, d: (batch,n) fp32 -> (C fp64 (batch,n,n), y fp64 (batch,n) or None)."""
    A = _c(A, np.float32)
    B = _c(B, np.float32)
    batch, n, n2 = A.shape
    assert n == n2 and B.shape == A.shape and n <= 32
    C = np.empty((batch, n, n), dtype=np.float64)
    y = None
    if x is not None:
        x = _c(x, np.float32)
        assert x.shape == (batch, n)
        if d is not None:
            d = _c(d, np.float32)
            assert d.shape == (batch, n)
        y = np.empty((batch, n), dtype=np.float64)
    lib().oracle_batched_gemm_f32(_p(A), _p(B), _p(C), _p(x), _p(d), _p(y), n, batch)
    return C, y


def tinympc_forward(Adyn, Bdyn, Kinf, x0, d, return_x=False):
    """Adyn (nx,nx), Bdyn (nx,nu), Kinf (nu,nx), x0 (batch,nx), d (batch,horizon,nu) fp32 -> u fp64."""
    Adyn = _c(Adyn, np.float32)
    Bdyn = _c(Bdyn, np.float32)
    Kinf = _c(Kinf, np.float32)
    x0 = _c(x0, np.float32)
    d = _c(d, np.float32)
    nx = Adyn.shape[0]
    nu = Bdyn.shape[1]
    batch, horizon, _ = d.shape
    assert Adyn.shape == (nx, nx) and Bdyn.shape == (nx, nu) and Kinf.shape == (nu, nx)
    assert x0.shape == (batch, nx) and d.shape == (batch, horizon, nu) and nx <= 64 and nu <= 64
    u = np.empty((batch, horizon, nu), dtype=np.float64)
    xs = np.empty((batch, horizon + 1, nx), dtype=np.float64) if return_x else None
    lib().oracle_tinympc_forward(_p(Adyn), _p(Bdyn), _p(Kinf), _p(x0), _p(d), _p(u), _p(xs), nx, nu, horizon, batch)
    return (u, xs) if return_x else u
