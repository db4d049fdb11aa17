"""ctypes loader for oracle/ngemm_oracle.c.  TEST INFRASTRUCTURE ONLY.

Marshals numpy arrays into the plain C functions; holds no arithmetic of its
own.  Layout conventions (problem statement, Sec. 2.1 of the paper): A is
row-major u8 [M x K]; B is the s8 operand the paper stores as [N x K], i.e. a
column-major K x N matrix, passed here as a numpy array of shape (N, ldb);
C is row-major [M x N].
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ngemm_oracle.c")
_LIB = os.path.join(_HERE, "libngemm_oracle.so")
_lib = None

_CFLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-shared", "-fPIC", "-Wall", "-Wextra"]


_CHECK_SRC = os.path.join(_HERE, "sanitize_check.c")
_CHECK_EXE = os.path.join(_HERE, "sanitize_check.bin")


def build(force=False):
    """Compile the C oracle with gcc (seconds); with force, also the plain (unsanitized) build of
    the C driver that tests/test_oracle_sanitized.py runs under the sanitizers."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *_CFLAGS, "-o", _LIB, _SRC, "-lm"])
    if force:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
                               "-o", _CHECK_EXE, _SRC, _CHECK_SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, p, f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_float
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_gemm_u8s8s32.argtypes = [i64, i64, i64, p, i64, i32, p, i64, i32, p, i64]
        lib.oracle_gemm_u8s8s64.argtypes = [i64, i64, i64, p, i64, i32, p, i64, i32, p, i64]
        lib.oracle_requant_s32u8.argtypes = [i64, i64, p, i64, f32, i32, p, i64]
        lib.oracle_gemm_u8s8u8_requant.argtypes = [i64, i64, i64, p, i64, i32, p, i64, i32,
                                                   f32, i32, p, i64]
        lib.oracle_gemm_u8s8s32_sampled.argtypes = [i64, p, i64, i32, p, i64, i32, i64, p, p, p]
        lib.oracle_gemm_u8s8u8_requant_channel.argtypes = [i64, i64, i64, p, i64, i32, p, i64, i32, p, p, p,
                                                           i32, i32, p, i64]
        lib.oracle_gemm_u8s8u8_requant_channel.restype = None
        lib.oracle_gemm_s8s8s32.argtypes = [i64, i64, i64, p, i64, i32, p, i64, i32, p, i64]
        lib.oracle_gemm_s8s8s32.restype = None
        lib.oracle_gemm_u8u8s32.argtypes = [i64, i64, i64, p, i64, i32, p, i64, i32, p, i64]
        lib.oracle_gemm_u8u8s32.restype = None
        lib.oracle_gemm_s16s16s32.argtypes = [i64, i64, i64, p, i64, i32, p, i64, i32, p, i64]
        lib.oracle_gemm_s16s16s32.restype = None
        for name in ("oracle_gemm_u8s8s32", "oracle_gemm_u8s8s64", "oracle_requant_s32u8",
                     "oracle_gemm_u8s8u8_requant", "oracle_gemm_u8s8s32_sampled"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def _check_ab(A, B):
    assert A.dtype == np.uint8 and A.ndim == 2 and (A.size == 0 or A.strides[1] == 1)
    assert B.dtype == np.int8 and B.ndim == 2 and (B.size == 0 or B.strides[1] == 1)
    M, K = A.shape
    N, Kb = B.shape
    assert K == Kb, "A is (M,K); B is passed as (N,K): column j of the K x N operand is row j"
    lda = A.strides[0] if M > 1 and K > 0 else K
    ldb = B.strides[0] if N > 1 and K > 0 else K
    return M, N, K, lda, ldb


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def gemm_u8s8s32(A, B, za=0, zb=0, out=None):
    """C (M,N) int32 = wrap32(sum_k (A[i,k]-za)(B[j,k]-zb)).  B has shape (N,K)."""
    M, N, K, lda, ldb = _check_ab(A, B)
    C = np.empty((M, N), dtype=np.int32) if out is None else out
    assert C.dtype == np.int32 and C.shape == (M, N) and C.strides[1] == 4
    _load().oracle_gemm_u8s8s32(M, N, K, _ptr(A), lda, int(za), _ptr(B), ldb, int(zb),
                                _ptr(C), C.strides[0] // 4)
    return C


def gemm_u8s8s64(A, B, za=0, zb=0):
    """Untruncated int64 sums (for the overflow-bound pins)."""
    M, N, K, lda, ldb = _check_ab(A, B)
    C = np.empty((M, N), dtype=np.int64)
    _load().oracle_gemm_u8s8s64(M, N, K, _ptr(A), lda, int(za), _ptr(B), ldb, int(zb),
                                _ptr(C), N)
    return C


def requant_s32u8(C32, scale, zc):
    assert C32.dtype == np.int32 and C32.ndim == 2 and C32.strides[1] == 4
    M, N = C32.shape
    out = np.empty((M, N), dtype=np.uint8)
    _load().oracle_requant_s32u8(M, N, _ptr(C32), C32.strides[0] // 4,
                                 float(np.float32(scale)), int(zc), _ptr(out), N)
    return out


def gemm_u8s8u8_requant(A, B, za, zb, scale, zc):
    M, N, K, lda, ldb = _check_ab(A, B)
    out = np.empty((M, N), dtype=np.uint8)
    _load().oracle_gemm_u8s8u8_requant(M, N, K, _ptr(A), lda, int(za), _ptr(B), ldb, int(zb),
                                       float(np.float32(scale)), int(zc), _ptr(out), N)
    return out


def gemm_u8s8s32_sampled(A, B, rows, cols, za=0, zb=0):
    """out[t] = C[rows[t], cols[t]] without forming C."""
    M, N, K, lda, ldb = _check_ab(A, B)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    assert rows.shape == cols.shape and rows.ndim == 1
    assert rows.size == 0 or (rows.min() >= 0 and rows.max() < M and cols.min() >= 0 and cols.max() < N)
    out = np.empty(rows.shape, dtype=np.int32)
    _load().oracle_gemm_u8s8s32_sampled(K, _ptr(A), lda, int(za), _ptr(B), ldb, int(zb),
                                        rows.size, _ptr(rows), _ptr(cols), _ptr(out))
    return out


def gemm_u8s8u8_requant_channel(A, B, za, zb, scale, zc, zb_vec=None, bias=None, relu=False):
    """Per-column scales (float32[N]), optional per-column B zero-points and biases (int32[N]),
    optional ReLU in the quantised domain."""
    M, N, K, lda, ldb = _check_ab(A, B)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    assert scale.shape == (N,)
    zbv = None if zb_vec is None else np.ascontiguousarray(zb_vec, dtype=np.int32)
    bv = None if bias is None else np.ascontiguousarray(bias, dtype=np.int32)
    assert zbv is None or zbv.shape == (N,)
    assert bv is None or bv.shape == (N,)
    out = np.empty((M, N), dtype=np.uint8)
    _load().oracle_gemm_u8s8u8_requant_channel(
        M, N, K, _ptr(A), lda, int(za), _ptr(B), ldb, int(zb),
        None if zbv is None else _ptr(zbv), _ptr(scale), None if bv is None else _ptr(bv),
        1 if relu else 0, int(zc), _ptr(out), N)
    return out


def gemm_s8s8s32(A, B, za=0, zb=0):
    """Signed variant: A int8 (M,K), B int8 (N,K)."""
    assert A.dtype == np.int8 and A.ndim == 2 and (A.size == 0 or A.strides[1] == 1)
    assert B.dtype == np.int8 and B.ndim == 2 and (B.size == 0 or B.strides[1] == 1)
    M, K = A.shape
    N, Kb = B.shape
    assert K == Kb
    lda = A.strides[0] if M > 1 and K > 0 else K
    ldb = B.strides[0] if N > 1 and K > 0 else K
    C = np.empty((M, N), dtype=np.int32)
    _load().oracle_gemm_s8s8s32(M, N, K, _ptr(A), lda, int(za), _ptr(B), ldb, int(zb), _ptr(C), N)
    return C


def gemm_u8u8s32(A, B, za=0, zb=0):
    """Unsigned-weight variant: A uint8 (M,K), B uint8 (N,K)."""
    assert A.dtype == np.uint8 and A.ndim == 2 and (A.size == 0 or A.strides[1] == 1)
    assert B.dtype == np.uint8 and B.ndim == 2 and (B.size == 0 or B.strides[1] == 1)
    M, K = A.shape
    N, Kb = B.shape
    assert K == Kb
    lda = A.strides[0] if M > 1 and K > 0 else K
    ldb = B.strides[0] if N > 1 and K > 0 else K
    C = np.empty((M, N), dtype=np.int32)
    _load().oracle_gemm_u8u8s32(M, N, K, _ptr(A), lda, int(za), _ptr(B), ldb, int(zb), _ptr(C), N)
    return C


def gemm_s16s16s32(A, B, za=0, zb=0):
    """16-bit variant: A int16 (M,K), B int16 (N,K); leading dimensions in elements."""
    assert A.dtype == np.int16 and A.ndim == 2 and (A.size == 0 or A.strides[1] == 2)
    assert B.dtype == np.int16 and B.ndim == 2 and (B.size == 0 or B.strides[1] == 2)
    M, K = A.shape
    N, Kb = B.shape
    assert K == Kb
    lda = A.strides[0] // 2 if M > 1 and K > 0 else K
    ldb = B.strides[0] // 2 if N > 1 and K > 0 else K
    C = np.empty((M, N), dtype=np.int32)
    _load().oracle_gemm_s16s16s32(M, N, K, _ptr(A), lda, int(za), _ptr(B), ldb, int(zb), _ptr(C), N)
    return C
