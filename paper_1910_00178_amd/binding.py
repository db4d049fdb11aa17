"""ctypes binding of the C ABI in include/ngemm.h.  Argument marshalling only.

Every function has the name and argument order of its C counterpart.  Device
pointers may be given as integers or as torch tensors (their data_ptr() is
taken); a stream may be an integer hipStream_t, a torch.cuda.Stream or None
(torch's current stream).  There is no CPU fallback: if the library is missing
or cannot be loaded, importing this module raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libngemm.so")

NGEMM_OK = 0
NGEMM_ERR_INVALID_ARG = -1
NGEMM_ERR_BAD_SHAPE = -2
NGEMM_ERR_BUFFER_TOO_SMALL = -3
NGEMM_ERR_DEVICE = -4
NGEMM_ERR_UNSUPPORTED_ARCH = -5
NGEMM_ERR_STATIC_LIMIT = -6
NGEMM_STATIC_MAX_M = 65536

NGEMM_KERNEL_AUTO = -1
NGEMM_KERNEL_SKINNY = 0
NGEMM_KERNEL_TILE_64 = 1
NGEMM_KERNEL_TILE_128 = 2
NGEMM_KERNEL_TILE_256 = 3
NGEMM_KERNEL_SPLIT_K = 4
NGEMM_KERNEL_TILE_192 = 5

EXPORTS = (
    "ngemm_status_string", "ngemm_create", "ngemm_destroy", "ngemm_set_kernel", "ngemm_tune_u8s8s32", "ngemm_tuned_kernel", "ngemm_set_max_workgroups",
    "ngemm_packed_b_bytes", "ngemm_pack_b", "ngemm_pack_b_u8", "ngemm_packed_b_free", "ngemm_packed_b_shape",
    "ngemm_workspace_bytes", "ngemm_run_u8s8s32", "ngemm_run_u8s8s32_static", "ngemm_run_s8s8s32", "ngemm_run_u8u8s32", "ngemm_packed_b_bytes_s16", "ngemm_pack_b_s16", "ngemm_run_s16s16s32", "ngemm_run_u8s8u8_requant",
    "ngemm_run_u8s8u8_requant_channel", "ngemm_unpacked_workspace_bytes", "ngemm_run_u8s8s32_unpacked",
    "ngemm_batched_workspace_bytes", "ngemm_run_batched_u8s8s32",
)


class ngemm_problem(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("A_dev", ctypes.c_void_p), ("lda", ctypes.c_int64),
                ("a_zero_point", ctypes.c_int32), ("b_zero_point", ctypes.c_int32),
                ("B", ctypes.c_void_p), ("C_dev", ctypes.c_void_p), ("ldc", ctypes.c_int64)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1910_00178_amd.build` "
                      "(there is no fallback path)")
_lib = ctypes.CDLL(LIB_PATH)

_i64, _i32, _p, _sz, _f32, _int = (ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t,
                                   ctypes.c_float, ctypes.c_int)
_lib.ngemm_status_string.restype = ctypes.c_char_p
_lib.ngemm_status_string.argtypes = [_int]
_lib.ngemm_create.argtypes = [ctypes.POINTER(_p), _int]
_lib.ngemm_destroy.argtypes = [_p]
_lib.ngemm_set_kernel.argtypes = [_p, _int]
_lib.ngemm_set_max_workgroups.argtypes = [_p, _int]
_lib.ngemm_packed_b_bytes.restype = _sz
_lib.ngemm_packed_b_bytes.argtypes = [_i64, _i64]
_lib.ngemm_pack_b.argtypes = [_p, _i64, _i64, _p, _i64, _p, _sz, _p, ctypes.POINTER(_p)]
_lib.ngemm_pack_b_u8.argtypes = [_p, _i64, _i64, _p, _i64, _p, _sz, _p, ctypes.POINTER(_p)]
_lib.ngemm_pack_b_u8.restype = _int
_lib.ngemm_packed_b_free.argtypes = [_p]
_lib.ngemm_packed_b_shape.argtypes = [_p, ctypes.POINTER(_i64), ctypes.POINTER(_i64)]
_lib.ngemm_workspace_bytes.restype = _sz
_lib.ngemm_workspace_bytes.argtypes = [_i64, _i64, _i64]
_lib.ngemm_run_u8s8s32.argtypes = [_p, _i64, _p, _i64, _i32, _p, _i32, _p, _i64, _p, _sz, _p]
_lib.ngemm_run_u8s8s32_static.argtypes = [_p, _i64, _p, _i64, _i32, _p, _i32, _p, _i64, _p]
_lib.ngemm_run_u8s8s32_static.restype = _int
_lib.ngemm_tune_u8s8s32.argtypes = [_p, _i64, _p, _i64, _i32, _p, _i32, _p, _i64, _p, _sz, _p, ctypes.POINTER(_int)]
_lib.ngemm_tune_u8s8s32.restype = _int
_lib.ngemm_tuned_kernel.argtypes = [_p, _i64, _i64, _i64, ctypes.POINTER(_int)]
_lib.ngemm_tuned_kernel.restype = _int
_lib.ngemm_run_s8s8s32.argtypes = [_p, _i64, _p, _i64, _i32, _p, _i32, _p, _i64, _p, _sz, _p]
_lib.ngemm_run_s8s8s32.restype = _int
_lib.ngemm_run_u8u8s32.argtypes = [_p, _i64, _p, _i64, _i32, _p, _i32, _p, _i64, _p, _sz, _p]
_lib.ngemm_run_u8u8s32.restype = _int
_lib.ngemm_packed_b_bytes_s16.restype = _sz
_lib.ngemm_packed_b_bytes_s16.argtypes = [_i64, _i64]
_lib.ngemm_pack_b_s16.argtypes = [_p, _i64, _i64, _p, _i64, _p, _sz, _p, ctypes.POINTER(_p)]
_lib.ngemm_pack_b_s16.restype = _int
_lib.ngemm_run_s16s16s32.argtypes = [_p, _i64, _p, _i64, _i32, _p, _i32, _p, _i64, _p, _sz, _p]
_lib.ngemm_run_s16s16s32.restype = _int
_lib.ngemm_run_u8s8u8_requant.argtypes = [_p, _i64, _p, _i64, _i32, _p, _i32, _f32, _i32, _p, _i64,
                                          _p, _sz, _p]
_lib.ngemm_run_u8s8u8_requant_channel.argtypes = [_p, _i64, _p, _i64, _i32, _p, _i32, _p, _p, _p, _i32, _i32,
                                                  _p, _i64, _p, _sz, _p]
_lib.ngemm_run_u8s8u8_requant_channel.restype = _int
_lib.ngemm_unpacked_workspace_bytes.restype = _sz
_lib.ngemm_unpacked_workspace_bytes.argtypes = [_i64, _i64, _i64]
_lib.ngemm_run_u8s8s32_unpacked.argtypes = [_p, _i64, _i64, _i64, _p, _i64, _i32, _p, _i64, _i32, _p, _i64,
                                            _p, _sz, _p]
_lib.ngemm_run_u8s8s32_unpacked.restype = _int
_lib.ngemm_batched_workspace_bytes.restype = _sz
_lib.ngemm_batched_workspace_bytes.argtypes = [_int, ctypes.POINTER(ngemm_problem)]
_lib.ngemm_run_batched_u8s8s32.argtypes = [_p, _int, ctypes.POINTER(ngemm_problem), _p, _sz, _p]
for _name in ("ngemm_create", "ngemm_destroy", "ngemm_set_kernel", "ngemm_set_max_workgroups", "ngemm_pack_b", "ngemm_packed_b_free",
              "ngemm_packed_b_shape", "ngemm_run_u8s8s32", "ngemm_run_u8s8u8_requant",
              "ngemm_run_batched_u8s8s32"):
    getattr(_lib, _name).restype = _int


class NgemmError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {ngemm_status_string(status)} ({status})")


def _dev(x):
    """Device address of a tensor, or the integer itself."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr() or None
    return int(x) or None


def _stream(s):
    if s is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if hasattr(s, "cuda_stream"):
        return s.cuda_stream or None
    return int(s) or None


def _check(status, where):
    if status != NGEMM_OK:
        raise NgemmError(status, where)


def ngemm_status_string(status):
    return _lib.ngemm_status_string(int(status)).decode()


def ngemm_create(device_ordinal=0):
    h = _p()
    _check(_lib.ngemm_create(ctypes.byref(h), int(device_ordinal)), "ngemm_create")
    return h


def ngemm_destroy(ctx):
    _check(_lib.ngemm_destroy(ctx), "ngemm_destroy")


def ngemm_set_kernel(ctx, kernel):
    _check(_lib.ngemm_set_kernel(ctx, int(kernel)), "ngemm_set_kernel")


def ngemm_set_max_workgroups(ctx, max_workgroups):
    _check(_lib.ngemm_set_max_workgroups(ctx, int(max_workgroups)), "ngemm_set_max_workgroups")


def ngemm_packed_b_bytes(K, N):
    return int(_lib.ngemm_packed_b_bytes(int(K), int(N)))


def ngemm_pack_b(ctx, K, N, B_dev, ldb, packed_dev, packed_bytes, hip_stream=None):
    h = _p()
    _check(_lib.ngemm_pack_b(ctx, int(K), int(N), _dev(B_dev), int(ldb), _dev(packed_dev), int(packed_bytes),
                             _stream(hip_stream), ctypes.byref(h)), "ngemm_pack_b")
    return h


def ngemm_pack_b_u8(ctx, K, N, B_dev, ldb, packed_dev, packed_bytes, hip_stream=None):
    h = _p()
    _check(_lib.ngemm_pack_b_u8(ctx, int(K), int(N), _dev(B_dev), int(ldb), _dev(packed_dev), int(packed_bytes),
                                _stream(hip_stream), ctypes.byref(h)), "ngemm_pack_b_u8")
    return h


def ngemm_packed_b_free(b):
    _check(_lib.ngemm_packed_b_free(b), "ngemm_packed_b_free")


def ngemm_packed_b_shape(b):
    K, N = _i64(), _i64()
    _check(_lib.ngemm_packed_b_shape(b, ctypes.byref(K), ctypes.byref(N)), "ngemm_packed_b_shape")
    return K.value, N.value


def ngemm_workspace_bytes(M, N, K):
    return int(_lib.ngemm_workspace_bytes(int(M), int(N), int(K)))


def ngemm_run_u8s8s32(ctx, M, A_dev, lda, a_zero_point, B, b_zero_point, C_dev, ldc,
                      workspace_dev=None, workspace_bytes=0, hip_stream=None):
    _check(_lib.ngemm_run_u8s8s32(ctx, int(M), _dev(A_dev), int(lda), int(a_zero_point), B, int(b_zero_point),
                                  _dev(C_dev), int(ldc), _dev(workspace_dev), int(workspace_bytes),
                                  _stream(hip_stream)), "ngemm_run_u8s8s32")


def ngemm_run_u8s8s32_static(ctx, M, A_dev, lda, a_zero_point, B, b_zero_point, C_dev, ldc, hip_stream=None):
    _check(_lib.ngemm_run_u8s8s32_static(ctx, int(M), _dev(A_dev), int(lda), int(a_zero_point), B, int(b_zero_point),
                                         _dev(C_dev), int(ldc), _stream(hip_stream)), "ngemm_run_u8s8s32_static")


def ngemm_tune_u8s8s32(ctx, M, A_dev, lda, a_zero_point, B, b_zero_point, C_dev, ldc,
                       workspace_dev=None, workspace_bytes=0, hip_stream=None):
    """Returns the NGEMM_KERNEL_* value found fastest (and remembered) for this shape."""
    best = _int(-1)
    _check(_lib.ngemm_tune_u8s8s32(ctx, int(M), _dev(A_dev), int(lda), int(a_zero_point), B, int(b_zero_point),
                                   _dev(C_dev), int(ldc), _dev(workspace_dev), int(workspace_bytes),
                                   _stream(hip_stream), ctypes.byref(best)), "ngemm_tune_u8s8s32")
    return best.value


def ngemm_tuned_kernel(ctx, M, N, K):
    k = _int(-1)
    _check(_lib.ngemm_tuned_kernel(ctx, int(M), int(N), int(K), ctypes.byref(k)), "ngemm_tuned_kernel")
    return k.value


def ngemm_run_s8s8s32(ctx, M, A_dev, lda, a_zero_point, B, b_zero_point, C_dev, ldc,
                      workspace_dev=None, workspace_bytes=0, hip_stream=None):
    _check(_lib.ngemm_run_s8s8s32(ctx, int(M), _dev(A_dev), int(lda), int(a_zero_point), B, int(b_zero_point),
                                  _dev(C_dev), int(ldc), _dev(workspace_dev), int(workspace_bytes),
                                  _stream(hip_stream)), "ngemm_run_s8s8s32")


def ngemm_run_u8u8s32(ctx, M, A_dev, lda, a_zero_point, B, b_zero_point, C_dev, ldc,
                      workspace_dev=None, workspace_bytes=0, hip_stream=None):
    _check(_lib.ngemm_run_u8u8s32(ctx, int(M), _dev(A_dev), int(lda), int(a_zero_point), B, int(b_zero_point),
                                  _dev(C_dev), int(ldc), _dev(workspace_dev), int(workspace_bytes),
                                  _stream(hip_stream)), "ngemm_run_u8u8s32")


def ngemm_packed_b_bytes_s16(K, N):
    return int(_lib.ngemm_packed_b_bytes_s16(int(K), int(N)))


def ngemm_pack_b_s16(ctx, K, N, B_dev, ldb, packed_dev, packed_bytes, hip_stream=None):
    h = _p()
    _check(_lib.ngemm_pack_b_s16(ctx, int(K), int(N), _dev(B_dev), int(ldb), _dev(packed_dev), int(packed_bytes),
                                 _stream(hip_stream), ctypes.byref(h)), "ngemm_pack_b_s16")
    return h


def ngemm_run_s16s16s32(ctx, M, A_dev, lda, a_zero_point, B, b_zero_point, C_dev, ldc,
                        workspace_dev=None, workspace_bytes=0, hip_stream=None):
    _check(_lib.ngemm_run_s16s16s32(ctx, int(M), _dev(A_dev), int(lda), int(a_zero_point), B, int(b_zero_point),
                                    _dev(C_dev), int(ldc), _dev(workspace_dev), int(workspace_bytes),
                                    _stream(hip_stream)), "ngemm_run_s16s16s32")


def ngemm_run_u8s8u8_requant(ctx, M, A_dev, lda, a_zero_point, B, b_zero_point, scale, c_zero_point,
                             C_dev, ldc, workspace_dev=None, workspace_bytes=0, hip_stream=None):
    _check(_lib.ngemm_run_u8s8u8_requant(ctx, int(M), _dev(A_dev), int(lda), int(a_zero_point), B,
                                         int(b_zero_point), float(scale), int(c_zero_point), _dev(C_dev),
                                         int(ldc), _dev(workspace_dev), int(workspace_bytes),
                                         _stream(hip_stream)), "ngemm_run_u8s8u8_requant")


def ngemm_run_u8s8u8_requant_channel(ctx, M, A_dev, lda, a_zero_point, B, b_zero_point, b_zero_points_dev,
                                     scales_dev, bias_dev, relu, c_zero_point, C_dev, ldc,
                                     workspace_dev=None, workspace_bytes=0, hip_stream=None):
    _check(_lib.ngemm_run_u8s8u8_requant_channel(ctx, int(M), _dev(A_dev), int(lda), int(a_zero_point), B,
                                                 int(b_zero_point), _dev(b_zero_points_dev), _dev(scales_dev),
                                                 _dev(bias_dev), int(bool(relu)), int(c_zero_point), _dev(C_dev),
                                                 int(ldc), _dev(workspace_dev), int(workspace_bytes),
                                                 _stream(hip_stream)), "ngemm_run_u8s8u8_requant_channel")


def ngemm_unpacked_workspace_bytes(M, N, K):
    return int(_lib.ngemm_unpacked_workspace_bytes(int(M), int(N), int(K)))


def ngemm_run_u8s8s32_unpacked(ctx, M, N, K, A_dev, lda, a_zero_point, B_dev, ldb, b_zero_point, C_dev, ldc,
                               workspace_dev, workspace_bytes, hip_stream=None):
    _check(_lib.ngemm_run_u8s8s32_unpacked(ctx, int(M), int(N), int(K), _dev(A_dev), int(lda), int(a_zero_point),
                                           _dev(B_dev), int(ldb), int(b_zero_point), _dev(C_dev), int(ldc),
                                           _dev(workspace_dev), int(workspace_bytes), _stream(hip_stream)),
           "ngemm_run_u8s8s32_unpacked")


def make_problems(items):
    """items: iterable of (M, A_dev, lda, za, zb, B_handle, C_dev, ldc) -> ctypes array."""
    items = list(items)
    arr = (ngemm_problem * len(items))()
    for t, (M, A, lda, za, zb, B, C, ldc) in enumerate(items):
        arr[t] = ngemm_problem(int(M), _dev(A), int(lda), int(za), int(zb),
                               B.value if hasattr(B, "value") else B, _dev(C), int(ldc))
    return arr


def ngemm_batched_workspace_bytes(problems):
    return int(_lib.ngemm_batched_workspace_bytes(len(problems), problems))


def ngemm_run_batched_u8s8s32(ctx, problems, workspace_dev=None, workspace_bytes=0, hip_stream=None):
    _check(_lib.ngemm_run_batched_u8s8s32(ctx, len(problems), problems, _dev(workspace_dev),
                                          int(workspace_bytes), _stream(hip_stream)),
           "ngemm_run_batched_u8s8s32")
