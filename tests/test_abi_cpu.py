"""CPU-side checks of the boundary: the library loads, exports every symbol the header
declares, and its pure host functions follow the documented sizes.  No compute calls."""
import ctypes
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ngemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ngemm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_1910_00178_amd as ng
    lib = ctypes.CDLL(ng.LIB_PATH)
    names = declared_functions()
    assert {"ngemm_create", "ngemm_pack_b", "ngemm_run_u8s8s32", "ngemm_destroy",
            "ngemm_run_u8s8u8_requant"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(ng.EXPORTS)


def test_packed_size_is_matrix_size():
    import paper_1910_00178_amd as ng
    # the pack-memory comparison of Sec. 5: a 512 x 512 int8 weight packs into its own size
    assert ng.ngemm_packed_b_bytes(512, 512) == 512 * 512 + 4 * 512
    for K, N in ((1, 1), (64, 32), (65, 33), (768, 3072), (1024, 4096), (8192, 8192), (0, 5), (5, 0)):
        Kp, Np = (K + 63) // 64 * 64, (N + 31) // 32 * 32
        assert ng.ngemm_packed_b_bytes(K, N) == Kp * Np + 4 * Np
    assert ng.ngemm_packed_b_bytes(-1, 4) == 0


def test_workspace_and_status_strings():
    import paper_1910_00178_amd as ng
    assert ng.ngemm_workspace_bytes(1, 10, 10) == 256
    assert ng.ngemm_workspace_bytes(1000, 10, 10) == 4096
    assert ng.ngemm_workspace_bytes(0, 10, 10) == 0
    # few tiles and a long K: room for the partial results of the K split, at most 4 MiB
    assert ng.ngemm_workspace_bytes(64, 64, 65536) == 256 + 64 * 64 * 64 * 4
    assert ng.ngemm_workspace_bytes(512, 512, 65536) == 2048 + 4 * 512 * 512 * 4
    assert ng.ngemm_workspace_bytes(512, 512, 1024) == 2048
    assert ng.ngemm_workspace_bytes(4096, 4096, 65536) == 16384
    seen = {ng.ngemm_status_string(s) for s in range(-6, 1)}
    assert len(seen) == 7 and "ok" in seen


def test_handles_reject_garbage_on_host():
    import paper_1910_00178_amd as ng
    lib = ctypes.CDLL(ng.LIB_PATH)
    lib.ngemm_destroy.argtypes = [ctypes.c_void_p]
    lib.ngemm_packed_b_free.argtypes = [ctypes.c_void_p]
    assert lib.ngemm_destroy(None) == 0
    assert lib.ngemm_packed_b_free(None) == 0
    buf = (ctypes.c_char * 128)()
    assert lib.ngemm_destroy(ctypes.addressof(buf)) == ng.NGEMM_ERR_INVALID_ARG
    assert lib.ngemm_packed_b_free(ctypes.addressof(buf)) == ng.NGEMM_ERR_INVALID_ARG


def test_unpack_helper_inverts_documented_layout():
    """The host-side inverse used by the GPU pack test, checked against a direct transcription
    of the header's byte-offset formula."""
    from gpu_util import unpack_packed
    rng = np.random.default_rng(3)
    K, N = 70, 37
    Kp, Np = 128, 64
    B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
    raw = np.zeros(Kp * Np + 4 * Np, dtype=np.uint8)
    for j in range(N):
        for k in range(K):
            off = 1024 * ((j // 32) * (Kp // 32) + k // 32) + 16 * (32 * ((k % 32) // 16) + j % 32) + k % 16
            raw[off] = B[j, k].view(np.uint8)
    raw[Kp * Np:].view(np.int32)[:N] = B.astype(np.int64).sum(1)
    back, pad_zero, colsum = unpack_packed(raw, K, N)
    assert np.array_equal(back, B) and pad_zero
    assert np.array_equal(colsum[:N], B.astype(np.int64).sum(1))
