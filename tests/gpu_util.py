"""Helpers for the GPU parity tests: move seeded inputs to the device, call the C ABI through
the Python binding, bring results back.  No arithmetic of the method lives here."""
import numpy as np
import torch

import paper_1910_00178_amd as ng

SENTINEL32 = -1234567
SENTINEL8 = 0xA5


class Runner:
    def __init__(self, device=0):
        self.device = device
        self.ctx = ng.ngemm_create(device)
        self._keep = []

    def close(self):
        ng.ngemm_destroy(self.ctx)
        self.ctx = None

    def set_kernel(self, k):
        ng.ngemm_set_kernel(self.ctx, k)

    def pack(self, B, ldb_pad=0):
        """B: numpy int8 (N, K).  Returns (handle, packed device tensor)."""
        N, K = B.shape
        if ldb_pad:
            Bh = np.full((N, K + ldb_pad), 77, dtype=np.int8)
            Bh[:, :K] = B
        else:
            Bh = np.ascontiguousarray(B)
        Bd = torch.from_numpy(Bh).cuda(self.device) if Bh.size else torch.empty(0, dtype=torch.int8, device="cuda")
        nbytes = ng.ngemm_packed_b_bytes(K, N)
        packed = torch.full((max(nbytes, 16),), 0x5A, dtype=torch.uint8, device="cuda")
        h = ng.ngemm_pack_b(self.ctx, K, N, Bd, K + ldb_pad, packed, nbytes)
        torch.cuda.synchronize()
        return h, packed

    def run(self, A, handle, N, za=0, zb=0, scale=None, zc=0, lda_pad=0, ldc_pad=0, a_byte_offset=0,
            A_dev=None, small_ws=False):
        """One GEMM through the C ABI.  Returns the M x N numpy result (int32 or uint8) after
        checking that nothing outside the M x N window of C was written."""
        M, K = A.shape
        lda = K + lda_pad
        if A_dev is None:
            Ah = np.full(M * lda + a_byte_offset + 64, 201, dtype=np.uint8)
            view = Ah[a_byte_offset:a_byte_offset + M * lda].reshape(M, lda)
            view[:, :K] = A
            # the allocation ends right after the last valid byte of the last row
            Ah = Ah[:a_byte_offset + (M - 1) * lda + K] if M > 0 else Ah[:0]
            Abuf = torch.from_numpy(np.ascontiguousarray(Ah)).cuda(self.device) if Ah.size else \
                torch.empty(16, dtype=torch.uint8, device="cuda")
            a_ptr = Abuf.data_ptr() + a_byte_offset
        else:
            Abuf = A_dev
            a_ptr = A_dev.data_ptr()
        ldc = N + ldc_pad
        rows = M + 1
        if scale is None:
            Cd = torch.full((rows, max(ldc, 1)), SENTINEL32, dtype=torch.int32, device="cuda")
        else:
            Cd = torch.full((rows, max(ldc, 1)), SENTINEL8, dtype=torch.uint8, device="cuda")
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        if small_ws:                                   # the row sums only: no room for a K split's partial results
            wsb = min(wsb, (4 * M + 255) // 256 * 256)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        if scale is None:
            ng.ngemm_run_u8s8s32(self.ctx, M, a_ptr, lda, za, handle, zb, Cd, ldc, ws, wsb)
        else:
            ng.ngemm_run_u8s8u8_requant(self.ctx, M, a_ptr, lda, za, handle, zb, scale, zc, Cd, ldc, ws, wsb)
        torch.cuda.synchronize()
        out = Cd.cpu().numpy()
        sent = SENTINEL32 if scale is None else SENTINEL8
        assert np.all(out[M:, :] == sent), "rows past M were written"
        assert np.all(out[:M, N:] == sent), "the gap of the leading dimension was written"
        del Abuf
        return np.ascontiguousarray(out[:M, :N])


def unpack_packed(packed_bytes, K, N):
    """Invert the documented packed layout on the host (numpy): returns (B (N,K) int8,
    padding-all-zero flag, colsum int32[Np])."""
    Kp = (K + 63) // 64 * 64
    Np = (N + 31) // 32 * 32
    raw = np.asarray(packed_bytes, dtype=np.uint8)
    body = raw[:Kp * Np].view(np.int8)
    colsum = raw[Kp * Np:Kp * Np + 4 * Np].view(np.int32)
    if Kp * Np == 0:
        return np.zeros((N, K), np.int8), True, colsum
    ns = Kp // 32
    # [panel][slice][half][col][16 k]
    f = body.reshape(Np // 32, ns, 2, 32, 16)
    full = f.transpose(0, 3, 1, 2, 4).reshape(Np, Kp)       # (column, k)
    pad_zero = not full[N:, :].any() and not full[:, K:].any()
    return np.ascontiguousarray(full[:N, :K]), pad_zero, colsum
