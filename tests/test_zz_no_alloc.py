"""The entry point that allocates nothing (ngemm_run_u8s8s32_static: row sums in a static device
array instead of a caller's workspace) against ngemm_run_u8s8s32, through the C ABI, bit for bit:
two calls in a row on one context, the second with a smaller input, with a weight zero-point so
that the scratch memory is really used (the 256 x 256 kernel reads its row sums from it)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_static_scratch_entry_matches_workspace_entry():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1910_00178_amd as ng
    from paper_1910_00178_amd import workloads as wl
    ctx = ng.ngemm_create(0)
    try:
        rng = wl.rng_for(6, 1)
        N, K = 520, 320
        B = wl.uniform_s8(rng, N, K)
        Bd = torch.from_numpy(B).cuda()
        nb = ng.ngemm_packed_b_bytes(K, N)
        packed = torch.empty(nb, dtype=torch.uint8, device="cuda")
        h = ng.ngemm_pack_b(ctx, K, N, Bd, K, packed, nb)
        # kernel forced to the 256 x 256 tiles (row sums by a pass of their own, through the scratch
        # memory), then the shape heuristic's choice; first the larger M, then the smaller one
        for kernel in (ng.NGEMM_KERNEL_TILE_256, ng.NGEMM_KERNEL_AUTO):
            ng.ngemm_set_kernel(ctx, kernel)
            for (M, za, zb) in ((1000, 131, -7), (300, 4, 5), (17, 255, -128)):
                print("static entry: kernel", kernel, "M", M, "za", za, "zb", zb, flush=True)
                A = wl.uniform_u8(rng, M, K)
                Ad = torch.from_numpy(A).cuda()
                wsb = ng.ngemm_workspace_bytes(M, N, K)
                ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
                want = torch.full((M + 1, N + 3), -77, dtype=torch.int32, device="cuda")
                got = torch.full((M + 1, N + 3), -77, dtype=torch.int32, device="cuda")
                ng.ngemm_run_u8s8s32(ctx, M, Ad, K, za, h, zb, want, N + 3, ws, wsb)
                ng.ngemm_run_u8s8s32_static(ctx, M, Ad, K, za, h, zb, got, N + 3)
                torch.cuda.synchronize()
                assert torch.equal(got, want), (kernel, M)
                assert int((got[:M, :N] != -77).sum()) > 0
        ng.ngemm_set_kernel(ctx, ng.NGEMM_KERNEL_AUTO)
        # beyond the static limit: a clear error, nothing launched
        C = torch.empty((1, N), dtype=torch.int32, device="cuda")
        with pytest.raises(ng.NgemmError) as e:
            ng.ngemm_run_u8s8s32_static(ctx, ng.NGEMM_STATIC_MAX_M + 1, Bd, K, 0, h, 0, C, N)
        assert e.value.status == ng.NGEMM_ERR_STATIC_LIMIT
        ng.ngemm_packed_b_free(h)
    finally:
        ng.ngemm_destroy(ctx)
