"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer and byte results must match bit for bit (tolerance 0): the integer sum
is unique and the requantise sequence is fixed operation by operation."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_1910_00178_amd import workloads as wl  # noqa: E402


@pytest.fixture(scope="module")
def rt():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1910_00178_amd as ng  # noqa: F401  (raises if the library is missing)
    from gpu_util import Runner
    r = Runner(0)
    yield r
    r.close()


def ng_mod():
    import paper_1910_00178_amd as ng
    return ng


TILE_KERNELS = (1, 2, 3, 4, 5)   # 4: the K split; it runs the 64 x 64 tiles where it cannot split; 5: 192 x 256 tiles


def check_problem(rt, oracle, prob, kernels, **kw):
    ng = ng_mod()
    want32 = oracle.gemm_u8s8s32(prob.A, prob.B, prob.za, prob.zb)
    h, packed = rt.pack(prob.B, ldb_pad=kw.pop("ldb_pad", 0))
    try:
        for k in kernels:
            if k == ng.NGEMM_KERNEL_SKINNY and prob.M > 32:
                continue
            rt.set_kernel(k)
            got = rt.run(prob.A, h, prob.N, prob.za, prob.zb, **kw)
            assert np.array_equal(got, want32), f"{prob.name} kernel {k}: {np.count_nonzero(got != want32)} mismatches"
            if prob.scale is not None:
                want8 = oracle.gemm_u8s8u8_requant(prob.A, prob.B, prob.za, prob.zb, prob.scale, prob.zc)
                got8 = rt.run(prob.A, h, prob.N, prob.za, prob.zb, scale=prob.scale, zc=prob.zc, **kw)
                assert np.array_equal(got8, want8), f"{prob.name} kernel {k} requant"
    finally:
        rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
        ng.ngemm_packed_b_free(h)


def test_pack_layout_roundtrip(rt):
    """The packed buffer follows the documented layout, pads with zeros, holds exact column sums,
    and is exactly the padded matrix plus 4 bytes per padded column (no blow-up)."""
    from gpu_util import unpack_packed
    ng = ng_mod()
    assert ng.ngemm_packed_b_bytes(512, 512) == 512 * 512 + 4 * 512
    rng = np.random.default_rng(5)
    for (N, K, pad) in ((64, 256, 0), (33, 65, 3), (1, 1, 0), (100, 1000, 7), (517, 129, 1), (31, 63, 0)):
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        h, packed = rt.pack(B, ldb_pad=pad)
        nbytes = ng.ngemm_packed_b_bytes(K, N)
        back, pad_zero, colsum = unpack_packed(packed.cpu().numpy()[:nbytes], K, N)
        assert np.array_equal(back, B)
        assert pad_zero
        assert np.array_equal(colsum[:N], B.astype(np.int64).sum(1).astype(np.int32))
        assert not colsum[N:].any()
        assert ng.ngemm_packed_b_shape(h) == (K, N)
        ng.ngemm_packed_b_free(h)


def test_config1_tiny(rt, oracle):
    p = wl.tiny()
    check_problem(rt, oracle, p, TILE_KERNELS + (-1,))
    check_problem(rt, oracle, p, TILE_KERNELS, lda_pad=5, ldc_pad=3, ldb_pad=9)


@pytest.mark.parametrize("index", [0, 1, 2])
def test_config2_bert_fc(rt, oracle, index):
    p = wl.bert_fc(index)
    check_problem(rt, oracle, p, TILE_KERNELS + (-1,))


@pytest.mark.parametrize("M", [1, 4, 16])
def test_config3_skinny_pack_once_reuse(rt, oracle, M):
    """Pack once, 1000 calls cycling through a pool of 16 inputs, every pool member verified,
    packed bytes unchanged at the end."""
    ng = ng_mod()
    probs = wl.skinny(M)
    B = probs[0].B
    N, K = B.shape
    h, packed = rt.pack(B)
    before = packed.clone()
    A_dev = [torch.from_numpy(p.A).cuda() for p in probs]
    # every output sits between two sentinel rows and has a sentinel column gap (ldc = N + 8)
    C_dev = [torch.full((M + 2, N + 8), -7, dtype=torch.int32, device="cuda") for _ in probs]
    for it in range(1000):
        t = it % len(probs)
        ng.ngemm_run_u8s8s32(rt.ctx, M, A_dev[t], K, 0, h, 0, C_dev[t][1:], N + 8)
    torch.cuda.synchronize()
    for t, p in enumerate(probs):
        got = C_dev[t].cpu().numpy()
        assert np.all(got[0] == -7) and np.all(got[M + 1] == -7) and np.all(got[:, N:] == -7), (M, t)
        assert np.array_equal(got[1:M + 1, :N], oracle.gemm_u8s8s32(p.A, B)), (M, t)
    assert torch.equal(before, packed)
    ng.ngemm_packed_b_free(h)


def test_config4_large_square(rt, oracle):
    """8192^3 in the benchmark's launch configuration: a slab of rows element by element, sampled
    elements over the whole matrix, and an exact Freivalds-style check of all of C."""
    ng = ng_mod()
    p = wl.large_square()
    n = p.M
    h, packed = rt.pack(p.B)
    Ad = torch.from_numpy(p.A).cuda()
    Cd = torch.empty((n, n), dtype=torch.int32, device="cuda")
    ng.ngemm_run_u8s8s32(rt.ctx, n, Ad, n, 0, h, 0, Cd, n)
    torch.cuda.synchronize()
    C = Cd.cpu().numpy()
    # (1) slab: rows straddling a 256-row tile boundary
    rows = np.r_[0:8, 252:260, n - 8:n]
    assert np.array_equal(C[rows], oracle.gemm_u8s8s32(np.ascontiguousarray(p.A[rows]), p.B))
    # (2) samples everywhere
    rng = np.random.default_rng(44)
    ri = rng.integers(0, n, size=20000)
    ci = rng.integers(0, n, size=20000)
    assert np.array_equal(C[ri, ci], oracle.gemm_u8s8s32_sampled(p.A, p.B, ri, ci))
    # (3) C x == A (B x) exactly in int64 for small random x: catches any single wrong element
    for s in range(4):
        x = np.random.default_rng(100 + s).integers(-8, 9, size=n).astype(np.int64)
        Bx = np.zeros(n, dtype=np.int64)
        for j0 in range(0, n, 1024):
            Bx += p.B[j0:j0 + 1024].astype(np.int64).T @ x[j0:j0 + 1024]
        lhs = np.zeros(n, dtype=np.int64)
        rhs = np.zeros(n, dtype=np.int64)
        for i0 in range(0, n, 1024):
            lhs[i0:i0 + 1024] = C[i0:i0 + 1024].astype(np.int64) @ x
            rhs[i0:i0 + 1024] = p.A[i0:i0 + 1024].astype(np.int64) @ Bx
        assert np.array_equal(lhs, rhs)
    ng.ngemm_packed_b_free(h)


def test_config5_batched_mixed(rt, oracle):
    ng = ng_mod()
    probs = wl.batched()
    handles, keep, items, outs = [], [], [], []
    for p in probs:
        h, packed = rt.pack(p.B)
        Ad = torch.from_numpy(p.A).cuda()
        Cd = torch.full((p.M, p.N), -9, dtype=torch.int32, device="cuda")
        handles.append(h)
        keep.append((packed, Ad))
        outs.append(Cd)
        items.append((p.M, Ad, p.K, p.za, p.zb, h, Cd, p.N))
    arr = ng.make_problems(items)
    wsb = ng.ngemm_batched_workspace_bytes(arr)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    ng.ngemm_run_batched_u8s8s32(rt.ctx, arr, ws, wsb)
    torch.cuda.synchronize()
    for p, Cd in zip(probs, outs):
        want = oracle.gemm_u8s8s32(p.A, p.B, p.za, p.zb)
        got = Cd.cpu().numpy()
        assert np.array_equal(got, want), f"{p.name} za={p.za} zb={p.zb}: {np.count_nonzero(got != want)} mismatches"
    for h in handles:
        ng.ngemm_packed_b_free(h)


def test_batched_degenerate_members(rt, oracle):
    """A batch mixing empty members (M = 0, N = 0, K = 0), skinny and tiled members, with and
    without a weight zero-point, several argument blocks' worth of each kind of them."""
    ng = ng_mod()
    rng = np.random.default_rng(91)
    shapes = [(0, 5, 7), (5, 0, 7), (5, 7, 0), (1, 1, 1), (33, 65, 129), (32, 64, 64), (70, 3, 300)]
    shapes += [(int(rng.integers(1, 90)), int(rng.integers(1, 90)), int(rng.integers(1, 200))) for _ in range(200)]
    items, outs, probs, keep, handles = [], [], [], [], []
    for t, (M, N, K) in enumerate(shapes):
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        za, zb = int(rng.integers(0, 256)), (0 if t % 3 == 0 else int(rng.integers(-128, 128)))
        h, packed = rt.pack(B)
        Ad = torch.from_numpy(A).cuda() if A.size else torch.empty(16, dtype=torch.uint8, device="cuda")
        Cd = torch.full((max(M, 1), max(N, 1)), -9, dtype=torch.int32, device="cuda")
        handles.append(h); keep.append((packed, Ad)); outs.append(Cd)
        probs.append((A, B, za, zb))
        items.append((M, Ad, K, za, zb, h, Cd, max(N, 1)))
    arr = ng.make_problems(items)
    wsb = ng.ngemm_batched_workspace_bytes(arr)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    ng.ngemm_run_batched_u8s8s32(rt.ctx, arr, ws, wsb)
    torch.cuda.synchronize()
    for (M, N, K), (A, B, za, zb), Cd in zip(shapes, probs, outs):
        got = Cd.cpu().numpy()
        if M == 0 or N == 0:
            assert np.all(got == -9)
            continue
        assert np.array_equal(got[:M, :N], oracle.gemm_u8s8s32(A, B, za, zb)), (M, N, K, za, zb)
    for h in handles:
        ng.ngemm_packed_b_free(h)


EDGE_DIMS = (1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 129, 255, 257)


def test_edge_shapes_all_kernels(rt, oracle):
    """Ragged tails in every dimension, every kernel, zero-points at their extremes, odd leading
    dimensions and a misaligned A pointer."""
    rng = np.random.default_rng(77)
    zps = ((0, 0), (128, 0), (255, -128), (0, 127), (77, -8), (1, 1))
    for t in range(60):
        M = int(rng.choice(EDGE_DIMS))
        N = int(rng.choice(EDGE_DIMS))
        K = int(rng.choice(EDGE_DIMS + (300, 513)))
        za, zb = zps[t % len(zps)]
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        p = wl.Problem(f"edge{t}_{M}x{N}x{K}", A, B, za=za, zb=zb,
                       scale=float(np.float32(0.004)) if t % 3 == 0 else None, zc=100)
        check_problem(rt, oracle, p, (0, 1, 2, 3, -1), lda_pad=int(rng.integers(0, 4)),
                      ldc_pad=int(rng.integers(0, 3)), a_byte_offset=int(rng.integers(0, 4)))


def test_large_tile_kernel_k_edges(rt, oracle):
    """The 256 x 256 kernel on 16-byte aligned rows (its copy path) around every boundary of its K
    pipeline: two full stages (the fewest it takes), odd and even numbers of full stages (A moves
    in double stages of 128 bytes; an odd last stage is fetched 64 bytes early), with and without
    a partial stage behind them, ragged M and N, int32 and requantised output, and B both packed
    and as a plain input."""
    ng = ng_mod()
    rng = np.random.default_rng(79)
    # K < 128 goes to the 32 x 32 x 32 form of the same tiling (the other kernel needs two full stages)
    ks = (16, 64, 100, 127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 383, 384, 449, 576, 639, 1000, 1088)
    dims = ((1, 260), (255, 1), (257, 250), (300, 513), (512, 256))
    for t, K in enumerate(ks):
        M, N = dims[t % len(dims)]
        za, zb = ((0, 0), (128, 0), (255, -128), (77, 9))[t % 4]
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        p = wl.Problem(f"kedge_{M}x{N}x{K}", A, B, za=za, zb=zb, scale=float(np.float32(0.003)), zc=31)
        check_problem(rt, oracle, p, (3, 5), lda_pad=(-K) % 16, ldb_pad=t % 3)   # 5: the 192 x 256 form of the same kernel
        if M > 32:
            ld = K + (-K) % 16
            Ah = np.zeros((M, ld), dtype=np.uint8); Ah[:, :K] = A
            Bh = np.zeros((N, ld), dtype=np.int8); Bh[:, :K] = B
            Ad, Bd = torch.from_numpy(Ah).cuda(), torch.from_numpy(Bh).cuda()
            wsb = ng.ngemm_unpacked_workspace_bytes(M, N, K)
            ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
            Cd = torch.full((M, N), -5, dtype=torch.int32, device="cuda")
            rt.set_kernel(3)
            try:
                ng.ngemm_run_u8s8s32_unpacked(rt.ctx, M, N, K, Ad, ld, za, Bd, ld, zb, Cd, N, ws, wsb)
                torch.cuda.synchronize()
            finally:
                rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
            assert np.array_equal(Cd.cpu().numpy(), oracle.gemm_u8s8s32(A, B, za, zb)), (M, N, K, "plain B")


def test_operands_beyond_4_gib(rt, oracle):
    """Maximum sizes: an A operand and a B operand of more than 4 GiB each (the 256 x 256 kernel
    addresses its copies with 32-bit offsets from each tile's first row / panel, the pack and the
    epilogue with 64-bit ones).  Sampled outputs, weighted towards the rows and columns past the
    4 GiB mark, against the oracle; zero-points on, so the row and column sums are covered too."""
    ng = ng_mod()
    rng = np.random.default_rng(80)
    big, small, K = 66000, 300, 65536
    for a_is_big in (True, False):
        M, N = (big, small) if a_is_big else (small, big)
        # rank-one-plus-noise operands: cheap to generate at this size, every row and column distinct
        A = (rng.integers(0, 256, size=(M, 1), dtype=np.uint8) + rng.integers(0, 256, size=(1, K), dtype=np.uint8))
        B = (rng.integers(-128, 128, size=(N, 1), dtype=np.int8) + rng.integers(-128, 128, size=(1, K), dtype=np.int8))
        assert A.dtype == np.uint8 and B.dtype == np.int8 and max(A.nbytes, B.nbytes) > 1 << 32
        za, zb = 117, -5
        Ad, Bd = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
        nbytes = ng.ngemm_packed_b_bytes(K, N)
        packed = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        h = ng.ngemm_pack_b(rt.ctx, K, N, Bd, K, packed, nbytes)
        del Bd
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        Cd = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
        rt.set_kernel(3)
        try:
            ng.ngemm_run_u8s8s32(rt.ctx, M, Ad, K, za, h, zb, Cd, N, ws, wsb)
            torch.cuda.synchronize()
        finally:
            rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
        nb = big - (1 << 32) // K                      # rows / columns past the 4 GiB mark
        far = rng.integers(big - nb, big, size=3000)
        anyb = rng.integers(0, big, size=3000)
        bi = np.concatenate([far, anyb, [0, big - 1, (1 << 32) // K - 1, (1 << 32) // K]])
        si = rng.integers(0, small, size=bi.size)
        ri, ci = (bi, si) if a_is_big else (si, bi)
        got = Cd[torch.from_numpy(ri).cuda(), torch.from_numpy(ci).cuda()].cpu().numpy()
        want = oracle.gemm_u8s8s32_sampled(A, B, ri, ci, za, zb)
        assert np.array_equal(got, want), ("A" if a_is_big else "B", np.count_nonzero(got != want))
        ng.ngemm_packed_b_free(h)
        del Ad, packed, Cd, ws, A, B


def test_skinny_all_row_counts(rt, oracle):
    rng = np.random.default_rng(78)
    for M in range(1, 33):
        K = int(rng.choice((64, 100, 1024, 2050)))
        N = int(rng.choice((32, 40, 4096 if M % 8 == 0 else 96)))
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        p = wl.Problem(f"skinny{M}", A, B, za=int(rng.integers(0, 256)), zb=int(rng.integers(-3, 4)),
                       scale=float(np.float32(0.002)), zc=128)
        check_problem(rt, oracle, p, (0,))


def test_skinny_wide_outputs_share_a_fragments(rt, oracle):
    """Outputs wide enough for the skinny kernel to give a workgroup 2 or 4 panels (one A
    fragment used against several panels), with a ragged last workgroup."""
    rng = np.random.default_rng(93)
    for (M, N, K) in ((9, 32768 + 40, 96), (16, 40000, 64), (17, 32768 + 72, 100), (32, 32768 + 8, 64), (3, 40000, 70),
                      (5, 9000, 200), (20, 8192 + 17, 64)):
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        p = wl.Problem(f"wide{M}x{N}x{K}", A, B, za=int(rng.integers(0, 256)), zb=int(rng.integers(-5, 6)),
                       scale=float(np.float32(0.01)), zc=100)
        check_problem(rt, oracle, p, (0,))


def test_streaming_skinny_single_calls(rt, oracle):
    """Outputs wide enough (2048 panels and more) for the streaming kernel: a whole panel per
    wavefront, A in LDS, a ragged last chunk and a ragged last panel, K tails, a K of one slice
    pair, the row paddings 8 / 16 / 32, zero-points of both operands, int32 and requantised
    outputs, an unaligned A."""
    rng = np.random.default_rng(2024)
    for (M, N, K, aoff) in ((1, 65536 + 5, 200, 0), (7, 65536 + 40, 64, 3), (16, 70001, 130, 0), (17, 65536 + 33, 1000, 1),
                            (32, 66000, 96, 0), (8, 65537, 1, 0), (9, 65600, 2048, 0)):
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        p = wl.Problem(f"stream{M}x{N}x{K}", A, B, za=int(rng.integers(0, 256)), zb=int(rng.integers(-5, 6)),
                       scale=float(np.float32(0.004)), zc=77)
        check_problem(rt, oracle, p, (0,), a_byte_offset=aoff, lda_pad=(5 if aoff else 0), ldc_pad=(3 if M == 7 else 0))
        p0 = wl.Problem(f"stream{M}x{N}x{K}_nozb", A, B, za=int(rng.integers(0, 256)), zb=0)
        check_problem(rt, oracle, p0, (0,))


def test_streaming_skinny_grouped(rt, oracle):
    """Grouped calls whose skinny members have panels enough for the streaming kernel: members of
    different M, N, K (tails in all three), with and without a weight zero-point, next to members
    the streaming kernel cannot serve (A too large for LDS, K = 0) and tiled members; more
    members than one argument block holds (84)."""
    ng = ng_mod()
    rng = np.random.default_rng(2025)
    shapes = []
    for t in range(100):
        M = int(rng.integers(1, 33))
        N = int(rng.integers(300, 1200))
        K = int(rng.choice((64, 65, 128, 200, 1000, 1024, 2048, 2100, 4096 + 7)))
        shapes.append((M, N, K))
    shapes += [(32, 400, 2048), (32, 400, 2049), (16, 300, 4096), (16, 300, 4097), (8, 100, 8192), (8, 100, 8200),
               (3, 50, 0), (40, 70, 300), (1, 1, 1)]
    items, outs, probs, keep, handles = [], [], [], [], []
    for t, (M, N, K) in enumerate(shapes):
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        za, zb = int(rng.integers(0, 256)), (0 if t % 2 == 0 else int(rng.integers(-128, 128)))
        h, packed = rt.pack(B)
        Ad = torch.from_numpy(A).cuda() if A.size else torch.empty(16, dtype=torch.uint8, device="cuda")
        Cd = torch.full((M + 1, N + 2), -9, dtype=torch.int32, device="cuda")
        handles.append(h); keep.append((packed, Ad)); outs.append(Cd)
        probs.append((A, B, za, zb))
        items.append((M, Ad, K, za, zb, h, Cd, N + 2))
    arr = ng.make_problems(items)
    ng.ngemm_run_batched_u8s8s32(rt.ctx, arr)
    torch.cuda.synchronize()
    for (M, N, K), (A, B, za, zb), Cd in zip(shapes, probs, outs):
        got = Cd.cpu().numpy()
        assert np.all(got[M:, :] == -9) and np.all(got[:, N:] == -9), (M, N, K)
        assert np.array_equal(got[:M, :N], oracle.gemm_u8s8s32(A, B, za, zb)), (M, N, K, za, zb)
    for h in handles:
        ng.ngemm_packed_b_free(h)


def test_batched_mixed_groups_over_the_member_limit(rt, oracle):
    """Grouped calls whose skinny and tiled members share one grid: 150 members (more than two argument
    blocks hold), skinny ones of few panels next to tiled ones, extreme zero-points on both kinds
    (the member record keeps 128 - za and zb as 16-bit values), long K on a few panels, sentinel rows
    and columns around every output."""
    ng = ng_mod()
    rng = np.random.default_rng(77)
    shapes = []
    for t in range(150):
        if t % 3 == 0:
            shapes.append((int(rng.integers(1, 33)), int(rng.integers(1, 200)), int(rng.integers(1, 700))))
        else:
            shapes.append((int(rng.integers(33, 200)), int(rng.integers(1, 200)), int(rng.integers(1, 400))))
    shapes += [(4, 40, 3000), (150, 3, 2700), (32, 33, 65), (33, 32, 64)]
    zps = [(0, -128), (255, 127), (0, 127), (255, -128)]
    items, outs, probs, keep, handles = [], [], [], [], []
    for t, (M, N, K) in enumerate(shapes):
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        za, zb = zps[t % 4] if t % 5 == 0 else (int(rng.integers(0, 256)), int(rng.integers(-128, 128)))
        h, packed = rt.pack(B)
        Ad = torch.from_numpy(A).cuda()
        Cd = torch.full((M + 1, N + 3), -9, dtype=torch.int32, device="cuda")
        handles.append(h); keep.append((packed, Ad)); outs.append(Cd)
        probs.append((A, B, za, zb))
        items.append((M, Ad, K, za, zb, h, Cd, N + 3))
    arr = ng.make_problems(items)
    ng.ngemm_run_batched_u8s8s32(rt.ctx, arr)
    torch.cuda.synchronize()
    for (M, N, K), (A, B, za, zb), Cd in zip(shapes, probs, outs):
        got = Cd.cpu().numpy()
        assert np.all(got[M:, :] == -9) and np.all(got[:, N:] == -9), (M, N, K)
        assert np.array_equal(got[:M, :N], oracle.gemm_u8s8s32(A, B, za, zb)), (M, N, K, za, zb)
    for h in handles:
        ng.ngemm_packed_b_free(h)


def test_extreme_values_and_wrap(rt, oracle):
    """All-255 x all-(-128)/127 operands: no 16-bit stage, exact at the int32 bound, wraps beyond."""
    for (K, b) in ((64, 127), (64, -128), (65793, -128), (65794, -128), (66311, 127), (66312, 127)):
        A = np.full((33, K), 255, np.uint8)
        B = np.full((40, K), b, np.int8)
        p = wl.Problem(f"extreme_K{K}_b{b}", A, B)
        check_problem(rt, oracle, p, (1, 3))
    A = np.full((8, 65794), 255, np.uint8)
    B = np.full((32, 65794), -128, np.int8)
    check_problem(rt, oracle, wl.Problem("extreme_skinny", A, B), (0,))


def test_degenerate_sizes(rt, oracle):
    ng = ng_mod()
    # K == 0: every element is the empty sum
    h, packed = rt.pack(np.zeros((5, 0), np.int8))
    got = rt.run(np.zeros((3, 0), np.uint8), h, 5, za=9, zb=4)
    assert np.array_equal(got, np.zeros((3, 5), np.int32))
    got = rt.run(np.zeros((40, 0), np.uint8), h, 5, za=9, zb=4)
    assert np.array_equal(got, np.zeros((40, 5), np.int32))
    # M == 0: nothing written
    got = rt.run(np.zeros((0, 0), np.uint8), h, 5)
    assert got.shape == (0, 5)
    ng.ngemm_packed_b_free(h)
    # N == 0
    h, packed = rt.pack(np.zeros((0, 16), np.int8))
    got = rt.run(np.ones((4, 16), np.uint8), h, 0)
    assert got.shape == (4, 0)
    ng.ngemm_packed_b_free(h)


def test_kernels_agree_with_each_other(rt, oracle):
    """Sec. 2.1: any tiling / reduction order gives the same integers."""
    ng = ng_mod()
    rng = np.random.default_rng(79)
    A = rng.integers(0, 256, size=(300, 1111), dtype=np.uint8)
    B = rng.integers(-128, 128, size=(555, 1111), dtype=np.int8)
    h, packed = rt.pack(B)
    res = []
    for k in TILE_KERNELS:
        rt.set_kernel(k)
        res.append(rt.run(A, h, 555, 13, -5))
    rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
    want = oracle.gemm_u8s8s32(A, B, 13, -5)
    assert len(res) == len(TILE_KERNELS)
    for k, got in zip(TILE_KERNELS, res):
        assert np.array_equal(got, res[0]), k
        assert np.array_equal(got, want), k
    ng.ngemm_packed_b_free(h)


def test_persistent_workgroups_many_tiles_each(rt, oracle):
    """Few persistent workgroups over many 256 x 256 (and 192 x 256) tiles: every workgroup walks several tiles,
    reusing its LDS ring and epilogue patches.  Ragged M, N, K, zero-points, a leading-dimension
    gap in C, and the requantised output."""
    ng = ng_mod()
    rng = np.random.default_rng(81)
    M, N, K = 1000, 1100, 2000 + 37
    A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
    p = wl.Problem("persistent", A, B, za=99, zb=-7, scale=float(np.float32(0.0005)), zc=120)
    try:
        for nwg in (1, 3, 7, 8):
            ng.ngemm_set_max_workgroups(rt.ctx, nwg)
            # lda_pad 27 keeps rows 16-byte aligned (K + 27 = 2064), so the direct-to-LDS kernel runs
            check_problem(rt, oracle, p, (3, 5), lda_pad=27, ldc_pad=5)      # 256 x 256 and 192 x 256 tiles
    finally:
        ng.ngemm_set_max_workgroups(rt.ctx, 0)


def test_long_pipeline_small_tile_kernel(rt, oracle):
    """Outputs with at most one 64 x 64 (128 x 128) tile per compute unit and K >= 512 take the
    long-pipeline variant of the small-tile kernels: even and odd numbers of stages, every count
    of sub-blocks in the partial stage, K tails, ragged M and N, several tiles per workgroup,
    both epilogues."""
    ng = ng_mod()
    rng = np.random.default_rng(98)
    shapes = ((64, 64, 512), (100, 130, 768), (130, 70, 1000), (65, 65, 576), (200, 300, 1300), (64, 128, 4096),
              (33, 1000, 640), (1024, 768, 1793), (129, 257, 704), (500, 640, 2048))
    for t, (M, N, K) in enumerate(shapes):
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        za, zb = int(rng.integers(0, 256)), (0 if t % 2 else int(rng.integers(-128, 128)))
        lda = (K + 15) // 16 * 16                      # 16-byte aligned rows: the direct-to-LDS kernels
        prob = wl.Problem("deep%d" % t, A, B, za, zb, 0.0003, 77)
        both = (ng.NGEMM_KERNEL_TILE_64, ng.NGEMM_KERNEL_TILE_128)     # 64 x 64 and 128 x 128 forms
        check_problem(rt, oracle, prob, both, lda_pad=lda - K)
        ng.ngemm_set_max_workgroups(rt.ctx, 3)
        try:
            check_problem(rt, oracle, prob, both, lda_pad=lda - K)
        finally:
            ng.ngemm_set_max_workgroups(rt.ctx, 0)


def test_row_sums_inside_tile_kernels(rt, oracle):
    """With a zero-point of B and 16-byte aligned rows of A the 64 x 64 and 128 x 128 kernels (many
    tiles per compute unit: the direct-to-LDS form; few: the long-pipeline form) add up the row sums
    themselves instead of reading them from a pass before the kernel: K with and without a tail
    (whose zero fill must not count), K below one stage, ragged M and N, int32 and u8 outputs, a
    zero-point per column, the signed-A entry point."""
    ng = ng_mod()
    rng = np.random.default_rng(84)
    shapes = ((1100, 1100, 200), (1100, 1100, 193), (2100, 2100, 130), (1100, 1200, 64), (1100, 1100, 40),
              (300, 200, 1000), (300, 200, 1024))
    for t, (M, N, K) in enumerate(shapes):
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        za, zb = int(rng.integers(0, 256)), (int(rng.integers(1, 128)) if t % 2 else int(rng.integers(-128, 0)))
        pad = (-K) % 16
        prob = wl.Problem("rows%d" % t, A, B, za, zb, 0.0004, 77)
        check_problem(rt, oracle, prob, (ng.NGEMM_KERNEL_TILE_64, ng.NGEMM_KERNEL_TILE_128), lda_pad=pad, ldc_pad=t % 2)
        # per-column zero-points of B through the same kernels
        zbv = rng.integers(-8, 9, size=N).astype(np.int32)
        scale = (10.0 ** rng.uniform(-4, -3, size=N)).astype(np.float32)
        h, packed = rt.pack(B)
        Ah = np.zeros((M, K + pad), np.uint8)
        Ah[:, :K] = A
        Ad = torch.from_numpy(Ah).cuda()
        sd, zd = torch.from_numpy(scale).cuda(), torch.from_numpy(zbv).cuda()
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        want = oracle.gemm_u8s8u8_requant_channel(A, B, za, 0, scale, 100, zb_vec=zbv, bias=None, relu=False)
        for k in (ng.NGEMM_KERNEL_TILE_64, ng.NGEMM_KERNEL_TILE_128):
            rt.set_kernel(k)
            try:
                Cd = torch.full((M, N), 0xA5, dtype=torch.uint8, device="cuda")
                ng.ngemm_run_u8s8u8_requant_channel(rt.ctx, M, Ad, K + pad, za, h, 0, zd, sd, None, False, 100, Cd, N, ws, wsb)
                torch.cuda.synchronize()
            finally:
                rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
            assert np.array_equal(Cd.cpu().numpy(), want), (M, N, K, k, "per-column zb")
        ng.ngemm_packed_b_free(h)
        if t < 3:
            As = (A.astype(np.int16) - 128).astype(np.int8)
            Asd = torch.from_numpy(np.pad(As, ((0, 0), (0, pad)))).cuda()
            h, packed = rt.pack(B)
            for k in (ng.NGEMM_KERNEL_TILE_64, ng.NGEMM_KERNEL_TILE_128):
                rt.set_kernel(k)
                try:
                    Cd = torch.full((M, N), -3, dtype=torch.int32, device="cuda")
                    ng.ngemm_run_s8s8s32(rt.ctx, M, Asd, K + pad, -5, h, zb, Cd, N, ws, wsb)
                    torch.cuda.synchronize()
                finally:
                    rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
                assert np.array_equal(Cd.cpu().numpy(), oracle.gemm_s8s8s32(As, B, -5, zb)), (M, N, K, k, "signed A")
            ng.ngemm_packed_b_free(h)


def test_split_k_kernel(rt, oracle):
    """Few 64 x 64 tiles and a long K: K is cut into parts over the workgroups; with room in the
    workspace the parts store their partial tiles and a second kernel sums them (int32 and u8
    outputs), with a workspace for the row sums only C is cleared and the parts add their partial
    tiles with atomic adds (bit-exact in any order).  Forced and by the heuristic; ragged
    M, N and K (a last part that is only a tail, parts with a partial stage), zero-points on,
    leading-dimension gaps with sentinels (the clearing must stay inside M x N), the wrap of the
    int32 sum across parts, the signed-A entry point, and the calls it cannot serve (u8 output,
    unaligned rows of A, short K), which must run the 64 x 64 tiles instead."""
    ng = ng_mod()
    rng = np.random.default_rng(83)
    shapes = ((64, 64, 4096), (100, 70, 5000), (33, 200, 8191), (256, 256, 16384), (65, 1, 2048 + 17),
              (40, 40, 66000), (200, 130, 2047), (64, 64, 2048), (129, 65, 12345), (500, 33, 4097), (33, 33, 262144 + 3),
              (16, 256, 16384), (1, 64, 9000), (32, 1024, 8192 + 5), (700, 520, 8192 + 64))
    for t, (M, N, K) in enumerate(shapes):
        za, zb = ((0, 0), (128, 0), (255, -128), (77, 9))[t % 4]
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        p = wl.Problem(f"splitk_{M}x{N}x{K}", A, B, za=za, zb=zb, scale=float(np.float32(0.0002)), zc=31)
        check_problem(rt, oracle, p, (ng.NGEMM_KERNEL_SPLIT_K, ng.NGEMM_KERNEL_AUTO), lda_pad=(-K) % 16, ldc_pad=5)
        check_problem(rt, oracle, p, (ng.NGEMM_KERNEL_SPLIT_K, ng.NGEMM_KERNEL_AUTO), lda_pad=(-K) % 16, ldc_pad=5,
                      small_ws=True)
        if t % 3 == 0:
            check_problem(rt, oracle, p, (ng.NGEMM_KERNEL_SPLIT_K,), lda_pad=(-K) % 16 + 3, ldc_pad=1)   # unaligned rows
    # fewer workgroups than compute units: fewer, longer parts
    for budget in (5, 8, 40):
        ng.ngemm_set_max_workgroups(rt.ctx, budget)
        try:
            for (M, N, K) in ((64, 64, 8192), (100, 70, 5000), (130, 130, 9000 + 3)):
                A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
                B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
                p = wl.Problem(f"splitk_budget{budget}_{M}x{N}x{K}", A, B, za=3, zb=-4, scale=float(np.float32(0.0002)), zc=9)
                check_problem(rt, oracle, p, (ng.NGEMM_KERNEL_SPLIT_K,), lda_pad=(-K) % 16)
        finally:
            ng.ngemm_set_max_workgroups(rt.ctx, 0)
    # the sum wraps at K = 65794 with these values, whatever the number of parts
    for (K, b) in ((65793, -128), (65794, -128), (66312, 127)):
        A = np.full((64, K), 255, dtype=np.uint8)
        B = np.full((70, K), b, dtype=np.int8)
        p = wl.Problem(f"splitk_wrap_{K}", A, B, za=0, zb=0)
        check_problem(rt, oracle, p, (ng.NGEMM_KERNEL_SPLIT_K,), lda_pad=(-K) % 16)
        check_problem(rt, oracle, p, (ng.NGEMM_KERNEL_SPLIT_K,), lda_pad=(-K) % 16, small_ws=True)
    # s8 x s8 through the same kernel
    M, N, K = 70, 90, 9000 + 16
    A = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
    B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
    h, packed = rt.pack(B)
    Ad = torch.from_numpy(A).cuda()
    wsb = ng.ngemm_workspace_bytes(M, N, K)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    Cd = torch.full((M, N), -3, dtype=torch.int32, device="cuda")
    rt.set_kernel(ng.NGEMM_KERNEL_SPLIT_K)
    try:
        ng.ngemm_run_s8s8s32(rt.ctx, M, Ad, K, -7, h, 11, Cd, N, ws, wsb)
        torch.cuda.synchronize()
    finally:
        rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
    assert np.array_equal(Cd.cpu().numpy(), oracle.gemm_s8s8s32(A, B, -7, 11))
    ng.ngemm_packed_b_free(h)


def test_per_channel_epilogue(rt, oracle):
    """Per-column scales, biases and B zero-points with and without the fused ReLU, on every
    kernel, against the oracle's per-column form; ragged shapes and odd leading dimensions."""
    ng = ng_mod()
    rng = np.random.default_rng(94)
    # the 65700-column case is wide enough for the streaming skinny kernel (one panel per wavefront)
    cases = [(7, 100, 300), (32, 4096, 128), (200, 333, 500), (300, 520, 1008), (64, 64, 64), (33, 1, 17), (260, 300, 1024),
             (3, 65700, 96)]
    for t, (M, N, K) in enumerate(cases):
        A = np.clip(np.rint(rng.normal(128, 40, size=(M, K))), 0, 255).astype(np.uint8)
        B = np.clip(np.rint(rng.normal(0, 30, size=(N, K))), -127, 127).astype(np.int8)
        za, zc = int(rng.integers(100, 156)), int(rng.integers(0, 200))
        zbv = rng.integers(-8, 9, size=N).astype(np.int32)
        bias = rng.integers(-20000, 20000, size=N).astype(np.int32)
        scale = (10.0 ** rng.uniform(-4, -2.5, size=N)).astype(np.float32)
        h, packed = rt.pack(B)
        lda, ldc = K + (t % 3), N + (t % 2) * 3
        Ah = np.zeros((M, lda), np.uint8)
        Ah[:, :K] = A
        Ad = torch.from_numpy(Ah).cuda()
        sd, bd, zd = torch.from_numpy(scale).cuda(), torch.from_numpy(bias).cuda(), torch.from_numpy(zbv).cuda()
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        kernels = (0,) if M <= 32 else (1, 2, 3)
        for k in kernels:
            rt.set_kernel(k)
            for (use_zbv, use_bias, relu, zb) in ((True, True, True, 0), (False, True, False, 3),
                                                  (True, False, False, 0), (False, False, True, 0)):
                Cd = torch.full((M + 1, ldc), 0xA5, dtype=torch.uint8, device="cuda")
                ng.ngemm_run_u8s8u8_requant_channel(rt.ctx, M, Ad, lda, za, h, zb, zd if use_zbv else None, sd,
                                                    bd if use_bias else None, relu, zc, Cd, ldc, ws, wsb)
                torch.cuda.synchronize()
                got = Cd.cpu().numpy()
                want = oracle.gemm_u8s8u8_requant_channel(A, B, za, zb, scale, zc, zb_vec=zbv if use_zbv else None,
                                                          bias=bias if use_bias else None, relu=relu)
                assert np.array_equal(got[:M, :N], want), (M, N, K, k, use_zbv, use_bias, relu)
                assert np.all(got[M:, :] == 0xA5) and np.all(got[:M, N:] == 0xA5)
        rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
        ng.ngemm_packed_b_free(h)


def test_requant_extremes(rt, oracle):
    """The requantising epilogues at the edges of their arithmetic: products of the accumulator and
    the scale at and beyond +-2^31 (where the rounded value leaves the int32 range), output
    zero-points at the ends of the int32 range, with and without ReLU, per tensor and per column,
    on every kernel."""
    ng = ng_mod()
    rng = np.random.default_rng(102)
    for (M, N, K) in ((16, 96, 64), (300, 300, 64)):
        za, zb = 77, 0
        A = np.full((M, K), za, dtype=np.uint8)
        A[:, 0] = za + 1                                    # c[i][j] = B[j][0]: every small integer occurs
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        B[:16, 0] = np.array([-128, -4, -3, -2, -1, 0, 1, 2, 3, 4, 5, 8, 16, 64, 127, -64], dtype=np.int8)
        h, packed = rt.pack(B)
        Ad = torch.from_numpy(A).cuda()
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        for k in ((0,) if M <= 32 else (1, 2, 3)):
            rt.set_kernel(k)
            for scale in (2.0 ** 30, 2.0 ** 29, 2.0 ** 24, 1.5 * 2.0 ** 29, 2.0 ** -30):
                for zc in (-2**31, -2**31 + 100, -2**31 + 300, -1, 0, 255, 2**31 - 1):
                    for relu in (False, True):
                        Cd = torch.full((M, N), 0x5A, dtype=torch.uint8, device="cuda")
                        if relu:
                            sv = torch.full((N,), scale, dtype=torch.float32, device="cuda")
                            ng.ngemm_run_u8s8u8_requant_channel(rt.ctx, M, Ad, K, za, h, zb, None, sv, None, True, zc,
                                                                Cd, N, ws, wsb)
                            want = oracle.gemm_u8s8u8_requant_channel(A, B, za, zb, np.full(N, scale, np.float32), zc,
                                                                      relu=True)
                        else:
                            ng.ngemm_run_u8s8u8_requant(rt.ctx, M, Ad, K, za, h, zb, scale, zc, Cd, N, ws, wsb)
                            want = oracle.gemm_u8s8u8_requant(A, B, za, zb, scale, zc)
                        torch.cuda.synchronize()
                        assert np.array_equal(Cd.cpu().numpy(), want), (M, N, K, k, scale, zc, relu)
        rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
        ng.ngemm_packed_b_free(h)


def test_signed_a_variant(rt, oracle):
    """s8 x s8 -> s32 on every kernel, ragged shapes, zero-points over the signed range."""
    ng = ng_mod()
    rng = np.random.default_rng(96)
    for t, (M, N, K) in enumerate(((3, 70, 333), (32, 96, 64), (100, 200, 300), (300, 333, 1024), (257, 65, 129))):
        A = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        za = int(rng.integers(-128, 128))
        zb = 0 if t % 2 else int(rng.integers(-128, 128))
        want = oracle.gemm_s8s8s32(A, B, za, zb)
        h, packed = rt.pack(B)
        Ad = torch.from_numpy(A).cuda()
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        for k in ((0,) if M <= 32 else (1, 2, 3)):
            rt.set_kernel(k)
            Cd = torch.full((M, N), -3, dtype=torch.int32, device="cuda")
            ng.ngemm_run_s8s8s32(rt.ctx, M, Ad, K, za, h, zb, Cd, N, ws, wsb)
            torch.cuda.synchronize()
            assert np.array_equal(Cd.cpu().numpy(), want), (M, N, K, k)
        rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
        # zero-point range of the signed operand
        for bad in (128, -129):
            try:
                ng.ngemm_run_s8s8s32(rt.ctx, M, Ad, K, bad, h, 0, Cd, N, ws, wsb)
                assert False
            except ng.NgemmError as e:
                assert e.status == ng.NGEMM_ERR_INVALID_ARG
        ng.ngemm_packed_b_free(h)


def test_unsigned_b_variant(rt, oracle):
    """u8 x u8 -> s32: the pack stores B - 128 with zero padding, every kernel, ragged shapes,
    zero-points over [0,255]; descriptors and entry points of the other type refuse each other."""
    from gpu_util import unpack_packed
    ng = ng_mod()
    rng = np.random.default_rng(97)
    for t, (M, N, K) in enumerate(((3, 70, 333), (16, 4096, 61), (100, 200, 300), (300, 333, 1024), (257, 65, 129))):
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(0, 256, size=(N, K), dtype=np.uint8)
        za = int(rng.integers(0, 256))
        zb = 128 if t == 2 else int(rng.integers(0, 256))       # 128: no row sums needed
        want = oracle.gemm_u8u8s32(A, B, za, zb)
        nbytes = ng.ngemm_packed_b_bytes(K, N)
        packed = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        Bd = torch.from_numpy(B).cuda()
        h = ng.ngemm_pack_b_u8(rt.ctx, K, N, Bd, K, packed, nbytes)
        torch.cuda.synchronize()
        back, pad_zero, colsum = unpack_packed(packed.cpu().numpy(), K, N)
        assert np.array_equal(back.astype(np.int16) + 128, B.astype(np.int16)) and pad_zero
        assert np.array_equal(colsum[:N], (B.astype(np.int64) - 128).sum(1).astype(np.int32))
        Ad = torch.from_numpy(A).cuda()
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        for k in ((0,) if M <= 32 else (1, 2, 3)):
            rt.set_kernel(k)
            Cd = torch.full((M, N), -3, dtype=torch.int32, device="cuda")
            ng.ngemm_run_u8u8s32(rt.ctx, M, Ad, K, za, h, zb, Cd, N, ws, wsb)
            torch.cuda.synchronize()
            assert np.array_equal(Cd.cpu().numpy(), want), (M, N, K, k)
        rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
        for call, args in ((ng.ngemm_run_u8s8s32, (za, h, 0)), (ng.ngemm_run_u8u8s32, (za, h, 256)),
                           (ng.ngemm_run_u8u8s32, (za, h, -1))):
            try:
                call(rt.ctx, M, Ad, K, *args, Cd, N, ws, wsb)
                assert False
            except ng.NgemmError as e:
                assert e.status == ng.NGEMM_ERR_INVALID_ARG
        ng.ngemm_packed_b_free(h)
    # a signed pack is refused by the unsigned entry point
    Bs = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
    h, _packed = rt.pack(Bs)
    try:
        ng.ngemm_run_u8u8s32(rt.ctx, M, Ad, K, za, h, 128, Cd, N, ws, wsb)
        assert False
    except ng.NgemmError as e:
        assert e.status == ng.NGEMM_ERR_INVALID_ARG
    ng.ngemm_packed_b_free(h)


def test_16bit_variant(rt, oracle):
    """s16 x s16 -> s32 through byte planes on the 8-bit matrix pipe: pack layout (two planes per
    32-element slice, zero padded, column sums of b - 128), parity on ragged shapes with K tails,
    zero-points over the int16 range, extreme values (wrap), several tiles per workgroup, and the
    refusals between descriptor types."""
    ng = ng_mod()
    rng = np.random.default_rng(101)
    shapes = ((1, 1, 1), (5, 7, 31), (64, 64, 32), (100, 130, 100), (130, 257, 320), (300, 200, 1000), (128, 128, 2048),
              (257, 129, 65), (70, 90, 128), (129, 64, 209), (40, 300, 448), (512, 640, 4096))
    for t, (M, N, K) in enumerate(shapes):
        if t == 3:      # extremes: every product near 2^30, sums wrap
            A = rng.choice(np.array([-32768, 32767], dtype=np.int16), size=(M, K))
            B = rng.choice(np.array([-32768, 32767], dtype=np.int16), size=(N, K))
        else:
            A = rng.integers(-32768, 32768, size=(M, K), dtype=np.int16)
            B = rng.integers(-32768, 32768, size=(N, K), dtype=np.int16)
        za = int(rng.integers(-32768, 32768)) if t % 3 else 0
        zb = 128 if t == 2 else (int(rng.integers(-32768, 32768)) if t % 2 else 0)
        want = oracle.gemm_s16s16s32(A, B, za, zb)
        lda = (K + 7) // 8 * 8
        Ah = np.full((M, lda), 1234, dtype=np.int16); Ah[:, :K] = A
        Ad = torch.from_numpy(Ah.reshape(-1)[:(M - 1) * lda + K].copy()).cuda()     # ends with the last valid element
        Bh = np.full((N, K + 3), -77, dtype=np.int16); Bh[:, :K] = B
        Bd = torch.from_numpy(Bh).cuda()
        nbytes = ng.ngemm_packed_b_bytes_s16(K, N)
        Kp, Np = (K + 31) // 32 * 32, (N + 31) // 32 * 32
        assert nbytes == 2 * Kp * Np + 4 * Np
        packed = torch.full((nbytes,), 0x5a, dtype=torch.uint8, device="cuda")
        h = ng.ngemm_pack_b_s16(rt.ctx, K, N, Bd, K + 3, packed, nbytes)
        torch.cuda.synchronize()
        # layout: fragment (panel, slice, plane) at 1024 * ((panel * nslices + slice) * 2 + plane),
        # byte 16 * (32 * ((k % 32) / 16) + j % 32) + k % 16 inside it
        raw = packed.cpu().numpy()
        frag = raw[:2 * Kp * Np].reshape(Np // 32, Kp // 32, 2, 2, 32, 16)      # panel, slice, plane, k-half, column, byte
        planes = frag.transpose(2, 0, 4, 1, 3, 5).reshape(2, Np, Kp)            # plane, column, k
        Bpad = np.zeros((Np, Kp), dtype=np.int16); Bpad[:N, :K] = B
        hi = ((Bpad.astype(np.int32) >> 8) & 255).astype(np.uint8)
        lo = ((Bpad.astype(np.int32) & 255) ^ 0x80).astype(np.uint8)
        mask = np.zeros((Np, Kp), dtype=bool); mask[:N, :K] = True
        assert np.array_equal(planes[0], np.where(mask, hi, 0)) and np.array_equal(planes[1], np.where(mask, lo, 0))
        colsum = raw[2 * Kp * Np:].view(np.int32)
        assert np.array_equal(colsum[:N], (B.astype(np.int64) - 128).sum(1).astype(np.int32)) and not colsum[N:].any()
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        for cap in (0, 2):
            ng.ngemm_set_max_workgroups(rt.ctx, cap)
            Cd = torch.full((M + 1, N + 2), -3, dtype=torch.int32, device="cuda")
            ng.ngemm_run_s16s16s32(rt.ctx, M, Ad, lda, za, h, zb, Cd, N + 2, ws, wsb)
            torch.cuda.synchronize()
            got = Cd.cpu().numpy()
            assert np.array_equal(got[:M, :N], want), (M, N, K, cap, np.count_nonzero(got[:M, :N] != want))
            assert (got[M:, :] == -3).all() and (got[:, N:] == -3).all()
        ng.ngemm_set_max_workgroups(rt.ctx, 0)
        # refusals: a 16-bit pack in an 8-bit call, zero-points out of range, unaligned rows
        for call, args in ((ng.ngemm_run_u8s8s32, (rt.ctx, M, Ad, lda, 0, h, 0, Cd, N + 2, ws, wsb)),
                           (ng.ngemm_run_s16s16s32, (rt.ctx, M, Ad, lda, 32768, h, 0, Cd, N + 2, ws, wsb)),
                           (ng.ngemm_run_s16s16s32, (rt.ctx, M, Ad, lda, 0, h, -32769, Cd, N + 2, ws, wsb)),
                           (ng.ngemm_run_s16s16s32, (rt.ctx, M, Ad, lda + 1, 0, h, 0, Cd, N + 2, ws, wsb))):
            try:
                call(*args)
                assert False
            except ng.NgemmError as e:
                assert e.status == ng.NGEMM_ERR_INVALID_ARG
        ng.ngemm_packed_b_free(h)
    # an 8-bit pack is refused by the 16-bit call
    h8, _pk = rt.pack(rng.integers(-128, 128, size=(N, K), dtype=np.int8))
    try:
        ng.ngemm_run_s16s16s32(rt.ctx, M, Ad, lda, 0, h8, 0, Cd, N + 2, ws, wsb)
        assert False
    except ng.NgemmError as e:
        assert e.status == ng.NGEMM_ERR_INVALID_ARG
    ng.ngemm_packed_b_free(h8)


def test_online_pack_path(rt, oracle):
    """Both operands as plain inputs.  Unaligned rows or M <= 32: B is packed into the workspace
    inside the call.  Rows of A and B 16-byte aligned and M > 32: the tile kernels read B from
    its plain storage (every tile size, K tails, ragged M and N, both zero-points)."""
    ng = ng_mod()
    rng = np.random.default_rng(95)
    cases = [(5, 100, 333, 7, -3, 0), (200, 333, 500, 131, 0, 0), (300, 300, 1024, 0, 9, 0), (40, 64, 0, 3, 3, 0),
             # (M, N, K, za, zb, pitch padding that makes the rows 16-byte aligned)
             (300, 300, 1024, 0, 9, 16), (200, 333, 500, 131, 0, 12), (100, 70, 40, 5, -7, 8),
             (33, 1000, 640, 250, 127, 0), (513, 257, 129, 128, -128, 15), (1024, 768, 768, 128, 0, 0)]
    for (M, N, K, za, zb, pad) in cases:
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        want = oracle.gemm_u8s8s32(A, B, za, zb)
        ld = K + pad
        Ah = np.full((M, ld), 99, dtype=np.uint8); Ah[:, :K] = A
        Bh = np.full((N, ld), 55, dtype=np.int8); Bh[:, :K] = B
        # the allocations end with the last valid byte of the last row
        Ad = torch.from_numpy(Ah.reshape(-1)[:(M - 1) * ld + K].copy()).cuda() if K else torch.empty(16, dtype=torch.uint8, device="cuda")
        Bd = torch.from_numpy(Bh.reshape(-1)[:(N - 1) * ld + K].copy()).cuda() if K else torch.empty(16, dtype=torch.int8, device="cuda")
        wsb = ng.ngemm_unpacked_workspace_bytes(M, N, K)
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        for k in ((-1,) if M <= 32 or pad == 0 and K % 16 else (-1, 1, 2, 3)):
            rt.set_kernel(k)
            Cd = torch.full((M + 1, N + 3), -5, dtype=torch.int32, device="cuda")
            ng.ngemm_run_u8s8s32_unpacked(rt.ctx, M, N, K, Ad, ld, za, Bd, ld, zb, Cd, N + 3, ws, wsb)
            torch.cuda.synchronize()
            got = Cd.cpu().numpy()
            assert np.array_equal(got[:M, :N], want), (M, N, K, pad, k)
            assert (got[M:, :] == -5).all() and (got[:, N:] == -5).all()
        rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
        try:
            ng.ngemm_run_u8s8s32_unpacked(rt.ctx, M, N, K, Ad, ld, za, Bd, ld, zb, Cd, N + 3, ws, wsb - 1)
            assert False, "a short workspace must be refused"
        except ng.NgemmError as e:
            assert e.status == ng.NGEMM_ERR_BUFFER_TOO_SMALL


def test_shape_tuning(rt, oracle):
    """ngemm_tune_u8s8s32 measures the kernels that can serve a shape, remembers the fastest for
    that (M, N, K), and later run calls with the automatic choice take it; results stay exact."""
    ng = ng_mod()
    rng = np.random.default_rng(99)
    for (M, N, K) in ((16, 512, 256), (300, 500, 700), (2048, 2048, 512), (40, 3000, 64)):
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        za, zb = 3, -2
        want = oracle.gemm_u8s8s32(A, B, za, zb)
        h, packed = rt.pack(B)
        Ad = torch.from_numpy(A).cuda()
        Cd = torch.full((M, N), -9, dtype=torch.int32, device="cuda")
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        assert ng.ngemm_tuned_kernel(rt.ctx, M, N, K) == ng.NGEMM_KERNEL_AUTO
        best = ng.ngemm_tune_u8s8s32(rt.ctx, M, Ad, K, za, h, zb, Cd, N, ws, wsb)
        allowed = (0, 1) if M <= 32 else (1, 2, 3)
        assert best in allowed, (M, N, K, best)
        assert ng.ngemm_tuned_kernel(rt.ctx, M, N, K) == best
        assert np.array_equal(Cd.cpu().numpy(), want)          # the tuning runs leave the result in C
        Cd.fill_(-9)
        ng.ngemm_run_u8s8s32(rt.ctx, M, Ad, K, za, h, zb, Cd, N, ws, wsb)
        torch.cuda.synchronize()
        assert np.array_equal(Cd.cpu().numpy(), want)
        try:
            ng.ngemm_tune_u8s8s32(rt.ctx, M, Ad, K, 256, h, zb, Cd, N, ws, wsb)
            assert False
        except ng.NgemmError as e:
            assert e.status == ng.NGEMM_ERR_INVALID_ARG
        ng.ngemm_packed_b_free(h)


def test_hip_graph_replays(rt, oracle):
    """Run calls captured in a HIP graph (the library allocates nothing and records no memset, so
    it can be captured): several replays with eager work and synchronisation in between, every
    replay checked against the oracle with fresh input contents."""
    ng = ng_mod()
    rng = np.random.default_rng(92)
    # the last two take the K split for the int32 output (C cleared and added to on every replay)
    cases = [(4, 4096, 1024, 0, 0), (300, 200, 500, 17, -3), (700, 520, 1024, 128, 0), (100, 70, 8192, 9, 5),
             (16, 256, 16384, 3, -2)]
    bufs = []
    for (M, N, K, za, zb) in cases:
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        h, packed = rt.pack(B)
        Ad = torch.zeros((M, K), dtype=torch.uint8, device="cuda")
        Cd = torch.zeros((M, N), dtype=torch.int32, device="cuda")
        C8 = torch.zeros((M, N), dtype=torch.uint8, device="cuda")
        wsb = ng.ngemm_workspace_bytes(M, N, K)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        bufs.append((B, h, packed, Ad, Cd, C8, ws, wsb))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()

    # the same problems once more through the batched entry point, into outputs of their own
    Cb = [torch.zeros((M, N), dtype=torch.int32, device="cuda") for (M, N, K, za, zb) in cases]
    arr = ng.make_problems([(M, b[3], K, za, zb, b[1], cb, N) for (M, N, K, za, zb), b, cb in zip(cases, bufs, Cb)])

    def launch_all():
        for (M, N, K, za, zb), (B, h, packed, Ad, Cd, C8, ws, wsb) in zip(cases, bufs):
            ng.ngemm_run_u8s8s32(rt.ctx, M, Ad, K, za, h, zb, Cd, N, ws, wsb)
            ng.ngemm_run_u8s8u8_requant(rt.ctx, M, Ad, K, za, h, zb, 0.0007, 128, C8, N, ws, wsb)
        ng.ngemm_run_batched_u8s8s32(rt.ctx, arr)

    with torch.cuda.stream(side):
        launch_all()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        launch_all()
    for rep in range(4):
        As = [rng.integers(0, 256, size=(M, K), dtype=np.uint8) for (M, N, K, za, zb) in cases]
        for A, b in zip(As, bufs):
            b[3].copy_(torch.from_numpy(A).cuda())     # eager work between replays
            b[4].fill_(-1)
            b[5].fill_(7)
        for cb in Cb:
            cb.fill_(-2)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for A, (M, N, K, za, zb), b in zip(As, cases, bufs):
            want = oracle.gemm_u8s8s32(A, b[0], za, zb)
            assert np.array_equal(b[4].cpu().numpy(), want), (rep, M, N, K)
            assert np.array_equal(Cb[cases.index((M, N, K, za, zb))].cpu().numpy(), want), (rep, M, N, K, "batched")
            assert np.array_equal(b[5].cpu().numpy(),
                                  oracle.gemm_u8s8u8_requant(A, b[0], za, zb, np.float32(0.0007), 128)), (rep, M, N, K)
    for b in bufs:
        ng.ngemm_packed_b_free(b[1])


def test_error_paths_launch_nothing(rt):
    ng = ng_mod()
    B = np.ones((8, 64), np.int8)
    h, packed = rt.pack(B)
    A = torch.zeros((40, 64), dtype=torch.uint8, device="cuda")
    C = torch.full((40, 8), 5, dtype=torch.int32, device="cuda")
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")

    def status(fn, *a, **k):
        try:
            fn(*a, **k)
        except ng.NgemmError as e:
            return e.status
        return 0

    run = ng.ngemm_run_u8s8s32
    assert status(run, rt.ctx, 40, A, 64, 256, h, 0, C, 8) == ng.NGEMM_ERR_INVALID_ARG
    assert status(run, rt.ctx, 40, A, 64, -1, h, 0, C, 8) == ng.NGEMM_ERR_INVALID_ARG
    assert status(run, rt.ctx, 40, A, 64, 0, h, 128, C, 8) == ng.NGEMM_ERR_INVALID_ARG
    assert status(run, rt.ctx, 40, A, 63, 0, h, 0, C, 8) == ng.NGEMM_ERR_BAD_SHAPE
    assert status(run, rt.ctx, 40, A, 64, 0, h, 0, C, 7) == ng.NGEMM_ERR_BAD_SHAPE
    assert status(run, rt.ctx, -1, A, 64, 0, h, 0, C, 8) == ng.NGEMM_ERR_BAD_SHAPE
    assert status(run, rt.ctx, 40, None, 64, 0, h, 0, C, 8) == ng.NGEMM_ERR_INVALID_ARG
    assert status(run, rt.ctx, 40, A, 64, 0, h, 0, None, 8) == ng.NGEMM_ERR_INVALID_ARG
    assert status(run, rt.ctx, 40, A, 64, 0, h, 3, C, 8, None, 0) == ng.NGEMM_ERR_INVALID_ARG
    assert status(run, rt.ctx, 40, A, 64, 0, h, 3, C, 8, ws, 16) == ng.NGEMM_ERR_BUFFER_TOO_SMALL
    rq = ng.ngemm_run_u8s8u8_requant
    C8 = torch.zeros((40, 8), dtype=torch.uint8, device="cuda")
    for bad in (0.0, -1.0, float("nan"), float("inf"), 2.0**31, 2.0**-31):
        assert status(rq, rt.ctx, 40, A, 64, 0, h, 0, bad, 0, C8, 8) == ng.NGEMM_ERR_INVALID_ARG
    rt.set_kernel(ng.NGEMM_KERNEL_SKINNY)
    assert status(run, rt.ctx, 40, A, 64, 0, h, 0, C, 8) == ng.NGEMM_ERR_INVALID_ARG
    rt.set_kernel(ng.NGEMM_KERNEL_AUTO)
    torch.cuda.synchronize()
    assert bool((C == 5).all())                      # nothing was launched by the failed calls
    # pack: buffer too small, bad ldb
    Bd = torch.zeros((8, 64), dtype=torch.int8, device="cuda")
    small = torch.zeros(64, dtype=torch.uint8, device="cuda")
    assert status(ng.ngemm_pack_b, rt.ctx, 64, 8, Bd, 64, small, 64) == ng.NGEMM_ERR_BUFFER_TOO_SMALL
    big = torch.zeros(ng.ngemm_packed_b_bytes(64, 8), dtype=torch.uint8, device="cuda")
    assert status(ng.ngemm_pack_b, rt.ctx, 64, 8, Bd, 63, big, big.numel()) == ng.NGEMM_ERR_BAD_SHAPE
    assert status(ng.ngemm_pack_b, rt.ctx, -1, 8, Bd, 64, big, big.numel()) == ng.NGEMM_ERR_BAD_SHAPE
    ng.ngemm_packed_b_free(h)
