#!/usr/bin/env python3
"""Benchmark of the gfx950 u8 x s8 -> s32 GEMM path on one MI355X.

Headline workload (config 4): M = N = K = 8192, uniform u8 x uniform s8, zero-points 0, int32
output.  A "step" is one ngemm_run_u8s8s32 call on operands already resident in HBM (B packed
once beforehand, as the method prescribes for the weight operand).  Prints ONE JSON line.

Extras in the same line: the skinny-M shapes (GB/s, as specified / with rotating weights so
that every byte comes from HBM / a large asymptote), the transformer FC shapes with int32 and
requantised u8 output, the batched odd shapes, and the pack kernel.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0     # MI355X dense INT8 matrix peak, TOP/s (published)
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E peak, GB/s (published)

# Figures that only a counter or trace run can give (HBM-side bytes per launch, kernel-only
# durations) are read from the rocprofv3 summaries under profiles/: lines of the form
# "bench_key <name> = <number>".  Each is reported with the file it came from; a missing file or
# key gives null.
PROFILES = os.path.join(ROOT, "profiles")


def profile_figure(fname, key):
    try:
        with open(os.path.join(PROFILES, fname)) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 4 and parts[0] == "bench_key" and parts[1] == key and parts[2] == "=":
                    return float(parts[3])
    except OSError:
        pass
    return None


def gpu_time_ms(fn, iters, warmup, torch):
    """Average milliseconds per call of fn(), HIP events on the current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def graph_time_ms(fn_seq, replays, torch):
    """Average milliseconds per call when `fn_seq` (a list of zero-argument launches on the
    current stream) is captured once into a HIP graph and replayed: removes the Python / ctypes
    cost per call, which is larger than these kernels."""
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        for f in fn_seq[:4]:
            f()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        for f in fn_seq:
            f()
    g.replay()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * len(fn_seq))


TRAFFIC_PROFILE = "large_square_8192_hbm_traffic.txt"
SKINNY_PROFILE = "skinny_4096x1024_kernel_trace.txt"
SECTIONS = ("skinny", "fc", "longk", "batched", "types")      # run by default
OPT_IN_SECTIONS = ("power",)                                    # only when named


class Bench:
    """Shared state of the sections: the context, torch, the binding and small helpers."""

    def __init__(self, ng, wl, torch, np, ctx):
        self.ng, self.wl, self.torch, self.np, self.ctx = ng, wl, torch, np, ctx

    def pack(self, B_np):
        ng, torch = self.ng, self.torch
        N, K = B_np.shape
        Bd = torch.from_numpy(B_np).cuda()
        nbytes = ng.ngemm_packed_b_bytes(K, N)
        packed = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        h = ng.ngemm_pack_b(self.ctx, K, N, Bd, K, packed, nbytes)
        torch.cuda.synchronize()
        return h, packed, Bd


def bench_headline(b, args, result):
    """Config 4.  Fills the contract's keys of `result`; returns (ops, n)."""
    ng, wl, torch, np, ctx = b.ng, b.wl, b.torch, b.np, b.ctx
    n = args.size
    prob = wl.large_square(n)
    h, packed, Bd = b.pack(prob.B)
    Ad = torch.from_numpy(prob.A).cuda()
    Cd = torch.empty((n, n), dtype=torch.int32, device="cuda")

    def step():
        ng.ngemm_run_u8s8s32(ctx, n, Ad, n, 0, h, 0, Cd, n)

    # An idle chip needs some 50 ms of this kernel before its clocks settle (the first launches run
    # up to 40 % longer): with fewer than 200 warm-up steps asked for, the difference is run first,
    # untimed and reported as clock_settle_steps, so that the K timed steps see the sustained state.
    settle = max(0, 200 - args.warmup)
    for _ in range(settle + args.warmup):
        step()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    kern_ms = ev0.elapsed_time(ev1) / args.steps
    ops = 2.0 * n * n * n
    tops = ops / (wall_ms * 1e-3) / 1e12
    kern_tops = ops / (kern_ms * 1e-3) / 1e12

    # correctness of the timed output on sampled elements (oracle, element by element)
    import oracle
    rng = np.random.default_rng(7)
    ri = rng.integers(0, n, size=4096)
    ci = rng.integers(0, n, size=4096)
    Cs = Cd[torch.from_numpy(ri).cuda(), torch.from_numpy(ci).cuda()].cpu().numpy()
    sample_ok = bool(np.array_equal(Cs, oracle.gemm_u8s8s32_sampled(prob.A, prob.B, ri, ci)))

    pack_ms = gpu_time_ms(lambda: ng.ngemm_packed_b_free(
        ng.ngemm_pack_b(ctx, n, n, Bd, n, packed, packed.numel())), 5, 1, torch)

    # plain device copy of known size: the achievable-copy ceiling, and the kernel whose
    # FETCH_SIZE / WRITE_SIZE readings calibrate those counters in the profiles
    csrc = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cdst = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    copy_ms = gpu_time_ms(lambda: cdst.copy_(csrc), 5, 2, torch)
    del csrc, cdst

    traffic = profile_figure(TRAFFIC_PROFILE, "traffic_bytes_per_launch") if n == 8192 else None
    result.update({
        "metric": "int8 GEMM TOPS (u8 x s8 -> s32, M=N=K=%d)" % n,
        "value": round(tops, 2),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "clock_settle_steps": settle,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 x int8 -> int32 (u8 operand shifted to s8)",
        "data": "synthetic (seeded uniform u8 / s8)",
        "config": {"workload": "large_square_%d" % n, "M": n, "N": n, "K": n, "za": 0, "zb": 0,
                   "kernel": "gemm_tile_x64_kernel (256 x 256 tiles, v_mfma_i32_16x16x64_i8)", "sampled_outputs_match_oracle": sample_ok},
        "roofline": {"bound": "mfma", "achieved": round(kern_tops, 2), "peak": INT8_MFMA_PEAK_TOPS,
                     "unit": "TOP/s", "frac": round(kern_tops / INT8_MFMA_PEAK_TOPS, 4),
                     "traffic": int(traffic) if traffic else None,
                     "traffic_source": ("profiles/%s (rocprofv3 --pmc runs of this script, not this run)" % TRAFFIC_PROFILE)
                     if traffic else None,
                     "kernel_ms": round(kern_ms, 5),
                     "algorithmic_ops_per_launch": ops,
                     "algorithmic_bytes_per_launch": 2 * n * n + 4 * n * n},
        "pack_b": {"ms": round(pack_ms, 4), "GBps": round(2.0 * n * n / (pack_ms * 1e-3) / 1e9, 1)},
        "copy_1GiB": {"ms": round(copy_ms, 4), "GBps_read_plus_write": round(2.0 * (1 << 30) / (copy_ms * 1e-3) / 1e9, 1)},
    })

    # ---------------- CPU baseline: the oracle as it stands, bounded sample ----------------
    if not args.no_cpu_baseline:
        cal_rows = 16 * oracle.num_threads()
        t = time.perf_counter()
        oracle.gemm_u8s8s32(np.ascontiguousarray(prob.A[:cal_rows]), prob.B)
        per_row = (time.perf_counter() - t) / cal_rows
        rows = int(max(oracle.num_threads(), min(n, args.cpu_seconds / max(per_row, 1e-9))))
        rows = max(oracle.num_threads(), rows // oracle.num_threads() * oracle.num_threads())
        rows = min(rows, n)
        t = time.perf_counter()
        oracle.gemm_u8s8s32(np.ascontiguousarray(prob.A[:rows]), prob.B)
        dt = time.perf_counter() - t
        result["cpu_baseline"] = {
            "value": round(2.0 * rows * n * n / dt / 1e12, 5), "unit": "TOPS",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "first %d rows of A against all of B (%d x %d x %d), %.1f s" % (rows, rows, n, n, dt)}

    del Ad, Cd
    ng.ngemm_packed_b_free(h)
    del packed, Bd
    torch.cuda.empty_cache()


def bench_skinny(b, args):
    """Config 3: (i) as specified, (ii) rotating weights (single calls and grouped calls),
    (iii) asymptotes."""
    ng, wl, torch, ctx = b.ng, b.wl, b.torch, b.ctx
    sk = {}
    per = 84                       # members of one grouped call (what one launch of the streaming kernel holds)
    ncopies = 3 * per              # distinct packed copies: 252 x 4 MiB, four times the 256 MiB memory-side cache
    for M in (1, 4, 16):
        probs = wl.skinny(M)
        B = probs[0].B
        N, K = B.shape
        hb, pk, _ = b.pack(B)
        A_dev = [torch.from_numpy(p.A).cuda() for p in probs]
        C = torch.empty((M, N), dtype=torch.int32, device="cuda")
        cnt = [0]

        def call():
            ng.ngemm_run_u8s8s32(ctx, M, A_dev[cnt[0] % 16], K, 0, hb, 0, C, N)
            cnt[0] += 1
        ms_eager = gpu_time_ms(call, 1000, 50, torch)
        seq = [(lambda t=t: ng.ngemm_run_u8s8s32(ctx, M, A_dev[t % 16], K, 0, hb, 0, C, N)) for t in range(250)]
        ms = graph_time_ms(seq, 4, torch)            # 1000 calls, one weight matrix, pool of 16 inputs
        abytes = K * N + M * K + 4 * M * N
        entry = {"as_specified_us": round(ms * 1e3, 3), "as_specified_GBps": round(abytes / (ms * 1e-3) / 1e9, 1),
                 "as_specified_eager_python_us": round(ms_eager * 1e3, 3),
                 "algorithmic_bytes": abytes}
        # rotating: distinct packed copies, so that every byte comes from HBM
        nb = ng.ngemm_packed_b_bytes(K, N)
        pool = torch.empty((ncopies, nb), dtype=torch.uint8, device="cuda")
        pool[:] = pk
        hs = []
        Bd2 = torch.from_numpy(B).cuda()
        for c in range(ncopies):
            hs.append(ng.ngemm_pack_b(ctx, K, N, Bd2, K, pool[c], nb))
        torch.cuda.synchronize()

        seq = [(lambda t=t: ng.ngemm_run_u8s8s32(ctx, M, A_dev[t % 16], K, 0, hs[t % ncopies], 0, C, N))
               for t in range(ncopies)]
        ms2 = graph_time_ms(seq, 6, torch)
        entry["rotating_weights_us"] = round(ms2 * 1e3, 3)
        entry["rotating_weights_GBps"] = round(abytes / (ms2 * 1e-3) / 1e9, 1)
        entry["rotating_frac_of_hbm_peak"] = round(abytes / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        # the same rotating GEMMs through the batched entry point, 84 independent problems per call
        # (one grouped launch each): what a server with many small GEMMs in flight would issue
        Cb = [torch.empty((M, N), dtype=torch.int32, device="cuda") for _ in range(per)]
        batches = [ng.make_problems([(M, A_dev[(g * per + t) % 16], K, 0, 0, hs[g * per + t], Cb[t], N)
                                     for t in range(per)]) for g in range(ncopies // per)]
        seqb = [(lambda arr=arr: ng.ngemm_run_batched_u8s8s32(ctx, arr)) for arr in batches]
        msb = graph_time_ms(seqb, 6, torch) / per
        entry["batched_members_per_call"] = per
        entry["rotating_weights_batched_us_per_gemm"] = round(msb * 1e3, 3)
        entry["rotating_weights_batched_GBps"] = round(abytes / (msb * 1e-3) / 1e9, 1)
        entry["rotating_batched_frac_of_hbm_peak"] = round(abytes / (msb * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        # kernel-only duration of the grouped launches (no gap between graph replays), from the trace summary
        # (the single calls are not quoted: a traced launch of a few us reads about 1.3 us too long)
        us = profile_figure(SKINNY_PROFILE, "rotating_batched_kernel_only_us_per_gemm_M%d" % M)
        if us:
            entry["rotating_batched_kernel_only_GBps_from_profile"] = round(abytes / (us * 1e-6) / 1e9, 1)
            entry["rotating_batched_kernel_only_frac_from_profile"] = round(abytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        for x in hs:
            ng.ngemm_packed_b_free(x)
        ng.ngemm_packed_b_free(hb)
        del pool
        sk["M%d" % M] = entry
    sk["kernel_only_source"] = "profiles/%s (rocprofv3 --kernel-trace of this section, not this run)" % SKINNY_PROFILE
    # launch floor: the smallest possible call through the same entry point, in the same graph
    tinyB = torch.zeros((32, 64), dtype=torch.int8, device="cuda")
    tb = ng.ngemm_packed_b_bytes(64, 32)
    tpk = torch.empty(tb, dtype=torch.uint8, device="cuda")
    th = ng.ngemm_pack_b(ctx, 64, 32, tinyB, 64, tpk, tb)
    tA = torch.zeros((1, 64), dtype=torch.uint8, device="cuda")
    tC = torch.empty((1, 32), dtype=torch.int32, device="cuda")
    msf = graph_time_ms([lambda: ng.ngemm_run_u8s8s32(ctx, 1, tA, 64, 0, th, 0, tC, 32)] * 250, 4, torch)
    sk["launch_floor_us_1x32x64"] = round(msf * 1e3, 3)
    ng.ngemm_packed_b_free(th)
    # asymptotes: the same kernel on weights large enough to leave launch and latency behind
    # (rotating copies, 512 MiB or more in all, so that every byte comes from HBM)
    for (Mb, Nb, Kb, ncp) in ((16, 16384, 4096, 8), (16, 32768, 8192, 3), (1, 32768, 8192, 3)):
        rngb = wl.rng_for(3, 90 + Mb)
        Bbig = wl.uniform_s8(rngb, Nb, Kb)
        Abig = torch.from_numpy(wl.uniform_u8(rngb, Mb, Kb)).cuda()
        nb = ng.ngemm_packed_b_bytes(Kb, Nb)
        pool = torch.empty((ncp, nb), dtype=torch.uint8, device="cuda")
        Bd2 = torch.from_numpy(Bbig).cuda()
        hs = [ng.ngemm_pack_b(ctx, Kb, Nb, Bd2, Kb, pool[c], nb) for c in range(ncp)]
        Cb = torch.empty((Mb, Nb), dtype=torch.int32, device="cuda")
        seq = [(lambda t=t: ng.ngemm_run_u8s8s32(ctx, Mb, Abig, Kb, 0, hs[t % ncp], 0, Cb, Nb))
               for t in range(4 * ncp)]
        ms3 = graph_time_ms(seq, 5, torch)
        ab = Kb * Nb + Mb * Kb + 4 * Mb * Nb
        sk["asymptote_M%d_N%d_K%d" % (Mb, Nb, Kb)] = {
            "us": round(ms3 * 1e3, 2), "GBps": round(ab / (ms3 * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(ab / (ms3 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        for x in hs:
            ng.ngemm_packed_b_free(x)
        del pool, Bd2, Bbig
    return sk


def bench_fc(b, args):
    """Config 2: the transformer FC shapes."""
    ng, wl, torch, ctx = b.ng, b.wl, b.torch, b.ctx
    fc = {}
    for idx in range(3):
        p = wl.bert_fc(idx)
        hb, pk, _ = b.pack(p.B)
        A = torch.from_numpy(p.A).cuda()
        C = torch.empty((p.M, p.N), dtype=torch.int32, device="cuda")
        C8 = torch.empty((p.M, p.N), dtype=torch.uint8, device="cuda")
        ms = graph_time_ms([lambda: ng.ngemm_run_u8s8s32(ctx, p.M, A, p.K, p.za, hb, p.zb, C, p.N)] * 50, 4, torch)
        ms8 = graph_time_ms([lambda: ng.ngemm_run_u8s8u8_requant(ctx, p.M, A, p.K, p.za, hb, p.zb, p.scale, p.zc,
                                                                 C8, p.N)] * 50, 4, torch)
        # per-column scales + bias + ReLU, and the online-pack path (B packed inside the call)
        sv = torch.full((p.N,), p.scale, dtype=torch.float32, device="cuda")
        bv = torch.zeros((p.N,), dtype=torch.int32, device="cuda")
        msc = graph_time_ms([lambda: ng.ngemm_run_u8s8u8_requant_channel(
            ctx, p.M, A, p.K, p.za, hb, p.zb, None, sv, bv, True, p.zc, C8, p.N)] * 50, 4, torch)
        Bdev = torch.from_numpy(p.B).cuda()
        uwb = ng.ngemm_unpacked_workspace_bytes(p.M, p.N, p.K)
        uws = torch.empty(uwb, dtype=torch.uint8, device="cuda")
        msu = graph_time_ms([lambda: ng.ngemm_run_u8s8s32_unpacked(
            ctx, p.M, p.N, p.K, A, p.K, p.za, Bdev, p.K, p.zb, C, p.N, uws, uwb)] * 50, 4, torch)
        # a weight zero-point (the row sums are formed inside these kernels: no extra launch)
        wsz = ng.ngemm_workspace_bytes(p.M, p.N, p.K)
        wz = torch.empty(max(wsz, 16), dtype=torch.uint8, device="cuda")
        msz = graph_time_ms([lambda: ng.ngemm_run_u8s8s32(ctx, p.M, A, p.K, p.za, hb, 5, C, p.N, wz, wsz)] * 50, 4, torch)
        # after shape tuning (the fastest kernel for this shape, measured on these operands)
        tuned = ng.ngemm_tune_u8s8s32(ctx, p.M, A, p.K, p.za, hb, p.zb, C, p.N)
        mst = graph_time_ms([lambda: ng.ngemm_run_u8s8s32(ctx, p.M, A, p.K, p.za, hb, p.zb, C, p.N)] * 50, 4, torch)
        o = 2.0 * p.M * p.N * p.K
        b32 = p.M * p.K + p.N * p.K + 4 * p.M * p.N
        b8 = p.M * p.K + p.N * p.K + p.M * p.N
        fc[p.name] = {"s32_us": round(ms * 1e3, 2), "s32_TOPS": round(o / (ms * 1e-3) / 1e12, 1),
                      "s32_GBps": round(b32 / (ms * 1e-3) / 1e9, 1),
                      "u8_us": round(ms8 * 1e3, 2), "u8_TOPS": round(o / (ms8 * 1e-3) / 1e12, 1),
                      "u8_GBps": round(b8 / (ms8 * 1e-3) / 1e9, 1),
                      "u8_per_channel_bias_relu_us": round(msc * 1e3, 2),
                      "s32_unpacked_b_us": round(msu * 1e3, 2),
                      "s32_weight_zero_point_5_us": round(msz * 1e3, 2),
                      "s32_tuned_us": round(mst * 1e3, 2), "tuned_kernel": int(tuned)}
        ng.ngemm_packed_b_free(hb)
    return fc


def bench_longk(b, args):
    """Few tiles, long K: K split over the workgroups (the heuristic's choice) against one
    workgroup per tile (M > 32) or the streaming kernel (M <= 32)."""
    ng, wl, torch, ctx = b.ng, b.wl, b.torch, b.ctx
    out = {}
    for (Ms, Ns, Ks) in ((64, 64, 65536), (256, 256, 16384), (512, 512, 16384), (100, 300, 30000), (16, 1024, 8192)):
        rngs = wl.rng_for(4, 70 + Ms)
        As = torch.from_numpy(wl.uniform_u8(rngs, Ms, Ks)).cuda()
        hb, pk, _ = b.pack(wl.uniform_s8(rngs, Ns, Ks))
        Cs = torch.empty((Ms, Ns), dtype=torch.int32, device="cuda")
        C8s = torch.empty((Ms, Ns), dtype=torch.uint8, device="cuda")
        wss = ng.ngemm_workspace_bytes(Ms, Ns, Ks)       # with room for the partial results (u8 output)
        wsd = torch.empty(max(wss, 16), dtype=torch.uint8, device="cuda")
        call = [lambda: ng.ngemm_run_u8s8s32(ctx, Ms, As, Ks, 0, hb, 0, Cs, Ns)] * 20
        call8 = [lambda: ng.ngemm_run_u8s8u8_requant(ctx, Ms, As, Ks, 128, hb, 0, 2.0e-4, 128, C8s, Ns, wsd, wss)] * 20
        ms_split = graph_time_ms(call, 10, torch)
        ms_split8 = graph_time_ms(call8, 10, torch)
        ng.ngemm_set_kernel(ctx, ng.NGEMM_KERNEL_SKINNY if Ms <= 32 else ng.NGEMM_KERNEL_TILE_64)
        ms_plain = graph_time_ms(call, 10, torch)
        ms_plain8 = graph_time_ms(call8, 10, torch)
        ng.ngemm_set_kernel(ctx, ng.NGEMM_KERNEL_AUTO)
        o = 2.0 * Ms * Ns * Ks
        out["%dx%dx%d" % (Ms, Ns, Ks)] = {"split_k_us": round(ms_split * 1e3, 2), "unsplit_us": round(ms_plain * 1e3, 2),
                                          "split_k_TOPS": round(o / (ms_split * 1e-3) / 1e12, 1),
                                          "u8_split_k_us": round(ms_split8 * 1e3, 2),
                                          "u8_unsplit_us": round(ms_plain8 * 1e3, 2)}
        ng.ngemm_packed_b_free(hb)
    return out


def bench_batched(b, args):
    """Config 5: 64 odd shapes in one call."""
    ng, wl, torch, ctx = b.ng, b.wl, b.torch, b.ctx
    probs = wl.batched()
    items, keep, hs = [], [], []
    for p in probs:
        hb, pk, _ = b.pack(p.B)
        A = torch.from_numpy(p.A).cuda()
        C = torch.empty((p.M, p.N), dtype=torch.int32, device="cuda")
        keep.append((pk, A, C))
        hs.append(hb)
        items.append((p.M, A, p.K, p.za, p.zb, hb, C, p.N))
    arr = ng.make_problems(items)
    wsb = ng.ngemm_batched_workspace_bytes(arr)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    msb = gpu_time_ms(lambda: ng.ngemm_run_batched_u8s8s32(ctx, arr, ws, wsb), 20, 3, torch)
    o = sum(2.0 * p.M * p.N * p.K for p in probs)
    by = sum(p.M * p.K + p.N * p.K + 4 * p.M * p.N for p in probs)
    for x in hs:
        ng.ngemm_packed_b_free(x)
    return {"ms": round(msb, 4), "TOPS": round(o / (msb * 1e-3) / 1e12, 2), "GBps": round(by / (msb * 1e-3) / 1e9, 1)}


def bench_types(b, args, extras):
    """The other entry points on the headline shape: signed A, unsigned B (shifted in the pack),
    requantised output, 16-bit operands, unpacked B, and the headline launch on constant operands."""
    ng, wl, torch, np, ctx = b.ng, b.wl, b.torch, b.np, b.ctx
    n = args.size
    ops = 2.0 * n * n * n
    rngt = wl.rng_for(4, 50)
    At = torch.from_numpy(wl.uniform_u8(rngt, n, n)).cuda()
    Bt = torch.from_numpy(wl.uniform_s8(rngt, n, n)).cuda()
    Ct = torch.empty((n, n), dtype=torch.int32, device="cuda")
    nb = ng.ngemm_packed_b_bytes(n, n)
    pks, pku = (torch.empty(nb, dtype=torch.uint8, device="cuda") for _ in range(2))
    hsg = ng.ngemm_pack_b(ctx, n, n, Bt, n, pks, nb)
    hun = ng.ngemm_pack_b_u8(ctx, n, n, Bt.view(torch.uint8), n, pku, nb)
    ms_ss = gpu_time_ms(lambda: ng.ngemm_run_s8s8s32(ctx, n, At.view(torch.int8), n, 0, hsg, 0, Ct, n), 100, 100, torch)
    ms_uu = gpu_time_ms(lambda: ng.ngemm_run_u8u8s32(ctx, n, At, n, 0, hun, 128, Ct, n), 100, 100, torch)
    ty = {"s8s8s32_TOPS": round(ops / (ms_ss * 1e-3) / 1e12, 1), "u8u8s32_TOPS": round(ops / (ms_uu * 1e-3) / 1e12, 1)}
    # requantised u8 output on the headline shape (per-tensor scale)
    C8t = torch.empty((n, n), dtype=torch.uint8, device="cuda")
    ms_q = gpu_time_ms(lambda: ng.ngemm_run_u8s8u8_requant(ctx, n, At, n, 128, hsg, 0, 2.0e-4, 128, C8t, n), 100, 100, torch)
    ty["u8s8u8_requant_TOPS"] = round(ops / (ms_q * 1e-3) / 1e12, 1)
    del C8t
    ng.ngemm_packed_b_free(hsg)
    ng.ngemm_packed_b_free(hun)
    # 16-bit operands through byte planes (four 8-bit matrix ops per block)
    A16 = torch.from_numpy(rngt.integers(-32768, 32768, size=(n, n), dtype=np.int16)).cuda()
    B16 = torch.from_numpy(rngt.integers(-32768, 32768, size=(n, n), dtype=np.int16)).cuda()
    nb16 = ng.ngemm_packed_b_bytes_s16(n, n)
    pk16 = torch.empty(nb16, dtype=torch.uint8, device="cuda")
    h16 = ng.ngemm_pack_b_s16(ctx, n, n, B16, n, pk16, nb16)
    wsb16 = ng.ngemm_workspace_bytes(n, n, n)
    ws16 = torch.empty(wsb16, dtype=torch.uint8, device="cuda")
    ms_16 = gpu_time_ms(lambda: ng.ngemm_run_s16s16s32(ctx, n, A16, n, 0, h16, 0, Ct, n, ws16, wsb16), 30, 30, torch)
    ty["s16s16s32_TOPS"] = round(ops / (ms_16 * 1e-3) / 1e12, 1)
    ng.ngemm_packed_b_free(h16)
    del A16, B16, pk16
    extras["other_integer_types_%d" % n] = ty
    # both operands as inputs: B read from its plain [N x K] storage, nothing packed
    uwb = ng.ngemm_unpacked_workspace_bytes(n, n, n)
    uws = torch.empty(uwb, dtype=torch.uint8, device="cuda")
    ms_un = gpu_time_ms(lambda: ng.ngemm_run_u8s8s32_unpacked(ctx, n, n, n, At, n, 0, Bt, n, 0, Ct, n, uws, uwb),
                        100, 100, torch)
    extras["unpacked_b_%d" % n] = {"ms": round(ms_un, 4), "TOPS": round(ops / (ms_un * 1e-3) / 1e12, 1)}
    # an output that 256 x 256 tiles leave compute units idle on (3072^3: 144 tiles): the heuristic's 192 x 256 tiles
    n3 = 3072
    A3 = torch.from_numpy(wl.uniform_u8(rngt, n3, n3)).cuda()
    B3 = torch.from_numpy(wl.uniform_s8(rngt, n3, n3)).cuda()
    nb3 = ng.ngemm_packed_b_bytes(n3, n3)
    pk3 = torch.empty(nb3, dtype=torch.uint8, device="cuda")
    h3 = ng.ngemm_pack_b(ctx, n3, n3, B3, n3, pk3, nb3)
    C3 = torch.empty((n3, n3), dtype=torch.int32, device="cuda")
    ms_a = gpu_time_ms(lambda: ng.ngemm_run_u8s8s32(ctx, n3, A3, n3, 0, h3, 0, C3, n3), 400, 400, torch)
    ng.ngemm_set_kernel(ctx, ng.NGEMM_KERNEL_TILE_256)
    ms_256 = gpu_time_ms(lambda: ng.ngemm_run_u8s8s32(ctx, n3, A3, n3, 0, h3, 0, C3, n3), 400, 400, torch)
    ng.ngemm_set_kernel(ctx, ng.NGEMM_KERNEL_AUTO)
    ng.ngemm_packed_b_free(h3)
    o3 = 2.0 * n3 ** 3
    extras["square_3072"] = {"heuristic_192x256_tiles_TOPS": round(o3 / (ms_a * 1e-3) / 1e12, 1),
                             "forced_256x256_tiles_TOPS": round(o3 / (ms_256 * 1e-3) / 1e12, 1)}
    del A3, B3, pk3, C3
    # The same launch on operands that do not change (A = 129, B = 1): on uniform data the chip runs
    # at its power cap (shader clock about 1.8 GHz), on such data at its full clock.  Context only.
    Ac = torch.full((n, n), 129, dtype=torch.uint8, device="cuda")
    Bc = torch.ones((n, n), dtype=torch.int8, device="cuda")
    hc = ng.ngemm_pack_b(ctx, n, n, Bc, n, pks, nb)
    ms_c = gpu_time_ms(lambda: ng.ngemm_run_u8s8s32(ctx, n, Ac, n, 0, hc, 0, Ct, n), 200, 200, torch)
    ng.ngemm_packed_b_free(hc)
    extras["power_limit_context_%d" % n] = {
        "constant_operands_TOPS": round(ops / (ms_c * 1e-3) / 1e12, 1),
        "constant_operands_frac_of_peak": round(ops / (ms_c * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS, 4),
        "matrix_pipe_only_rates": "profiles/large_square_8192_power_and_time_budget.txt"}


def smi_sample():
    """One reading of rocm-smi (a child process; read-only queries): shader clock in MHz, socket
    power in W, junction temperature in C; None for what it does not print."""
    import re
    import subprocess
    try:
        out = subprocess.run(["rocm-smi", "--showclocks", "--showpower", "--showtemp"], stdout=subprocess.PIPE,
                             stderr=subprocess.STDOUT, text=True, timeout=20).stdout
    except Exception:
        return None
    sclk = re.search(r"sclk clock level[^\n]*\((\d+)Mhz\)", out)
    pw = re.search(r"Power \(W\)\s*:\s*([0-9.]+)", out)
    tj = re.search(r"junction\) \(C\)\s*:\s*([0-9.]+)", out)
    return {"sclk_MHz": int(sclk.group(1)) if sclk else None, "power_W": float(pw.group(1)) if pw else None,
            "junction_C": float(tj.group(1)) if tj else None}


def bench_power(b, args):
    """What the headline figure rests on, measured here: (1) the sustained rate, shader clock and
    power of the headline launch on uniform and on constant operands (rocm-smi sampled from a
    thread while the launches run); (2) the launch time as a function of K at M = N = 8192, fitted
    as tiles-per-workgroup x (fixed + stages x per-stage), which splits the time of the headline
    launch into its main loop and everything else (fill, epilogue, hand-over between tiles)."""
    import statistics
    import threading
    ng, wl, torch, np, ctx = b.ng, b.wl, b.torch, b.np, b.ctx
    n = args.size
    out = {}
    rng = wl.rng_for(4, 60)
    nb = ng.ngemm_packed_b_bytes(n, n)
    pk = torch.empty(nb, dtype=torch.uint8, device="cuda")
    C = torch.empty((n, n), dtype=torch.int32, device="cuda")
    for name, A_np, B_np in (("uniform", wl.uniform_u8(rng, n, n), wl.uniform_s8(rng, n, n)),
                             ("constant", np.full((n, n), 129, np.uint8), np.ones((n, n), np.int8))):
        A = torch.from_numpy(A_np).cuda()
        Bd = torch.from_numpy(B_np).cuda()
        h = ng.ngemm_pack_b(ctx, n, n, Bd, n, pk, nb)
        torch.cuda.synchronize()
        seconds = 4.0
        t_end = time.time() + seconds
        samples = []

        def sampler():
            time.sleep(1.0)
            while time.time() < t_end - 0.3:
                r = smi_sample()
                if r:
                    samples.append(r)
                time.sleep(0.25)
        th = threading.Thread(target=sampler)
        th.start()
        calls = 0
        t0 = time.time()
        while time.time() < t_end:
            for _ in range(100):
                ng.ngemm_run_u8s8s32(ctx, n, A, n, 0, h, 0, C, n)
            torch.cuda.synchronize()
            calls += 100
        dt = time.time() - t0
        th.join()
        ng.ngemm_packed_b_free(h)

        def med(key):
            v = [x[key] for x in samples if x.get(key) is not None]
            return round(statistics.median(v), 1) if v else None
        out[name] = {"TOPS_sustained": round(2.0 * n ** 3 * calls / dt / 1e12, 1), "seconds": round(dt, 2),
                     "smi_samples": len(samples), "sclk_MHz_median": med("sclk_MHz"),
                     "power_W_median": med("power_W"), "junction_C_median": med("junction_C")}
        del A, Bd
    # K sweep on uniform operands
    sweep = {}
    ks = (1024, 2048, 4096, 8192, 16384)
    ncus = torch.cuda.get_device_properties(0).multi_processor_count
    tiles_per_wg = math.ceil((n // 256) ** 2 / ncus)
    for K in ks:
        A = torch.from_numpy(wl.uniform_u8(rng, n, K)).cuda()
        Bd = torch.from_numpy(wl.uniform_s8(rng, n, K)).cuda()
        nbk = ng.ngemm_packed_b_bytes(K, n)
        pkk = torch.empty(nbk, dtype=torch.uint8, device="cuda")
        h = ng.ngemm_pack_b(ctx, K, n, Bd, K, pkk, nbk)
        reps = max(40, int(200 * 8192 / K))
        ms = gpu_time_ms(lambda: ng.ngemm_run_u8s8s32(ctx, n, A, K, 0, h, 0, C, n), reps, reps, torch)
        sweep[K] = ms * 1e3
        ng.ngemm_packed_b_free(h)
        del A, Bd, pkk
    xs = [K / 64.0 for K in ks]
    ys = [sweep[K] / tiles_per_wg for K in ks]
    mx, my = sum(xs) / len(xs), sum(ys) / len(ys)
    slope = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sum((x - mx) ** 2 for x in xs)
    icpt = my - slope * mx
    sclk = out["uniform"].get("sclk_MHz_median")
    fit = {"us_per_launch_by_K": {str(K): round(v, 2) for K, v in sweep.items()}, "tiles_per_workgroup": tiles_per_wg,
           "fixed_us_per_tile": round(icpt, 3), "us_per_stage_of_64": round(slope, 5),
           "main_loop_share_at_8192": round(128 * slope / (icpt + 128 * slope), 4),
           "residual_us_max": round(max(abs(y - (icpt + slope * x)) for x, y in zip(xs, ys)) * tiles_per_wg, 2)}
    if sclk:
        ideal = 1024.0 / sclk          # 64 matrix ops of 16 cycles per stage and wavefront, at the sampled clock (us)
        fit["ideal_us_per_stage_at_sampled_clock"] = round(ideal, 5)
        fit["matrix_pipe_share_of_main_loop"] = round(ideal / slope, 4)
    out["k_sweep_fit"] = fit
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the clocks of an idle MI355X take some 50 ms of this kernel to settle: the defaults warm up
    # long enough for the timed steps to see the sustained state (0.2 s in all)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--size", type=int, default=8192, help="square size of the headline workload")
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload")
    ap.add_argument("--sections", default="all",
                    help="comma-separated extras to run, of: %s (default all of these), %s (only when named)"
                    % (", ".join(SECTIONS), ", ".join(OPT_IN_SECTIONS)))
    ap.add_argument("--skip-headline", action="store_true",
                    help="run the chosen extras only (to profile one kernel class); the line then carries no "
                         "headline value")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=16.0, help="target oracle wall time")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    want = set(SECTIONS) if args.sections == "all" else set(x for x in args.sections.split(",") if x)
    if args.no_extras:
        want = set()
    unknown = want - set(SECTIONS) - set(OPT_IN_SECTIONS)
    if unknown:
        print("bench.py: unknown section(s) %s" % ", ".join(sorted(unknown)), file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1910_00178_amd as ng
    from paper_1910_00178_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    ctx = ng.ngemm_create(0)
    b = Bench(ng, wl, torch, np, ctx)

    result = {}
    if not args.skip_headline:
        bench_headline(b, args, result)
    else:
        result["metric"] = "extras only (--skip-headline)"
        result["value"] = None
    if want:
        extras = {}
        if "skinny" in want:
            extras["skinny"] = bench_skinny(b, args)
        if "fc" in want:
            extras["bert_fc"] = bench_fc(b, args)
        if "longk" in want:
            extras["underfilled_long_k"] = bench_longk(b, args)
        if "batched" in want:
            extras["batched_64_odd_shapes"] = bench_batched(b, args)
        if "types" in want:
            bench_types(b, args, extras)
        if "power" in want:
            extras["power_and_time_budget_%d" % args.size] = bench_power(b, args)
        result["extras"] = extras

    ng.ngemm_destroy(ctx)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
