#!/usr/bin/env python3
"""Benchmark of the partition-local epoch (halo gather from the two-tier cache + GCN/SAGE forward and
backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C2]

A step is one full epoch over one synthetic partition: for every layer the halo rows are gathered from
the GPU tier (device copy) and the pinned-host tier (side stream), then the layer runs; loss; backward.
All inputs that the method keeps on the device are resident in HBM before the timed region; the host
tier is in pinned host memory because that is where the method keeps it.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
FP32_MATRIX_PEAK_TFLOPS = 157.3
BF16_MATRIX_PEAK_TFLOPS = 2500.0
L2_PEAK_GBPS = 8 * 2048 * 2.4          # 8 L2s x 2 KB per clock x 2.4 GHz = 39 322 GB/s (equally 256 CUs x 64 B per clock)


def spmm_launches(cfg, part, orders):
    """(layer, backward) -> (F, n_out, n_in_touched) of every SpMM launch of one epoch."""
    import numpy as np
    L = len(cfg.dims) - 1
    touched_fwd = int(np.unique(part.col).size)                 # source rows that any edge reads
    touched_bwd = int((np.diff(part.rowptr) > 0).sum())
    out = {}
    for l in range(L):
        fi, fo = cfg.dims[l], cfg.dims[l + 1]
        agg = orders[l] == 1
        out[(l, 0)] = (fi if agg else fo, part.n_loc, touched_fwd)
        if agg:
            if l > 0:                                            # dX = A_hat^T dM over the local columns
                out[(l, 1)] = (fi, part.n_loc, touched_bwd)
        else:                                                    # dT = A_hat^T dZ over all columns
            out[(l, 1)] = (fo, part.n_cols, touched_bwd)
    return out


def spmm_min_bytes(part, F, n_out, n_in_touched, es):
    """Compulsory traffic of one SpMM launch: every index once, every needed source row once, every
    output row once (nnz*4 + (n_out+1)*8 + touched*F*s + n_out*F*s)."""
    return part.nnz * 4 + (n_out + 1) * 8 + n_in_touched * F * es + n_out * F * es


def gemm_report(cfg, part, orders, kernels, f32_product):
    """The first layer's forward transform: the METHOD's FLOP rate (2 M N K per product, whatever the implementation
    spends on it) against the peak of the matrix instruction for the operands' own type - fp32 157.3 TFLOP/s, bf16
    2500 - and, beside it, the work the implementation gives the matrix cores: the split form of the fp32 product
    issues six bf16 piece products per fp32 product, so its instruction-level rate is six times the method's and is
    measured against the bf16 peak.  The second figure is implementation work, not the method's."""
    rec = [k for k in kernels if k["kind"] == "gemm" and k["layer"] == 0 and not k["backward"]]
    if not rec:
        return None
    rows = part.n_loc if orders[0] == 1 else part.n_cols
    mult = 2 if cfg.kind == "sage" else 1                    # GraphSAGE adds the self transform over the local rows
    flops = 2.0 * rows * cfg.dims[0] * cfg.dims[1] + (mult - 1) * 2.0 * part.n_loc * cfg.dims[0] * cfg.dims[1]
    tf = flops / (rec[0]["ms"] * 1e-3) / 1e12
    split = cfg.dtype == "f32" and (f32_product == "split" or
                                    (f32_product == "auto" and rows * cfg.dims[0] * cfg.dims[1] >= 1 << 28))
    method_peak = FP32_MATRIX_PEAK_TFLOPS if cfg.dtype == "f32" else BF16_MATRIX_PEAK_TFLOPS
    out = {"kernel": "transform of layer 0 (forward)", "gflop": flops / 1e9, "ms": rec[0]["ms"],
           "method_tflops": tf, "method_peak_tflops": method_peak, "method_frac_of_peak": tf / method_peak,
           "method_peak_is": "fp32 matrix instruction" if cfg.dtype == "f32" else "bf16 matrix instruction"}
    if split:
        out.update({"product_form": "three bf16 pieces per operand, six piece products per fp32 product",
                    "instruction_work_tflops": 6.0 * tf, "instruction_peak_tflops": BF16_MATRIX_PEAK_TFLOPS,
                    "instruction_work_frac_of_bf16_peak": 6.0 * tf / BF16_MATRIX_PEAK_TFLOPS,
                    "method_frac_of_bf16_peak": tf / BF16_MATRIX_PEAK_TFLOPS,
                    "note": "the factor 6 is implementation work; SQ_VALU_MFMA_BUSY_CYCLES of the same kernels is in "
                            "profiles/gemm_C2_C4_mfma_counters.txt"})
    else:
        out["product_form"] = "fp32 matrix instruction" if cfg.dtype == "f32" else "bf16 matrix instruction"
    return out


def f32_product_check(cfg):
    """Both forms of the fp32 product on one product of the first layer's shape (4096 rows): the largest deviation from an
    fp64 product of the same operands, relative to the largest result.  Untimed; shows in the benchmark line itself
    that the form the library chooses is as close to the exact product as the fp32 matrix instruction."""
    import torch
    from paper_2508_13716_amd import binding as B
    if cfg.dtype != "f32":
        return None
    M, K, N = 4096, cfg.dims[0], cfg.dims[1]
    lda = (K + 3) // 4 * 4
    gen = torch.Generator(device="cuda").manual_seed(1)
    A = torch.randn((M, lda), device="cuda", generator=gen)
    W = torch.randn((K, N), device="cuda", generator=gen)
    ref = A[:, :K].double() @ W.double()
    wsb = B.gemm_workspace_bytes(0, M, N, K)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    out = {}
    for name, mode in (("fp32_instruction", B.F32_PRODUCT_NATIVE), ("three_bf16_pieces", B.F32_PRODUCT_SPLIT)):
        Cd = torch.empty((M, N), device="cuda")
        B.gemm(0, 0, M, N, K, A, lda, W, N, Cd, N, B.F32, out_f32=1, ws=ws, ws_bytes=wsb, stream=torch.cuda.current_stream(),
               f32_product=mode)
        torch.cuda.synchronize()
        out[name] = float((Cd.double() - ref).abs().max() / ref.abs().max())
    out["product"] = f"{M} x {N} x {K}, standard normal operands"
    return out


def gather_peaks(steps, sweep=False):
    """What the memory levels deliver for the aggregation's access pattern, measured now on this GPU: 128-byte lines at
    random line numbers, 16 loads in flight per lane, nothing else (capgnn_gather_peak), on tables that fit an L2
    (2 MB), the Infinity Cache (128 MB) and neither (2 GB).  GB/s."""
    import torch
    from paper_2508_13716_amd import binding as B
    st = torch.cuda.Stream()
    wgs = 256 * 16
    out_buf = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    res = {}
    sizes = [("l2_2MB", 2 << 20, 64), ("infinity_cache_128MB", 128 << 20, 32), ("hbm_2GB", 2 << 30, 16)]
    if sweep:
        sizes = [(f"{b >> 10}KB", b, 64 if b <= (4 << 20) else 24) for b in (16 << 10, 256 << 10, 1 << 20, 2 << 20, 4 << 20, 8 << 20, 32 << 20,
                                                                              128 << 20, 512 << 20, 2 << 30)]
    for name, nbytes, iters in sizes:
        table = torch.zeros(nbytes // 4, dtype=torch.float32, device="cuda")
        B.gather_peak(table, nbytes // 128, wgs, iters, out_buf, st)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        moved = 0.0
        for _ in range(max(3, steps // 4)):
            moved += B.gather_peak(table, nbytes // 128, wgs, iters, out_buf, st)
        e1.record(st)
        torch.cuda.synchronize()
        res[name] = moved / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del table
    res["published_l2_peak"] = L2_PEAK_GBPS
    res["note"] = ("published: 8 XCDs x 2 KB per clock per L2 x 2.4 GHz (= 256 compute units x 64 B per clock into their L1s); "
                   "the measured rows are this GPU's rates for scattered 128-byte lines")
    return res


def cpu_baseline(prob, n_agg, threads=None, sample=None):
    """The oracle as it stands, timed on the host cores on `prob` (one full fp64 epoch).  threads: None = all cores."""
    from oracle import oracle as orc
    from tests import oracle_side as O
    all_cores = orc.max_threads()
    if threads is not None:
        orc.set_threads(threads)
    try:
        t0 = time.perf_counter()
        O.oracle_epoch(prob)
        dt = time.perf_counter() - t0
    finally:
        if threads is not None:
            orc.set_threads(all_cores)
    part, cfg = prob.part, prob.cfg
    return {"value": part.nnz * n_agg / dt / 1e9, "unit": "GEdges/s (edges aggregated per epoch / epoch wall time)",
            "cores": all_cores if threads is None else threads, "kind": "oracle",
            "sample": sample or f"the whole of {cfg.name} ({part.n_loc} local, {part.n_halo} halo, {part.nnz} edges), one full fp64 oracle epoch, {dt:.2f} s",
            "epoch_s_on_sample": dt}


def bench_cache_update(args):
    """Throughput of the cache write path (vertex update into both tiers, bounded-staleness list) on the
    configuration's halo set; one JSON line.  Not the headline metric: a measurement of its own."""
    import numpy as np
    import torch
    from paper_2508_13716_amd import binding as B, synth
    cfg = synth.CONFIGS[args.config]
    part = synth.partition_for(cfg)
    L = len(cfg.dims) - 1
    dt = B.BF16 if cfg.dtype == "bf16" else B.F32
    es = 2 if cfg.dtype == "bf16" else 4
    cap = synth.cap_gpu_for(cfg, part)
    c = B.Cache(part.halo_gid, part.halo_prio, cap, cfg.dims[:L], dt, B.MAP_DIRECT)
    tier, _ = c.query(np.arange(part.n_halo))
    st = torch.cuda.Stream()
    ids_out = torch.empty(max(part.n_halo, 1), dtype=torch.int64, device="cuda")

    def timeit(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(st):
            e0.record(st)
            for _ in range(args.steps):
                fn()
            e1.record(st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    layers = []
    for l in range(L):
        F = cfg.dims[l]
        ld = synth.pad_to(F, 16 // es)
        rec = {"layer": l, "F": F}
        for key, sel in (("gpu_tier", np.nonzero(tier == 0)[0]), ("host_tier", np.nonzero(tier == 1)[0])):
            if len(sel) == 0:
                continue
            ids = torch.from_numpy(np.random.default_rng(l).permutation(sel).astype(np.int64)).cuda()
            rows = torch.randn(len(sel), ld, device="cuda").to(torch.bfloat16 if es == 2 else torch.float32)
            torch.cuda.synchronize()
            ms = timeit(lambda: B.cache_update(c, l, ids, len(sel), rows, ld, 3, stream=st))
            nbytes = len(sel) * F * es
            rec[key] = {"rows": int(len(sel)), "ms": ms, "written_GBps": nbytes / ms / 1e6,
                        "read_plus_written_GBps": 2 * nbytes / ms / 1e6}
        rec["stale_list_ms"] = timeit(lambda: B.cache_stale(c, l, 10, 2, ids_out, stream=st))
        layers.append(rec)
    print(json.dumps({"metric": "cache update throughput", "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "data": "synthetic",
                      "config": {"workload": f"{cfg.name}: {part.n_halo} halo vertices, GPU tier {cap} rows, dims {cfg.dims[:L]}, {cfg.dtype}"},
                      "hbm_peak_GBps": HBM_PEAK_GBPS, "layers": layers}))
    c.close()


def bench_policy(args):
    """Hit-rate curves of the policy layer (overlap-ratio priority against FIFO and LRU on the two-level
    structure) on a random 4-way partition of a synthetic power-law graph; one JSON line."""
    import numpy as np
    import torch
    from paper_2508_13716_amd import binding as B, synth
    n, nnz, P = 233_000, 11_500_000, 4          # Reddit's vertex count, a tenth of its edges
    sets, _ = synth.make_halo_sets(n, nnz, P, seed=synth.BASE_SEED * 10 + 9)
    flat = np.concatenate(sets)
    ids_d = torch.from_numpy(flat).cuda()
    R = torch.empty(n, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    B.overlap_ratio(ids_d, len(flat), n, R)
    torch.cuda.synchronize()
    t_overlap = time.perf_counter() - t0
    hist = np.bincount(R.cpu().numpy(), minlength=P + 1).tolist()
    union = int((R > 0).sum().item())
    rate = lambda c: (c[0] + c[1]) / max(1, sum(c))
    curves = []
    for frac in (0.02, 0.05, 0.1, 0.2, 0.4, 0.6, 0.8, 1.0):
        cap_g = int(frac * union)
        cap_l = cap_g // 8 if frac < 1.0 else cap_g
        t0 = time.perf_counter()
        row = {"global_capacity": cap_g, "local_capacity": cap_l}
        for name, pid in (("jaca", B.POLICY_JACA), ("low_overlap_first", B.POLICY_JACA_LOW), ("fifo", B.POLICY_FIFO), ("lru", B.POLICY_LRU)):
            row[name] = round(rate(B.policy_simulate(sets, pid, cap_l, cap_g, 3)), 4)
        row["simulate_s"] = round(time.perf_counter() - t0, 3)
        curves.append(row)
    print(json.dumps({"metric": "cache hit rate by policy", "unit": "fraction of halo requests served by a cache", "n_gpus": 1,
                      "data": "synthetic", "config": {"workload": f"random {P}-way partition of a power-law graph, {n} vertices, {nnz} edges; "
                                                                  f"{len(flat)} halo requests per epoch, {union} distinct halo vertices"},
                      "overlap_ratio_histogram": hist, "overlap_ratio_kernel_ms": t_overlap * 1e3, "curves": curves}))


def bench_zipf_requests(args):
    """C5's second reading: a request list of 2 M ids drawn with replacement, Zipf(1.1) over the halo vertices ranked
    by priority, served from a cache whose GPU tier holds the top 10 %.  Reports the measured hit fraction next to
    the closed form H_{k,s} / H_{N,s}, and the rate of the request-list gather (lookup + copy); one JSON line."""
    import numpy as np
    import torch
    from paper_2508_13716_amd import binding as B, synth
    N, k, s_exp, F = 2_000_000, 200_000, 1.1, 512
    p = np.arange(1, N + 1, dtype=np.float64) ** -s_exp
    p /= p.sum()
    rng = synth.rng_for(synth.BASE_SEED * 10 + 5, 90)
    gid = rng.permutation(N).astype(np.int64) * 3 + 11
    prio = (1e15 * p).astype(np.int64)                      # strictly decreasing: rank = halo-local index
    c = B.Cache(gid, prio, k, [F], B.BF16, B.MAP_HASH)
    c.set_miss_mode(B.MISS_ZEROCOPY)                         # a request list is served by one kernel, misses read pinned memory
    req_h = rng.choice(N, size=N, p=p)
    hits_expected = float((p[:k]).sum())
    st = torch.cuda.Stream()
    out = torch.empty((N, F), dtype=torch.bfloat16, device="cuda")
    res = {}
    for name, ids_h, by_gid in (("halo_local_index_direct", req_h.astype(np.int64), False), ("global_id_hash", gid[req_h], True)):
        ids = torch.from_numpy(ids_h).cuda()
        rc, stats = B.halo_gather(c, 0, ids, N, out, F, by_gid=by_gid, stream=st, want_stats=True)
        for _ in range(args.warmup):
            B.halo_gather(c, 0, ids, N, out, F, by_gid=by_gid, stream=st)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(args.steps):
            B.halo_gather(c, 0, ids, N, out, F, by_gid=by_gid, stream=st)
        e1.record(st)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        res[name] = {"ms": round(ms, 3), "hit_fraction": stats.hits / N, "rows_per_s": N / ms * 1e3,
                     "out_GBps": N * F * 2 / ms / 1e6}
    c.close()
    print(json.dumps({"metric": "request-list halo gather, Zipf(1.1) requests", "unit": "ms per 2 M requests", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "dtype": "bf16 rows (bit copies)", "data": "synthetic",
                      "config": {"workload": f"{N} halo vertices, GPU tier = top {k} by priority, {N} requests with replacement, "
                                             f"rows of {F} bf16; host-tier rows are read from pinned memory by the same kernel"},
                      "hit_fraction_closed_form": hits_expected, "lookups": res}))


def bench_mfma_peak(args):
    """What the matrix cores deliver with register-resident operands (fp32 and bf16 instructions); one JSON line."""
    import torch
    from paper_2508_13716_amd import binding as B
    st = torch.cuda.Stream()
    wgs, iters = 256 * 8, 4096
    out = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    res = {}
    for name, dt, peak in (("f32", B.F32, 157.3), ("bf16", B.BF16, BF16_MATRIX_PEAK_TFLOPS)):
        B.mfma_peak(dt, wgs, iters, out, st)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        flop = 0.0
        for _ in range(args.steps):
            flop += B.mfma_peak(dt, wgs, iters, out, st)
        e1.record(st)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        res[name] = {"tflops": flop / ms / 1e9, "data_sheet_tflops": peak, "frac": flop / ms / 1e9 / peak}
    print(json.dumps({"metric": "matrix-instruction throughput, register-resident operands", "unit": "TFLOP/s", "n_gpus": 1,
                      "steps": args.steps, "data": "synthetic", "config": {"workload": f"{wgs} workgroups x 4 waves x {4 * iters} instructions"},
                      "measured": res}))


def bench_products(args):
    """The dense products of a configuration's layers, alone, operands resident, in both forms of the fp32 product
    (fp32 matrix instruction / three bf16 pieces): time, rate, and distance from an fp64 product of the same operands."""
    import torch
    from paper_2508_13716_amd import binding as B, synth
    cfg = synth.CONFIGS[args.config]
    if cfg.dtype != "f32":
        print("bench.py --what products: the two product forms exist for fp32 configurations (C1, C2, C3)", file=sys.stderr)
        sys.exit(2)
    n_cols, n_loc = cfg.n_loc + cfg.n_halo, cfg.n_loc

    def pad(n):                                             # rows of whole, odd numbers of 128-byte lines
        b = (n * 4 + 127) // 128 * 128
        return (b + 128 if b % 256 == 0 else b) // 4

    def run(ta, tb, M, N, K, mode):
        sa, sb = ((K, M) if ta else (M, K)), ((N, K) if tb else (K, N))
        lda, ldb, ldc = pad(sa[1]), (pad(sb[1]) if ta else sb[1]), pad(N)
        g = torch.Generator(device="cuda").manual_seed(M + 3 * N + 7 * K)
        A = torch.randn((sa[0], lda), device="cuda", generator=g)
        Bm = torch.randn((sb[0], ldb), device="cuda", generator=g)
        Cd = torch.empty((M, ldc), device="cuda")
        wsb = B.gemm_workspace_bytes(ta, M, N, K)
        ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
        st = torch.cuda.Stream()
        call = lambda: B.gemm(ta, tb, M, N, K, A, lda, Bm, ldb, Cd, ldc, B.F32, out_f32=1, ws=ws, ws_bytes=wsb, stream=st,
                              f32_product=mode)
        for _ in range(args.warmup):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(args.steps):
            call()
        e1.record(st)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        Ad, Bd = A[:, :sa[1]].double(), Bm[:, :sb[1]].double()
        ref = (Ad.T if ta else Ad) @ (Bd.T if tb else Bd)
        err = float((Cd[:, :N].double() - ref).abs().max() / ref.abs().max())
        return {"ms": ms, "tflops": 2e-9 * M * N * K / ms, "err": err}

    out = []
    for l in range(len(cfg.dims) - 1):
        fi, fo = cfg.dims[l], cfg.dims[l + 1]
        for name, ta, tb, M, N, K in ((f"layer {l}: X W", 0, 0, n_cols, fo, fi), (f"layer {l}: X^T dT", 1, 0, fi, fo, n_cols),
                                      (f"layer {l}: dT W^T", 0, 1, n_loc, fi, fo)):
            out.append({"product": name, "M": M, "N": N, "K": K, "trans_a": ta, "trans_b": tb,
                        "fp32_instruction": run(ta, tb, M, N, K, B.F32_PRODUCT_NATIVE),
                        "three_bf16_pieces": run(ta, tb, M, N, K, B.F32_PRODUCT_SPLIT)})
    print(json.dumps({"metric": "dense products alone, both forms of the fp32 product", "unit": "ms / TFLOP/s / max error over max |result|",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
                      "config": {"workload": f"{args.config}: {n_loc} local + {cfg.n_halo} halo rows, dims {list(cfg.dims)}"},
                      "products": out}))


def bench_spmm_launch(args):
    """One aggregation launch alone, repeated: the dominant launch of a configuration (or --F / --direction), on the
    configuration's graph, with scratch, exactly as the layer code calls it.  Before it, two calibration launches of
    known size for counter runs: capgnn_gather_peak over a 2 GB table (reads its requested bytes from memory: the table
    is 500 times the L2s) and a 1 GiB fill (writes 1 GiB).  One JSON line."""
    import numpy as np
    import torch
    from paper_2508_13716_amd import binding as B, synth
    cfg = synth.CONFIGS[args.config]
    part = synth.partition_for(cfg)
    bf = cfg.dtype == "bf16"
    dt, tdt, es = (B.BF16, torch.bfloat16, 2) if bf else (B.F32, torch.float32, 4)
    F = args.F or {"C1": 128, "C2": 256, "C3": 256, "C4": 256, "C5": 512}[args.config]
    kind = B.NORM_SYM if cfg.kind == "gcn" else B.NORM_MEAN
    r, c = B.norm_scales(kind, part.n_loc, part.n_halo, part.rowptr, part.halo_degree if part.n_halo else None)
    g = B.Graph(part.n_loc, part.n_halo, part.rowptr, part.col, r, c, None, B.GRAPH_SYMMETRIC if part.symmetric else 0)
    st = torch.cuda.Stream()
    # calibration launches
    table = torch.zeros((2 << 30) // 4, dtype=torch.float32, device="cuda")
    outp = torch.empty(4096 * 256, dtype=torch.float32, device="cuda")
    cal_read = B.gather_peak(table, (2 << 30) // 128, 4096, 16, outp, st)
    torch.cuda.synchronize()
    del table
    filled = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    filled.fill_(1.0)
    torch.cuda.synchronize()
    del filled
    # the layer code's pitch: whole, odd numbers of 128-byte lines when the graph has a column-blocked copy
    wsb = B.spmm_workspace_bytes(g, F, dt)
    pitch = (F * es + 15) // 16 * 16
    if wsb > part.n_cols * F * es:
        pitch = (pitch + 127) // 128 * 128
        pitch += 128 if pitch % 256 == 0 else 0
    ld = pitch // es
    fwd = args.direction == "fwd"
    n_in, n_out = (part.n_cols, part.n_loc) if fwd else (part.n_loc, part.n_cols)
    X = torch.randn(n_in, ld, device="cuda").to(tdt)
    Y = torch.empty(n_out, ld, device="cuda", dtype=tdt)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    call = (lambda: B.spmm_fwd(g, X, ld, Y, ld, F, dt, st, ws=ws, ws_bytes=wsb)) if fwd else \
           (lambda: B.spmm_bwd(g, X, ld, Y, ld, F, dt, st, ws=ws, ws_bytes=wsb))
    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(args.steps):
        call()
    e1.record(st)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    touched = int(np.unique(part.col).size) if fwd else int((np.diff(part.rowptr) > 0).sum())
    bmin = spmm_min_bytes(part, F, n_out, touched, es)
    print(json.dumps({"metric": "one aggregation launch alone", "unit": "ms per launch", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "dtype": cfg.dtype, "data": "synthetic",
                      "config": {"workload": f"{cfg.name} {args.direction} F={F}: {n_out} output rows, {n_in} source rows, {part.nnz} entries, pitch {pitch} B"},
                      "ms": ms, "gedges_s": part.nnz / ms / 1e6, "algorithmic_bytes": bmin,
                      "requested_bytes": part.nnz * F * es, "requested_GBps": part.nnz * F * es / ms / 1e6,
                      "launches": args.steps + args.warmup,
                      "calibration": {"gather_peak_2GB_table_read_bytes": cal_read, "fill_written_bytes": (1 << 28) * 4}}))
    g.close()


def bench_spmm_ranges(args):
    """What tiling the sources of a low-degree aggregation to a cache level could give at best: the configuration's
    forward launch against the same launch cut into --ranges launches, range k keeping only the entries whose source row
    lies in the k-th part of the operand (so each launch gathers from 1/ranges of it).  The cut launches write every
    output row once per range and nothing adds them up: their summed time is a lower bound for a tiled kernel, which
    would also have to carry or re-read the partial sums.  One JSON line."""
    import numpy as np
    import torch
    from paper_2508_13716_amd import binding as B, synth
    cfg = synth.CONFIGS[args.config]
    part = synth.partition_for(cfg)
    bf = cfg.dtype == "bf16"
    dt, tdt, es = (B.BF16, torch.bfloat16, 2) if bf else (B.F32, torch.float32, 4)
    F = args.F or 256
    kind = B.NORM_SYM if cfg.kind == "gcn" else B.NORM_MEAN
    r, c = B.norm_scales(kind, part.n_loc, part.n_halo, part.rowptr, part.halo_degree if part.n_halo else None)
    st = torch.cuda.Stream()
    ld = (F * es + 15) // 16 * 16 // es
    X = torch.randn(part.n_cols, ld, device="cuda").to(tdt)
    Y = torch.empty(part.n_loc, ld, device="cuda", dtype=tdt)

    def time_graph(rowptr, col):
        g = B.Graph(part.n_loc, part.n_halo, rowptr, col, r, c, None, 0)
        wsb = B.spmm_workspace_bytes(g, F, dt)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        for _ in range(args.warmup):
            B.spmm_fwd(g, X, ld, Y, ld, F, dt, st, ws=ws, ws_bytes=wsb)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(args.steps):
            B.spmm_fwd(g, X, ld, Y, ld, F, dt, st, ws=ws, ws_bytes=wsb)
        e1.record(st)
        torch.cuda.synchronize()
        g.close()
        return e0.elapsed_time(e1) / args.steps

    whole = time_graph(part.rowptr, part.col)
    row_of = np.repeat(np.arange(part.n_loc, dtype=np.int32), np.diff(part.rowptr))
    cuts = []
    for k in range(args.ranges):
        lo, hi = part.n_cols * k // args.ranges, part.n_cols * (k + 1) // args.ranges
        keep = (part.col >= lo) & (part.col < hi)
        rp = np.zeros(part.n_loc + 1, np.int64)
        np.cumsum(np.bincount(row_of[keep], minlength=part.n_loc), out=rp[1:])
        ms = time_graph(rp, part.col[keep])
        cuts.append({"source_rows": [int(lo), int(hi)], "operand_MB": (hi - lo) * ld * es / 1e6, "entries": int(keep.sum()), "ms": ms})
        print(f"range {k}: {cuts[-1]}", file=sys.stderr, flush=True)
    print(json.dumps({"metric": "aggregation launch whole against cut into source ranges", "unit": "ms", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "dtype": cfg.dtype, "data": "synthetic",
                      "config": {"workload": f"{cfg.name} fwd F={F}: {part.n_loc} output rows, {part.n_cols} source rows, {part.nnz} entries"},
                      "whole_ms": whole, "ranges": args.ranges, "cut_ms_sum": sum(c["ms"] for c in cuts), "cuts": cuts,
                      "note": "the cut launches write each output row once per range and do not add the partial sums"}))


def bench_rapa(args):
    """RAPA's subgraph adjustment end to end on a synthetic 4-way partition with uneven shares: influence scores on the
    GPU (Eq. 6), Alg. 2 / Alg. 3 in the library with equal GPUs (every rate 1), pruning, and the measured epoch time of
    every subgraph on this GPU before and after.  What the method promises is a smaller spread of the per-subgraph cost;
    the measured spread is printed beside the cost model's.  One JSON line."""
    import dataclasses
    import numpy as np
    import torch
    from paper_2508_13716_amd import binding as B, harness as H, synth
    P = 4
    parts, _ = synth.make_partitioned_graph(600000, 12000000, P, seed=synth.BASE_SEED * 10 + 21, shares=[4, 3, 2, 1])
    dims = [128, 256, 47]

    def epoch_ms(part):
        cfg = synth.Config(part.name, "sage", part.n_loc, part.n_halo, part.nnz, dims, "f32", 1.0, seed=synth.BASE_SEED * 10 + 22)
        dp = H.DeviceProblem(H.make_problem(cfg, part=part))
        for _ in range(args.warmup):
            dp.run_epoch()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            dp.run_epoch()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        dp.close()
        return ms

    n_inner, e_inner, he, scores = [], [], [], []
    for p in parts:
        ei, cnt = B.halo_edge_counts(p.n_loc, p.n_halo, p.rowptr, p.col)
        n_inner.append(p.n_loc); e_inner.append(ei); he.append(cnt)
        din = np.maximum(np.diff(p.rowptr), 1)
        dout = np.maximum(np.bincount(p.col, minlength=p.n_cols), 1)
        count = np.concatenate([np.ones(p.n_loc), p.halo_prio.astype(np.float64)])
        g = B.Graph(p.n_loc, p.n_halo, p.rowptr, p.col)
        S = torch.zeros(p.n_cols, device="cuda")
        B.influence_score(g, torch.from_numpy((1.0 / np.sqrt(din)).astype(np.float32)).cuda(),
                          torch.from_numpy((1.0 / np.sqrt(dout)).astype(np.float32)).cuda(),
                          torch.from_numpy(count.astype(np.float32)).cuda(), S)
        torch.cuda.synchronize()
        g.close()
        scores.append(S.cpu().numpy()[p.n_loc:])
    dev = [B.RapaDevice(1.0, 1.0, 1.0, 1.0, 1.0, 1e18) for _ in range(P)]
    # the cost model (Eq. 3-4) of the subgraphs as they are, all rate ratios 1: the threshold is 1 % of its mean (the
    # evaluation's setting)
    alpha = 0.5
    lam0 = np.array([alpha * (e_inner[i] + int(he[i].sum())) + (1 - alpha) * n_inner[i] + int(he[i].sum()) * (2.0 * (1 - 1.0 / P) + 1.0 / P)
                     for i in range(P)])
    res = B.rapa_adjust(n_inner, e_inner, he, scores, dev,
                        B.RapaParams(0.5, 0.01 * float(np.mean(lam0)), 8, 12, 4, dims[0], 100.0 * 2 ** 20, 1000))
    before = [epoch_ms(p) for p in parts]
    pruned = []
    for i, p in enumerate(parts):
        rp, cl, _ = B.prune_halo(p.n_loc, p.n_halo, p.rowptr, p.col, res["keep"][i])
        k = res["keep"][i].astype(bool)
        pruned.append(dataclasses.replace(p, name=p.name + "-pruned", n_halo=int(k.sum()), rowptr=rp, col=cl,
                                          halo_gid=p.halo_gid[k], halo_prio=p.halo_prio[k], halo_degree=p.halo_degree[k]))
    after = [epoch_ms(p) for p in pruned]
    print(json.dumps({
        "metric": "per-subgraph epoch ms before / after RAPA's subgraph adjustment", "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{P}-way random partition (shares 4:3:2:1) of a power-law graph, 600000 vertices, "
                               f"{sum(p.nnz for p in parts)} edges in the subgraphs; GraphSAGE {dims}; equal GPUs, alpha 0.5, "
                               "epsilon 1 % of the mean cost"},
        "sweeps": res["sweeps"], "r": res["r"],
        "subgraphs": [{"n_inner": int(n_inner[i]), "halo": [int(parts[i].n_halo), int(pruned[i].n_halo)],
                       "edges": [int(parts[i].nnz), int(pruned[i].nnz)], "cost_model": [float(lam0[i]), float(res["lam"][i])],
                       "epoch_ms": [before[i], after[i]]} for i in range(P)],
        "cost_model_sigma": [float(np.std(lam0)), float(res["sigma"])],
        "epoch_ms_sigma": [float(np.std(before)), float(np.std(after))],
        "epoch_ms_max": [max(before), max(after)],
        "note": "with equal GPUs the adjustment can only shed halo vertices of the costliest subgraphs; the slowest subgraph bounds "
                "a synchronous epoch, so epoch_ms_max is the figure that matters"}))


def bench_reorder(args):
    """Aggregation time of one SpMM launch (forward and transposed, hidden width 256) before and after the
    vertices are stored in a locality order, on the named config's graph (--config; 'clustered' = a graph with
    geometric locality whose numbering hides it); one JSON line."""
    import torch
    from paper_2508_13716_amd import binding as B, synth
    F = 256
    if args.config == "clustered":
        part = synth.make_clustered_partition("clustered", 1_300_000, 26, 4000, seed=synth.BASE_SEED * 10 + 7)
        kind, bf = B.NORM_SYM, True
        workload = f"clustered ring-window graph, labels shuffled: {part.n_loc} vertices, {part.nnz} entries"
    else:
        cfg = synth.CONFIGS[args.config]
        part = synth.partition_for(cfg)
        kind, bf = (B.NORM_SYM if cfg.kind == "gcn" else B.NORM_MEAN), cfg.dtype == "bf16"
        workload = f"{args.config}: {part.n_loc} local + {part.n_halo} halo vertices, {part.nnz} entries"
    dt, tdt, es = (B.BF16, torch.bfloat16, 2) if bf else (B.F32, torch.float32, 4)
    st = torch.cuda.Stream()

    def timeit(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(args.steps):
            fn()
        e1.record(st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    def measure(rowptr, col, halo_degree):
        r, c = B.norm_scales(kind, part.n_loc, part.n_halo, rowptr, halo_degree)
        g = B.Graph(part.n_loc, part.n_halo, rowptr, col, r, c, None, B.GRAPH_SYMMETRIC if part.symmetric else 0)
        X = torch.randn(part.n_cols, F, device="cuda").to(tdt)
        Y = torch.empty(part.n_loc, F, device="cuda", dtype=tdt)
        dY = torch.randn(part.n_loc, F, device="cuda").to(tdt)
        dX = torch.empty(part.n_cols, F, device="cuda", dtype=tdt)
        wsb = B.spmm_workspace_bytes(g, F, dt)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        tf = timeit(lambda: B.spmm_fwd(g, X, F, Y, F, F, dt, st, ws=ws, ws_bytes=wsb))
        tb = timeit(lambda: B.spmm_bwd(g, dY, F, dX, F, F, dt, st, ws=ws, ws_bytes=wsb))
        g.close()
        gathered = part.nnz * F * es
        return {"spmm_fwd_ms": round(tf, 4), "spmm_bwd_ms": round(tb, 4), "fwd_gather_GBps": round(gathered / tf / 1e6, 1),
                "bwd_gather_GBps": round(gathered / tb / 1e6, 1)}

    hd = part.halo_degree if part.n_halo else None
    out = {"original": measure(part.rowptr, part.col, hd)}
    for name, mid in (("popularity", B.RELABEL_POPULARITY), ("bfs", B.RELABEL_BFS)):
        t0 = time.perf_counter()
        o = B.locality_order(mid, part.n_loc, part.n_halo, part.rowptr, part.col)
        rp, cl, _ = B.relabel_csr(part.n_loc, part.n_halo, part.rowptr, part.col, o)
        host_s = time.perf_counter() - t0
        out[name] = measure(rp, cl, None if hd is None else hd[o[part.n_loc:] - part.n_loc])
        out[name]["host_order_and_relabel_s"] = round(host_s, 2)
    print(json.dumps({"metric": "SpMM time before / after vertex reordering", "unit": "ms per launch", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "dtype": "bf16" if bf else "f32", "data": "synthetic",
                      "config": {"workload": workload, "F": F}, "orders": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default=None, help="one workload only (C1..C5); default: C2 as the headline line with C1, C3, C4, C5 under 'configs'")
    ap.add_argument("--what", default="epoch", choices=["epoch", "cache_update", "policy", "reorder", "zipf_requests", "mfma_peak", "products", "gather_peak", "spmm", "spmm_ranges", "rapa"],
                    help="epoch (default): the headline benchmark; cache_update: throughput of the cache write path; "
                         "policy: hit-rate curves of the cache policies; reorder: SpMM before / after vertex reordering "
                         "(--config C2..C5 or clustered); zipf_requests: request-list gather under Zipf(1.1) requests")
    ap.add_argument("--miss-mode", type=int, default=None, help="0 zero-copy kernel, 1 staged DMA, 2 staged DMA prefetched one epoch ahead (default 2)")
    ap.add_argument("--reorder", default="none", choices=["none", "popularity", "bfs"],
                    help="store the vertices in a locality order before the graph handle is built (epoch benchmark)")
    ap.add_argument("--orders", default=None, help="comma list of 1 (aggregate first) / 2 (transform first) per layer")
    ap.add_argument("--f32-product", default="auto", choices=["auto", "native", "split"],
                    help="how products of fp32 operands are formed: the fp32 matrix instruction, three bf16 pieces per operand "
                         "on the bf16 matrix cores, or (default) the library's choice by size")
    ap.add_argument("--plain", action="store_true", help="epoch benchmark: the eager epochs only (no graph replay, no vertex-update leg, no second timing with the GPU tier Alg. 1 grants): what the kernel traces and counter runs under profiles/ use")
    ap.add_argument("--F", type=int, default=0, help="--what spmm: width of the launch (default: the configuration's dominant launch)")
    ap.add_argument("--direction", default="fwd", choices=["fwd", "bwd"], help="--what spmm: forward or transposed aggregation")
    ap.add_argument("--ranges", type=int, default=5, help="--what spmm_ranges: number of source ranges the launch is cut into")
    ap.add_argument("--cpu-scale", type=float, default=None,
                    help="share of the workload the oracle is timed on (0 = skip; default: the whole workload, 0.1-27 s per configuration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the partition-local step on ONE GPU; --gpus > 1 is not part of it "
              "(no collectives, no sharding across GPUs).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2508_13716_amd import binding as B, harness as H, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    B.lib()
    if args.what != "epoch" and args.config is None:
        args.config = "C2"
    if args.what == "cache_update":
        return bench_cache_update(args)
    if args.what == "reorder":
        return bench_reorder(args)
    if args.what == "zipf_requests":
        return bench_zipf_requests(args)
    if args.what == "spmm_ranges":
        return bench_spmm_ranges(args)
    if args.what == "rapa":
        return bench_rapa(args)
    if args.what == "spmm":
        return bench_spmm_launch(args)
    if args.what == "mfma_peak":
        return bench_mfma_peak(args)
    if args.what == "gather_peak":
        print(json.dumps({"metric": "scattered 128-byte-line gather rate by table size", "unit": "GB/s", "n_gpus": 1,
                          "data": "synthetic", "measured": gather_peaks(args.steps, sweep=True)}))
        return
    if args.what == "products":
        return bench_products(args)
    if args.what == "policy":
        return bench_policy(args)

    peaks = gather_peaks(args.steps)
    if args.config is not None:
        out = epoch_record(args.config, args, peaks, headline=True)
    else:
        # the headline line is C2's; the other four named workloads ride along, each measured the same way
        out = epoch_record("C2", args, peaks, headline=True)
        out["configs"] = {}
        for name in ("C1", "C3", "C4", "C5"):
            rec = epoch_record(name, args, peaks, headline=False)
            out["configs"][name] = rec
    out["gather_peaks_GBps"] = peaks
    print(json.dumps(out))


def traffic_for(key):
    """(bytes per launch beyond L2, where it comes from) for a launch key of profiles/traffic_per_launch.txt, or (None, None):
    a PROFILED CONSTANT (two rocprofv3 --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size), not
    measured in this run; the file names the commit the counters were taken at."""
    tpath = os.path.join(ROOT, "profiles", "traffic_per_launch.txt")
    if not os.path.exists(tpath):
        return None, None
    taken_at = None
    for line in open(tpath):
        if line.startswith("# taken at"):
            taken_at = line[2:].strip()
        parts = line.split()
        if len(parts) >= 2 and parts[0] == key:
            return float(parts[1]), f"profiled constant from profiles/traffic_per_launch.txt ({taken_at or 'commit not recorded'}); not measured in this run"
    return None, None


def epoch_record(name, args, peaks, headline):
    """Builds the named workload, times args.steps epochs, and returns its record (the whole JSON line when headline)."""
    import numpy as np
    import torch
    from paper_2508_13716_amd import binding as B, harness as H, synth
    cfg = synth.CONFIGS[name]
    prob = H.make_problem(cfg)
    if args.reorder != "none":
        prob, _ = H.relabel_problem(prob, B.RELABEL_POPULARITY if args.reorder == "popularity" else B.RELABEL_BFS)
    part = prob.part
    orders = [int(x) for x in args.orders.split(",")] if args.orders else None
    f32p = {"auto": B.F32_PRODUCT_AUTO, "native": B.F32_PRODUCT_NATIVE, "split": B.F32_PRODUCT_SPLIT}[args.f32_product]
    miss_mode = B.MISS_PIPELINED if args.miss_mode is None else args.miss_mode

    def timed(dp, steps):
        for _ in range(args.warmup):
            dp.run_epoch()
        torch.cuda.synchronize()
        acc, stage, dev_epochs = {}, {}, []
        t0 = time.perf_counter()
        for _ in range(steps):
            loss, times = dp.run_epoch(want_times=True)
            per_epoch = {}
            for r in times["records"]:      # several records of one epoch may share a key (the GEMMs of one layer)
                key = (r["kind"], r["layer"], r["backward"])
                per_epoch[key] = per_epoch.get(key, 0.0) + r["ms"]
            for key, ms in per_epoch.items():
                acc.setdefault(key, []).append(ms)
            dev_epochs.append(times["total_ms"])
            for k in ("pick_cache_ms", "communication_ms", "aggregation_ms", "combine_ms", "loss_ms", "other_ms", "total_ms"):
                stage[k] = stage.get(k, 0.0) + times[k] / steps
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, acc, stage, dev_epochs, loss

    dp = H.DeviceProblem(prob, orders=orders, miss_mode=miss_mode, f32_product=f32p)
    res_orders = dp.resolved_orders()
    es = dp.es
    ms_per_step, acc, stage, dev_epochs, loss = timed(dp, args.steps)

    launches = spmm_launches(cfg, part, res_orders)
    # the method's own count: one aggregation per layer forward, one transposed aggregation per layer
    # backward except the first layer (whose input needs no gradient) - whatever association is run
    n_agg = 2 * dp.L - 1
    edges_per_epoch = part.nnz * n_agg
    kernels = []
    for (kind, layer, bwd), v in sorted(acc.items(), key=lambda kv: -sum(kv[1])):
        # a record may cover more than one launch of the same kind (e.g. the GEMMs of one layer)
        kernels.append({"kind": kind, "layer": layer, "backward": bwd, "ms": float(np.mean(v))})
    spmm_recs = [k for k in kernels if k["kind"] in ("spmm_fwd", "spmm_bwd")]
    # the dominant launch: the slowest forward aggregation (the transposed launch of the same layer takes about as long -
    # on a symmetric graph it is the same launch - and the choice must not flip between runs)
    fwd_recs = [k for k in spmm_recs if k["kind"] == "spmm_fwd"]
    dom = fwd_recs[0] if fwd_recs else (spmm_recs[0] if spmm_recs else kernels[0])
    F, n_out, touched = launches[(dom["layer"], dom["backward"])]
    bmin = spmm_min_bytes(part, F, n_out, touched, es)
    bgather = part.nnz * (4 + F * es) + n_out * F * es
    achieved = bmin / (dom["ms"] * 1e-3) / 1e9
    traffic, traffic_src = traffic_for(f"{cfg.name}:{dom['kind']}:L{dom['layer']}:F{F}")
    spmm_ms = sum(k["ms"] for k in spmm_recs)
    hit_bytes = sum(2 * dp.cache.cap_gpu * cfg.dims[l] * es for l in range(dp.L)) if dp.cache else 0
    miss_bytes = sum((part.n_halo - dp.cache.cap_gpu) * cfg.dims[l] * es for l in range(dp.L)) if dp.cache else 0
    hit_ms = sum(k["ms"] for k in kernels if k["kind"] == "gather_hit")
    staged_ms = sum(k["ms"] for k in kernels if k["kind"] == "gather_staged")
    miss_ms = sum(k["ms"] for k in kernels if k["kind"] == "gather_miss")
    pipelined_mode = miss_mode == B.MISS_PIPELINED
    copy_rate = ((hit_bytes + (2 * miss_bytes if (staged_ms or pipelined_mode) else 0)) / ((hit_ms + staged_ms) * 1e-3) / 1e9
                 if hit_ms + staged_ms else None)
    # which memory level serves the gather: the column-blocked kernel walks 4 MB panels (an L2); the one-wave-per-row
    # kernel gathers from the whole operand
    operand_bytes = touched * F * es
    blocked = bool(B.spmm_workspace_bytes(dp.graph, F, dp.dtype) > operand_bytes)     # partial rows for every source block
    level = "l2_2MB" if blocked else ("infinity_cache_128MB" if operand_bytes <= (256 << 20) else "hbm_2GB")
    gather_rate = part.nnz * F * es / (dom["ms"] * 1e-3) / 1e9

    out = {
        "metric": "aggregation GEdges/s + achieved HBM GB/s; partition epoch ms (fwd+bwd)",
        "value": edges_per_epoch / (ms_per_step * 1e-3) / 1e9,
        "unit": "GEdges/s (edges aggregated per epoch / epoch wall time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if cfg.dtype == "f32" else "bf16 storage, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {part.n_loc} local + {part.n_halo} halo vertices, {part.nnz} edges, "
                               f"{cfg.kind} dims {cfg.dims}, GPU tier {dp.cache.cap_gpu if dp.cache else 0} halo rows",
                   "orders": ["agg_first" if o == 1 else "xform_first" for o in res_orders],
                   "f32_product": args.f32_product,
                   "spmm_launches_per_epoch": len(launches), "loss": loss, "vertex_order": args.reorder,
                   "host_tier": {0: "kernel reads pinned memory", 1: "DMA into a staging area, same epoch",
                                 2: "DMA into a staging area, one epoch ahead (pipelined)"}[dp.miss_mode] if dp.cache else None},
        "epoch_ms_device": stage.get("total_ms"),
        "epoch_ms_device_median": float(np.median(dev_epochs)), "epoch_ms_device_min": float(np.min(dev_epochs)),
        "stages_ms": {k: round(v, 4) for k, v in stage.items()},
        "aggregation_gedges_s_kernel_only": part.nnz * len(launches) / (spmm_ms * 1e-3) / 1e9 if spmm_ms else None,
        # pipelined mode: one launch per layer copies the GPU tier's rows and the staged host rows (read + written bytes)
        "gather": {"device_copy_GBps": copy_rate, "device_copy_frac_of_hbm_peak": copy_rate / HBM_PEAK_GBPS if copy_rate else None,
                   "hit_bytes": hit_bytes,
                   "miss_host_link_GBps": miss_bytes / (miss_ms * 1e-3) / 1e9 if miss_ms else None,
                   "miss_bytes": miss_bytes},
        "gemm": gemm_report(cfg, part, res_orders, kernels, args.f32_product),
        "kernels": kernels[:12 if headline else 6],
        "roofline": {"kernel": f"{dom['kind']} layer {dom['layer']} F={F}", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "traffic_source": traffic_src,
                     "traffic_frac_of_hbm_peak": traffic / (dom["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS if traffic else None,
                     "algorithmic_bytes": bmin, "gathered_bytes_no_reuse": bgather, "ms": dom["ms"],
                     "gedges_s": part.nnz / (dom["ms"] * 1e-3) / 1e9,
                     "note": "achieved = algorithmic bytes (every index, needed source row and output row once) / launch time"},
        # the roof the same launch actually sits on: what the CUs request (every entry's feature bytes) against the rate the
        # serving memory level delivers for scattered 128-byte lines, measured in this run (gather_peaks_GBps)
        "roofline_gather": {"kernel": f"{dom['kind']} layer {dom['layer']} F={F}",
                            "bound": {"l2_2MB": "l2", "infinity_cache_128MB": "infinity cache", "hbm_2GB": "hbm, scattered lines"}[level],
                            "achieved": gather_rate, "peak": peaks[level], "unit": "GB/s", "frac": gather_rate / peaks[level],
                            "peak_is": f"capgnn_gather_peak on a {level.split('_')[-1]} table, this run",
                            "frac_of_published_l2_peak": gather_rate / L2_PEAK_GBPS,
                            "kernel_form": "column-blocked (4 MB source panels)" if blocked else "one wave per row"},
    }
    if headline:
        out["env"] = {"device": torch.cuda.get_device_name(0), "hip": torch.version.hip, "torch": torch.__version__,
                      "host_cores": os.cpu_count()}
        out["f32_product_max_rel_err"] = f32_product_check(cfg)
    # the same epoch replayed as a HIP graph (one launch per epoch): what a launch-bound partition gains, and the launch
    # gaps of the others.  With a host tier the two-stream epoch is recorded: every replay consumes the rows the run
    # before it prefetched and prefetches the next ones (the eager epochs above have primed it)
    host_tier = bool(dp.cache and dp.cache.cap_gpu < part.n_halo)
    if not args.plain and (headline or not host_tier):
        eg, loss_dev = dp.capture_epoch(two_streams=host_tier)
        for _ in range(args.warmup):
            eg.launch(dp.stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            eg.launch(dp.stream)
        torch.cuda.synchronize()
        gms = (time.perf_counter() - t0) * 1e3 / args.steps
        out["graph_replay"] = {"ms_per_step": gms, "gedges_s": edges_per_epoch / (gms * 1e-3) / 1e9, "loss": float(loss_dev.cpu()[0]),
                               "streams_recorded": 2 if host_tier else 1,
                               "note": "capgnn_epoch_graph_launch: the same kernels in the same order, one launch per epoch; wall time"
                                       + ("; the runtime runs the recorded host-tier copies and the kernels one after the other, so the "
                                          "eager two-stream epoch, whose copies overlap the kernels, stays the faster path" if host_tier else "")}
        eg.close()
        out["eager"] = {"ms_per_step": ms_per_step, "gedges_s": out["value"]}
        if gms < ms_per_step:
            # the faster of the library's two ways to run the same epoch is the configuration's figure; the per-kernel
            # times, stages and rooflines of this record come from the eager run (a graph has no events inside)
            out["ms_per_step"], out["value"] = gms, edges_per_epoch / (gms * 1e-3) / 1e9
            out["config"]["timed_path"] = "HIP graph replay (capgnn_epoch_graph_launch)"
        else:
            out["config"]["timed_path"] = "eager (capgnn_epoch)"
    # Alg. 1 on this GPU: how many halo rows its memory would cache
    if dp.cache and dp.cache.cap_gpu < part.n_halo:
        free_b, total_b = torch.cuda.mem_get_info()
        cap = B.cal_capacity(total_b / 2 ** 30, 4096.0, cfg.dims[:dp.L], part.n_halo, es)
        out["alg1_capacity"] = {"gpu_memory_GiB": total_b / 2 ** 30, "reserved_MB": 4096, "rows": cap, "halo_rows": part.n_halo,
                                "note": "Alg. 1 (cal_capacity) with this GPU's memory"}
        if cap >= part.n_halo and not headline and not args.plain:
            # the same workload with the GPU tier Alg. 1 grants here: every halo row is a hit, no host-link traffic
            dp.close()
            del dp
            torch.cuda.empty_cache()
            import copy
            prob_all = copy.copy(prob)
            prob_all.cap_gpu = part.n_halo
            dp = H.DeviceProblem(prob_all, orders=orders, miss_mode=miss_mode, f32_product=f32p)
            ms2, _, stage2, _, _ = timed(dp, args.steps)
            out["alg1_capacity"].update({"epoch_ms_wall": ms2, "epoch_ms_device": stage2.get("total_ms"),
                                         "gedges_s": edges_per_epoch / (ms2 * 1e-3) / 1e9})
    dp.close()
    del dp
    torch.cuda.empty_cache()
    if headline and part.n_halo and len(cfg.dims) > 2 and not args.plain:
        # JACA refreshes the cached hidden-layer halo rows as training goes on (section "Vertex Importance and Vertex
        # Update"): the same epoch with every halo row of every hidden-layer table rewritten before each epoch
        upd = {}
        for mode, mname in ((B.MISS_PIPELINED, "pipelined"), (B.MISS_STAGED, "staged")):
            dpu = H.DeviceProblem(prob, orders=orders, miss_mode=mode, f32_product=f32p)
            ids = torch.arange(part.n_halo, dtype=torch.int64, device="cuda")
            rows = {l: H.np_to_dev(prob.tables[l]) for l in range(1, dpu.L)}
            torch.cuda.synchronize()

            def step(it):
                for l, r in rows.items():
                    B.cache_update(dpu.cache, l, ids, part.n_halo, r, r.shape[1], it, stream=dpu.stream)
                dpu.run_epoch()

            for it in range(args.warmup):
                step(it)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for it in range(args.steps):
                step(args.warmup + it)
            torch.cuda.synchronize()
            upd[mname + "_ms"] = (time.perf_counter() - t0) * 1e3 / args.steps
            dpu.close()
            del dpu, rows
            torch.cuda.empty_cache()
        upd["rows_rewritten_per_epoch"] = part.n_halo * (len(cfg.dims) - 2)
        upd["note"] = ("update + epoch, wall; in pipelined mode the prefetched copy of the host tier is patched by the update, "
                       "not fetched again")
        out["epoch_with_vertex_update"] = upd
    if args.cpu_scale is None or args.cpu_scale > 0:
        scale = args.cpu_scale
        if scale is None or scale >= 1.0:
            out["cpu_baseline"] = cpu_baseline(prob, n_agg)
        else:
            sprob = H.make_problem(cfg.scaled(scale))
            out["cpu_baseline"] = cpu_baseline(sprob, n_agg, sample=f"{cfg.name} at {scale:g} of its vertices and edges "
                                               f"({sprob.part.n_loc} local, {sprob.part.n_halo} halo, {sprob.part.nnz} edges; same average degree and widths), one full fp64 oracle epoch")
        if name in ("C1", "C2", "C3"):
            # the single-thread leg, on a bounded sample of the same shape (the whole of C1)
            s1 = 1.0 if name == "C1" else 0.1
            sprob = prob if s1 >= 1.0 else H.make_problem(cfg.scaled(s1))
            out["cpu_baseline_1_thread"] = cpu_baseline(
                sprob, n_agg, threads=1,
                sample=None if s1 >= 1.0 else f"{cfg.name} at {s1:g} of its vertices and edges ({sprob.part.n_loc} local, "
                                              f"{sprob.part.n_halo} halo, {sprob.part.nnz} edges; same average degree and widths), one full fp64 oracle epoch")
    return out


if __name__ == "__main__":
    main()
