#!/usr/bin/env python3
"""Benchmark of the fused SVD-factored gated MLP forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--repeats R] [--workload prefill|wide|mlp_small|decode|xuv]
                    [--r R] [--M M] [--fused] [--one-kernel-decode] [--sweep] [--shape d,r,n] [--roofs]
                    [--no-cpu-baseline] [--no-dense] [--no-decode] [--no-configs] [--no-roofs]

A step is one pass of the whole hot path (svdmlp_forward: rank-r strips, gate/up second stage with
the SiLU gate, down projection) over one batch of seeded synthetic input already resident in HBM.
Prints ONE JSON line.  `value` is TFLOP/s of the prefill workload (algorithmic FLOPs 6 M r (d + ffn)
divided by the step time); the same line also carries the other configurations (`configs`: the prefill
rank sweep, the wide layer, the 128-row layer and the decode shapes, each with its rate and fraction of
its roof), a dense bf16 MLP on the same GPU (third-party GEMMs through torch), the roofline of the
dominant kernel against the published and the measured peak, and the CPU oracle timed on the host cores.

Timing protocol: W untimed warm-up steps, then R (default 10) batches of exactly K steps, each batch
between two HIP events on the launch stream with a device synchronisation on both sides;
`ms_per_step` is the MEDIAN batch (per step), `ms_per_step_min` the fastest, `ms_per_step_first_batch`
the first one (what a single short batch straight after the warm-up reads while the clocks are still
settling: about 15 % slower at K = 20).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2510_25977_amd import binding as B  # noqa: E402
from paper_2510_25977_amd import costmodel as cm  # noqa: E402
from paper_2510_25977_amd import synth  # noqa: E402

METRIC = "SVD-MLP forward TFLOP/s (prefill) + GB/s (decode), % of roofline"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def measured_traffic(kernel, profile):
    """HBM-side bytes per launch of `kernel` from the rocprofv3 --pmc summary `profile` under profiles/ (FETCH_SIZE /
    WRITE_SIZE scaled by a copy of known size; the file says how): the line "  <kernel> ... read X MB  written Y MB"."""
    path = os.path.join(ROOT, "profiles", profile)
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"^\s*" + re.escape(kernel) + r"\S*\s.*?read\s+([0-9.]+) MB\s+written\s+([0-9.]+) MB", text, re.M)
    if not m:
        return None
    return {"read_MB": float(m.group(1)), "written_MB": float(m.group(2)), "source": "profiles/" + profile}


def time_batches(fn, steps, warmup, repeats=10):
    """W untimed warm-up steps, then `repeats` batches of exactly `steps` steps, each between two events on the current
    stream, with a synchronisation before and after.  Returns per-step milliseconds: median, min, first, all."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    per = []
    wall = []
    for _ in range(max(1, repeats)):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        wall.append((time.perf_counter() - t0) * 1e3 / steps)
        per.append(e0.elapsed_time(e1) / steps)
    return {"median": statistics.median(per), "min": min(per), "first": per[0], "all": per,
            "wall_median": statistics.median(wall), "repeats": len(per)}


def time_steps(fn, steps, warmup, repeats=3):
    t = time_batches(fn, steps, warmup, repeats)
    return t["median"], t["wall_median"]


def make_ctx(gi, dev, max_M, flags=0):
    f = {k: v.to(dev) for k, v in gi.factors().items()}
    return B.SvdMlp(max_M=max_M, flags=flags, keep_factors=False, **f)


def bench_forward(gi, dev, steps, warmup, profile=True, flags=0, repeats=10):
    """Time the forward of one context (time_batches); then once more with the library recording a HIP event before
    and after every kernel on the launch stream, which gives the per-kernel averages (the event packets between the
    kernels cost a few microseconds per launch, so that pass is slower; both step times are reported)."""
    dims = gi.dims
    mlp = make_ctx(gi, dev, dims["M"], flags=flags)
    X = gi.X.to(dev)
    Y = torch.empty_like(X)
    t = time_batches(lambda: mlp(X, Y), steps, warmup, repeats)
    kernels, ms_ev = {}, None
    if profile:
        n_ev = max(steps, 20)
        B.svdmlp_profile_begin(mlp.ctx, n_ev)
        ms_ev = time_batches(lambda: mlp(X, Y), n_ev, 0, 1)["median"]
        kernels, nf = B.svdmlp_profile_end(mlp.ctx)
    path = mlp.last_path
    mlp.close()
    return t, kernels, path, ms_ev


def bench_xuv(dev, M, steps, warmup, dense=True, shape=(8192, 4096, 16384)):
    """Stand-alone factored layer O = (X U) V at the shapes of the paper's kernel evaluation (Sec. 5.2:
    X[M,8192] U[8192,4096] V[4096,16384], M = 1K .. 32K; Sec. 5.3: X[4096,7168] U[7168,4096] V[4096,18432]);
    FLOPs 2 M r (d + n).  Beside it (third party, torch.matmul): the dense product X W that the factors replace,
    and the factored layer as two separate GEMMs with T = X U written out by one and read back by the other."""
    d, r, n = shape
    li = synth.make_linear_gaussian(M, d, n, r)
    mlp = B.SvdMlp(max_M=M, Ug=li.U.to(dev), Vg=li.V.to(dev), kind=B.SVDMLP_LINEAR, keep_factors=True)
    X = li.X.to(dev)
    O = torch.empty((M, n), dtype=torch.bfloat16, device=dev)
    ms, wall_ms = time_steps(lambda: mlp(X, O), steps, warmup)
    B.svdmlp_profile_begin(mlp.ctx, steps)
    ms_ev, _ = time_steps(lambda: mlp(X, O), steps, 0, repeats=1)
    kernels, _ = B.svdmlp_profile_end(mlp.ctx)
    path = mlp.last_path
    U, V = mlp.tensors[0], mlp.tensors[1]
    out = dict(M=M, d=d, r=r, n=n, ms=ms, wall_ms=wall_ms, ms_ev=ms_ev, kernels=kernels, path=path, flops=2 * M * r * (d + n))
    if dense:
        T = torch.empty((M, r), dtype=torch.bfloat16, device=dev)

        def two_gemms():
            torch.matmul(X, U, out=T)
            torch.matmul(T, V, out=O)

        ums, _ = time_steps(two_gemms, max(5, steps // 3), max(3, warmup // 2))
        out["unfused"] = dict(ms_per_step=ums, TFLOPs=2 * M * r * (d + n) / ums / 1e9,
                              provider="two torch.matmul calls, T through HBM (third-party GEMM)")
        W = torch.randn((d, n), dtype=torch.bfloat16, device=dev) * (d ** -0.5)
        dms, _ = time_steps(lambda: torch.matmul(X, W, out=O), max(5, steps // 3), max(3, warmup // 2))
        out["dense"] = dict(ms_per_step=dms, TFLOPs=2 * M * d * n / dms / 1e9, flops=2 * M * d * n,
                            provider="torch.matmul (third-party GEMM)")
        del W, T
        # Alg. 1 of the paper (fusion without the cached strip): every block of B_N output columns recomputes T = X U.
        # Built from this library's own kernels: one context whose V is a single block, run once per block.
        B_N = max(512, r)   # a context's rank may not exceed its output width
        nblk = (n + B_N - 1) // B_N
        blk = B.SvdMlp(max_M=M, Ug=U, Vg=V[:, :B_N].contiguous(), kind=B.SVDMLP_LINEAR, keep_factors=False)
        Ob = torch.empty((M, B_N), dtype=torch.bfloat16, device=dev)

        def recompute():
            for _ in range(nblk):
                blk(X, Ob)

        rms, _ = time_steps(recompute, max(3, steps // 10), 2)
        blk.close()
        out["naive_recompute"] = dict(ms_per_step=rms, blocks=nblk, B_N=B_N, flops=nblk * 2 * M * r * d + 2 * M * r * n,
                                      provider="this library's kernels, T recomputed for every block of B_N output columns "
                                               "(paper Alg. 1); timing only, every block multiplies by the same V block")
        # Block-size comparison (the paper's Table 3 varies B_M on Trainium): the same layer with both products on
        # 128 x 128 tiles; operand bytes a CU must pull in per MFMA halve from the 128- to the 256-row tile.
        small = B.SvdMlp(max_M=M, Ug=U, Vg=V, kind=B.SVDMLP_LINEAR, keep_factors=False, flags=B.FLAG_TILE_128)
        sms, _ = time_steps(lambda: small(X, O), max(5, steps // 3), max(3, warmup // 2))
        small.close()
        out["tile_rows"] = {"128": dict(ms_per_step=sms, operand_bytes_per_mfma=512),
                            "256 (planner's choice at this M)": dict(ms_per_step=ms, operand_bytes_per_mfma=256)}
    mlp.close()
    return out


def copy_calibration(dev, reps=5):
    """A plain device-to-device copy of known size (256 MiB read + 256 MiB written per launch)."""
    n = 256 << 20
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    return dict(bytes_read=n, bytes_written=n, launches=reps, kernel="torch Tensor.copy_ (uint8, 256 MiB)")


def rotating_contexts(gi, dev, max_M, nsets, flags=0):
    """`nsets` contexts over the same factor values at different addresses (one re-tiled copy each)."""
    f = {k: v.to(dev) for k, v in gi.factors().items()}
    ctxs = [B.SvdMlp(max_M=max_M, keep_factors=False, flags=flags, **f) for _ in range(nsets)]
    del f
    return ctxs


def bench_rotating(ctxs, gi, dev, M, steps, warmup, repeats, warm_too=True):
    """A weight-bandwidth-bound shape measured cold to the 256 MB memory-side cache: the forwards rotate through
    independent factor sets (one context each, more than 2x the cache in total), so every forward streams its
    weights from HBM.  The single-set time (warm in that cache) and its per-kernel split are reported beside it."""
    dims = gi.dims
    X = gi.X[:M].contiguous().to(dev)
    Y = torch.empty_like(X)
    n = [0]
    nsets = len(ctxs)

    def step():
        ctxs[n[0] % nsets](X, Y)
        n[0] += 1

    t = time_batches(step, steps, warmup, repeats)
    nbytes = cm.gated_mlp_bytes(M, dims["d"], dims["ffn"], dims["r"])
    out = dict(M=M, ms_per_step=t["median"], ms_per_step_min=t["min"], steps_per_batch=steps, repeats=t["repeats"],
               GBps=nbytes / t["median"] / 1e6, frac_of_hbm_peak=nbytes / t["median"] / 1e6 / PEAK_HBM_GBS, bytes=nbytes,
               factor_sets=nsets)
    if warm_too:
        tw = time_batches(lambda: ctxs[0](X, Y), steps, warmup, max(3, repeats // 2))
        # once more for the per-kernel split (the events cost a few microseconds per launch: not the pass that is timed)
        B.svdmlp_profile_begin(ctxs[0].ctx, steps)
        time_batches(lambda: ctxs[0](X, Y), steps, 0, 1)
        kernels, _ = B.svdmlp_profile_end(ctxs[0].ctx)
        out.update(warm_single_set_ms=tw["median"], warm_GBps=nbytes / tw["median"] / 1e6, warm_kernels_ms=kernels)
    return out


def bench_decode_rotating(dev, M, steps, warmup, nsets=12, flags=0, r=None, repeats=10):
    gi = synth.make_workload("decode", M=M, r=r)
    ctxs = rotating_contexts(gi, dev, max(16, M), nsets, flags)
    out = bench_rotating(ctxs, gi, dev, M, steps, warmup, repeats)
    for c in ctxs:
        c.close()
    return out


def measure_roofs(dev, quick=True):
    """What this machine delivers with kernels that do one thing only (svdmlp_roof_* of the library): a streaming
    read of a buffer larger than the memory-side cache (HBM), the same over a buffer that fits it, a register-resident
    MFMA issue loop, and a chain of four dependent launches of an empty kernel of the decode path's launch shape."""
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    s = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    out = {"compute_units": cus}
    big = torch.full(((1536 << 20),), 1, dtype=torch.uint8, device=dev)
    for name, nbytes in (("hbm_read", big.numel()), ("memory_side_cache_read", 96 << 20)):
        t = time_batches(lambda: B.svdmlp_roof_read(big.data_ptr(), nbytes, sink.data_ptr(), cus * 8, s),
                         4 if nbytes > (1 << 30) else 40, 2, 5)
        out[name] = {"bytes": nbytes, "ms": t["median"], "GBps": nbytes / t["median"] / 1e6, "GBps_best": nbytes / t["min"] / 1e6}
    del big
    iters = 8000
    t = time_batches(lambda: B.svdmlp_roof_mfma(iters, sink.data_ptr(), cus, s), 3, 2, 5)
    fl = cus * 8 * 4 * iters * 32768
    out["mfma_bf16"] = {"flop": fl, "ms": t["median"], "TFLOPs": fl / t["median"] / 1e9, "TFLOPs_best": fl / t["min"] / 1e9,
                        "note": "v_mfma_f32_32x32x16_bf16, constant register operands, two waves per SIMD"}
    # the same issue loop on other operand values: the matrix cores' clock is power-limited and their power follows the
    # number of operand bits that toggle, so zeros run at the full clock and data like real activations and weights slower
    for name, mode, note in (("mfma_bf16_zero_operands", B.ROOF_OPERANDS_ZERO, "all-zero register operands"),
                             ("mfma_bf16_random_operands", B.ROOF_OPERANDS_RANDOM,
                              "register operands uniform in (-1, 1), different in every lane: the roof of a product of real data")):
        t = time_batches(lambda: B.svdmlp_roof_mfma_operands(iters, mode, sink.data_ptr(), cus, s), 3, 2, 5)
        out[name] = {"flop": fl, "ms": t["median"], "TFLOPs": fl / t["median"] / 1e9, "TFLOPs_best": fl / t["min"] / 1e9, "note": note}

    # the phase skeleton of the 256 x 256 tile kernels on LDS-resident operands, nothing copied
    steps = 4000
    flp = cus * 8 * 16 * steps * 32768
    for name, mode in (("tile_skeleton_zero_operands", B.ROOF_OPERANDS_ZERO), ("tile_skeleton_random_operands", B.ROOF_OPERANDS_RANDOM)):
        t = time_batches(lambda: B.svdmlp_roof_pingpong(steps, mode, sink.data_ptr(), cus, s), 3, 2, 5)
        out[name] = {"flop": flp, "ms": t["median"], "TFLOPs": flp / t["median"] / 1e9, "TFLOPs_best": flp / t["min"] / 1e9,
                     "note": "eight waves in two alternating phases (12 LDS frag reads / 16 MFMAs), two barriers per step, no copies"}

    # SiLU on one wave of each SIMD under the MFMAs of the other: each half alone, then both
    mi, vi = 6000, 160     # 12000 MFMAs (384 k clocks of matrix core) and 5120 SiLU evaluations per lane
    co = {}
    for name, a, b in (("mfma_only", mi, 0), ("silu_only", 0, vi), ("both", mi, vi)):
        co[name + "_ms"] = time_batches(lambda: B.svdmlp_roof_coexec(a, b, sink.data_ptr(), cus, s), 3, 2, 5)["median"]
    co["overlap"] = (co["mfma_only_ms"] + co["silu_only_ms"] - co["both_ms"]) / min(co["mfma_only_ms"], co["silu_only_ms"])
    co["note"] = "overlap 1 = the shorter half hides completely under the longer one, 0 = they run one after the other"
    out["silu_under_partner_mfma"] = co

    # Dependent launches.  Enqueued from one library call (no interpreter between them) an empty kernel costs what the
    # HIP runtime needs to submit it; replayed from a recorded graph, what the device needs between two dependent kernels.
    n_chain = 400
    t = time_batches(lambda: B.svdmlp_roof_empty_chain(4 * n_chain, 256, 512, s), 3, 2, 5)
    out["four_dependent_empty_launches_us"] = {"median": t["median"] * 1e3 / n_chain, "min": t["min"] * 1e3 / n_chain,
                                               "shape": "256 workgroups x 512 threads, 1600 launches from one library call"}
    out["one_empty_launch_us"] = {"median": t["median"] * 1e3 / n_chain / 4, "min": t["min"] * 1e3 / n_chain / 4}
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        B.svdmlp_roof_empty_chain(4, 256, 512, side.cuda_stream)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            B.svdmlp_roof_empty_chain(4 * n_chain, 256, 512, side.cuda_stream)
    torch.cuda.synchronize()
    t = time_batches(graph.replay, 3, 2, 5)
    out["four_dependent_empty_launches_in_a_graph_us"] = {"median": t["median"] * 1e3 / n_chain, "min": t["min"] * 1e3 / n_chain}
    del graph

    # The floor of a forward that is four dependent launches over the decode shape's factors: four launches that only
    # stream the bytes of the four phases (8.4, 29.4, 14.7 and 4.2 MB), 24 such groups over distinct parts of a 1.5 GB
    # buffer so that every byte comes from HBM.
    big = torch.full(((1536 << 20),), 1, dtype=torch.uint8, device=dev)
    phases = [2 * 4096 * 1024, 2 * 2 * 512 * 14336, 2 * 14336 * 512, 2 * 512 * 4096]
    groups = 24

    # replayed from a recorded graph, so that the interpreter's call overhead (3 us per launch) is not what is timed
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            off = 0
            for _ in range(groups):
                for nbytes in phases:
                    n = nbytes // 32768 * 32768
                    B.svdmlp_roof_read(big.data_ptr() + off, n, sink.data_ptr(), cus * 4, side.cuda_stream)
                    off = (off + n + (1 << 20)) // 4096 * 4096
    torch.cuda.synchronize()
    t = time_batches(graph.replay, 3, 2, 5)
    out["decode_shape_four_read_only_launches_us"] = {
        "median": t["median"] * 1e3 / groups, "min": t["min"] * 1e3 / groups, "bytes": sum(phases),
        "note": "four dependent kernels that stream the phases' factor bytes from HBM and do nothing else (graph replay)"}
    del graph
    del big
    assert int(sink.abs().sum().item()) == 0   # the sinks are never written
    return out


def bench_dense(dev, M, d, ffn, steps, warmup):
    """Uncompressed bf16 gated MLP with torch.matmul (hipBLASLt / rocBLAS): third-party, for comparison only."""
    g = torch.Generator(device="cpu").manual_seed(synth.BASE_SEED)
    Wg = (torch.randn(d, ffn, generator=g) / d ** 0.5).to(torch.bfloat16).to(dev)
    Wu = (torch.randn(d, ffn, generator=g) / d ** 0.5).to(torch.bfloat16).to(dev)
    Wd = (torch.randn(ffn, d, generator=g) / ffn ** 0.5).to(torch.bfloat16).to(dev)
    X = torch.randn(M, d, generator=g).to(torch.bfloat16).to(dev)

    def step():
        return (torch.nn.functional.silu(X @ Wg) * (X @ Wu)) @ Wd

    ms, _ = time_steps(step, steps, warmup)
    fl = cm.dense_mlp_flops(M, d, ffn)
    return dict(ms_per_step=ms, TFLOPs=fl / ms / 1e9, flops=fl, provider="torch.matmul (third-party GEMM)")


def bench_unfused(gi, dev, steps, warmup):
    """The same factored MLP as six separate GEMMs plus one elementwise kernel (torch.matmul / torch ops: third party),
    every intermediate (T, G, P, H, Td) through HBM: the counterpart of the paper's unfused "XUV" baseline."""
    f = {k: v.to(dev) for k, v in gi.factors().items()}
    X = gi.X.to(dev)

    def step():
        G = (X @ f["Ug"]) @ f["Vg"]
        P = (X @ f["Uu"]) @ f["Vu"]
        return ((torch.nn.functional.silu(G) * P) @ f["Ud"]) @ f["Vd"]

    ms, _ = time_steps(step, steps, warmup)
    return dict(ms_per_step=ms, provider="six torch.matmul calls + silu * mul (third-party kernels)")


def _oracle_rows(oracle, X, a, rows):
    t0 = time.perf_counter()
    oracle.gated(X[:rows], **a)
    return time.perf_counter() - t0


def cpu_baseline(gi, target_seconds=10.0):
    """The fp64 oracle as it stands, timed on the host cores on a bounded sample of rows of the same workload: with all
    the threads its OpenMP row loop takes, and with one thread (omp_set_num_threads of the OpenMP runtime the oracle is
    linked against; the oracle itself is not touched)."""
    import ctypes
    import oracle
    a = {k: synth.to_f64(v) for k, v in gi.factors().items()}
    X = synth.to_f64(gi.X)
    dims = gi.dims
    fl_row = cm.gated_mlp_flops(1, dims["d"], dims["ffn"], dims["r"])
    cores = oracle.threads()

    def sample(threads, budget):
        probe = min(X.shape[0], max(threads, 8))
        dt = _oracle_rows(oracle, X, a, probe)
        rows = int(min(X.shape[0], max(probe, budget / max(dt / probe, 1e-9))))
        rows = max(threads, rows // threads * threads) if rows >= threads else rows
        rows = min(rows, X.shape[0])
        dt = _oracle_rows(oracle, X, a, rows)
        return rows, dt

    rows, dt = sample(cores, target_seconds)
    out = dict(value=fl_row * rows / dt / 1e12, unit="TFLOP/s", cores=cores, kind="oracle",
               sample=f"first {rows} of {X.shape[0]} rows of the same workload, fp64, {dt:.1f} s", seconds=dt)
    try:
        omp = ctypes.CDLL("libgomp.so.1")
        omp.omp_set_num_threads(1)
        try:
            if oracle.threads() == 1:
                rows1, dt1 = sample(1, target_seconds * 0.6)
                out["one_thread"] = dict(value=fl_row * rows1 / dt1 / 1e12, unit="TFLOP/s", cores=1,
                                         sample=f"first {rows1} rows, fp64, {dt1:.1f} s", seconds=dt1)
        finally:
            omp.omp_set_num_threads(cores)
    except OSError:
        pass
    return out


def bench_configs(dev, steps, warmup, repeats, skip=()):
    """The other configurations of the metric, each timed like the headline: the prefill shape at r = 256 and 1024,
    the wide layer, the 128-row layer (cold to the memory-side cache) and the decode shape at M = 1, 4, 16 (cold)."""
    rows = []
    for name, kw in (("prefill", dict(r=256)), ("prefill", dict(r=1024)), ("wide", {})):
        gi = synth.make_workload(name, **kw)
        dm = gi.dims
        t, kernels, path, _ = bench_forward(gi, dev, steps, warmup, profile=True, repeats=repeats)
        fl = cm.gated_mlp_flops(dm["M"], dm["d"], dm["ffn"], dm["r"])
        rows.append({"workload": f"{name}: d={dm['d']} ffn={dm['ffn']} r={dm['r']} M={dm['M']}", "bound": "mfma",
                     "ms_per_step": t["median"], "ms_per_step_min": t["min"], "TFLOPs": fl / t["median"] / 1e9,
                     "frac_of_bf16_mfma_peak": fl / t["median"] / 1e9 / PEAK_BF16_TFLOPS, "kernels_ms": kernels, "path": path})
        del gi
        torch.cuda.empty_cache()
    # 128-row layer: 15.7 MB of factors per set; 40 sets pass twice the memory-side cache
    gi = synth.make_workload("mlp_small")
    dm = gi.dims
    ctxs = rotating_contexts(gi, dev, dm["M"], 40)
    b = bench_rotating(ctxs, gi, dev, dm["M"], max(steps, 100), warmup, repeats)
    for c in ctxs:
        c.close()
    b.update(workload=f"mlp_small: d={dm['d']} ffn={dm['ffn']} r={dm['r']} M={dm['M']}", bound="hbm",
             TFLOPs=cm.gated_mlp_flops(dm["M"], dm["d"], dm["ffn"], dm["r"]) / b["ms_per_step"] / 1e9)
    rows.append(b)
    del ctxs
    torch.cuda.empty_cache()
    if "decode" not in skip:
        gi = synth.make_workload("decode", M=16)
        dm = gi.dims
        ctxs = rotating_contexts(gi, dev, 16, 12)
        for M in (1, 4, 16):
            b = bench_rotating(ctxs, gi, dev, M, max(steps, 200), warmup, repeats, warm_too=(M == 16))
            b.update(workload=f"decode: d={dm['d']} ffn={dm['ffn']} r={dm['r']} M={M}", bound="hbm")
            rows.append(b)
        for c in ctxs:
            c.close()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--repeats", type=int, default=10, help="timed batches of --steps steps; the median batch is reported")
    ap.add_argument("--roofs", action="store_true", help="only the roof microbenchmarks (one JSON line)")
    ap.add_argument("--no-roofs", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the other configurations (`configs` of the line)")
    ap.add_argument("--workload", default="prefill", choices=["prefill", "wide", "mlp_small", "decode", "xuv"])
    ap.add_argument("--r", type=int, default=None)
    ap.add_argument("--M", type=int, default=None)
    ap.add_argument("--shape", default=None, help="xuv workload: d,r,n (default 8192,4096,16384)")
    ap.add_argument("--sweep", action="store_true", help="xuv workload: M = 1K .. 32K, one table")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--one-kernel-decode", action="store_true", help="decode through the single persistent kernel")
    ap.add_argument("--fused", action="store_true",
                    help="tiled path with the gated activation kept in registers (one fused kernel) instead of staged")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (known size) so that a rocprofv3 --pmc run of this "
                         "command can scale FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (rows of X are independent, so the forward shards over rows with no "
              "communication and one GPU shows its share at the real shape); --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    B.lib()  # fail loudly if the HIP library is missing

    if args.workload == "xuv":
        shape = tuple(int(v) for v in args.shape.split(",")) if args.shape else (8192, 4096, 16384)
        if args.sweep:
            rows = []
            for Ms in (1024, 2048, 4096, 8192, 16384, 32768):
                x = bench_xuv(dev, Ms, max(5, args.steps // 3), max(3, args.warmup // 2), dense=not args.no_dense, shape=shape)
                row = {"M": Ms, "ms": x["ms"], "TFLOPs": x["flops"] / x["ms"] / 1e9, "kernels_ms": x["kernels"]}
                if "dense" in x:
                    row.update(dense_ms=x["dense"]["ms_per_step"], unfused_ms=x["unfused"]["ms_per_step"],
                               speedup_vs_dense=x["dense"]["ms_per_step"] / x["ms"],
                               speedup_vs_unfused=x["unfused"]["ms_per_step"] / x["ms"])
                rows.append(row)
                torch.cuda.empty_cache()
            avg = lambda key: sum(r_[key] for r_ in rows) / len(rows)
            out = {"metric": METRIC, "value": avg("TFLOPs"), "unit": "TFLOP/s", "n_gpus": 1, "steps": max(5, args.steps // 3),
                   "warmup": max(3, args.warmup // 2), "ms_per_step": avg("ms"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                   "dtype": "bf16", "data": "synthetic",
                   "config": {"workload": f"xuv sweep: (X U) V, X[M,{shape[0]}] U[{shape[0]},{shape[1]}] V[{shape[1]},{shape[2]}], "
                                          "M = 1K .. 32K; value = mean over M"},
                   "sweep": rows}
            if not args.no_dense:
                out["mean_speedup_vs_dense"] = avg("speedup_vs_dense")
                out["mean_speedup_vs_unfused"] = avg("speedup_vs_unfused")
            print(json.dumps(out))
            return
        x = bench_xuv(dev, args.M or 4096, args.steps, args.warmup, dense=not args.no_dense, shape=shape)
        k = x["kernels"]
        kfl = {"k_s1": 2 * x["M"] * x["d"] * x["r"], "k_in": 2 * x["M"] * x["d"] * x["r"], "k_out": 2 * x["M"] * x["r"] * x["n"],
               "k_s5": 2 * x["M"] * x["r"] * x["n"]}
        kfl.update({"k_stream_d1": kfl["k_s1"], "k_stream_d5": kfl["k_out"]})
        kname = max((n_ for n_ in k if n_ in kfl), key=k.get)
        out = {"metric": METRIC, "value": x["flops"] / x["ms"] / 1e9, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
               "warmup": args.warmup, "ms_per_step": x["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
               "dtype": "bf16", "data": "synthetic",
               "config": {"workload": f"xuv: factored layer (X U) V, X[{x['M']},{x['d']}] U[{x['d']},{x['r']}] V[{x['r']},{x['n']}]",
                          "path": " + ".join(k)},
               "flops_per_step": x["flops"], "frac_of_bf16_mfma_peak": x["flops"] / x["ms"] / 1e9 / PEAK_BF16_TFLOPS,
               "wall_ms_per_step": x["wall_ms"], "ms_per_step_with_kernel_events": x["ms_ev"], "kernels_ms": k,
               "roofline": {"bound": "mfma", "kernel": kname, "achieved": kfl[kname] / k[kname] / 1e9, "peak": PEAK_BF16_TFLOPS,
                            "unit": "TFLOP/s", "frac": kfl[kname] / k[kname] / 1e9 / PEAK_BF16_TFLOPS, "traffic": None,
                            "per_kernel_TFLOPs": {n_: kfl[n_] / v / 1e9 for n_, v in k.items() if v and n_ in kfl}}}
        if x["path"] == 7:   # up to 128 rows: weight-streaming kernels, bound by the bytes of the factors
            kb = {"k_stream_d1": 2 * x["d"] * x["r"], "k_stream_d5": 2 * x["r"] * x["n"]}
            nbytes = 2 * x["r"] * (x["d"] + x["n"]) + 2 * x["M"] * (x["d"] + x["n"])
            out["roofline"] = {"bound": "hbm", "kernel": kname, "achieved": kb[kname] / k[kname] / 1e6, "peak": PEAK_HBM_GBS,
                               "unit": "GB/s", "frac": kb[kname] / k[kname] / 1e6 / PEAK_HBM_GBS, "traffic": None,
                               "whole_forward_GBps": nbytes / x["ms"] / 1e6,
                               "note": "single factor set (warm in the memory-side cache if it fits); per-kernel time from HIP events"}
        if "dense" in x:
            out["dense_baseline"] = x["dense"]
            out["dense_baseline"]["speedup_of_factored"] = x["dense"]["ms_per_step"] / x["ms"]
            out["unfused_baseline"] = x["unfused"]
            out["unfused_baseline"]["speedup_of_this_library"] = x["unfused"]["ms_per_step"] / x["ms"]
            out["naive_recompute_baseline"] = x["naive_recompute"]
            out["naive_recompute_baseline"]["speedup_of_this_library"] = x["naive_recompute"]["ms_per_step"] / x["ms"]
            out["tile_rows"] = x["tile_rows"]
        print(json.dumps(out))
        return

    if args.roofs:
        print(json.dumps({"metric": "roof microbenchmarks", "peak_bf16_TFLOPs": PEAK_BF16_TFLOPS, "peak_hbm_GBps": PEAK_HBM_GBS,
                          "measured": measure_roofs(dev)}))
        return
    roofs = None if args.no_roofs else measure_roofs(dev)

    gi = synth.make_workload(args.workload, M=args.M, r=args.r)
    dims = gi.dims
    M, d, ffn, r = dims["M"], dims["d"], dims["ffn"], dims["r"]
    flops = cm.gated_mlp_flops(M, d, ffn, r)
    nbytes = cm.gated_mlp_bytes(M, d, ffn, r)

    dflags = B.FLAG_STREAM_ONE_KERNEL if args.one_kernel_decode else 0
    ms_ev = None
    if args.workload == "decode":
        dec = bench_decode_rotating(dev, M, max(args.steps, 200), args.warmup, flags=dflags, r=args.r, repeats=args.repeats)
        t = {"median": dec["ms_per_step"], "min": dec["ms_per_step_min"], "first": None, "wall_median": dec["ms_per_step"],
             "repeats": dec["repeats"]}
        kernels, path = dec["warm_kernels_ms"], (4 if dflags else 3)
    else:
        t, kernels, path, ms_ev = bench_forward(gi, dev, args.steps, args.warmup, flags=B.FLAG_TILED_FUSED if args.fused else 0,
                                                repeats=args.repeats)
        dec = None
    ms = t["median"]

    out = {
        "metric": METRIC,
        "value": flops / ms / 1e9 if args.workload != "decode" else nbytes / ms / 1e6,
        "unit": "TFLOP/s" if args.workload != "decode" else "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: gated SVD-MLP d={d} ffn={ffn} r={r} M={M}", "M": M, "d": d, "ffn": ffn,
                   "r": r, "path": {2: "mfma-tiled, fused", 3: "weight-streaming, 4 launches", 4: "weight-streaming, 1 launch",
                            5: "mfma-tiled, staged"}.get(path, str(path))},
        "timing": {"protocol": "warm-up, then `repeats` batches of `steps` forwards, each between two HIP events on the launch "
                               "stream with a synchronisation on both sides; ms_per_step = median batch / steps",
                   "repeats": t["repeats"], "ms_per_step_min": t["min"], "ms_per_step_first_batch": t["first"],
                   "value_at_min": (flops / t["min"] / 1e9 if args.workload != "decode" else nbytes / t["min"] / 1e6),
                   "value_first_batch": (flops / t["first"] / 1e9 if t["first"] else None)},
        "flops_per_step": flops, "algorithmic_bytes_per_step": nbytes,
        "frac_of_bf16_mfma_peak": flops / ms / 1e9 / PEAK_BF16_TFLOPS,
        "wall_ms_per_step": t["wall_median"],
        "kernels_ms": kernels,
    }
    if roofs is not None:
        out["measured_roofs"] = roofs
        if args.workload != "decode":
            out["frac_of_measured_mfma_peak"] = flops / ms / 1e9 / roofs["mfma_bf16"]["TFLOPs"]
            out["frac_of_measured_mfma_peak_random_operands"] = flops / ms / 1e9 / roofs["mfma_bf16_random_operands"]["TFLOPs"]
    if args.workload != "decode":
        out["ms_per_step_with_kernel_events"] = ms_ev

    # roofline of the dominant kernel (HIP-event average over a timed region of the same forwards)
    if path in (3, 4):   # weight-streaming path: HBM-bound
        rd = dims.get("r_down", r)
        kbytes = {"k_decode": nbytes,                                           # the whole forward is one launch
                  "k_stream_d1": 2 * (2 * d * r) + 2 * (M * d + M * 2 * r),     # Ug, Uu once; X in, T out
                  "k_stream_d2": 2 * (2 * r * ffn) + 2 * (M * 2 * r + M * ffn), # Vg, Vu once; T in, H out
                  "k_stream_d4": 2 * (ffn * rd) + 2 * (M * ffn + M * rd),       # Ud once; H in, Td out
                  "k_stream_d5": 2 * (rd * d) + 2 * (M * rd + M * d)}           # Vd once; Td in, Y out
        cand = {k_: v for k_, v in kernels.items() if k_ in kbytes}
        kname = "k_stream_d2" if args.workload == "decode" and "k_stream_d2" in cand else max(cand, key=cand.get)
        k_ms = kernels.get(kname, 0.0)
        k_bytes = kbytes[kname]
        traffic = measured_traffic(kname, "decode_m16_all_kernels.txt") if (M, d, ffn, r) == (16, 4096, 14336, 512) else None
        if traffic:
            traffic["algorithmic_MB"] = k_bytes / 1e6
        out["roofline"] = {"bound": "hbm", "kernel": kname, "achieved": k_bytes / k_ms / 1e6 if k_ms else None,
                           "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": k_bytes / k_ms / 1e6 / PEAK_HBM_GBS if k_ms else None,
                           "traffic": traffic,
                           "whole_forward_GBps": nbytes / ms / 1e6,
                           "note": "per-kernel time from HIP events" + (" of the warm single-set run" if args.workload == "decode" else "")}
        if roofs is not None and k_ms:
            out["roofline"]["measured_peak"] = roofs["hbm_read"]["GBps"]
            out["roofline"]["frac_of_measured_peak"] = k_bytes / k_ms / 1e6 / roofs["hbm_read"]["GBps"]
    else:
        rd = dims.get("r_down", r)
        kflops = {"k_s1": 2 * M * d * 2 * r, "k_in": 2 * M * d * 2 * r,   # X [Ug|Uu]
                  "k_fused": 4 * M * ffn * r + 2 * M * ffn * rd,   # gate + up second stage, down first stage
                  "k_gate_up": 4 * M * ffn * r,             # gate + up second stage
                  "k_down1": 2 * M * ffn * rd,              # down first stage
                  "k_s5": 2 * M * rd * d, "k_out": 2 * M * rd * d}
        # bytes each kernel has to move at least: its factor panels and rank-r strips once, X in, Y out; the ffn-wide
        # activation H and the split-K partial sums are the implementation's own traffic and count as nothing
        kalg = {"k_s1": 2 * (M * d + 2 * d * r), "k_in": 2 * (M * d + 2 * d * r),
                "k_gate_up": 2 * (M * 2 * r + 2 * r * ffn), "k_fused": 2 * (M * 2 * r + 2 * r * ffn + ffn * rd),
                "k_down1": 2 * (ffn * rd), "k_s5": 2 * (M * rd + rd * d + M * d), "k_out": 2 * (M * rd + rd * d + M * d)}
        cand = {k: v for k, v in kernels.items() if k in kflops}
        kname = max(cand, key=cand.get) if cand else "k_gate_up"   # the dominant kernel: the longest one
        k_ms = kernels.get(kname, 0.0)
        k_flops = kflops[kname]
        traffic = None
        if args.workload == "wide" and M == 2048 and not args.fused:
            traffic = measured_traffic(kname, "wide_all_kernels.txt")
        if args.workload == "prefill" and M == 4096 and not args.fused:
            traffic = measured_traffic(kname, f"prefill_r{r}_all_kernels.txt")
        if traffic:
            traffic["algorithmic_MB"] = kalg[kname] / 1e6
            traffic["times_algorithmic"] = (traffic["read_MB"] + traffic["written_MB"]) / (kalg[kname] / 1e6)
        out["roofline"] = {"bound": "mfma", "kernel": kname, "achieved": k_flops / k_ms / 1e9 if k_ms else None,
                           "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                           "frac": k_flops / k_ms / 1e9 / PEAK_BF16_TFLOPS if k_ms else None,
                           "traffic": traffic,
                           "per_kernel_TFLOPs": {k: kflops[k] / v / 1e9 for k, v in cand.items() if v}}
        if roofs is not None and k_ms:
            out["roofline"]["measured_peak"] = roofs["mfma_bf16"]["TFLOPs"]
            out["roofline"]["frac_of_measured_peak"] = k_flops / k_ms / 1e9 / roofs["mfma_bf16"]["TFLOPs"]
            out["roofline"]["measured_peak_random_operands"] = roofs["mfma_bf16_random_operands"]["TFLOPs"]
            out["roofline"]["frac_of_measured_peak_random_operands"] = k_flops / k_ms / 1e9 / roofs["mfma_bf16_random_operands"]["TFLOPs"]

    if dec is not None:
        out["decode"] = dec
    elif not args.no_decode and args.no_configs:
        out["decode"] = bench_decode_rotating(dev, 16, max(args.steps, 200), args.warmup, flags=dflags, repeats=args.repeats)
    if not args.no_configs and args.workload == "prefill" and args.r in (None, 512) and args.M in (None, 4096) and not args.fused:
        del gi
        torch.cuda.empty_cache()
        out["configs"] = bench_configs(dev, args.steps, args.warmup, max(3, args.repeats // 2),
                                       skip=("decode",) if args.no_decode else ())
        for row in out["configs"]:
            if row["workload"].startswith("decode") and row["M"] == 16:
                out["decode"] = row
        gi = synth.make_workload(args.workload, M=args.M, r=args.r)
    if "decode" in out and roofs is not None:
        out["decode"]["measured_hbm_peak_GBps"] = roofs["hbm_read"]["GBps"]
        out["decode"]["frac_of_measured_hbm_peak"] = out["decode"]["GBps"] / roofs["hbm_read"]["GBps"]
        # the floor of a forward that is four dependent launches: four kernels that only stream the phases' bytes
        floor_us = roofs["decode_shape_four_read_only_launches_us"]["median"]
        out["decode"]["floor_four_read_only_launches_us"] = floor_us
        out["decode"]["frac_of_hbm_peak_at_that_floor"] = out["decode"]["bytes"] / floor_us / 1e3 / PEAK_HBM_GBS
    if not args.no_dense and args.workload != "decode":
        out["dense_baseline"] = bench_dense(dev, M, d, ffn, max(5, args.steps // 3), max(3, args.warmup // 2))
        out["dense_baseline"]["speedup_of_factored"] = out["dense_baseline"]["ms_per_step"] / ms
        out["unfused_baseline"] = bench_unfused(gi, dev, max(5, args.steps // 3), max(3, args.warmup // 2))
        out["unfused_baseline"]["speedup_of_this_library"] = out["unfused_baseline"]["ms_per_step"] / ms
    out["paper_context"] = {"kernel_speedup_vs_nki": 1.35, "e2e_speedup": 1.21, "hardware": "AWS Trainium trn1",
                            "note": "paper figures for its own kernels; not the target"}
    if args.copy_calibration:
        out["copy_calibration"] = copy_calibration(dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(gi if args.workload != "decode" else synth.make_workload("decode", M=16))
    print(json.dumps(out))

if __name__ == "__main__":
    main()
