#!/usr/bin/env python3
"""Benchmark of the PowerSGD+ compressor hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic gradients:
psgd_compress (or psgd_compress_refresh when step % tau == 0, Algorithm 2) followed by
psgd_decompress.  Inputs are resident in HBM before the timed region; three gradient sets are
rotated so that a step never finds its gradients in the 256 MB memory-side cache.

The headline workload is the largest single-GPU configuration: the 7B-shaped sweep (224 matrices,
bf16 gradients, r = 64, one worker = one GPU's share of a data-parallel job), run with the deferred
residual (psgd_options.lazy_residual; `--plain` runs the immediate form, which the line reports
beside it either way).  The smaller configurations are run after it and reported as sub-objects
(`--only` skips them).

Prints ONE JSON line (see the fields below).  `value` is gigabytes of gradient compressed per
second: N * sum_l rows_l*cols_l * sizeof(G) * steps / time.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5a", "c5a_bf16"])
    ap.add_argument("--only", action="store_true", help="the named workload only, no sub-objects for the others")
    ap.add_argument("--plain", action="store_true",
                    help="time the immediate residual (E_{t+1} written by a pass of its own) instead of the deferred one")
    ap.add_argument("--sets", type=int, default=3, help="rotating gradient sets")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decompress", action="store_true")
    ap.add_argument("--rank", type=int, default=0, help="override the compression rank (sweep r = 8..64)")
    ap.add_argument("--lazy", action="store_true", help="(default now; kept for old command lines)")
    ap.add_argument("--no-qr", action="store_true",
                    help="signal factors = scaled Gaussian columns (orthonormal up to O(sqrt(k/rows))) instead of a "
                         "QR: keeps rocsolver out of counter-collection runs")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the library's plain copy kernel on 256 MiB three times (counter calibration)")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark, run the plain streaming kernels of libpsgd_ceilings.so (the access "
                         "patterns of the passes without the arithmetic) and print what HBM gives them, one JSON line")
    return ap.parse_args()


def run_ceilings():
    """Measured HBM ceilings for the access patterns of the three passes (GB/s), HIP-event timed."""
    import ctypes as C
    import torch
    torch.cuda.set_device(0)
    path = os.path.join(ROOT, "paper_2509_11254_amd", "libpsgd_ceilings.so")
    if not os.path.exists(path):
        raise FileNotFoundError(path + " is missing: run `python -m paper_2509_11254_amd.build`")
    lib = C.CDLL(path)
    vp = C.c_void_p
    lib.ceil_flat_read.argtypes = [vp, C.c_int, vp, C.c_size_t, vp]
    lib.ceil_flat_copy.argtypes = [vp, C.c_int, vp, vp, C.c_size_t]
    lib.ceil_flat_rmw.argtypes = [vp, C.c_int, vp, C.c_size_t]
    lib.ceil_flat_write.argtypes = [vp, C.c_int, vp, C.c_size_t]
    lib.ceil_form.argtypes = [vp, C.c_int, C.POINTER(vp), C.c_int, vp, vp, C.c_size_t]
    lib.ceil_tile_read.argtypes = [vp, C.c_int, vp, C.c_int, C.c_int, C.c_int, vp]
    lib.ceil_flat_read_nt.argtypes = [vp, C.c_int, vp, C.c_size_t, vp]
    lib.ceil_flat_rmw_nt.argtypes = [vp, C.c_int, vp, C.c_size_t]
    lib.ceil_tile_write.argtypes = [vp, C.c_int, vp, C.c_int, C.c_int, C.c_int]
    lib.ceil_form_tile.argtypes = [vp, C.c_int, vp, vp, C.c_int, C.c_int, C.c_int]
    lib.ceil_walk_32x256.argtypes = [vp, C.c_int, vp, vp, C.c_int, C.c_int, C.c_int, vp]
    st = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(16, device="cuda")

    def timed(fn, reps=10):
        for i in range(3):
            rc = fn(i)
            if rc != 0:
                raise RuntimeError("ceilings kernel failed: HIP error %d" % rc)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(reps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    out = {}
    n = 512 * 1024 * 1024                                   # 2 GiB of fp32
    big = torch.randn(n, device="cuda")
    big2 = torch.empty_like(big)
    for grid in (2048, 4096, 8192):
        ms = timed(lambda i: lib.ceil_flat_read(st, grid, big.data_ptr(), n, sink.data_ptr()))
        out["flat_read_2GiB_grid%d" % grid] = n * 4 / ms / 1e6
        ms = timed(lambda i: lib.ceil_flat_copy(st, grid, big.data_ptr(), big2.data_ptr(), n))
        out["flat_copy_2GiB_grid%d" % grid] = 2 * n * 4 / ms / 1e6
        ms = timed(lambda i: lib.ceil_flat_write(st, grid, big2.data_ptr(), n))
        out["flat_write_2GiB_grid%d" % grid] = n * 4 / ms / 1e6
        ms = timed(lambda i: lib.ceil_flat_rmw(st, grid, big2.data_ptr(), n))
        out["flat_rmw_in_place_2GiB_grid%d" % grid] = 2 * n * 4 / ms / 1e6
        ms = timed(lambda i: lib.ceil_flat_read_nt(st, grid, big.data_ptr(), n, sink.data_ptr()))
        out["flat_read_nontemporal_2GiB_grid%d" % grid] = n * 4 / ms / 1e6
        ms = timed(lambda i: lib.ceil_flat_rmw_nt(st, grid, big2.data_ptr(), n))
        out["flat_rmw_in_place_nontemporal_x4_2GiB_grid%d" % grid] = 2 * n * 4 / ms / 1e6
    del big, big2
    # pass 1 of config 2 without the product: 8 fp32 arrays of 4096^2 + E -> M, three rotating sets
    m = 4096 * 4096
    sets = [[torch.randn(m, device="cuda") for _ in range(8)] for _ in range(3)]
    e = torch.randn(m, device="cuda")
    o = torch.empty(m, device="cuda")
    for grid in (1024, 2048, 4096):
        def f(i):
            tab = (vp * 8)(*[t.data_ptr() for t in sets[i % 3]])
            return lib.ceil_form(st, grid, tab, 8, e.data_ptr(), o.data_ptr(), m)
        out["form_8xf32_plus_E_store_4096sq_grid%d" % grid] = m * 40 / timed(f, 20) / 1e6
    del sets
    # tile-pattern reads of 96 matrices of 4096 x 4096 fp32 (6.4 GB), two workgroups per CU
    mats = [torch.randn(4096, 4096, device="cuda") for _ in range(96)]
    tab = torch.tensor([x.data_ptr() for x in mats], dtype=torch.int64, device="cuda")
    for colmode, name in ((0, "tile_read_rowmode_128rows_x_256B"), (1, "tile_read_colmode_64rows_x_512B")):
        ms = timed(lambda i: lib.ceil_tile_read(st, colmode, tab.data_ptr(), len(mats), 4096, 4096, sink.data_ptr()), 5)
        out[name] = len(mats) * 4096 * 4096 * 4 / ms / 1e6
    for pat, name in ((0, "tile_write_128x128_accumulator_layout"), (1, "tile_write_64x256_1KB_per_wave_store"),
                      (2, "tile_write_128x256_accumulator_layout_8_columns_per_lane")):
        ms = timed(lambda i: lib.ceil_tile_write(st, pat, tab.data_ptr(), len(mats), 4096, 4096), 5)
        out[name] = len(mats) * 4096 * 4096 * 4 / ms / 1e6
    gmats = [torch.randn(4096, 4096, device="cuda").bfloat16() for _ in range(48)]
    gtab = torch.tensor([x.data_ptr() for x in gmats], dtype=torch.int64, device="cuda")
    for rot, name in ((0, "form_tile_bf16_plus_E_in_place_rowmode_in_step"), (1, "form_tile_bf16_plus_E_in_place_rowmode_rotated")):
        ms = timed(lambda i: lib.ceil_form_tile(st, rot, gtab.data_ptr(), tab.data_ptr(), len(gmats), 4096, 4096), 5)
        out[name] = len(gmats) * 4096 * 4096 * 10 / ms / 1e6
    for which, name, bpe in ((0, "walk_32x256_bf16_plus_E_in_place_rotated", 10), (1, "walk_32x256_bf16_plus_E_in_place_rotated_nt_store", 10),
                             (2, "walk_256cols_down_32rows_read_only", 4), (3, "walk_256cols_down_32rows_read_only_2_in_flight", 4)):
        ms = timed(lambda i: lib.ceil_walk_32x256(st, which, gtab.data_ptr(), tab.data_ptr(), len(gmats), 4096, 4096, sink.data_ptr()), 5)
        out[name] = len(gmats) * 4096 * 4096 * bpe / ms / 1e6
    print(json.dumps({"metric": "measured HBM ceilings of plain streaming kernels", "unit": "GB/s",
                      "peak_nominal": HBM_PEAK_GBPS, "values": {k: round(v, 1) for k, v in out.items()}}))


def make_workload(name, rank):
    from paper_2509_11254_amd import synth
    wl = {"c1": synth.config1, "c2": synth.config2, "c3": synth.config3, "c4": synth.config4,
          "c5a": synth.config5a, "c5a_bf16": lambda: synth.config5a(synth.BF16)}[name]()
    if rank > 0:
        wl.r = rank
    return wl


def host_info():
    model = None
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"nproc": os.cpu_count(), "cpu_model": model}


def cpu_baseline(wl, sets, E, Q, torch, seconds=12.0):
    """The fp64 NumPy oracle, as it stands, on a bounded sample of the same workload: SSP-Comp steps on the first layer
    of each distinct shape, round after round with the oracle's own E and Q carried along, until `seconds` are used."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import psgd_oracle as orc
    seen, sample = set(), []
    for l, spec in enumerate(wl.layers):
        if (spec.rows, spec.cols) not in seen:
            seen.add((spec.rows, spec.cols))
            sample.append(l)
    state = {}
    for l in sample:
        spec = wl.layers[l]
        g = [x.float().cpu().numpy().astype(np.float64) for x in sets[0][l]]
        e = [E[l].cpu().numpy().astype(np.float64)] * wl.n_workers
        if spec.transposed:
            g = [x.T for x in g]
            e = [x.T for x in e]
        state[l] = (g, e, Q[l].cpu().numpy().astype(np.float64))
    t_total, bytes_total, rounds = 0.0, 0.0, 0
    while t_total < seconds:
        for l in sample:
            spec = wl.layers[l]
            g, e, q = state[l]
            t0 = time.perf_counter()
            out = orc.compress_step(1, None, wl.r, q, g, e)
            t_total += time.perf_counter() - t0
            state[l] = (g, out.e_next, out.comp.q)
            bytes_total += spec.rows * spec.cols * wl.n_workers * (2 if wl.grad_dtype == "bf16" else 4)
        rounds += 1
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    out = {"value": bytes_total / t_total / 1e9, "unit": "GB/s", "cores": int(threads), "kind": "oracle",
           "sample": "%d SSP-Comp steps (all %d workers, fp64 NumPy) on each of the layers %s of %s, one per distinct "
                     "shape: %.1f s; the rate of the whole batch is this one extrapolated (same shapes)" % (
                         rounds, wl.n_workers, [wl.layers[l].name or l for l in sample], wl.name, t_total)}
    out.update(host_info())
    return out


def read_traffic(tag):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary of this workload, if there
    is one (the counters are collected in a run of their own, not in this one)."""
    path = os.path.join(ROOT, "profiles", "sweep1_%s_pmc.txt" % tag)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1]), "profiles/sweep1_%s_pmc.txt" % tag
    except OSError:
        pass
    return None, None


def run_c5b(torch):
    """Config 5b, a demonstration rather than a rate: the least-squares problem (N = 16, A_i 512 x 256, X 256 x 128,
    r = 4) run for 2000 steps as PowerSGD and as PowerSGD+ (tau = 10), every compressor and optimizer step through the
    library; reported: the gradient norms at the start and at the end, and the wall time per step."""
    from paper_2509_11254_amd import demo_least_squares, synth
    problem = synth.least_squares_problem(steps=2000)
    res = {"workload": "c5b_least_squares_n16_512x256_x256x128_r4", "steps": 2000, "tau": problem.tau, "mu": problem.mu,
           "sigma": problem.sigma, "eta_scale": problem.eta_scale}
    for tag, tau in (("powersgd", None), ("powersgd_plus", problem.tau)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        hist = demo_least_squares.run(problem, tau, 2000, record_every=500)
        dt = time.perf_counter() - t0
        res["grad_norm_%s" % tag] = hist
        res["final_grad_norm_%s" % tag] = hist[-1]
        res["wall_ms_per_step_%s" % tag] = 1e3 * dt / 2000
    return res


def run_workload(name, args, primary):
    """Times one workload; returns (the fields of its bench line, objects the CPU baseline needs)."""
    import torch
    from paper_2509_11254_amd import psgd, synth

    wl = make_workload(name, args.rank if primary else 0)
    gd = psgd.PSGD_BF16 if wl.grad_dtype == synth.BF16 else psgd.PSGD_F32
    sg = 2 if wl.grad_dtype == synth.BF16 else 4
    layers = [(s.rows, s.cols, wl.r, gd) for s in wl.layers]
    # the deferred residual pays where a step is bound by the bytes of the streaming passes (the batched bf16 sets);
    # on a single small matrix the immediate form is the faster one
    lazy = (not args.plain) and name in ("c3", "c4")
    steps = args.steps if primary else max(5, min(args.steps, 20))
    warmup = args.warmup if primary else max(2, min(args.warmup, 5))
    # (q_resident: this loop never writes the Q buffers between the library's calls)
    comp = psgd.Compressor(layers, wl.n_workers, lazy_residual=lazy, q_resident=True)
    comp_other = psgd.Compressor(layers, wl.n_workers, lazy_residual=not lazy, q_resident=True)
    planes = 3 if wl.grad_dtype == synth.F32 else 2
    sets, E, Q, P, OUT = synth.device_gradients(wl, args.sets, torch, args.no_qr)
    elems = sum(s.rows * s.cols for s in wl.layers)
    grad_bytes = elems * wl.n_workers * sg
    tau = wl.tau

    def step(c, t):
        G = sets[t % args.sets]
        if t % tau == 0:
            c.compress_refresh(G, E, Q, P)
        else:
            c.compress(G, E, Q, P)
        if not args.no_decompress:
            # Delta_hat of the factors this step's compress call produced: the library reads its own operand copies
            # of them (P = Q = NULL in the ABI) instead of packing the P and Q buffers again
            c.decompress(None, None, OUT)

    if args.calibrate_copy and primary:
        a = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            psgd.copy_bytes(b, a, a.numel())
        torch.cuda.synchronize()
        del a, b
    t = 0
    for _ in range(warmup):
        step(comp, t)
        t += 1
    torch.cuda.synchronize()
    # only the dominant kernel (pass 1) is timed inside the measured region, and only on every fourth step: a timed
    # launch costs two event records, about 6 microseconds of idle GPU each (3 % of a config-2 step); the other
    # kernels are timed in the breakdown loop below
    comp.profile_enable(steps + 64)
    n_refresh = sum(1 for k in range(t, t + steps) if k % tau == 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        comp.profile_select(["sweep1"] if k % 4 == 0 else [])
        step(comp, t)
        t += 1
    if lazy:
        comp.flush_residual(E)          # E_{t+1} of the last step: the deferred form owes it until here
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = comp.profile_read()
    comp.profile_enable(0)

    # ---- breakdown outside the timed region
    def timed(fn, n):
        torch.cuda.synchronize()
        a = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - a) / n * 1e3

    n_b = max(3, min(20, steps))

    def ssp_loop(c, is_lazy):
        def body(_):
            for i in range(n_b):
                c.compress(sets[i % args.sets], E, Q, P)
            if is_lazy:
                c.flush_residual(E)
        return body
    def kernel_times(c, is_lazy):
        c.profile_select(list(psgd.PROF_TAGS))
        c.profile_enable(4 * n_b + 8)
        for i in range(n_b):
            c.compress(sets[i % args.sets], E, Q, P)
        if is_lazy:
            c.flush_residual(E)
        torch.cuda.synchronize()
        d = c.profile_read()
        c.profile_enable(0)
        return d
    # (each context in one stretch: with q_resident the Q buffers must not be written by anyone else in between)
    ssp_ms = timed(ssp_loop(comp, lazy), 1) / n_b
    per_kernel = {"lazy" if lazy else "plain": kernel_times(comp, lazy)}
    for i in range(2):
        comp_other.compress(sets[i % args.sets], E, Q, P)
    if not lazy:
        comp_other.flush_residual(E)
    ssp_other_ms = timed(ssp_loop(comp_other, not lazy), 1) / n_b
    per_kernel["plain" if lazy else "lazy"] = kernel_times(comp_other, not lazy)
    ssp_lazy_ms, ssp_plain_ms = (ssp_ms, ssp_other_ms) if lazy else (ssp_other_ms, ssp_ms)
    comp_plain = comp_other if lazy else comp
    comp_plain.workspace_reset()
    extra = {}
    if primary:
        # the same step as the two halves a data-parallel job runs per worker (P averaged between them)
        def halves(i):
            comp_plain.compress_project(sets[i % args.sets], E, Q, P)
            comp_plain.compress_finish(E, Q, P)
        halves(0)
        extra["ssp_step_two_halves_ms"] = timed(halves, n_b)
        # the same step recorded into a HIP graph once and replayed (kernel launches only)
        comp_plain.compress(sets[0], E, Q, P)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            comp_plain.compress(sets[0], E, Q, P)
        gr.replay()
        extra["ssp_step_graph_replay_ms"] = timed(lambda i: gr.replay(), n_b)
        del gr
    # SVD-Comp steps, one call per synchronised interval as in a schedule with tau > 1 (the library looks at the
    # iteration bound it fetched behind the previous refresh only if that copy has arrived)
    n_r = max(2, min(4, n_b))
    for i in range(2):                                 # (a layer's first two refreshes on a workspace run the whole budget)
        comp_plain.compress_refresh(sets[i % args.sets], E, Q, P)
    st_next = [comp_plain.status(l) for l in range(len(wl.layers))]
    it_next = [s_.refresh_iters_next for s_ in st_next]
    refresh_ms = sum(timed(lambda i: comp_plain.compress_refresh(sets[i % args.sets], E, Q, P), 1) for _ in range(n_r)) / n_r
    # cheaper refresh (Remark 2): one subspace iteration from a random start = randomized range finder
    comp_rf = psgd.Compressor(layers, wl.n_workers, refresh_iters=1, refresh_warm_start=False, q_resident=True)
    comp_rf.compress_refresh(sets[0], E, Q, P)
    rangefinder_ms = sum(timed(lambda i: comp_rf.compress_refresh(sets[i % args.sets], E, Q, P), 1) for _ in range(n_r)) / n_r
    del comp_rf

    def k_of(st):
        k = st.refresh_iters_next
        return k if 0 < k <= 16 else (16 if k <= 0 else min(16, st.refresh_iters_no_gap))
    # The same step early in a run: E reset to zero, then refreshes with three SSP-Comp steps between them; the third
    # one (the first whose iteration count is the layer's own) is timed.  The refresh timed above meets the state
    # after this benchmark's long stretch of error feedback (||E|| of the order of ||M||, the spectrum flat at the
    # cut), where the count that keeps Eq. (6)'s error is the whole budget.
    for e_buf in E:
        e_buf.zero_()
    comp_plain.workspace_reset()
    for i in range(2):
        comp_plain.compress_refresh(sets[i % args.sets], E, Q, P)
        for j in range(3):
            comp_plain.compress(sets[(i + j + 1) % args.sets], E, Q, P)
    k_early = [k_of(comp_plain.status(l)) for l in range(len(wl.layers))]
    refresh_early_ms = timed(lambda i: comp_plain.compress_refresh(sets[2 % args.sets], E, Q, P), 1)
    # refresh arithmetic: block width b, k iterations of two products of 2 m n b flops each (+ the forming product)
    b_w = min(wl.r + max(8, wl.r // 4) + 7 & ~7, min(s.n for s in wl.layers))
    # iterations per layer as the device decides them: the count for the subspace if within the budget of 16, else
    # the count for the error
    k_layers = [k_of(s_) for s_ in st_next]
    k_run = sum(k_layers) / len(k_layers)
    refresh_flops = sum(4.0 * s.rows * s.cols * b_w * k for s, k in zip(wl.layers, k_layers))
    cp_w = (b_w + 31) // 32 * 32
    plane_products = 3 if planes == 2 else 6
    dec_ms = timed(lambda i: comp_plain.decompress(P, Q, OUT), n_b)
    comp_plain.compress(sets[0], E, Q, P)
    dec_last_ms = timed(lambda i: comp_plain.decompress(None, None, OUT), n_b)
    if primary:
        # decompress fused with the momentum-SGD update (Eq. (7c)): reads and writes m and X, 16 bytes per element
        MOM = [torch.zeros_like(e) for e in E]
        XW = [torch.randn_like(e) for e in E]
        msgd_ms = timed(lambda i: comp_plain.decompress_msgd(P, Q, MOM, XW, 0.9, 1e-3), n_b)
        extra.update(decompress_msgd_ms=msgd_ms, decompress_msgd_GBps=16.0 * elems / (msgd_ms * 1e-3) / 1e9,
                     decompress_msgd_frac_of_hbm_peak=16.0 * elems / (msgd_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS)
        # ... and with Adam (second moment as well: 24 bytes per element); the step counter advances as in a run
        M2 = [torch.zeros_like(e) for e in E]
        adam_ms = timed(lambda i: comp_plain.decompress_adam(P, Q, MOM, M2, XW, i + 1, 1e-3), n_b)
        extra.update(decompress_adam_ms=adam_ms, decompress_adam_GBps=24.0 * elems / (adam_ms * 1e-3) / 1e9,
                     decompress_adam_frac_of_hbm_peak=24.0 * elems / (adam_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS)
        del MOM, M2, XW

    # ---- roofline of the dominant kernel: the first streaming pass (reads N gradients + E, writes M; with the
    # deferred residual also the kept factors of the step before).  Event pairs recorded inside the timed region;
    # the SSP-only loop is the fallback when the timed region held no SSP step.
    mode = "lazy" if lazy else "plain"
    s1_ms, s1_n = prof["sweep1"] if prof["sweep1"][1] > 0 else per_kernel[mode]["sweep1"]
    per_launch_ms = s1_ms / max(1, s1_n)
    s1_bytes = comp.kernel_bytes("sweep1")
    achieved = s1_bytes / (per_launch_ms * 1e-3) / 1e9 if per_launch_ms > 0 else 0.0
    # (the counter files were taken on the default form of each workload: deferred residual where it applies)
    traffic, traffic_src = read_traffic(name) if lazy == (name in ("c3", "c4")) else (None, None)
    kernels = {}
    for tag, d in per_kernel.items():
        for kname, (ms, n) in d.items():
            if n > 0:
                kernels["%s_%s_ms" % (kname, tag)] = ms / n
    algo = comp.algorithmic_bytes
    out = {
        "metric": "compress GB/s of gradient",
        "value": grad_bytes * steps / elapsed / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": elapsed / steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        # elementwise arithmetic (error feedback, residual) in fp32; the three m*n*r contractions on the bf16 matrix
        # cores with operands split into `planes` bf16 planes and fp32 accumulation; r x r pieces in fp64
        "dtype": "f32" if planes == 3 else "bf16x2",
        "data": "synthetic",
        "config": dict(wl.describe(), refresh_steps_in_timed_region=n_refresh, gradient_sets=args.sets,
                       decompress_in_step=not args.no_decompress, deferred_residual=bool(lazy),
                       mfma_operand_planes=planes, error_buffer_dtype="f32",
                       factors_from_workspace=True),    # q_resident = 1, decompress with P = Q = NULL
        "roofline": {"bound": "hbm",
                     "kernel": "form_row_kernel / prod_kernel FORM (M = mean G + E formed and stored, P = M Q%s)" % (
                         "; the owed residual of the step before applied on the way in" if lazy else ""),
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_src,
                     "bytes_per_launch": s1_bytes, "ms_per_launch": per_launch_ms},
        "breakdown": dict(kernels, ssp_step_ms=ssp_ms, ssp_step_deferred_residual_ms=ssp_lazy_ms,
                          ssp_step_immediate_residual_ms=ssp_plain_ms,
                          ssp_step_algorithmic_GBps=algo / (ssp_ms * 1e-3) / 1e9,
                          ssp_step_frac_of_hbm_peak=algo / (ssp_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                          refresh_step_ms=refresh_ms, refresh_ms_per_layer=refresh_ms / len(wl.layers),
                          refresh_iterations_mean=k_run, refresh_iterations_max=max(k_layers), refresh_block_width=b_w,
                          refresh_early_in_a_run_step_ms=refresh_early_ms, refresh_early_in_a_run_ms_per_layer=refresh_early_ms / len(wl.layers),
                          refresh_early_in_a_run_iterations_mean=sum(k_early) / len(k_early),
                          refresh_iterations_for_the_subspace_min=min(it_next), refresh_iterations_for_the_subspace_max=max(it_next),
                          refresh_iterations_no_gap_max=max(s_.refresh_iters_no_gap for s_ in st_next),
                          refresh_algorithmic_TFLOPs=refresh_flops / (refresh_ms * 1e-3) / 1e12,
                          refresh_plane_product_TFLOPs=refresh_flops * plane_products * cp_w / b_w / (refresh_ms * 1e-3) / 1e12,
                          refresh_plane_product_frac_of_bf16_mfma_peak=refresh_flops * plane_products * cp_w / b_w / (refresh_ms * 1e-3) / 1e12 / 2500.0,
                          rangefinder_refresh_step_ms=rangefinder_ms,
                          rangefinder_refresh_ms_per_layer=rangefinder_ms / len(wl.layers),
                          decompress_ms=dec_ms, decompress_of_last_factors_ms=dec_last_ms,
                          decompress_GBps=4.0 * elems / (dec_last_ms * 1e-3) / 1e9, **extra),
    }
    return out, (wl, sets, E, Q)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if args.ceilings:
        run_ceilings()
        return
    import gc
    import torch
    torch.cuda.set_device(0)
    out, (wl, sets, E, Q) = run_workload(args.workload, args, True)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, sets, E, Q, torch)
    del wl, sets, E, Q
    if not args.only:
        others = {}
        for name in ("c2", "c3", "c5a", "c5a_bf16"):
            if name == args.workload:
                continue
            gc.collect()
            torch.cuda.empty_cache()
            sub, keep = run_workload(name, args, False)
            del keep
            others[name] = {k: sub[k] for k in ("value", "unit", "steps", "ms_per_step", "dtype", "config", "roofline", "breakdown")}
        others["c5b"] = run_c5b(torch)
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
