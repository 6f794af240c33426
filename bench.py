"""Benchmark of the batch-SOM epoch on one MI355X.

A step is one whole epoch (weight preparation, BMU search, exact re-decision of near-ties, per-BMU accumulation in a
second pass over the samples, neighbourhood update) over the full sample matrix, which is resident in HBM before the
timed region starts.  Prints ONE JSON line; `value` is presented samples per second.  The timed epochs ask the library
for no statistics (`som_epoch` with stats = NULL: the distances to the BMUs, which only the quantisation error needs, are
then not formed); `final_qe` comes from one separate search after the timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3      # MI355X dense float32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
METRIC = "samples/sec per batch-SOM epoch (BMU+update), 1024 nodes x 50 features"


def stream_bench(args, wl, X, W0, sig, som, pkg, torch) -> int:
    """Host-resident X through som_epoch_host; reports whole-epoch samples/s and the copy stream's GB/s."""
    Xh = X if args.stream in ("mmap", "file") else torch.from_numpy(X)
    if args.stream == "pinned":
        Xh = Xh.pin_memory()
    Wd = torch.from_numpy(W0).cuda()
    # what the host link itself sustains on this machine: plain copies of 1 GiB from pinned memory, best of three
    probe_h = torch.empty(1 << 28, dtype=torch.float32).pin_memory()
    probe_d = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    link_peak = 0.0
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        probe_d.copy_(probe_h, non_blocking=True)
        torch.cuda.synchronize()
        link_peak = max(link_peak, probe_h.numel() * 4 / (time.perf_counter() - t0) / 1e9)
    del probe_h, probe_d
    lattice = wl.topology in ("rect", "hex")
    if lattice:
        G = torch.from_numpy(pkg.topology.graph_distances(wl.topology, lattice=wl.lattice)).cuda()
    else:
        G = torch.empty((wl.k, wl.k), dtype=torch.float32, device="cuda")

    def epoch(e):
        if not lattice:                      # data-driven graph, rebuilt on the device from the current weights
            som.som_topology(Wd, wl.topology, G)
        if args.stream == "file":
            return som.som_epoch_file(Xh, 0, wl.n, wl.d, Wd, G, float(sig[min(e, len(sig) - 1)]), chunk_rows=args.chunk_rows)
        return som.som_epoch_host(Xh, Wd, G, float(sig[min(e, len(sig) - 1)]), chunk_rows=args.chunk_rows)

    for e in range(args.warmup):
        epoch(e)
    Wd.copy_(torch.from_numpy(W0))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    h2d_ms = 0.0
    for e in range(args.steps):
        st = epoch(e)
        h2d_ms += st.ms_h2d
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    nbytes = wl.n * wl.d * 4
    out = {
        "metric": METRIC + " (host-resident samples, chunked loading path)", "value": wl.n * args.steps / dt,
        "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / max(args.steps, 1), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16x2-split MFMA scores (float32 accumulate), f32 re-decision and distances, f64 sums and update" if args.search == "auto" and wl.d >= 4 and wl.k > 1
                 else "f32 MFMA scores, f32 re-decision and distances, f64 sums and update",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.k}-node {wl.topology} map, {wl.n} x {wl.d} float32 samples in {args.stream} "
                               f"host memory, chunks of {args.chunk_rows} rows", "samples": wl.n, "chunk_rows": args.chunk_rows},
        "host_link": {"bytes_per_epoch": nbytes, "copy_stream_GBps": nbytes * args.steps / (h2d_ms * 1e-3) / 1e9 if h2d_ms else None,
                      "end_to_end_GBps": nbytes * args.steps / dt / 1e9, "pinned_copy_peak_GBps": link_peak,
                      "end_to_end_frac_of_pinned_copy_peak": nbytes * args.steps / dt / 1e9 / link_peak,
                      "chunks_per_epoch": -(-wl.n // args.chunk_rows)},
    }
    som.close()
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=40,
                    help="untimed epochs first; the GPU needs about 20 ms of load after idling before its clocks "
                         "settle (the first launches of a run are up to 13 %% slower)")
    ap.add_argument("--workload", default="cfg1", choices=["cfg0", "cfg1", "cfg2", "cfg3", "cfg4", "scale"],
                    help="cfg1 is the headline workload; 'scale' is the default point of the paper's speed runs "
                         "(uniform data, Section 4.2.1), to be varied with --rows / --features / --grid")
    ap.add_argument("--features", type=int, default=None, help="override the feature count D (scale workload)")
    ap.add_argument("--grid", type=int, default=None, help="override the lattice side length, K = side^2 (scale workload)")
    ap.add_argument("--search", default="auto", choices=["auto", "float32"],
                    help="BMU score arithmetic: auto = bf16 parts on the bf16 matrix pipe for 4 <= D <= 64, float32 MFMA "
                         "otherwise; float32 = float32 MFMA for every shape (same results either way)")
    ap.add_argument("--topology", default=None, choices=["rect", "hex", "mst", "rng"],
                    help="override the workload's map topology (mst and rng are rebuilt on the device every epoch)")
    ap.add_argument("--stream", default=None, choices=["pinned", "pageable", "mmap", "file"],
                    help="keep X in host memory (or, mmap / file, in a file written to --mmap-dir first and then mapped, "
                         "or read with pread by som_epoch_file) and run the chunked loading path instead")
    ap.add_argument("--mmap-dir", default="/tmp", help="where --stream mmap writes its sample file (deleted afterwards)")
    ap.add_argument("--chunk-rows", type=int, default=4_000_000,
                    help="chunk length of the loading path in rows (cfg4 as configured: 64000000)")
    ap.add_argument("--rows", type=int, default=None, help="override the workload's sample count")
    ap.add_argument("--cpu-rows", type=int, default=1_000_000, help="rows of the workload the CPU oracle is timed on")
    ap.add_argument("--no-float32-reference", action="store_true",
                    help="skip the extra epochs that time the float32 search for the roofline's reference entry")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device-to-device copy of X (known size) for scaling hardware counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2604_26555_amd as pkg
    from synth import draw_initial_rows, draw_subset, linear_sigma, make_workload

    over = {}
    if args.features:
        over["d"] = args.features
    if args.grid:
        over.update(k=args.grid * args.grid, lattice=(args.grid, args.grid), sigma=(args.grid / 2.0, 1.0))
    if args.topology:
        over["topology"] = args.topology
    wl = make_workload(args.workload, n=args.rows, **over)
    t0 = time.time()
    mmap_path = None
    if args.stream == "mmap":
        # the paper's disk-backed regime (Section 3.3.2): the matrix lives in a file and is mapped, never loaded whole
        mmap_path = os.path.join(args.mmap_dir, f"som_bench_{os.getpid()}.f32")
        Xw = np.lib.format.open_memmap(mmap_path, mode="w+", dtype=np.float32, shape=(wl.n, wl.d))
        wl.data().fill(Xw)
        Xw.flush()
        del Xw
        X = np.load(mmap_path, mmap_mode="r")
    elif args.stream == "file":
        # the same file, handed to the library as a descriptor: chunks are read with pread into the staging buffers
        mmap_path = os.path.join(args.mmap_dir, f"som_bench_{os.getpid()}.f32")
        Xw = np.memmap(mmap_path, mode="w+", dtype=np.float32, shape=(wl.n, wl.d))
        wl.data().fill(Xw)
        Xw.flush()
        init_rows = draw_initial_rows(wl.seed, wl.n, wl.k)
        W0_file = np.ascontiguousarray(Xw[np.sort(init_rows)])
        del Xw
        X = os.open(mmap_path, os.O_RDONLY)
    elif args.stream and wl.n * wl.d * 4 > (8 << 30):
        # a large host-resident matrix: one anonymous allocation, filled in place by the host's cores (the generators
        # are seeded per block of rows, so the data do not depend on how the work is cut)
        from concurrent.futures import ThreadPoolExecutor
        X = np.empty((wl.n, wl.d), dtype=np.float32)
        gen = wl.data()
        piece = 1 << 22
        done = [0]

        def fill_piece(lo):
            gen.fill(X[lo:lo + piece], lo)
            done[0] += 1
            if done[0] % 32 == 0:
                print(f"[bench] {done[0] * piece} rows generated after {time.time() - t0:.0f}s", file=sys.stderr, flush=True)

        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 8)) as pool:
            list(pool.map(fill_piece, range(0, wl.n, piece)))
    elif not args.stream and wl.n * wl.d * 4 > (48 << 30):
        # Too large to hold twice on the host: the matrix is generated in pieces (the generators are seeded per
        # block of rows, so the data do not depend on how they are cut) and goes to the device piece by piece; a
        # 10^9 x 50 matrix (200 GB, the upper end of the paper's sample axis) stays resident in the 288 GB of HBM.
        from concurrent.futures import ThreadPoolExecutor
        X = None
        Xd = torch.empty((wl.n, wl.d), dtype=torch.float32, device="cuda")
        piece = 1 << 24
        gen = wl.data()
        starts = list(range(0, wl.n, piece))
        with ThreadPoolExecutor(max_workers=8) as pool:
            pending = []
            for i, lo in enumerate(starts):
                pending.append((lo, pool.submit(gen.rows, lo, min(wl.n, lo + piece))))
                if len(pending) >= 8 or i + 1 == len(starts):
                    for plo, fut in pending:
                        blk = fut.result()
                        Xd[plo:plo + len(blk)].copy_(torch.from_numpy(blk))
                    pending = []
                    print(f"[bench] {min(wl.n, lo + piece)} rows on the device after {time.time() - t0:.0f}s", file=sys.stderr, flush=True)
    else:
        X = wl.data().rows(0, wl.n)
    init_rows = draw_initial_rows(wl.seed, wl.n, wl.k)
    if args.stream == "file":
        W0 = W0_file[np.argsort(np.argsort(init_rows))]
    elif X is not None:
        W0 = np.ascontiguousarray(X[init_rows])
    else:
        W0 = Xd[torch.from_numpy(init_rows).cuda()].cpu().numpy()
    sig = linear_sigma(wl.sigma[0], wl.sigma[1], max(args.steps, 1))
    print(f"[bench] generated {wl.name}: {wl.n} x {wl.d} in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    som = pkg.Som(0)
    som.som_set_search(args.search)
    if args.stream:
        try:
            return stream_bench(args, wl, X, W0, sig, som, pkg, torch)
        finally:
            if mmap_path:
                if args.stream == "file":
                    os.close(X)
                del X
                os.remove(mmap_path)
    if X is not None:
        Xd = torch.from_numpy(X).cuda()
    Wd = torch.from_numpy(W0).cuda()
    lattice_G = None
    if wl.topology in ("rect", "hex"):
        lattice_G = torch.from_numpy(pkg.topology.graph_distances(wl.topology, lattice=wl.lattice)).cuda()

    Gd = lattice_G if lattice_G is not None else torch.empty((wl.k, wl.k), dtype=torch.float32, device="cuda")
    # random selector (Eq. 1-2): a fresh subset of m = max(1, floor(N rho)) rows per epoch, drawn on the host
    # beforehand and resident on the device like the samples
    m_sel = wl.n if wl.rho >= 1.0 else max(1, int(wl.n * wl.rho))
    subsets = None
    if m_sel < wl.n:
        subsets = [torch.from_numpy(draw_subset(wl.seed, e, wl.n, m_sel).astype(np.int32)).cuda()
                   for e in range(max(args.steps, args.warmup))]

    def epoch(e):
        # data-driven graphs (Algorithms 1 and 2) are rebuilt on the device from the current weights every epoch
        if lattice_G is None:
            som.som_topology(Wd, wl.topology, Gd)
        som.som_epoch(Xd, Wd, Gd, float(sig[min(e, len(sig) - 1)]), idx=subsets[e] if subsets else None, want_stats=False)

    for e in range(args.warmup):
        epoch(e)
    som.som_sync()
    Wd.copy_(torch.from_numpy(W0))
    torch.cuda.synchronize()

    som.som_profile(True)
    # the epochs are enqueued back to back inside one bracket, synchronised on both sides
    torch.cuda.synchronize()
    ts = time.perf_counter()
    for e in range(args.steps):
        epoch(e)
    som.som_sync()
    torch.cuda.synchronize()
    gpu_s = time.perf_counter() - ts
    kernel_ms = som.som_profile_read()
    som.som_profile(False)

    m = m_sel
    ms_per_step = 1e3 * gpu_s / max(args.steps, 1)
    value = m * args.steps / gpu_s if gpu_s > 0 else 0.0
    # (the library runs more than 2^27 rows as several launches of the kernel: the figure is the kernel time per epoch)
    avg_kernel_ms = float(np.sum(kernel_ms)) / max(args.steps, 1) if kernel_ms else float("nan")
    flops = 2.0 * m * wl.k * wl.d                          # algorithmic: 2 K D per presented sample
    achieved = flops / (avg_kernel_ms * 1e-3) / 1e12 if kernel_ms else float("nan")
    # which matrix pipe the dominant kernel runs on decides the peak it is priced against
    split = args.search == "auto" and wl.d >= 4 and wl.k > 1       # (what SOM_SEARCH_AUTO means in the library)
    if split:
        # MFMAs of 32 nodes x 32 samples x 16 slots the kernel issues per 32 x 32 block: three per whole 16-feature block
        # (hi.hi, lo.hi, hi.lo), one packed block for a remainder of 1..4 features (D <= 64); chunks of 64 features above
        if wl.d <= 64:
            tail = 1 <= wl.d % 16 <= 4
            n_mfma = 3 * (wl.d // 16) + 1 if tail else 3 * ((wl.d + 15) // 16)
        else:
            n_mfma = 12 * ((wl.d + 63) // 64)
        kpad = (wl.k + 127) // 128 * 128
        issued = 2.0 * m * kpad * 16 * n_mfma
        roof = {"bound": "mfma", "kernel": ("bmu_split_kernel + bmu_list_kernel" if wl.d <= 64 else "bmu_split_convert_kernel + bmu_split_wide_kernel + bmu_list_kernel") +
                          " (scores from bf16 parts on the bf16 matrix pipe + arg-max; the marks of the samples to re-decide compacted into a list)",
                "achieved": achieved, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_MFMA_TFLOPS if kernel_ms else None,
                "issued": issued / (avg_kernel_ms * 1e-3) / 1e12 if kernel_ms else None,
                "issued_frac": issued / (avg_kernel_ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS if kernel_ms else None,
                "mfma_per_block": n_mfma,
                "note": "achieved = algorithmic 2 m K D float32 flops per launch; issued = the bf16 MFMA flops the kernel "
                        "executes for them (mfma_per_block instructions of 32 x 32 x 16 per 32 nodes x 32 samples, K padded to 128); "
                        "under this kernel the chip holds its power limit at a shader clock of about 1.9 GHz, the peak assumes 2.4"}
    else:
        roof = {"bound": "mfma", "kernel": "bmu_kernel (fused float32 score contraction + arg-max)",
                "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_FP32_MFMA_TFLOPS if kernel_ms else None}
    roof.update({"avg_kernel_ms": avg_kernel_ms, "launches": len(kernel_ms)})
    if split and kernel_ms:
        # What the bf16 pipe sustains on this machine under its power limit (random operands, two wavefronts per SIMD): MFMAs
        # alone, and with six vector instructions beside each (the search's fold has four to five).  Each loop runs for
        # about 0.6 s; the last launches count.  The published peak is one MFMA per 13.3 ns and SIMD (2.4 GHz).
        def sustained(fold_steps):
            iters, last = 20000, []
            t_end = time.perf_counter() + 0.6
            while time.perf_counter() < t_end:
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                som.som_mfma_rate_probe(fold_steps, 2, iters)
                b.record()
                torch.cuda.synchronize()
                last.append(a.elapsed_time(b))
            return float(np.median(last[-5:])) * 1e6 / (8.0 * iters * 2)
        simds = 4 * torch.cuda.get_device_properties(0).multi_processor_count
        ns_alone, ns_valu = sustained(0), sustained(2)
        ns_kernel = avg_kernel_ms * 1e6 / (issued / (2.0 * 32 * 32 * 16) / simds)
        roof["power_limit"] = {"mfma_alone_ns": ns_alone, "mfma_with_6_vector_instructions_ns": ns_valu, "peak_ns": 13.333,
                               "mfma_alone_frac_of_peak": 13.333 / ns_alone, "with_6_vector_instructions_frac_of_peak": 13.333 / ns_valu,
                               "search_kernel_ns_per_mfma": ns_kernel,
                               "note": "nanoseconds per v_mfma_f32_32x32x16_bf16 and SIMD: sustained by som_mfma_rate_probe on random "
                                       "operands for 0.6 s each, and averaged over the whole search kernel (its prologue and epilogue "
                                       "included)"}
    # the float32 search on the same workload, for reference (same results; its own kernel, its own peak)
    if split and not args.no_float32_reference and flops * (args.warmup + args.steps) < 2e15:
        som.som_set_search("float32")
        W_keep = Wd.clone()
        Wd.copy_(torch.from_numpy(W0))
        for e in range(min(args.warmup, 10)):
            epoch(e)
        som.som_sync()
        Wd.copy_(torch.from_numpy(W0))
        n_ref = min(args.steps, 10)
        som.som_profile(True)
        torch.cuda.synchronize()
        ts = time.perf_counter()
        for e in range(n_ref):
            epoch(e)
        som.som_sync()
        torch.cuda.synchronize()
        ref_s = time.perf_counter() - ts
        ref_ms = som.som_profile_read()
        som.som_profile(False)
        som.som_set_search(args.search)
        Wd.copy_(W_keep)
        if ref_ms:
            k_ms = float(np.sum(ref_ms)) / max(n_ref, 1)
            roof["float32_search"] = {"kernel": "bmu_kernel (float32 MFMA)", "ms_per_step": 1e3 * ref_s / max(n_ref, 1),
                                      "avg_kernel_ms": k_ms, "achieved": flops / (k_ms * 1e-3) / 1e12,
                                      "peak": PEAK_FP32_MFMA_TFLOPS, "frac": flops / (k_ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
                                      "steps": n_ref}
    traffic = None
    # measured off-line with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a plain copy); see profiles/
    pmc = os.path.join(ROOT, "profiles", f"epoch_{wl.name}_hbm_traffic.md")
    if os.path.exists(pmc) and args.rows is None and not over:
        for line in open(pmc):
            if line.startswith("traffic_bytes_per_launch_bmu_kernel:"):
                traffic = float(line.split(":")[1])
    roof["traffic"] = traffic

    if args.copy_calibration:
        Xcopy = torch.empty_like(Xd)
        Xcopy.copy_(Xd)                      # reads and writes X.numel() * 4 bytes
        torch.cuda.synchronize()
        del Xcopy
    qe = torch.zeros(2, dtype=torch.float64, device="cuda")
    b_final, _, _ = som.som_bmu(Xd, Wd, qe=qe)    # quantisation error of the final weights over all rows
    final_qe = float(qe[0].item()) / wl.n

    # the other stages on their own, outside the timed region: the accumulation (HBM-bound in principle: one row and
    # one BMU index read per sample) over all rows with the final BMUs, and the update
    S_t = torch.empty((wl.k, wl.d), dtype=torch.float64, device="cuda")
    n_t = torch.empty((wl.k,), dtype=torch.int64, device="cuda")
    W_t = Wd.clone()

    def event_ms(fn, reps=5):
        fn()
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in pairs:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in pairs]))

    acc_ms = event_ms(lambda: som.som_accumulate(Xd, b_final, wl.k, S_t, n_t, zero_first=True))
    upd_ms = event_ms(lambda: som.som_neighborhood_update(S_t, n_t, Gd, float(sig[-1]), W_t))
    read_ms = event_ms(lambda: som.som_read_probe(Xd))
    # the whole search (weight preparation, search kernel, re-decision) with and without the distances to the BMUs, which
    # only statistics need: the timed epochs run without them
    d2_t = torch.empty(b_final.numel(), dtype=torch.float32, device="cuda")
    search_plain_ms = event_ms(lambda: som.som_bmu(Xd, Wd, idx=subsets[0] if subsets else None, bmu=b_final[:m_sel]))
    search_dist_ms = event_ms(lambda: som.som_bmu(Xd, Wd, idx=subsets[0] if subsets else None, bmu=b_final[:m_sel], d2=d2_t[:m_sel], qe=qe))
    del d2_t
    acc_bytes = wl.n * (wl.d * 4 + 4)
    read_GBps = Xd.numel() * 4 / (read_ms * 1e-3) / 1e9
    stages = {"accumulate_ms": acc_ms, "accumulate_GBps": acc_bytes / (acc_ms * 1e-3) / 1e9,
              "accumulate_frac_of_hbm_peak": acc_bytes / (acc_ms * 1e-3) / 8e12, "update_ms": upd_ms,
              "search_ms": search_plain_ms, "search_with_distances_ms": search_dist_ms,
              "plain_read_of_X_ms": read_ms, "plain_read_GBps": read_GBps, "plain_read_frac_of_hbm_peak": read_GBps / 8e3,
              "accumulate_frac_of_plain_read": acc_bytes / (acc_ms * 1e-3) / 1e9 / read_GBps,
              "note": "stand-alone som_accumulate over all rows with the final BMUs (algorithmic bytes: one row + "
                      "one int32 per sample) and som_neighborhood_update, HIP events, median of 5; plain_read = a kernel "
                      "that only streams X through 16-byte loads (som_read_probe), the rate this GPU's memory system delivers; "
                      "search_ms = som_bmu on the final weights (preparation, search, re-decision) as the timed epochs run it, "
                      "search_with_distances_ms = the same with d2 and the quantisation-error sums asked for"}

    out = {
        "metric": METRIC, "value": value, "unit": "samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("bf16x2-split MFMA scores (float32 accumulate), f32 re-decision and distances, f64 sums and update" if split
                  else "f32 MFMA scores, f32 re-decision and distances, f64 sums and update"),
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.k}-node {wl.topology} map, {wl.n} x {wl.d} float32 samples resident in HBM"
                               f"{'' if m_sel == wl.n else f' ({m_sel} drawn per epoch)'}, "
                               f"sigma {wl.sigma[0]}->{wl.sigma[1]} over {args.steps} epochs",
                   "samples": wl.n, "presented_per_epoch": m_sel, "features": wl.d, "nodes": wl.k, "topology": wl.topology,
                   "final_qe": final_qe, "topology_rebuilt_on_device_each_epoch": lattice_G is None,
                   "search": "bf16 parts on the bf16 matrix pipe, re-decision in float32" if split else "float32 MFMA"},
        "roofline": roof,
        "stages": stages,
    }

    if not args.no_cpu_baseline:
        import oracle
        n_cpu = min(args.cpu_rows, wl.n)
        G_or = oracle.graph_distances(wl.topology, W=W0, lattice=wl.lattice)
        Xc = X[:n_cpu] if X is not None else wl.data().rows(0, n_cpu)
        # whole epochs of the oracle, each from the previous one's weights, until about ten seconds have passed
        tc = time.perf_counter()
        Wc, n_ep = W0, 0
        while n_ep < len(sig) and (n_ep == 0 or time.perf_counter() - tc < 10.0):
            Wc = oracle.epoch_grouped(Xc, None, Wc, G_or, float(sig[n_ep]))["W"].astype(np.float32)
            n_ep += 1
        dt = time.perf_counter() - tc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": n_cpu * n_ep / dt, "unit": "samples/s", "cores": cores, "kind": "oracle",
                               "sample": f"{n_ep} epoch(s) of the float64 oracle (BLAS distance product, grouped update, fixed "
                                         f"initial graph) on the first {n_cpu} rows of {wl.name}, {dt:.1f}s"}
    som.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
