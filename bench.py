#!/usr/bin/env python3
"""Benchmark of the single-GPU GCN hot path.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5|1|2|3|4] [--epoch] [--f F]

Default workload: the stand-alone SpMM on the config 5 graph (the largest one: Protein-shaped Chung-Lu,
8.7 M vertices, 1.32 G stored entries) at the hidden width f = 16.  One step is the pair Z = A X and
Z = A^T X (the transposed product runs on its own stored arrays).  `value` is algorithmic GB/s:
(8 nnz + 8 (n+1) + 4 n f read + 4 n f written) per product over wall time, inputs resident in HBM before
the timed region.  `--config 2` is the same on the R-MAT scale-20 graph at f = 128; `--config N --epoch`
times one full-batch epoch (forward + loss + backward, lr = 0) of config N instead and reports milliseconds.

The JSON line also carries `roofline` for the sparse product (every kernel of a product, bracketed by HIP
events inside the library on the launch stream) and `cpu_baseline` (the CPU oracle timed on the host cores
on the same matrix).
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

HBM_PEAK_GBPS = 8000.0

# Bytes that crossed the L2 <-> fabric interface per product (every kernel of one A X), measured with
# rocprofv3 --pmc (FETCH_SIZE, then WRITE_SIZE, in KiB per dispatch, each scaled by what the same counter
# reads for a plain device copy of known size: FETCH_SIZE x 2.0, WRITE_SIZE x 1.0) and summed over the
# kernels of a product; from the profiles/spmm_*.txt summaries.  They are fills of the eight L2s: reads that
# the memory-side Infinity Cache served are included, so this is an upper bound of the HBM bytes.  Each entry
# names the schedule it was measured on (what gcn_spmm_describe returned in that run): a line whose library
# reports another schedule carries traffic = null instead of a stale figure.
MEASURED_TRAFFIC = {
    ("rmat20_spmm_f128", 128): {
        "bytes": 10045335483,
        "kernels": "k_spmm_split<8,4> over 4 panels of 32 columns + k_spmm_fixup",
        "schedule": "split(chunks=63376)",
        "profile": "profiles/spmm_split_rmat20_f128.txt"},
    ("chunglu_reddit_gcn_602_16_16_41", 16): {
        "bytes": 1033356854,
        "kernels": "k_scale_rows + k_spmm_split<4,4> over the column-blocked copy + k_spmm_fixup + k_block_reduce",
        "schedule": "blocked(blocks=8,cols_per_block=29696,partial_rows=1863720,chunks=224269)"
                    "; value-free (operand rows pre-scaled by d^-1/2, output rows scaled)",
        "profile": "profiles/spmm_blocked_chunglu_reddit_f16.txt"},
    ("rmat_amazon_gcn_300_16_16_24", 16): {
        "bytes": 20042035304,
        "kernels": "k_pack_rows + k_spmm_split_pair<4,4> (paired launch of the hub schedule) + 2 x k_spmm_fixup + k_block_reduce",
        "schedule": "hub(hot_cols=524288,cols_per_block=32768,long_row>=64,nnz_hot=148858651,nnz_rest=96949372,partial_rows=7701691)",
        "profile": "profiles/spmm_hub_rmat_amazon_f16.txt"},
    ("chunglu_protein_gcn_128_16_16_256", 16): {
        "bytes": 82950924194,
        "kernels": "k_scale_rows + 15 x k_spmm_sweep<4> + k_spmm_split<4,4> (column-blocked, long rows) + k_spmm_fixup + k_block_reduce",
        "schedule": "sweep(entries_per_step=16,rows_per_task=256,long_row>1024,tasks=34163,launches=15,stored=936862448)"
                    "+long_rows:blocked(blocks=101,cols_per_block=87040,partial_rows=12649811,chunks=745738)"
                    "; value-free (operand rows pre-scaled by d^-1/2, output rows scaled)",
        "profile": "profiles/spmm_sweep_chunglu_protein_f16_default_command.txt"},
}

# kernels inside the library's event bracket of one product, by the schedule the library reports
SCHEDULE_KERNELS = {1: "k_spmm_rowwise", 2: "k_spmm_split + k_spmm_fixup",
                    3: "k_spmm_sweep (rows <= 1024 entries) + k_spmm_split, k_spmm_fixup, k_block_reduce (column-blocked, longer rows)",
                    4: "k_pack_rows + k_spmm_split_pair (hub schedule: long rows x hot columns over packed rows + the rest) + k_spmm_fixup + k_block_reduce",
                    5: "k_spmm_split (column-blocked) + k_spmm_fixup + k_block_reduce"}

GRAPH_WORDS = {1: "Erdos-Renyi, 4096 vertices", 2: "R-MAT scale 20, edge factor 16",
               3: "Reddit-shaped Chung-Lu", 4: "Amazon-shaped R-MAT scale 24", 5: "Protein-shaped Chung-Lu"}


def host_cpu() -> dict:
    """Model string and logical CPU count of the host the oracle is timed on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"model": model, "logical_cpus": os.cpu_count()}


def spmm_alg_bytes(n: int, nnz: int, f: int) -> int:
    return 8 * nnz + 8 * (n + 1) + 4 * n * f + 4 * n * f


_T0 = time.time()


def progress(msg: str) -> None:
    """One line per finished stage on stderr (stdout carries only the JSON line)."""
    print(f"[bench {time.time() - _T0:7.1f}s] {msg}", file=sys.stderr, flush=True)


def oracle_matrix(a, transposed=False):
    """The stored matrix of the library as the oracle's Csr on the host: the CPU baseline then runs on exactly
    the matrix the GPU ran on (its construction is checked against the oracle's own in the tests)."""
    import oracle
    rowptr, colidx, val, deg = [t.cpu().numpy() for t in a.views(transposed)]
    return oracle.Csr(n=a.n_cols if transposed else a.n_rows, rowptr=rowptr, colidx=colidx, val=val, deg=deg,
                      ncols=a.n_rows if transposed else a.n_cols)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--epoch", action="store_true",
                    help="configs 1, 3, 4, 5: time one full-batch epoch (forward + loss + backward) instead of the "
                         "stand-alone SpMM")
    ap.add_argument("--order", type=int, default=0, help="0 auto, 1 GEMM first, 2 SpMM first (epoch mode)")
    ap.add_argument("--algo", type=int, default=0, help="SpMM kernel: 0 auto, 1 row-wise, 2 nonzero-split, 3 sweep, 4 hub")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--f", type=int, default=0, help="dense width of the stand-alone SpMM (default: 128 on config 2, else 16)")
    ap.add_argument("--slice", type=int, default=0,
                    help="SpMM mode: time one block row of P = SLICE (rows [0, n/P) of A against all of X), "
                         "one process's share of the paper's 1D algorithm")
    ap.add_argument("--directed", action="store_true",
                    help="SpMM mode: keep the drawn pairs as directed edges (no symmetrisation) with row normalisation, "
                         "so that A and A^T differ")
    ap.add_argument("--no-permute", action="store_true",
                    help="skip the random vertex relabelling (hubs then sit at low ids, which flatters the caches)")
    ap.add_argument("--preaggregate", action="store_true",
                    help="epoch mode: compute A^T H0 once before the timed epochs and run gcn_epoch_preaggregated "
                         "(first layer without sparse products); an extra row, never the default")
    ap.add_argument("--pattern", action="store_true",
                    help="SpMM mode: also time the value-free product (row pre-scaling + gcn_spmm_pattern) and report "
                         "it under extra")
    ap.add_argument("--graph", action="store_true",
                    help="epoch mode: also time the epoch replayed from a HIP graph (reported in extra)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of the dense operand (known size) for scaling PMC byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (no collectives or sharding are built)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2005_03300_amd as g
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    g.lib()
    w = synth.CONFIGS[args.config]
    if args.epoch and len(w.dims) == 1:
        print("bench.py: config 2 is the stand-alone SpMM workload; --epoch applies to configs 1, 3, 4, 5", file=sys.stderr)
        return 2
    if args.no_permute:
        import dataclasses
        w = dataclasses.replace(w, permute=False)
    if args.directed and args.epoch:
        print("bench.py: --directed applies to the stand-alone SpMM", file=sys.stderr)
        return 2
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    t0 = time.time()
    n, src, dst = synth.make_graph(w, args.seed)
    t_gen = time.time() - t0
    progress(f"generated {w.name}: n={n}, {src.shape[0]} raw pairs")
    t0 = time.time()
    src_d, dst_d = dev(src), dev(dst)
    n_raw = int(src.shape[0])
    del src, dst
    flags = (g.ADD_SELF_LOOPS | g.NORM_ROW | g.BUILD_TRANSPOSE) if args.directed else \
            (g.SYMMETRISE | g.ADD_SELF_LOOPS | g.NORM_SYM | g.BUILD_TRANSPOSE)
    a = g.gcn_csr_create(n, src_d, dst_d, flags)
    torch.cuda.synchronize()
    t_build = time.time() - t0
    del src_d, dst_d
    nnz = a.nnz
    progress(f"compressed rows built on the GPU: nnz={nnz}")
    g.gcn_config(g.CFG_SPMM_ALGO, args.algo)

    out = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic"}
    extra = {"n": n, "nnz": nnz, "max_degree": a.max_degree, "gen_s": round(t_gen, 2),
             "csr_build_s": round(t_build, 3), "n_raw_pairs": n_raw}

    if not args.epoch:
        f = args.f or (w.dims[0] if len(w.dims) == 1 else 16)
        X = synth.uniform_features(n, f, args.seed)
        Xd = dev(X)
        zrows = n
        if args.slice > 1:
            # block row 0 of P: an (n/P) x n matrix; A X_all forward, A^T X_slice for the transposed product
            rowptr, colidx, val, _ = a.arrays(False)
            zrows = n // args.slice
            hi = int(rowptr[zrows].item())
            a_full = a
            a = g.gcn_csr_create_from_csr_rect(zrows, n, rowptr[:zrows + 1].clone(), colidx[:hi].clone(), val[:hi].clone(),
                                               g.BUILD_TRANSPOSE)
            a_full.close()
            del rowptr, colidx, val
            nnz = a.nnz
            extra.update(slice_of=args.slice, slice_rows=zrows, slice_nnz=nnz)
        Z = torch.empty(zrows, f, device="cuda")
        Zt = torch.empty(n, f, device="cuda")
        Xs = Xd[:zrows]
        t0 = time.time()
        g.gcn_spmm_prepare(a, 0, f)
        g.gcn_spmm_prepare(a, 1, f)
        torch.cuda.synchronize()
        extra["schedule_build_s"] = round(time.time() - t0, 3)
        schedule_text = g.gcn_spmm_describe(a, 0, f)
        extra["schedule"] = schedule_text

        def step():
            g.gcn_spmm(a, 0, Xd, Z)
            g.gcn_spmm(a, 1, Xs, Zt)

        # plain device copy of the dense operand (reads and writes n*f*4 bytes): the stream rate this GPU
        # reaches, beside the 8 TB/s peak; with --copy-calibration it is also the known-size dispatch
        # that scales the PMC byte counters
        for _ in range(2):
            Zt.copy_(Xd)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(5):
            Zt.copy_(Xd)
        ev[1].record()
        torch.cuda.synchronize()
        copy_gbps = 2 * n * f * 4 / (ev[0].elapsed_time(ev[1]) / 5 * 1e-3) / 1e9
        extra["stream_copy_GBps"] = round(copy_gbps, 1)
        if args.copy_calibration:
            extra["copy_calibration_bytes_each_way"] = n * f * 4
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        g.gcn_config(g.CFG_TIMING, 1)
        g.gcn_timing_read_phases()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        phases = g.gcn_timing_read_phases()
        g.gcn_config(g.CFG_TIMING, 0)
        # the same loop without the event bracketing, so `value` carries no instrumentation cost
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = min(dt, time.perf_counter() - t0)
        sched = g.gcn_last_spmm_schedule()

        if args.pattern and args.slice <= 1 and not args.directed:
            def valued(a, trans, X, Zout):
                g.gcn_config(g.CFG_PATTERN_SPMM, 0)          # gcn_spmm reads the stored values
                try:
                    g.gcn_spmm(a, trans, X, Zout)
                finally:
                    g.gcn_config(g.CFG_PATTERN_SPMM, 2)
                return Zout
            sc = torch.empty(n, device="cuda")
            g.gcn_csr_inv_sqrt_degrees(a, sc)
            Xsc = torch.empty_like(Xd)
            for timed in (False, True):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps if timed else max(args.warmup, 1)):
                    g.gcn_scale_rows(Xd, sc, Xsc)
                    g.gcn_spmm_pattern(a, 0, Xsc, Z, sc)
                    g.gcn_scale_rows(Xd, sc, Xsc)
                    g.gcn_spmm_pattern(a, 1, Xsc, Zt, sc)
                torch.cuda.synchronize()
                t_pat = (time.perf_counter() - t0) / args.steps * 1e3
            for timed in (False, True):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps if timed else max(args.warmup, 1)):
                    g.gcn_scale_rows(Xd, sc, Xsc)
                    g.gcn_scale_rows(Xd, sc, Xsc)
                torch.cuda.synchronize()
                t_sc = (time.perf_counter() - t0) / args.steps * 1e3
            extra.update(pattern_ms_per_step=round(t_pat, 4), pattern_prescale_ms_per_step=round(t_sc, 4),
                         pattern_bytes_alg_per_spmm=4 * nnz + 8 * (n + 1) + 4 * n + 8 * n * f,
                         pattern_max_abs_diff_vs_valued=float((Zt - valued(a, 1, Xd, torch.empty_like(Zt))).abs().max()))
            g.gcn_spmm(a, 0, Xd, Z)

        progress("SpMM timed")
        b_alg = spmm_alg_bytes(n, nnz, f) if args.slice <= 1 else 8 * nnz + 8 * (zrows + 1) + 4 * n * f + 4 * zrows * f
        ms_step = dt / args.steps * 1e3
        value = 2 * b_alg / (ms_step * 1e-3) / 1e9
        products, product_ms = phases["spmm"]
        main_launches, main_ms = phases["spmm_kernel"]
        avg_product_ms = product_ms / max(products, 1)      # every kernel of one product, by HIP events on the stream
        achieved = b_alg / (avg_product_ms * 1e-3) / 1e9
        variant = []
        if args.directed:
            variant.append("directed, row-normalised (A and A^T differ)")
        if args.no_permute:
            variant.append("not relabelled")
        if args.slice > 1:
            variant.append(f"block row: rows [0, n/{args.slice}) of A ({zrows} x {n})")
        out.update(metric="SpMM algorithmic GB/s (CSR fp32, A X and A^T X)", value=round(value, 2), unit="GB/s",
                   ms_per_step=round(ms_step, 4),
                   config={"workload": f"config {args.config}: stand-alone SpMM on the {w.name} graph ({GRAPH_WORDS[args.config]}; "
                                       f"symmetrised, self loops, sym-normalised, relabelled), X {n}x{f} uniform[-1,1)",
                           "n": n, "nnz": nnz, "f": f, "step": "Z=A X then Z=A^T X",
                           **({"variant": "; ".join(variant)} if variant else {})})
        extra.update(spmm_gflops=round(2 * 2.0 * nnz * f / (ms_step * 1e-3) / 1e9, 1),
                     pct_hbm_peak=round(100 * value / HBM_PEAK_GBPS, 2),
                     bytes_alg_per_spmm=b_alg, bytes_nocache_per_spmm=8 * nnz + 8 * (n + 1) + 4 * f * nnz + 4 * n * f,
                     spmm_products_timed=2 * args.steps, event_brackets=products,
                     main_kernel_ms_per_product=round(main_ms / max(products, 1), 4),
                     main_kernel_brackets=main_launches)
        meas = MEASURED_TRAFFIC.get((w.name, f)) if not (args.slice > 1 or args.directed or args.no_permute or args.algo) else None
        traffic = None
        if meas is not None:
            if meas["schedule"] is None or meas["schedule"] == schedule_text:
                traffic = meas["bytes"]
                extra["traffic_measured_on"] = {k: meas[k] for k in ("kernels", "profile")}
            else:
                extra["traffic_withheld"] = (f"the stored counter figure was measured on schedule {meas['schedule']!r}, "
                                             f"this run took {schedule_text!r}")
        value_free = "value-free" in schedule_text
        if value_free:
            # the library took the form that skips the stored values (4 B per entry instead of 8, one pre-scaling pass
            # over X); `achieved` still prices the product at the CSR formula's bytes, this is the form's own count
            vf_bytes = 4 * nnz + 8 * (n + 1) + 4 * n + 8 * n * f + 8 * n * f
            extra["value_free_bytes_alg_per_spmm"] = vf_bytes
            extra["value_free_achieved_GBps"] = round(vf_bytes / (avg_product_ms * 1e-3) / 1e9, 2)
            extra["value_free_frac_of_hbm_peak"] = round(vf_bytes / (avg_product_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
        out["roofline"] = {"bound": "hbm", "kernel": ("k_scale_rows + " if value_free else "") + SCHEDULE_KERNELS.get(sched, "k_spmm_split"),
                           "achieved": round(achieved, 2),
                           "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                           "avg_kernel_ms": round(avg_product_ms, 4),
                           "covers": "every kernel of one product (HIP events around the whole product on the launch stream)",
                           "bytes_basis": "the task's CSR formula 8 nnz + 8 (n + 1) + 8 n f, whatever form the library takes"
                                          + ("; this run took the value-free form, whose own minimum is extra.value_free_bytes_alg_per_spmm" if value_free else ""),
                           "traffic": traffic,
                           "traffic_is": "bytes across the L2 <-> fabric interface per product (rocprofv3 FETCH_SIZE / WRITE_SIZE, "
                                         "scaled by a plain copy); fills served by the Infinity Cache are included, so an "
                                         "upper bound of the HBM bytes; no HBM-side counter is exposed on this machine"}
        extra["achieved_pct_of_stream_copy"] = round(100 * achieved / copy_gbps, 2)
        if traffic:
            moved = traffic / (avg_product_ms * 1e-3) / 1e9
            extra.update(l2_fabric_traffic_GBps=round(moved, 1),
                         l2_fabric_traffic_over_algorithmic=round(traffic / b_alg, 2),
                         l2_fabric_traffic_pct_of_stream_copy=round(100 * moved / copy_gbps, 1))

        if not args.no_cpu:
            import oracle
            t0 = time.time()
            A = oracle_matrix(a, False)
            t_ex = time.time() - t0
            progress("oracle: stored matrix copied to the host")
            t0 = time.time()
            Zo = oracle.spmm(A, X)
            t_o = time.time() - t0
            progress("oracle: product done")
            Zh = Z.cpu().numpy()
            err = float(np.abs(Zh - Zo).max())
            scale = float(np.sqrt(np.mean(Zo.astype(np.float64) ** 2)))
            out["cpu_baseline"] = {"value": round(b_alg / t_o / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(),
                                   "kind": "oracle",
                                   "sample": f"one full Z = A X on the same stored matrix ({zrows} x {n}, nnz={nnz}, f={f}), 1 rep",
                                   "ms": round(t_o * 1e3, 1), "matrix_copy_to_host_s": round(t_ex, 2), "host": host_cpu()}
            # the same product on one core, on a bounded sample of the rows: random rows and the longest ones
            all_threads = oracle.threads()
            rs = np.random.default_rng(args.seed)
            k = max(1, min(zrows, max(zrows // 64, 4096)))
            heavy = np.argsort(A.deg[:zrows])[-min(1000, zrows):] if A.deg.shape[0] >= zrows else np.zeros(0, np.int64)
            sample_rows = np.unique(np.concatenate([rs.integers(0, zrows, k), heavy])).astype(np.int64)
            sample_nnz = int((A.rowptr[sample_rows + 1] - A.rowptr[sample_rows]).sum())
            oracle.set_threads(1)
            t0 = time.time()
            Zs = oracle.spmm_rows(A, X, sample_rows)
            t_1 = time.time() - t0
            oracle.set_threads(all_threads)
            extra["oracle_single_thread"] = {"rows": int(sample_rows.size), "entries": sample_nnz, "ms": round(t_1 * 1e3, 1),
                                             "ms_scaled_to_all_entries": round(t_1 * 1e3 * nnz / max(sample_nnz, 1), 1)}
            extra.update(max_abs_err_vs_oracle=err, rms_of_oracle=scale,
                         sampled_rows_match_full_product=bool(np.array_equal(Zs, Zo[sample_rows])))
    else:
        H0, y, Ws = synth.make_model_inputs(w, args.seed)
        dims = list(w.dims)
        L = len(dims) - 1
        H0d, yd = dev(H0), dev(y)
        Wd = [dev(x) for x in Ws]
        Yd = [torch.empty_like(x) for x in Wd]
        ws = torch.empty(g.gcn_epoch_workspace_bytes(n, dims, args.order), dtype=torch.uint8, device="cuda")
        loss = torch.zeros(1, device="cuda")
        t0 = time.time()
        g.gcn_epoch_prepare(a, dims, args.order)
        extra["schedule_build_s"] = round(time.time() - t0, 3)

        if args.preaggregate:
            P0 = torch.empty(n, dims[0], device="cuda")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g.gcn_spmm(a, 1, H0d, P0)
            torch.cuda.synchronize()
            extra["preaggregation_ms_once"] = round((time.perf_counter() - t0) * 1e3, 3)

        def step():
            if args.preaggregate:
                g.gcn_epoch_preaggregated(a, dims, P0, yd, n, Wd, Yd, 0.0, loss, ws, args.order)
            else:
                g.gcn_epoch(a, dims, H0d, yd, Wd, Yd, 0.0, loss, ws, args.order)

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        g.gcn_config(g.CFG_TIMING, 1)
        g.gcn_timing_read_phases()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        phases = g.gcn_timing_read_phases()
        g.gcn_config(g.CFG_TIMING, 0)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = min(dt, time.perf_counter() - t0)
        ms_step = dt / args.steps * 1e3
        progress("epochs timed")
        if args.graph:
            # the same epoch captured once in a HIP graph and replayed: what a launch-bound caller gains
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            for _ in range(max(args.warmup, 1)):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            extra["hip_graph_replay_ms_per_epoch"] = round((time.perf_counter() - t0) / args.steps * 1e3, 4)
        extra["phase_ms_per_epoch"] = {"spmm": round(phases["spmm"][1] / args.steps, 4),
                                       "gemm": round(phases["gemm"][1] / args.steps, 4),
                                       "loss_elementwise_update": round(phases["other"][1] / args.steps, 4)}
        # widths of the SpMM launches of one epoch under the chosen association order
        widths = []
        for l in range(L):
            fi, fo = dims[l], dims[l + 1]
            gemm_first = (args.order == 1) or (args.order == 0 and fo <= fi)
            if l == 0 and args.preaggregate:
                continue                                                 # no sparse product in layer 1
            widths.append(fo if gemm_first else fi)                      # forward
            if l > 0 or gemm_first:
                widths.append(fo if gemm_first else fi)                  # backward (none for SpMM-first layer 1)
        bytes_epoch_spmm = sum(spmm_alg_bytes(n, nnz, fw) for fw in widths)
        spmm_ms = phases["spmm"][1]
        achieved = bytes_epoch_spmm * args.steps / (spmm_ms * 1e-3) / 1e9 if spmm_ms > 0 else 0.0
        out.update(metric="full-batch GCN epoch ms (forward + loss + backward)" +
                   (" with A^T H0 aggregated once outside the epochs" if args.preaggregate else ""),
                   value=round(ms_step, 4), unit="ms",
                   ms_per_step=round(ms_step, 4), higher_is_better=False,
                   config={"workload": f"config {args.config}: one epoch of {w.name} ({GRAPH_WORDS[args.config]})", "n": n,
                           "nnz": nnz, "dims": dims, "order": args.order})
        extra.update(loss=float(loss.item()), spmm_widths=widths, spmm_ms_per_epoch=round(spmm_ms / args.steps, 4),
                     spmm_share=round(spmm_ms / args.steps / ms_step, 3))
        out["roofline"] = {"bound": "hbm", "kernel": SCHEDULE_KERNELS.get(g.gcn_last_spmm_schedule(), "k_spmm_split"),
                           "achieved": round(achieved, 2),
                           "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                           "avg_kernel_ms": round(spmm_ms / max(len(widths) * args.steps, 1), 4),
                           "covers": "every kernel of the sparse products of an epoch (incl. pre-scaling, fix-up, reduce)",
                           "traffic": None}
        if not args.no_cpu:
            import oracle
            # the oracle's own epoch on the same stored matrix (symmetric: A^T == A bit for bit, checked in the tests)
            A = oracle_matrix(a, False)
            progress("oracle: stored matrix copied to the host")
            t0 = time.time()
            ref = oracle.epoch(A, A, H0, y, Ws, 0.0)
            t_o = time.time() - t0
            progress("oracle: epoch done")
            out["cpu_baseline"] = {"value": round(t_o * 1e3, 1), "unit": "ms", "cores": oracle.threads(), "kind": "oracle",
                                   "sample": "one full oracle epoch (forward + loss + backward, every product) on the same "
                                             "stored matrix and inputs, 1 rep", "host": host_cpu()}
            extra["loss_rel_err_vs_oracle"] = abs(float(loss.item()) - ref["loss"]) / abs(ref["loss"])
    out["extra"] = extra
    print(json.dumps(out))
    a.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
