#!/usr/bin/env python3
"""Benchmark of the Ozaki scheme II FP64 GEMM path on one MI355X.

One "step" = one oz2_dgemm call (all stages of Algorithm 1) on the headline workload
m = n = k = 16384, phi = 0.5, 16 moduli, inputs resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c3|c2|c1|c5a|c5b] [--moduli N]
                  [--no-cpu-baseline] [--no-context]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense INT8 matrix peak, TOP/s
HBM_PEAK_GBPS = 8000.0         # MI355X HBM3E peak

GEMM_SOURCE = os.path.join(ROOT, "paper_2504_08009_amd", "csrc", "oz2_stage2.hip")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gemm_hbm_traffic.txt")


def gemm_source_hash():
    import hashlib
    with open(GEMM_SOURCE, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def measured_traffic(key):
    """HBM-side bytes per GEMM launch from the rocprofv3 counter runs summarised in profiles/gemm_hbm_traffic.txt
    (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a plain copy of known size).  The
    file names the hash of the GEMM source it was taken on; for any other source the figure would be stale and None
    is returned."""
    try:
        entries = {}
        with open(TRAFFIC_FILE) as f:
            for line in f:
                line = line.split("#")[0].strip()
                if "=" in line:
                    k, v = [t.strip() for t in line.split("=", 1)]
                    entries[k] = v
    except OSError:
        return None
    if entries.get("gemm_source_sha256_16") != gemm_source_hash():
        return None
    try:
        fetch = float(entries[key + ".fetch_size_raw_GiB"]) * float(entries["fetch_size_scale"])
        write = float(entries[key + ".write_size_raw_GiB"]) * float(entries["write_size_scale"])
        return {"bytes": round((fetch + write) * 2**30), "read_GiB": round(fetch, 2), "written_GiB": round(write, 2),
                "algorithmic_GiB": float(entries[key + ".algorithmic_GiB"]),
                "source": "profiles/gemm_hbm_traffic.txt (GEMM source %s)" % entries["gemm_source_sha256_16"]}
    except (KeyError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--moduli", type=int, default=0)
    ap.add_argument("--mnk", default="", help="override the shape of the workload: m,n,k (same phi and seed)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context", action="store_true")
    ap.add_argument("--shift-mode", type=int, default=0,
                    help="0: shifts from maxima (Section 3, default); 1: Cauchy-Schwarz bound; 2: INT8-product bound (Section 4.1)")
    ap.add_argument("--product-format", type=int, default=-1,
                    help="0: INT32 product planes; 1: UINT8 residue planes (library default)")
    ap.add_argument("--gemm-algorithm", type=int, default=-1,
                    help="-1: library default (Strassen form of the INT8 products for large sizes); 0: classical; 1: Strassen form")
    ap.add_argument("--round-sync", type=int, default=-1,
                    help="bound (polls) of a wait of the GEMM's round synchronisation; 0 switches it off, 1 makes every "
                         "first wait run to its bound (library default 4096)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one captured HIP graph of the call instead of eager calls (small sizes)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of A (known size) so that rocprofv3 byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path needs no exchange between GPUs: each would take "
              "its own tile of C with its own panels of A and B). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2504_08009_amd as oz
    from paper_2504_08009_amd import inputs

    cfg = inputs.CONFIGS[args.workload]
    m, n, k, phi = cfg["m"], cfg["n"], cfg["k"], cfg["phi"]
    if args.mnk:
        m, n, k = [int(v) for v in args.mnk.split(",")]
    N = args.moduli or (16 if args.workload == "c4" else cfg["N"][len(cfg["N"]) // 2])
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    print("bench: generating inputs on the host ...", file=sys.stderr, flush=True)
    t0 = time.time()
    A = inputs.block(cfg["seed"], 0, m, k, phi)
    B = inputs.block(cfg["seed"], 1, k, n, phi)
    gen_s = time.time() - t0
    dA = torch.from_numpy(A.T).to(dev).t()   # A is column-major: A.T is a C-contiguous view
    dB = torch.from_numpy(B.T).to(dev).t()
    dC = torch.empty((n, m), dtype=torch.float64, device=dev).t()
    fmt = args.product_format if args.product_format >= 0 else oz.OZ2_PRODUCT_RESIDUE_U8
    oz.oz2_set_product_format(fmt)
    oz.oz2_set_gemm_algorithm(args.gemm_algorithm)
    oz.oz2_set_shift_mode(args.shift_mode)
    if args.round_sync >= 0:
        oz.oz2_set_round_sync(args.round_sync)
    ws = oz.Workspace(m, n, k, N, device=dev, product_format=fmt)
    strassen = oz.oz2_gemm_algorithm_for(m, n, k, N) == oz.OZ2_GEMM_STRASSEN
    stream = torch.cuda.current_stream()

    hip = ctypes.CDLL("libamdhip64.so")
    def new_event():
        ev = ctypes.c_void_p()
        rc = hip.hipEventCreate(ctypes.byref(ev))
        assert rc == 0, "hipEventCreate failed"
        return ev
    def elapsed(a, b):
        ms = ctypes.c_float()
        rc = hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, "hipEventElapsedTime failed"
        return ms.value

    def step(events=None):
        oz.oz2_set_stage_events(events)
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N, stream)

    def timed_ms(call, reps=5):
        """average milliseconds of `call` over reps launches, HIP events on the stream the library launches on"""
        call()
        torch.cuda.synchronize()
        a, b = new_event(), new_event()
        sp = ctypes.c_void_p(stream.cuda_stream)
        assert hip.hipEventRecord(a, sp) == 0
        for _ in range(reps):
            call()
        assert hip.hipEventRecord(b, sp) == 0
        torch.cuda.synchronize()
        return elapsed(a, b) / reps

    print("bench: timing %d steps ..." % args.steps, file=sys.stderr, flush=True)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[new_event() for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step([e.value for e in evs[s]])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    oz.oz2_set_stage_events(None)
    # the same K calls once more with no event between the stages: the three events recorded inside every call of
    # the timed region cost a few microseconds each, which the launch-bound small workloads feel (reported beside
    # the headline figure, which stays the instrumented one)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step()
    torch.cuda.synchronize()
    plain_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    if args.graph:
        # the stage times above come from the eager pass; the headline time from replays of one captured call
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
            oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N, torch.cuda.current_stream())
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

    stage_ms = np.array([[elapsed(e[i], e[i + 1]) for i in range(3)] for e in evs])
    avg = stage_ms.mean(axis=0)
    ms_per_step = wall * 1e3 / args.steps
    tflops = 2.0 * m * n * k / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the INT8 GEMM of stage 2 (one launch per step)
    gemm_ms = float(avg[1])
    # INT8 operations the launch executes: 2 m n k per modulus as printed in Algorithm 1 line 6; in the Strassen
    # form seven products of half the (padded) size per modulus, 7/8 of that
    if strassen:
        up = lambda v, a: (v + a - 1) // a * a
        mh, nh, kh = up((m + 1) // 2, 256), up((n + 1) // 2, 256), up((k + 1) // 2, 64)
        gemm_ops = 7 * 2.0 * mh * nh * kh * N
    else:
        gemm_ops = 2.0 * m * n * k * N
    gemm_tops = gemm_ops / (gemm_ms * 1e-3) / 1e12
    planes = 1.75 if strassen else 1.0   # plane bytes of the conversion and CRT passes relative to the classical form
    s1_bytes = (16 + planes * N) * (m * k + k * n) + 4 * (m + n)
    s3_bytes = ((1 if fmt == oz.OZ2_PRODUCT_RESIDUE_U8 else 4) * planes * N + 8) * m * n + 4 * (m + n)
    roofline = {"bound": "mfma", "kernel": "gemm_i8_kernel", "achieved": round(gemm_tops, 2),
                "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": round(gemm_tops / INT8_MFMA_PEAK_TOPS, 4),
                "traffic": None, "avg_launch_ms": round(gemm_ms, 4)}
    if strassen:
        # achieved / frac count the INT8 operations the launch executes (what the matrix cores do); the count of
        # Algorithm 1 line 6 as printed, 2 m n k N, over the same time is given beside them
        alg_tops = 2.0 * m * n * k * N / (gemm_ms * 1e-3) / 1e12
        roofline["achieved_as_2mnkN"] = round(alg_tops, 2)
        roofline["frac_as_2mnkN"] = round(alg_tops / INT8_MFMA_PEAK_TOPS, 4)
        roofline["note"] = "achieved counts the INT8 operations executed: 7 half-size products per modulus, 7/8 of 2mnkN"
    if not args.mnk and args.shift_mode == 0 and N == (16 if args.workload == "c4" else cfg["N"][len(cfg["N"]) // 2]):
        # a counter measurement, not made in this run: valid only for the GEMM source it was taken on
        tr = measured_traffic("%s.%s.%s" % (args.workload, "strassen" if strassen else "classical",
                                            "u8" if fmt == oz.OZ2_PRODUCT_RESIDUE_U8 else "int32"))
        if tr:
            roofline["traffic"] = tr["bytes"]
            roofline["traffic_unit"] = ("bytes per launch leaving the L2 (reads %.1f GiB + writes %.1f GiB; algorithmic "
                                        "minimum %g GiB)" % (tr["read_GiB"], tr["written_GiB"], tr["algorithmic_GiB"]))
            roofline["traffic_source"] = tr["source"]
        else:
            roofline["traffic_source"] = "none for this build (profiles/gemm_hbm_traffic.txt names another GEMM source or has no entry)"
    # The memory-bound stages: bytes the launches of this form move (the Strassen form writes and reads 7/4 of the
    # plane bytes) and the bytes of the method itself, (16 + N)(mk + kn) for lines 1-5 read twice and (N + 8) mn for
    # lines 8-11, both over the measured stage time and against the HBM peak.  The practical ceiling on this card
    # is what a plain device copy sustains (context.device_copy_GBps_same_gpu, about 0.62 of the peak).
    own1 = (16 + N) * (m * k + k * n) + 4 * (m + n)
    own3 = ((1 if fmt == oz.OZ2_PRODUCT_RESIDUE_U8 else 4) * N + 8) * m * n + 4 * (m + n)
    gbps = lambda b, ms: b / (ms * 1e-3) / 1e9
    stages = {
        "stage1_convert_ms": round(float(avg[0]), 4),
        "stage2_gemm_ms": round(gemm_ms, 4),
        "stage3_crt_ms": round(float(avg[2]), 4),
        "stage1_algorithmic_GBps": round(gbps(s1_bytes, avg[0]), 1),
        "stage3_algorithmic_GBps": round(gbps(s3_bytes, avg[2]), 1),
        "stage1_frac_of_hbm_peak_moved_bytes": round(gbps(s1_bytes, avg[0]) / HBM_PEAK_GBPS, 4),
        "stage3_frac_of_hbm_peak_moved_bytes": round(gbps(s3_bytes, avg[2]) / HBM_PEAK_GBPS, 4),
        "stage1_frac_of_hbm_peak_method_bytes": round(gbps(own1, avg[0]) / HBM_PEAK_GBPS, 4),
        "stage3_frac_of_hbm_peak_method_bytes": round(gbps(own3, avg[2]) / HBM_PEAK_GBPS, 4),
        "hbm_peak_GBps": HBM_PEAK_GBPS,
    }

    out = {
        "metric": "emulated FP64 TFLOPS (2mnk/t) at m=n=k=16384 per #moduli; max rel err",
        "value": round(tflops, 3), "unit": "TFLOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "%s: m=%d n=%d k=%d phi=%g, %d moduli, seed %d" % (args.workload, m, n, k, phi, N, cfg["seed"]),
                   "num_moduli": N, "entry_point": "oz2_dgemm" + (" (HIP graph replay)" if args.graph else ""), "shift_mode": args.shift_mode,
                   "product_format": "uint8 residues" if fmt == oz.OZ2_PRODUCT_RESIDUE_U8 else "int32",
                   "gemm_algorithm": "strassen (one level, in the residue rings)" if strassen else "classical",
                   "workspace_GiB": round(ws.nbytes / 2**30, 2), "host_input_generation_s": round(gen_s, 1)},
        "roofline": roofline, "stages": stages,
        "without_stage_events": {"ms_per_step": round(plain_ms, 4),
                                 "value": round(2.0 * m * n * k / (plain_ms * 1e-3) / 1e12, 3),
                                 "note": "the same K calls timed again with no HIP event recorded between the stages"},
    }

    # accuracy + CPU baseline: the oracle on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        # sample size: about 5e11 residue multiply-adds for the oracle (10-20 s on 16 cores)
        nr = 1
        while 2 * (2 * nr) ** 2 * k * N <= 5.5e11 and 2 * nr <= m:
            nr *= 2
        nc = min(n, 2 * nr)
        print("bench: oracle on a %d x %d sample of C ..." % (nr, nc), file=sys.stderr, flush=True)
        rng = np.random.default_rng(1)
        rows = np.sort(rng.choice(m, size=min(nr, m), replace=False))
        cols = np.sort(rng.choice(n, size=min(nc, n), replace=False))
        Asub = np.asfortranarray(A[rows, :])
        Bsub = np.asfortranarray(B[:, cols])
        t0 = time.perf_counter()
        if args.shift_mode == 2:   # the shifts of this mode depend on every row and column
            ref = orc.dgemm(A, B, N, rows=rows, cols=cols, mode=2).C
        else:
            ref = orc.dgemm(Asub, Bsub, N, mode=args.shift_mode).C
        cpu_s = time.perf_counter() - t0
        Cx, S = orc.exact(Asub, Bsub)
        got = dC[torch.from_numpy(rows).to(dev)][:, torch.from_numpy(cols).to(dev)].cpu().numpy()
        out["cpu_baseline"] = {
            "value": round(2.0 * len(rows) * len(cols) * k / cpu_s / 1e12, 6), "unit": "TFLOPS",
            "cores": min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))),
            "kind": "oracle",
            "sample": "%d random rows x %d random columns of C, full k=%d, %d moduli: %.1f s" % (len(rows), len(cols), k, N, cpu_s),
        }
        out["accuracy"] = {
            "max_abs_diff_vs_oracle_over_absAabsB": float(np.max(np.abs(got - ref) / S)),
            "bit_identical_with_oracle": bool(np.array_equal(got, ref)),
            "max_componentwise_err_vs_exact": float(np.max(np.abs(got - Cx) / S)),
            "max_rel_err_vs_exact": float(np.max(np.abs(got - Cx) / np.maximum(np.abs(Cx), 1e-300))),
        }

    # the metric is quoted per number of moduli: same workload, N = 14 .. 18 (a few calls each, outside the
    # timed region of the headline number above)
    if args.workload == "c4" and not args.no_context and not args.mnk:
        per_n, err_n = {}, {}
        for Nx in (14, 15, 17, 18):
            del ws
            ws = oz.Workspace(m, n, k, Nx, device=dev, product_format=fmt)
            ms_n = timed_ms(lambda: oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, Nx, stream))
            per_n[str(Nx)] = round(2.0 * m * n * k / (ms_n * 1e-3) / 1e12, 2)
            if not args.no_cpu_baseline:
                # error of the same sample of C against the exact product (the reference was formed above)
                gx = dC[torch.from_numpy(rows).to(dev)][:, torch.from_numpy(cols).to(dev)].cpu().numpy()
                err_n[str(Nx)] = float(np.max(np.abs(gx - Cx) / S))
        per_n[str(N)] = round(tflops, 2)
        out["emulated_TFLOPS_per_num_moduli"] = dict(sorted(per_n.items()))
        if not args.no_cpu_baseline:
            err_n[str(N)] = out["accuracy"]["max_componentwise_err_vs_exact"]
            out["max_componentwise_err_per_num_moduli"] = dict(sorted(err_n.items()))
        if strassen:
            # the same call with Algorithm 1 line 6 as printed (one full-size INT8 product per modulus)
            oz.oz2_set_gemm_algorithm(oz.OZ2_GEMM_CLASSICAL)
            cl_t = timed_ms(lambda: oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N, stream)) * 1e-3
            oz.oz2_set_gemm_algorithm(args.gemm_algorithm)
            out["classical_form_%d_moduli" % N] = {"ms_per_call": round(cl_t * 1e3, 3),
                                                   "emulated_TFLOPS": round(2.0 * m * n * k / cl_t / 1e12, 2)}
        del ws
        ws = oz.Workspace(m, n, k, N, device=dev, product_format=fmt)
        oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC.data_ptr(), m, N, stream)
        torch.cuda.synchronize()

    # context: the paper's tables time the Cauchy-Schwarz ("fast") and INT8-product ("accu") variants; same
    # workload with 14 moduli in those modes
    if args.workload == "c4" and not args.no_context and args.shift_mode == 0 and not args.no_cpu_baseline and not args.mnk:
        del ws
        ws = oz.Workspace(m, n, k, 14, device=dev, product_format=fmt)
        dC2 = torch.empty((n, m), dtype=torch.float64, device=dev).t()
        for mode, label in ((1, "cauchy_schwarz_mode_14_moduli"), (2, "int8_product_mode_14_moduli")):
            oz.oz2_set_shift_mode(mode)
            mode_t = timed_ms(lambda: oz.oz2_dgemm(m, n, k, dA.data_ptr(), m, dB.data_ptr(), k, dC2.data_ptr(), m, 14, stream)) * 1e-3
            oz.oz2_set_shift_mode(0)
            g2 = dC2[torch.from_numpy(rows).to(dev)][:, torch.from_numpy(cols).to(dev)].cpu().numpy()
            out[label] = {
                "emulated_TFLOPS": round(2.0 * m * n * k / mode_t / 1e12, 2),
                "max_componentwise_err_vs_exact": float(np.max(np.abs(g2 - Cx) / S)),
            }
        del ws
        # context: the symmetric rank-k update A A^T of the same A (half the conversion, about half the tiles);
        # TFLOPS counted with the flops of the full product so that it compares with the lines above
        ws = oz.Workspace(m, m, k, N, device=dev, product_format=fmt)
        dC2 = torch.zeros((m, m), dtype=torch.float64, device=dev).t()
        syrk_t = timed_ms(lambda: oz.oz2_dsyrk("L", "N", m, k, 1.0, dA.data_ptr(), m, 0.0, dC2.data_ptr(), m, N, stream)) * 1e-3
        out["dsyrk_lower_%d_moduli" % N] = {"ms_per_call": round(syrk_t * 1e3, 3),
                                            "TFLOPS_as_full_product": round(2.0 * m * m * k / syrk_t / 1e12, 2)}
        # context: the triangular product B := A_lower * B in place (same sizes; half of the inner dimension
        # is zero by structure)
        if m == k:
            dB2 = dB.clone()
            trmm_t = timed_ms(lambda: oz.oz2_dtrmm("L", "L", "N", "N", m, n, 1.0, dA.data_ptr(), m, dB2.data_ptr(), k, N, stream)) * 1e-3
            out["dtrmm_left_lower_%d_moduli" % N] = {"ms_per_call": round(trmm_t * 1e3, 3),
                                                     "TFLOPS_as_full_product": round(2.0 * m * n * k / trmm_t / 1e12, 2)}
            del dB2
        del dC2, ws
        ws = oz.Workspace(m, n, k, N, device=dev, product_format=fmt)

    if args.calibrate_copy:
        tmp = torch.empty_like(dA)
        tmp.copy_(dA)   # 8*m*k bytes read, 8*m*k bytes written
        torch.cuda.synchronize()
        del tmp

    if not args.no_context:
        # context only: native FP64 GEMM of the same shape on the same GPU
        torch.matmul(dA, dB)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            Cn = torch.matmul(dA, dB)
        e1.record()
        torch.cuda.synchronize()
        nat_ms = e0.elapsed_time(e1) / 3
        out["context"] = {"native_fp64_gemm_TFLOPS_same_gpu": round(2.0 * m * n * k / (nat_ms * 1e-3) / 1e12, 2),
                          "paper_GH200_OSII_fast_16_n16384_TFLOPS": 70.4, "paper_GH200_DGEMM_n16384_TFLOPS": 60.9}
        # context only: what a plain device copy of A (read 8mk bytes, write 8mk bytes) sustains on this card, the
        # practical ceiling for the memory-bound stages
        tmp = torch.empty_like(dA)
        tmp.copy_(dA)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            tmp.copy_(dA)
        e1.record()
        torch.cuda.synchronize()
        out["context"]["device_copy_GBps_same_gpu"] = round(2 * 8.0 * m * k / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e9, 1)
        del tmp
        # context only: the vendor library's INT8 GEMM with INT32 output on one plane of the same shape (random
        # bytes, both operands with the inner dimension contiguous: its faster layout)
        try:
            ia = torch.randint(-128, 128, (m, k), dtype=torch.int8, device=dev)
            ib = torch.randint(-128, 128, (n, k), dtype=torch.int8, device=dev).t()
            torch._int_mm(ia, ib)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(3):
                torch._int_mm(ia, ib)
            e1.record()
            torch.cuda.synchronize()
            out["context"]["vendor_int8_gemm_TOPs_same_gpu"] = round(2.0 * m * n * k / (e0.elapsed_time(e1) / 3 * 1e-3) / 1e12, 1)
            del ia, ib
        except Exception:   # not every build of the framework carries this routine
            pass
        sink = torch.empty(512 * 256, dtype=torch.int32, device=dev)
        clocks = torch.zeros(2, dtype=torch.int64, device=dev)
        for label, rnd in (("constant", 0), ("random", 1), ("fresh_random", 2)):
            iters = 200000
            oz.oz2_calibrate_mfma(512, 2000, rnd, sink.data_ptr(), clocks.data_ptr(), stream)
            torch.cuda.synchronize()
            e0.record()
            oz.oz2_calibrate_mfma(512, iters, rnd, sink.data_ptr(), clocks.data_ptr(), stream)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            cyc, ref = [int(v) for v in clocks.cpu()]
            out["context"]["mfma_only_%s_operands_TOPs" % label] = round(512 * 4 * iters * 8 * 65536.0 / (ms * 1e-3) / 1e12, 1)
            out["context"]["mfma_only_%s_operands_GHz" % label] = round(cyc / max(ref, 1) * 0.1, 3)
        # the GEMM against what the matrix cores of this card sustain on random INT8 operands with no memory
        # traffic at all (the card is power-capped well below the published peak)
        # (random: two operand fragments reused by every instruction; fresh_random: eight per operand in changing
        # pairs, as in a product, where no instruction finds its operands in the matrix core's input latches)
        cal = out["context"].get("mfma_only_random_operands_TOPs")
        if cal:
            out["roofline"]["frac_of_mfma_only_random_operands"] = round(gemm_tops / cal, 4)
        cal = out["context"].get("mfma_only_fresh_random_operands_TOPs")
        if cal:
            out["roofline"]["frac_of_mfma_only_fresh_random_operands"] = round(gemm_tops / cal, 4)
        if not args.no_cpu_baseline:
            gotn = Cn[torch.from_numpy(rows).to(dev)][:, torch.from_numpy(cols).to(dev)].cpu().numpy()
            out["context"]["native_fp64_max_componentwise_err_vs_exact"] = float(np.max(np.abs(gotn - Cx) / S))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
