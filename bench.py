"""Benchmark of the ADC-scan hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input:
  PQ 8x8 (default workload, BASELINE config 1): tables for 1000 queries, float ADC scan of
  25 M codes, top-100.
The 16x4 Quick-ADC-style pipeline (config 2: tables, qmax pre-scan, 8-bit tables, integer scan
to top-1000, float rerank to top-100) is timed the same way and reported in "pq16x4".
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def read_traffic(name):
    """Per-launch HBM bytes measured with rocprofv3 --pmc, stored as text under profiles/."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def cpu_baseline(codes_h, luts_h, gpu_dist, gpu_ids, sample_q, topk):
    """Time the oracle's scan on the host cores for the first sample_q queries; check the GPU result on them."""
    from oracle import pq_oracle as orc
    threads = orc.set_threads(0)
    luts_s = np.ascontiguousarray(luts_h[:sample_q])
    t0 = time.perf_counter()
    od, oi = orc.adc_scan_topk_f32(codes_h, orc.CODES_U8, luts_s, topk)
    dt = time.perf_counter() - t0
    ok = bool(np.allclose(gpu_dist[:sample_q], od, rtol=1e-5, atol=0) and (gpu_ids[:sample_q] == oi).mean() > 0.98)
    # one thread, for comparison with single-core figures in the literature (a few queries are enough)
    one_q = min(16, sample_q)
    orc.set_threads(1)
    t0 = time.perf_counter()
    orc.adc_scan_topk_f32(codes_h, orc.CODES_U8, np.ascontiguousarray(luts_h[:one_q]), topk)
    dt1 = time.perf_counter() - t0
    orc.set_threads(threads)
    return {"value": codes_h.shape[0] * sample_q / dt / 1e9, "unit": "G codes/s", "cores": threads, "kind": "oracle",
            "sample": f"first {sample_q} of the queries over all {codes_h.shape[0]} codes, {dt:.1f} s wall",
            "gpu_matches_oracle_on_sample": ok,
            "one_core": {"value": codes_h.shape[0] * one_q / dt1 / 1e9, "unit": "G codes/s", "cores": 1,
                         "sample": f"first {one_q} queries, {dt1:.1f} s wall"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--n", type=int, default=25_000_000)
    ap.add_argument("--nq", type=int, default=1000)
    ap.add_argument("--topk", type=int, default=100)
    ap.add_argument("--cand", type=int, default=1000, help="candidates kept by the 16x4 integer scan before the rerank")
    ap.add_argument("--cpu-queries", type=int, default=1000, help="queries of the workload the oracle is timed on")
    ap.add_argument("--skip-16x4", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--skip-streaming", action="store_true")
    ap.add_argument("--ivf", action="store_true", help="also time ivf_adc_search on config 4 (allocates 8 GB of codes)")
    ap.add_argument("--ivf-n", type=int, default=1_000_000_000)
    ap.add_argument("--config3", action="store_true", help="also time config 3 (d=960, 16x8 codes, 1 M codes)")
    ap.add_argument("--encode", action="store_true", help="also time pq_encode (d=128 mixture vectors, 8x8 and 16x4 codebooks)")
    ap.add_argument("--encode-n", type=int, default=4_000_000)
    ap.add_argument("--derived", action="store_true", help="also time pq_derived_search (64-bit codes of four 16-bit indexes, k=65536)")
    ap.add_argument("--derived-r2", type=int, default=10000)
    ap.add_argument("--lut-shapes", action="store_true", help="also time the Tables step alone at the shapes of configs 1, 3, 4")
    ap.add_argument("--streaming-n", type=int, nargs="+", default=[100_000_000, 1_000_000_000])
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain copy kernel of this many MiB (counter calibration under rocprofv3)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1712_02912_amd import binding, datagen

    ctx = binding.Context(0)
    mix = datagen.sift_like()
    queries_h = mix.sample(args.nq, datagen.SEED_QUERIES)
    queries = torch.from_numpy(queries_h).cuda()

    def sync():
        torch.cuda.synchronize()

    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        ctx.pq_calibration_copy(src, dst)
        sync()
        del src, dst

    # ---------------------------------------------------------------- PQ 8x8 float scan
    cb8 = torch.from_numpy(datagen.sampled_codebooks(mix, 8, 256)).cuda()
    codes8_h = datagen.random_codes(args.n, 8)
    codes8 = torch.from_numpy(codes8_h).cuda()
    out = (torch.empty((args.nq, args.topk), dtype=torch.float32, device="cuda"),
           torch.empty((args.nq, args.topk), dtype=torch.int64, device="cuda"))

    def step8():
        luts = ctx.pq_build_luts(queries, cb8)
        ctx.pq_adc_scan_topk(codes8, binding.CODES_U8, luts, args.topk, out=out)
        return luts

    ctx.pq_set_profiling(True)
    for _ in range(args.warmup):
        step8()
    sync()
    # duration of the scan kernel of every timed step, from the HIP events the library records around the
    # launch on its own stream (reading them waits for that step's kernel only)
    kernel_ms = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        luts8 = step8()
        kernel_ms.append(ctx.pq_last_scan_kernel_ms())
    sync()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    scan_ms = float(np.mean(kernel_ms))
    alg_bytes = float(args.n) * 8 * args.nq
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9
    result = {
        "metric": "adc_codes_scanned_per_s", "value": args.n * args.nq / (ms_per_step * 1e-3) / 1e9,
        "unit": "G codes/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "PQ 8x8 float ADC scan (BASELINE config 1): N=%d uniform random codes, %d queries, "
                               "fp32 LUTs 8x256 built each step, top-%d" % (args.n, args.nq, args.topk)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic("scan_f32_pq8x8_config1_pmc.txt"),
                     "kernel": ("scan_tuned_kernel<F32Q_M8 (8x8 float, 8-bit lower bounds, 16 queries per pass), lists for top<=%d, groups of 2 sub-tiles>"
                                if args.nq >= 249 else
                                "scan_tuned_kernel<F32P_M8 (8x8 float, 16-bit lower bounds, 8 queries per pass), lists for top<=%d>")
                               % (128 if args.topk <= 128 else 1024), "kernel_ms": scan_ms,
                     "algorithmic_bytes": alg_bytes,
                     # what binds this kernel: issue slots of the 1024 SIMDs.  One sub-tile of the 16-query loop (128 codes x 16
                     # queries) is 60 three-operand vector instructions (4 cycles each), 4 two-operand ones (2 cycles) and 16
                     # ds_read_b128 (8 SIMD cycles each, measured): 376 cycles; peak = every SIMD issuing all the time at 2.4 GHz
                     "issue_model": ({"bound": "alu", "unit": "G SIMD cycles per launch",
                                      "achieved": args.n * ((args.nq + 15) // 16) / 128 * 376 / 1e9,
                                      "peak": 1024 * scan_ms * 1e-3 * 2.4e9 / 1e9,
                                      "frac": args.n * ((args.nq + 15) // 16) / 128 * 376 / (1024 * scan_ms * 1e-3 * 2.4e9)}
                                     if args.nq >= 249 and args.n >= 65536 else None),
                     "note": "algorithmic bytes = 8 B per code per query pass; one pass over a chunk serves 8 or 16 queries and "
                             "concurrent blocks share chunks through L2, so the HBM bytes really moved (traffic) are far below "
                             "the algorithmic figure and frac exceeds 1; the kernel is bound by LDS reads and vector issue"},
    }

    # ---------------------------------------------------------------- PQ 16x4 Quick-ADC-style pipeline
    if not args.skip_16x4:
        cb16 = torch.from_numpy(datagen.sampled_codebooks(mix, 16, 16)).cuda()
        codes4 = torch.from_numpy(datagen.random_codes(args.n, 8, seed=datagen.SEED_CODES + 1)).cuda()
        fmt = binding.CODES_U4_PACKED

        def step16():
            luts = ctx.pq_build_luts(queries, cb16)
            qmax = ctx.pq_qmax_prescan(codes4, fmt, luts, 2 * args.cand, args.cand)
            qluts, _, _ = ctx.pq_quantize_luts(luts, qmax)
            _, cand = ctx.pq_adc_scan_topk(codes4, fmt, qluts, args.cand)
            return ctx.pq_rerank_f32(codes4, fmt, luts, cand, args.topk)

        for _ in range(args.warmup):
            step16()
        sync()
        kernel16_ms = []
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step16()
            kernel16_ms.append(ctx.pq_last_scan_kernel_ms())
        sync()
        ms16 = (time.perf_counter() - t0) * 1e3 / args.steps
        scan16_ms = float(np.mean(kernel16_ms))
        ach16 = alg_bytes / (scan16_ms * 1e-3) / 1e9
        result["pq16x4"] = {"value": args.n * args.nq / (ms16 * 1e-3) / 1e9, "unit": "G codes/s", "ms_per_step": ms16,
                            "dtype": "u8 tables, integer sums", "workload": "PQ 16x4 packed codes (BASELINE config 2): "
                            "tables, qmax pre-scan, 8-bit tables, integer scan top-%d, fp32 rerank top-%d" % (args.cand, args.topk),
                            "roofline": {"bound": "hbm", "achieved": ach16, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                         "frac": ach16 / HBM_PEAK_GBS, "kernel": ("scan_tuned_kernel<U4Q_M16 (8-bit lower bounds, 16 queries per pass), lists for top<=%d>" if args.nq >= 249
                                                    else "scan_tuned_kernel<U4_M16, lists for top<=%d>") % (128 if args.cand <= 128 else 1024), "kernel_ms": scan16_ms,
                                         "traffic": read_traffic("scan_u4_pq16x4_config2_pmc.txt")}}
        del codes4

    # ---------------------------------------------------------------- streaming mode (few queries, codes from HBM)
    if not args.skip_streaming:
        stream = {"note": "random 8-byte codes, top-%d; one pass over the codes serves up to 8 queries (16 from 249 queries on); GB/s = code bytes of all "
                          "passes / scan kernel time (with one pass every byte comes from HBM exactly once; with 8 passes the "
                          "concurrent passes share fetches, so the figure is algorithmic); call_ms = whole pq_adc_scan_topk call "
                          "(first bounds, scan, merge); both sizes exceed the 256 MB Infinity Cache" % args.topk, "cases": []}
        for ns in args.streaming_n:
            gen = torch.Generator(device="cuda").manual_seed(datagen.SEED_CODES + 2)
            codes_s = torch.randint(0, 256, (ns, 8), dtype=torch.uint8, device="cuda", generator=gen)
            for nq_s in (1, 8, 64, 256):   # (256 queries: past the streaming shape, 16 queries per pass)
                luts_s = ctx.pq_build_luts(queries[:nq_s].contiguous(), cb8)
                ms, calls = [], []
                for _ in range(4):
                    sync()
                    t0 = time.perf_counter()
                    ctx.pq_adc_scan_topk(codes_s, binding.CODES_U8, luts_s, args.topk)
                    sync()
                    calls.append((time.perf_counter() - t0) * 1e3)
                    ms.append(ctx.pq_last_scan_kernel_ms())
                k_ms = float(np.mean(ms[1:]))
                passes = (nq_s + 15) // 16 if nq_s >= 249 else (nq_s + 7) // 8
                gbs = ns * 8.0 * passes / (k_ms * 1e-3) / 1e9
                stream["cases"].append({"codes": ns, "queries": nq_s, "passes_over_the_codes": passes, "kernel_ms": k_ms,
                                        "call_ms": float(np.median(calls[1:])), "GB/s": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS,
                                        "G codes/s": ns * nq_s / (k_ms * 1e-3) / 1e9})
            del codes_s
        result["streaming_pq8x8"] = stream

    # ---------------------------------------------------------------- config 3 (d=960, 16x8), on request
    if args.config3:
        mix3 = datagen.gist_like()
        q3 = torch.from_numpy(mix3.sample(args.nq, datagen.SEED_QUERIES)).cuda()
        cb3 = torch.from_numpy(datagen.sampled_codebooks(mix3, 16, 256)).cuda()
        n3 = 1_000_000
        codes3 = torch.from_numpy(datagen.random_codes(n3, 16, seed=datagen.SEED_CODES + 4)).cuda()

        def step3():
            l3 = ctx.pq_build_luts(q3, cb3)
            return ctx.pq_adc_scan_topk(codes3, binding.CODES_U8, l3, args.topk)

        step3()
        sync()
        k3 = []
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step3()
            k3.append(ctx.pq_last_scan_kernel_ms())
        sync()
        ms3 = (time.perf_counter() - t0) * 1e3 / args.steps
        result["config3_pq16x8_d960"] = {"workload": "N=%d 16-byte codes, %d queries of d=960, tables 16x256 built each step, top-%d"
                                         % (n3, args.nq, args.topk), "ms_per_step": ms3, "scan_kernel_ms": float(np.mean(k3)),
                                         "G codes/s": n3 * args.nq / (ms3 * 1e-3) / 1e9,
                                         "algorithmic GB/s (16 B per code per query)": n3 * 16.0 * args.nq / (float(np.mean(k3)) * 1e-3) / 1e9}

    # ---------------------------------------------------------------- Tables step alone, on request
    if args.lut_shapes:
        shapes = {"config1": (1000, 128, 8, 256), "config3": (1000, 960, 16, 256), "config4_coarse": (10000, 128, 1, 65536),
                  "config4_residual_tables_40k_pairs": (40000, 128, 8, 256)}
        tables = {}
        gen = torch.Generator(device="cuda").manual_seed(datagen.SEED_DATA + 9)
        for name, (nq_t, d_t, m_t, k_t) in shapes.items():
            q_t = torch.rand((nq_t, d_t), device="cuda", generator=gen)
            cb_t = torch.rand((m_t, k_t, d_t // m_t), device="cuda", generator=gen)
            ctx.pq_build_luts(q_t, cb_t)
            sync()
            t0 = time.perf_counter()
            for _ in range(5):
                ctx.pq_build_luts(q_t, cb_t)
            sync()
            ms = (time.perf_counter() - t0) * 1e3 / 5
            tables[name] = {"nq": nq_t, "d": d_t, "m": m_t, "k": k_t, "ms": ms, "TFLOP/s (2*nq*d*k, fp64 MFMA)": 2.0 * nq_t * d_t * k_t / ms / 1e9,
                            "frac_of_fp64_mfma_peak": 2.0 * nq_t * d_t * k_t / ms / 1e9 / 78.6}
        result["tables_step"] = tables

    # ---------------------------------------------------------------- encoder, on request
    if args.encode:
        ne = args.encode_n
        x_e = torch.from_numpy(mix.sample(ne, datagen.SEED_DATA + 11)).cuda()
        enc = {}
        for name, cb_e, fmt_e in (("pq8x8", cb8, binding.CODES_U8),
                                  ("pq16x4", torch.from_numpy(datagen.sampled_codebooks(mix, 16, 16)).cuda(), binding.CODES_U4_PACKED)):
            ctx.pq_encode(x_e, cb_e, fmt_e)
            sync()
            t0 = time.perf_counter()
            for _ in range(3):
                ctx.pq_encode(x_e, cb_e, fmt_e)
            sync()
            ms = (time.perf_counter() - t0) * 1e3 / 3
            flops = 2.0 * ne * 128 * cb_e.shape[1]
            enc[name] = {"vectors": ne, "ms": ms, "M vectors/s": ne / ms / 1e3, "TFLOP/s (2*n*d*k, fp64 MFMA)": flops / ms / 1e9,
                         "frac_of_fp64_mfma_peak": flops / ms / 1e9 / 78.6}
        result["encode"] = enc
        del x_e

    # ---------------------------------------------------------------- derived quantizers, on request
    if args.derived:
        cb16_h, cbar_h = datagen.clustered_codebooks(mix, 4, 65536)
        cb16, cbar = torch.from_numpy(cb16_h).cuda(), torch.from_numpy(cbar_h).cuda()
        gen = torch.Generator(device="cuda").manual_seed(datagen.SEED_CODES + 5)
        codes16 = torch.randint(-32768, 32768, (args.n, 4), dtype=torch.int16, device="cuda", generator=gen)
        times, kms = [], []
        for _ in range(1 + args.steps):
            sync()
            t0 = time.perf_counter()
            _, _, _, ncand, _ = ctx.pq_derived_search(codes16, cbar, cb16, queries, args.derived_r2, args.topk)
            sync()
            times.append((time.perf_counter() - t0) * 1e3)
            kms.append(ctx.pq_last_scan_kernel_ms())
        ms_d = float(np.mean(times[1:]))
        result["derived_pq4x8_16"] = {
            "workload": "N=%d codes of four 16-bit indexes (k=65536, derived 8-bit quantizers), %d queries, r2=%d, top-%d"
                        % (args.n, args.nq, args.derived_r2, args.topk),
            "ms_per_call": ms_d, "counting_pass_kernel_ms": float(np.mean(kms[1:])),
            "G codes/s": args.n * args.nq / (ms_d * 1e-3) / 1e9,
            "candidates_per_query_mean": float(ncand.double().mean().item()),
            "algorithmic GB/s (8 B per code per query, one pass)": args.n * 8.0 * args.nq / (ms_d * 1e-3) / 1e9}
        del codes16, cb16

    # ---------------------------------------------------------------- IVF-ADC (BASELINE config 4), on request
    if args.ivf:
        nt, nlist, nq_i, nprobe = args.ivf_n, 65536, 10000, 64
        coarse = torch.from_numpy(mix.sample(nlist, datagen.SEED_DATA + 7)).cuda()
        sizes = datagen.zipf_list_sizes(nt, nlist)
        offsets = torch.from_numpy(datagen.offsets_from_sizes(sizes)).cuda()
        gen = torch.Generator(device="cuda").manual_seed(datagen.SEED_CODES + 3)
        codes_i = torch.randint(0, 256, (nt, 8), dtype=torch.uint8, device="cuda", generator=gen)
        cb_r = cb8 * 0.25   # residual codebooks: same shape, smaller scale
        q_i = torch.from_numpy(mix.sample(nq_i, datagen.SEED_QUERIES + 1)).cuda()
        times = []
        for _ in range(3):
            sync()
            t0 = time.perf_counter()
            _, _, probes = ctx.ivf_adc_search(coarse, offsets, codes_i, None, cb_r, binding.CODES_U8, q_i, nprobe, args.topk,
                                              return_probes=True)
            sync()
            times.append((time.perf_counter() - t0) * 1e3)
        scanned = int(torch.from_numpy(sizes).cuda()[probes.long()].sum().item())
        result["ivf_config4"] = {"workload": "N=%d codes in %d Zipf-sized lists, %d queries, nprobe %d, top-%d" %
                                 (nt, nlist, nq_i, nprobe, args.topk), "ms_per_call": min(times[1:]),
                                 "code_query_pairs": scanned, "G codes/s": scanned / (min(times[1:]) * 1e-3) / 1e9}
        del codes_i

    # ---------------------------------------------------------------- oracle on the host cores
    if not args.skip_cpu:
        sync()
        result["cpu_baseline"] = cpu_baseline(codes8_h, luts8.cpu().numpy(), out[0].cpu().numpy(), out[1].cpu().numpy(),
                                              min(args.cpu_queries, args.nq), args.topk)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
