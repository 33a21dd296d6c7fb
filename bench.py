"""Benchmark of the ADC-scan hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input, inputs resident in HBM:
  headline (BASELINE config 1): tables for 1000 queries + float ADC scan of 25 M 8-byte codes + top-100.
Beside it, each as an object of the same JSON line:
  config1_encoded      the same step on codes encoded from mixture vectors (pq_encode on the GPU);
  pq16x4 / pq16x4_encoded   config 2: tables, qmax pre-scan, 8-bit tables, integer scan top-1000, fp32 rerank top-100;
  streaming_pq8x8 / streaming_pq16x4   few queries over 25 M / 10^8 / 10^9 codes: every byte from HBM once per pass;
  config3_pq16x8_d960  config 3: d = 960, 16 x 256, 1 M encoded codes, 1000 queries (+ the Tables step alone);
  ivf_config4          config 4: 10^9 codes in 65 536 Zipf-sized lists, 10 000 queries, nprobe 64;
  ivf_quick_adc_config4  the same index searched with Quick ADC (16 x 4 codes, 8-bit tables, integer scan, float rerank);
  cpu_baseline         the oracle's scan on the host cores (a bounded sample of config 1).
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
FP64_MFMA_PEAK_TFLOPS = 78.6
# LDS read peak: 256 compute units x 256 bytes per clock (a 16-byte read of a 64-lane wave occupies the LDS of a
# compute unit for 4 clocks) x 2.4 GHz
LDS_PEAK_GBS = 256 * 256 * 2.4


def read_profile_traffic(name):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE) and stored as text under profiles/.
    Returns (bytes or None, description of the source)."""
    path = os.path.join(ROOT, "profiles", name)
    traffic, commit = None, "unknown"
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = float(line.split(":", 1)[1])
                if line.startswith("source_commit:"):
                    commit = line.split(":", 1)[1].strip()
    except OSError:
        return None, None
    if traffic is None:
        return None, None
    return traffic, "profiles/%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of commit %s; not measured in this run)" % (name, commit)


def scan_roofline(n, code_bytes, lookups_per_code, kernel_ms, info, profile):
    """Roofline of a flat scan launch.  Algorithmic bytes = code bytes of every pass over the codes the launched
    kernel makes (a pass serves `queries_per_pass` queries); the LDS figure counts one 16-byte read per lookup."""
    passes = info["passes"]
    alg = float(passes) * n * code_bytes
    sec = kernel_ms * 1e-3
    achieved = alg / sec / 1e9
    traffic, source = read_profile_traffic(profile) if profile else (None, None)
    lds_bytes = float(passes) * n * lookups_per_code * 16.0
    return {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic, "traffic_source": source,
            "hbm_traffic_frac": (traffic / sec / 1e9 / HBM_PEAK_GBS) if traffic else None,
            "kernel": info["kernel"], "kernel_ms": kernel_ms, "queries_per_pass": info["queries_per_pass"],
            "passes_over_the_codes": passes, "algorithmic_bytes": alg,
            "lds": {"bound": "lds", "achieved": lds_bytes / sec / 1e9, "peak": LDS_PEAK_GBS, "unit": "GB/s",
                    "frac": lds_bytes / sec / 1e9 / LDS_PEAK_GBS,
                    "note": "table lookups of the scan loop only: %d reads of 16 bytes per code and pass" % lookups_per_code},
            "note": "algorithmic bytes = code bytes x passes over the codes; when the codes fit the 256 MB Infinity Cache "
                    "(25 M codes = 200 MB) later passes are served from it and the HBM bytes really moved are `traffic`; "
                    "what binds the many-query kernel is LDS reads and vector issue (see `lds`)"}


def pruning_stats(info, n, nq, codes_per_lane=2):
    lanes = float(info["passes"]) * n / codes_per_lane
    return {"parked_lanes": info["parked_lanes"], "share_of_lanes_parked": info["parked_lanes"] / lanes if lanes else None,
            "inserted_keys": info["inserted_keys"], "share_of_pairs_inserted": info["inserted_keys"] / (float(n) * nq)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (after an idle spell the GPU needs some 15 calls, about 45 ms of work, to reach its steady clock: the headline kernel
    # falls from 3.15 to 2.53 ms over them.  The defaults time the steady state; the whole timed region is ~60 ms.)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--n", type=int, default=25_000_000)
    ap.add_argument("--nq", type=int, default=1000)
    ap.add_argument("--topk", type=int, default=100)
    ap.add_argument("--cand", type=int, default=1000, help="candidates kept by the 16x4 integer scan before the rerank")
    ap.add_argument("--cpu-queries", type=int, default=1000, help="queries of the workload the oracle is timed on")
    ap.add_argument("--skip-16x4", action="store_true")
    ap.add_argument("--skip-encoded", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--skip-streaming", action="store_true")
    ap.add_argument("--skip-config3", action="store_true")
    ap.add_argument("--skip-ivf", action="store_true")
    ap.add_argument("--ivf-n", type=int, default=1_000_000_000)
    ap.add_argument("--ivf-cpu-queries", type=int, default=100)
    ap.add_argument("--skip-ivf-quick", action="store_true", help="no Quick ADC leg on config 4's index")
    ap.add_argument("--ivf-quick-only", action="store_true", help="config 4's index searched with Quick ADC only")
    ap.add_argument("--ivf-quick-init", type=int, default=1024, help="codes scanned for the qmax bound of the Quick ADC IVF leg")
    ap.add_argument("--ivf-quick-kprime", type=int, default=128, help="candidates per (query, list) pair of the Quick ADC IVF leg")
    ap.add_argument("--encode", action="store_true", help="also time pq_encode (d=128 mixture vectors, 8x8 and 16x4 codebooks)")
    ap.add_argument("--encode-n", type=int, default=4_000_000)
    ap.add_argument("--derived", action="store_true", help="also time pq_derived_search (64-bit codes of four 16-bit indexes, k=65536)")
    ap.add_argument("--derived-r2", type=int, default=10000)
    ap.add_argument("--lut-shapes", action="store_true", help="also time the Tables step alone at the shapes of configs 1, 3, 4")
    ap.add_argument("--streaming-n", type=int, nargs="+", default=[25_000_000, 100_000_000, 1_000_000_000])
    ap.add_argument("--streaming-queries", type=int, nargs="+", default=None,
                    help="numbers of queries of the streaming cases (default: 1 8 64 256 for 8x8, 1 8 for 16x4)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run one plain copy kernel of this many MiB (counter calibration under rocprofv3)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1712_02912_amd import binding, datagen

    ctx = binding.Context(0)
    ctx.pq_set_profiling(True)
    mix = datagen.sift_like()
    queries_h = mix.sample(args.nq, datagen.SEED_QUERIES)
    queries = torch.from_numpy(queries_h).cuda()
    U8, U4 = binding.CODES_U8, binding.CODES_U4_PACKED

    def sync():
        torch.cuda.synchronize()

    w_aux = max(1, args.warmup // 4)   # warm-up steps of the legs that follow the headline one

    def timed_steps(step, warmup, steps):
        """ms per step (wall clock around `steps` steps, synchronised on both sides), mean duration of the scan kernel
        (HIP events recorded by the library on its stream around every launch) and what that kernel was."""
        for _ in range(warmup):
            step()
        sync()
        kernel_ms = []
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
            kernel_ms.append(ctx.pq_last_scan_kernel_ms())
        sync()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        return ms, float(np.mean(kernel_ms)), ctx.pq_last_scan_info()

    def encoded_codes(cb, fmt, n, seed, mixture=mix, chunk=1 << 20):
        """n mixture vectors drawn on the GPU in chunks and encoded there with pq_encode."""
        m = cb.shape[0]
        out = torch.empty((n, m // 2 if fmt == U4 else m), dtype=torch.uint8, device="cuda")
        for i, a in enumerate(range(0, n, chunk)):
            b = min(n, a + chunk)
            out[a:b] = ctx.pq_encode(mixture.sample_device(b - a, seed + i), cb, fmt)
        sync()
        return out

    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        ctx.pq_calibration_copy(src, dst)
        sync()
        del src, dst

    # ---------------------------------------------------------------- PQ 8x8 float scan (config 1)
    cb8 = torch.from_numpy(datagen.sampled_codebooks(mix, 8, 256)).cuda()
    codes8_h = datagen.random_codes(args.n, 8)
    codes8 = torch.from_numpy(codes8_h).cuda()
    out = (torch.empty((args.nq, args.topk), dtype=torch.float32, device="cuda"),
           torch.empty((args.nq, args.topk), dtype=torch.int64, device="cuda"))
    state = {}

    def step8(codes=codes8):
        state["luts8"] = ctx.pq_build_luts(queries, cb8)
        ctx.pq_adc_scan_topk(codes, U8, state["luts8"], args.topk, out=out)

    ms_per_step, scan_ms, info = timed_steps(step8, args.warmup, args.steps)
    luts8 = state["luts8"]
    gpu_dist8, gpu_ids8 = out[0].cpu().numpy(), out[1].cpu().numpy()
    pairs = float(args.n) * args.nq
    result = {
        "metric": "adc_codes_scanned_per_s", "value": pairs / (ms_per_step * 1e-3) / 1e9,
        "unit": "G codes/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "PQ 8x8 float ADC scan (BASELINE config 1): N=%d uniform random codes, %d queries, "
                               "fp32 LUTs 8x256 built each step, top-%d" % (args.n, args.nq, args.topk)},
        "roofline": scan_roofline(args.n, 8, 8, scan_ms, info, "scan_f32_pq8x8_config1_pmc.txt"),
        "pruning": pruning_stats(info, args.n, args.nq),
    }

    if not args.skip_encoded:
        codes8e = encoded_codes(cb8, U8, args.n, datagen.SEED_DATA + 100)
        ms_e, scan_e, info_e = timed_steps(lambda: step8(codes8e), w_aux, args.steps)
        result["config1_encoded"] = {
            "workload": "as the headline, on codes of N mixture vectors (drawn on the GPU, 64-component mixture as the queries) "
                        "encoded by pq_encode against the same codebooks (256 mixture samples per sub-space)",
            "ms_per_step": ms_e, "value": pairs / (ms_e * 1e-3) / 1e9, "unit": "G codes/s",
            "slowdown_vs_uniform_codes": ms_e / ms_per_step,
            "roofline": scan_roofline(args.n, 8, 8, scan_e, info_e, None), "pruning": pruning_stats(info_e, args.n, args.nq)}
        del codes8e

    # ---------------------------------------------------------------- PQ 16x4 Quick-ADC-style pipeline (config 2)
    cb16 = torch.from_numpy(datagen.sampled_codebooks(mix, 16, 16)).cuda()
    if not args.skip_16x4:
        def make_step16(codes4):
            def step16():
                luts = ctx.pq_build_luts(queries, cb16)
                qmax = ctx.pq_qmax_prescan(codes4, U4, luts, 2 * args.cand, args.cand)
                qluts, _, _ = ctx.pq_quantize_luts(luts, qmax)
                _, cand = ctx.pq_adc_scan_topk(codes4, U4, qluts, args.cand)
                return ctx.pq_rerank_f32(codes4, U4, luts, cand, args.topk)
            return step16

        codes4 = torch.from_numpy(datagen.random_codes(args.n, 8, seed=datagen.SEED_CODES + 1)).cuda()
        ms16, scan16_ms, info16 = timed_steps(make_step16(codes4), args.warmup, args.steps)
        workload16 = ("PQ 16x4 packed codes (BASELINE config 2): tables, qmax pre-scan, 8-bit tables, integer scan top-%d, "
                      "fp32 rerank top-%d" % (args.cand, args.topk))
        result["pq16x4"] = {"value": pairs / (ms16 * 1e-3) / 1e9, "unit": "G codes/s", "ms_per_step": ms16,
                            "dtype": "u8 tables, integer sums", "workload": workload16 + "; uniform random codes",
                            "roofline": scan_roofline(args.n, 8, 8, scan16_ms, info16, "scan_u4_pq16x4_config2_pmc.txt"),
                            "pruning": pruning_stats(info16, args.n, args.nq)}
        del codes4
        if not args.skip_encoded:
            codes4e = encoded_codes(cb16, U4, args.n, datagen.SEED_DATA + 200)
            ms16e, scan16e, info16e = timed_steps(make_step16(codes4e), w_aux, args.steps)
            result["pq16x4_encoded"] = {"value": pairs / (ms16e * 1e-3) / 1e9, "unit": "G codes/s", "ms_per_step": ms16e,
                                        "workload": workload16 + "; codes of N mixture vectors encoded by pq_encode (16 mixture samples per sub-space as codebooks)",
                                        "slowdown_vs_uniform_codes": ms16e / ms16,
                                        "roofline": scan_roofline(args.n, 8, 8, scan16e, info16e, None),
                                        "pruning": pruning_stats(info16e, args.n, args.nq)}
            del codes4e

    # ---------------------------------------------------------------- streaming mode (few queries, codes from HBM)
    if not args.skip_streaming:
        note = ("random 8-byte codes, top-%d; a pass over the codes serves up to 8 queries (16 from 249 queries on); GB/s = code "
                "bytes of all passes / time.  With one pass (1 or 8 queries) every byte is fetched exactly once; 10^8 and 10^9 "
                "codes exceed the 256 MB Infinity Cache, 25 M codes (200 MB) fit it, so their repeated calls are partly served "
                "from it.  kernel_ms = the scan kernel (HIP events on the library's stream); call_ms = the whole "
                "pq_adc_scan_topk call, first kernel to last (events on the same stream): first bounds, scan, merge" % args.topk)
        s8 = {"note": note, "cases": []}
        s16 = {"note": note + "; 16x4: packed 4-bit codes, u8 tables (tables, pre-scan and quantisation outside the call)", "cases": []}
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for ns in args.streaming_n:
            codes_s = datagen.random_codes_device(ns, 8, datagen.SEED_CODES + 2)
            for which, nqs in (("8x8", args.streaming_queries or (1, 8, 64, 256)), ("16x4", args.streaming_queries or (1, 8))):
                if which == "16x4" and args.skip_16x4:
                    continue
                for nq_s in nqs:
                    q_s = queries[:nq_s].contiguous()
                    if which == "8x8":
                        fmt, tabs = U8, ctx.pq_build_luts(q_s, cb8)
                    else:
                        fmt = U4
                        l16 = ctx.pq_build_luts(q_s, cb16)
                        tabs, _, _ = ctx.pq_quantize_luts(l16, ctx.pq_qmax_prescan(codes_s, U4, l16, 2 * args.topk, args.topk))
                    kms, cms = [], []
                    for _ in range(8):
                        sync()
                        ev[0].record()
                        ctx.pq_adc_scan_topk(codes_s, fmt, tabs, args.topk)
                        ev[1].record()
                        sync()
                        cms.append(ev[0].elapsed_time(ev[1]))
                        kms.append(ctx.pq_last_scan_kernel_ms())
                    inf = ctx.pq_last_scan_info()
                    k_ms, c_ms = float(np.mean(kms[3:])), float(np.median(cms[3:]))
                    passes = inf["passes"]
                    gbs_k = ns * 8.0 * passes / (k_ms * 1e-3) / 1e9
                    gbs_c = ns * 8.0 * passes / (c_ms * 1e-3) / 1e9
                    (s8 if which == "8x8" else s16)["cases"].append({
                        "codes": ns, "queries": nq_s, "passes_over_the_codes": passes, "kernel": inf["kernel"],
                        "kernel_ms": k_ms, "call_ms": c_ms, "kernel_GB/s": gbs_k, "kernel_frac_of_hbm_peak": gbs_k / HBM_PEAK_GBS,
                        "call_GB/s": gbs_c, "call_frac_of_hbm_peak": gbs_c / HBM_PEAK_GBS,
                        "every_byte_from_hbm_once": bool(passes == 1 and ns * 8 > (256 << 20)),
                        "G codes/s (call)": ns * nq_s / (c_ms * 1e-3) / 1e9})
            del codes_s
        result["streaming_pq8x8"] = s8
        if not args.skip_16x4:
            result["streaming_pq16x4"] = s16

    # ---------------------------------------------------------------- config 3 (d=960, 16x8, encoded)
    c3 = None
    if not args.skip_config3:
        mix3 = datagen.gist_like()
        q3_h = mix3.sample(args.nq, datagen.SEED_QUERIES)
        q3 = torch.from_numpy(q3_h).cuda()
        cb3 = torch.from_numpy(datagen.sampled_codebooks(mix3, 16, 256)).cuda()
        n3 = 1_000_000
        codes3 = encoded_codes(cb3, U8, n3, datagen.SEED_DATA + 300, mixture=mix3, chunk=1 << 17)

        def step3(codes=codes3):
            state["l3"] = ctx.pq_build_luts(q3, cb3)
            state["r3"] = ctx.pq_adc_scan_topk(codes, U8, state["l3"], args.topk)

        ms3, k3, info3 = timed_steps(step3, w_aux, args.steps)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        tms = []
        for _ in range(6):
            sync()
            ev[0].record()
            ctx.pq_build_luts(q3, cb3)
            ev[1].record()
            sync()
            tms.append(ev[0].elapsed_time(ev[1]))
        t_ms = float(np.median(tms[1:]))
        flops3 = 2.0 * args.nq * 960 * 256
        result["config3_pq16x8_d960"] = {
            "workload": "BASELINE config 3: N=%d 16-byte codes encoded by pq_encode from a 128-component mixture in [0,1]^960, "
                        "%d queries, tables 16x256 built each step, top-%d" % (n3, args.nq, args.topk),
            "ms_per_step": ms3, "value": n3 * float(args.nq) / (ms3 * 1e-3) / 1e9, "unit": "G codes/s",
            "roofline": scan_roofline(n3, 16, 16, k3, info3, None), "pruning": pruning_stats(info3, n3, args.nq, codes_per_lane=1),
            "tables_step": {"ms": t_ms, "TFLOP/s": flops3 / t_ms / 1e9, "bound": "mfma (fp64)", "peak": FP64_MFMA_PEAK_TFLOPS,
                            "frac": flops3 / t_ms / 1e9 / FP64_MFMA_PEAK_TFLOPS, "output_GB/s": args.nq * 16 * 256 * 4 / t_ms / 1e6,
                            "note": "2*nq*d*k = 0.49 GFLOP and 16.4 MB of tables: a launch of ~%d us is bound by its own ramp and by "
                                    "writing the tables, not by the matrix cores" % round(t_ms * 1e3)}}
        c3 = (mix3, q3, cb3, n3)
        del codes3

    # ---------------------------------------------------------------- Tables step alone, on request
    if args.lut_shapes:
        shapes = {"config1": (1000, 128, 8, 256), "config3": (1000, 960, 16, 256), "config4_coarse": (10000, 128, 1, 65536),
                  "config4_residual_tables_640k_pairs": (640000, 128, 8, 256)}
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
                            "frac_of_fp64_mfma_peak": 2.0 * nq_t * d_t * k_t / ms / 1e9 / FP64_MFMA_PEAK_TFLOPS}
        result["tables_step"] = tables

    # ---------------------------------------------------------------- encoder, on request
    if args.encode:
        ne = args.encode_n
        x_e = mix.sample_device(ne, datagen.SEED_DATA + 11)
        enc = {}
        for name, cb_e, fmt_e in (("pq8x8", cb8, U8), ("pq16x4", cb16, U4)):
            ctx.pq_encode(x_e, cb_e, fmt_e)
            sync()
            t0 = time.perf_counter()
            for _ in range(3):
                ctx.pq_encode(x_e, cb_e, fmt_e)
            sync()
            ms = (time.perf_counter() - t0) * 1e3 / 3
            flops = 2.0 * ne * 128 * cb_e.shape[1]
            enc[name] = {"vectors": ne, "ms": ms, "M vectors/s": ne / ms / 1e3, "TFLOP/s (2*n*d*k, fp64 MFMA)": flops / ms / 1e9,
                         "frac_of_fp64_mfma_peak": flops / ms / 1e9 / FP64_MFMA_PEAK_TFLOPS}
        result["encode"] = enc
        del x_e

    # ---------------------------------------------------------------- derived quantizers, on request
    if args.derived:
        cb16_h, cbar_h = datagen.clustered_codebooks(mix, 4, 65536)
        cbd, cbar = torch.from_numpy(cb16_h).cuda(), torch.from_numpy(cbar_h).cuda()
        gen = torch.Generator(device="cuda").manual_seed(datagen.SEED_CODES + 5)
        codes16 = torch.randint(-32768, 32768, (args.n, 4), dtype=torch.int16, device="cuda", generator=gen)
        times, kms = [], []
        for _ in range(1 + args.steps):
            sync()
            t0 = time.perf_counter()
            _, _, _, ncand, _ = ctx.pq_derived_search(codes16, cbar, cbd, queries, args.derived_r2, args.topk)
            sync()
            times.append((time.perf_counter() - t0) * 1e3)
            kms.append(ctx.pq_last_scan_kernel_ms())
        ms_d = float(np.mean(times[1:]))
        result["derived_pq4x8_16"] = {
            "workload": "N=%d codes of four 16-bit indexes (k=65536, derived 8-bit quantizers), %d queries, r2=%d, top-%d"
                        % (args.n, args.nq, args.derived_r2, args.topk),
            "ms_per_call": ms_d, "counting_pass_kernel_ms": float(np.mean(kms[1:])),
            "G codes/s": args.n * args.nq / (ms_d * 1e-3) / 1e9,
            "candidates_per_query_mean": float(ncand.double().mean().item())}
        del codes16, cbd

    # ---------------------------------------------------------------- IVF-ADC (config 4)
    ivf = None
    ivf_quick = None
    if not args.skip_ivf:
        nt, nlist, nq_i, nprobe = args.ivf_n, 65536, 10000, 64
        coarse_h = mix.sample(nlist, datagen.SEED_DATA + 7)
        coarse = torch.from_numpy(coarse_h).cuda()
        sizes = datagen.zipf_list_sizes(nt, nlist)
        offsets_h = datagen.offsets_from_sizes(sizes)
        offsets = torch.from_numpy(offsets_h).cuda()
        codes_i = datagen.random_codes_device(nt, 8, datagen.SEED_CODES + 3)
        cb_r = cb8 * 0.25   # residual codebooks: same shape, smaller scale
        q_i_h = mix.sample(nq_i, datagen.SEED_QUERIES + 1)
        q_i = torch.from_numpy(q_i_h).cuda()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        if not args.ivf_quick_only:
            times, kms = [], []
            for _ in range(6):
                sync()
                ev[0].record()
                d_i, i_i, probes = ctx.ivf_adc_search(coarse, offsets, codes_i, None, cb_r, U8, q_i, nprobe, args.topk, return_probes=True)
                ev[1].record()
                sync()
                times.append(ev[0].elapsed_time(ev[1]))
                kms.append(ctx.pq_last_scan_kernel_ms())
            scanned = int(torch.from_numpy(sizes).cuda()[probes.long()].sum().item())
            ms_i, k_i = float(np.median(times[2:])), float(np.mean(kms[2:]))
            inf_i = ctx.pq_last_scan_info()
            result["ivf_config4"] = {
                "workload": "BASELINE config 4: N=%d uniform random 8-byte codes in %d Zipf-sized lists, %d queries in one call, nprobe %d, "
                            "top-%d" % (nt, nlist, nq_i, nprobe, args.topk),
                "ms_per_call": ms_i, "queries_per_s": nq_i / (ms_i * 1e-3), "code_query_pairs": scanned,
                "value": scanned / (ms_i * 1e-3) / 1e9, "unit": "G codes/s",
                "scan_kernel": inf_i["kernel"], "scan_kernel_ms": k_i, "queries_per_pass_over_a_list": inf_i["queries_per_pass"],
                "scan_kernel_code_bytes_GB/s": scanned * 8.0 / inf_i["queries_per_pass"] / (k_i * 1e-3) / 1e9,
                "scan_kernel_frac_of_hbm_peak": scanned * 8.0 / inf_i["queries_per_pass"] / (k_i * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "note": "scan_kernel_ms covers both scan kernels (long lists, short lists); code bytes they pass = pairs x 8 B / pairs per work "
                        "item (an upper estimate of the sharing: items of a list with fewer probing queries are not full)"}
            ivf = (coarse_h, offsets_h, codes_i, cb_r.cpu().numpy(), q_i_h, probes.cpu().numpy(), d_i.cpu().numpy(), i_i.cpu().numpy(), nprobe)
        # the same index with Quick ADC in the Scan step: the 8 bytes of a code read as 16 packed 4-bit indexes
        cb_q_h = datagen.sampled_codebooks(mix, 16, 16) * np.float32(0.25)
        cb_q = torch.from_numpy(cb_q_h).cuda()
        times, kms = [], []
        for _ in range(0 if args.skip_ivf_quick else 5):
            sync()
            ev[0].record()
            d_k, i_k, probes_k = ctx.ivf_quick_adc_search(coarse, offsets, codes_i, None, cb_q, q_i, nprobe, args.ivf_quick_init,
                                                          args.ivf_quick_kprime, args.topk, return_probes=True)
            ev[1].record()
            sync()
            times.append(ev[0].elapsed_time(ev[1]))
            kms.append(ctx.pq_last_scan_kernel_ms())
        if not args.skip_ivf_quick:
            scanned = int(torch.from_numpy(sizes).cuda()[probes_k.long()].sum().item())
            ms_k, k_k = float(np.median(times[2:])), float(np.mean(kms[2:]))
            inf_k = ctx.pq_last_scan_info()
            result["ivf_quick_adc_config4"] = {
                "workload": "config 4's index with Quick ADC in the Scan step: N=%d packed 16x4 codes (the same 8 bytes per code) in %d "
                            "Zipf-sized lists, %d queries in one call, nprobe %d, init %d, kprime %d, top-%d"
                            % (nt, nlist, nq_i, nprobe, args.ivf_quick_init, args.ivf_quick_kprime, args.topk),
                "ms_per_call": ms_k, "queries_per_s": nq_i / (ms_k * 1e-3), "code_query_pairs": scanned,
                "value": scanned / (ms_k * 1e-3) / 1e9, "unit": "G codes/s",
                "scan_kernel": inf_k["kernel"], "scan_kernel_ms": k_k, "queries_per_pass_over_a_list": inf_k["queries_per_pass"],
                "passes_over_a_list_per_work_item": inf_k["passes"],
                "note": "scan_kernel_ms covers the two integer scan kernels (work items of long and of short lists); every work item reads its "
                        "codes twice (counting pass, collecting pass)"}
            ivf_quick = (coarse_h, offsets_h, codes_i, cb_q_h, q_i_h, probes_k.cpu().numpy(), d_k.cpu().numpy(), i_k.cpu().numpy(), nprobe,
                         args.ivf_quick_init, args.ivf_quick_kprime)

    # ---------------------------------------------------------------- oracle on the host cores
    if not args.skip_cpu:
        sync()
        result["cpu_baseline"] = cpu_baseline(codes8_h, luts8.cpu().numpy(), gpu_dist8, gpu_ids8, min(args.cpu_queries, args.nq), args.topk)
        if c3 is not None:
            result["config3_pq16x8_d960"]["cpu_baseline"] = cpu_baseline_config3(ctx, c3, args.topk)
        if ivf is not None:
            result["ivf_config4"]["cpu_baseline"] = cpu_baseline_ivf(ivf, min(args.ivf_cpu_queries, 10000), args.topk)
        if ivf_quick is not None:
            result["ivf_quick_adc_config4"]["cpu_baseline"] = cpu_baseline_ivf_quick(ivf_quick, min(args.ivf_cpu_queries // 2, 10000), args.topk)
    print(json.dumps(result))


def ids_agree(gpu_ids, orc_ids):
    return bool((gpu_ids == orc_ids).mean() > 0.98)


def cpu_baseline(codes_h, luts_h, gpu_dist, gpu_ids, sample_q, topk):
    """Time the oracle's scan on the host cores for the first sample_q queries; check the GPU result on them."""
    from oracle import pq_oracle as orc
    threads = orc.set_threads(0)
    luts_s = np.ascontiguousarray(luts_h[:sample_q])
    t0 = time.perf_counter()
    od, oi = orc.adc_scan_topk_f32(codes_h, orc.CODES_U8, luts_s, topk)
    dt = time.perf_counter() - t0
    ok = bool(np.allclose(gpu_dist[:sample_q], od, rtol=1e-5, atol=0) and ids_agree(gpu_ids[:sample_q], oi))
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


def cpu_baseline_config3(ctx, c3, topk, sample_q=100):
    """Config 3's shape on the oracle: uniform random 16-byte codes (made by the input generator, so that nothing the
    oracle reads comes from the GPU encoder), tables built by the GPU, first sample_q queries; the GPU scans the same
    input for the comparison."""
    import torch
    from oracle import pq_oracle as orc
    from paper_1712_02912_amd import binding, datagen
    mix3, q3, cb3, n3 = c3
    codes_h = datagen.random_codes(n3, 16, seed=datagen.SEED_CODES + 4)
    luts = ctx.pq_build_luts(q3[:sample_q].contiguous(), cb3)
    gd, gi = ctx.pq_adc_scan_topk(torch.from_numpy(codes_h).cuda(), binding.CODES_U8, luts, topk)
    torch.cuda.synchronize()
    threads = orc.set_threads(0)
    t0 = time.perf_counter()
    od, oi = orc.adc_scan_topk_f32(codes_h, orc.CODES_U8, luts.cpu().numpy(), topk)
    dt = time.perf_counter() - t0
    ok = bool(np.allclose(gd.cpu().numpy(), od, rtol=1e-5, atol=0) and ids_agree(gi.cpu().numpy(), oi))
    return {"value": n3 * sample_q / dt / 1e9, "unit": "G codes/s", "cores": threads, "kind": "oracle",
            "sample": f"{sample_q} queries over {n3} uniform random 16-byte codes, {dt:.1f} s wall", "gpu_matches_oracle_on_sample": ok}


def cpu_baseline_ivf(ivf, sample_q, topk):
    """The oracle's inverted-list scan for the first sample_q queries of config 4, on the lists the GPU probed (their
    codes are copied back from the device-resident array the input generator filled); parity on those queries."""
    from oracle import pq_oracle as orc
    coarse_h, offsets_h, codes_dev, cb_h, q_h, probes, gd, gi, nprobe = ivf
    pr = probes[:sample_q]
    lists = np.unique(pr)
    sizes = (offsets_h[lists + 1] - offsets_h[lists]).astype(np.int64)
    sub_off = np.zeros(len(lists) + 1, np.int64)
    np.cumsum(sizes, out=sub_off[1:])
    sub_codes = np.empty((int(sub_off[-1]), codes_dev.shape[1]), np.uint8)
    sub_ids = np.empty(int(sub_off[-1]), np.int64)
    for j, l in enumerate(lists):
        a, b = int(offsets_h[l]), int(offsets_h[l + 1])
        sub_codes[sub_off[j]:sub_off[j + 1]] = codes_dev[a:b].cpu().numpy()
        sub_ids[sub_off[j]:sub_off[j + 1]] = np.arange(a, b)
    remap = np.searchsorted(lists, pr).astype(np.int32)
    threads = orc.set_threads(0)
    t0 = time.perf_counter()
    od, oi = orc.ivf_scan(q_h[:sample_q], coarse_h[lists], sub_off, sub_codes, sub_ids, cb_h, orc.CODES_U8, remap, topk)
    dt = time.perf_counter() - t0
    pairs = int(sizes[remap].sum())
    ok = bool(np.allclose(gd[:sample_q], od, rtol=1e-5, atol=0) and ids_agree(gi[:sample_q], oi))
    return {"value": pairs / dt / 1e9, "unit": "G codes/s", "cores": threads, "kind": "oracle",
            "sample": f"first {sample_q} of the 10000 queries on the lists the GPU probed ({pairs} code-query pairs, tables on residuals included), {dt:.1f} s wall",
            "queries_per_s": sample_q / dt, "gpu_matches_oracle_on_sample": ok}


def cpu_baseline_ivf_quick(ivf, sample_q, topk):
    """The oracle's IVF search with Quick ADC for the first sample_q queries, on the lists the GPU probed; the GPU's
    distances and ids must equal the oracle's exactly (integer stages, float sums rounded once on both sides)."""
    from oracle import pq_oracle as orc
    coarse_h, offsets_h, codes_dev, cb_h, q_h, probes, gd, gi, nprobe, init, kprime = ivf
    pr = probes[:sample_q]
    lists = np.unique(pr)
    sizes = (offsets_h[lists + 1] - offsets_h[lists]).astype(np.int64)
    sub_off = np.zeros(len(lists) + 1, np.int64)
    np.cumsum(sizes, out=sub_off[1:])
    sub_codes = np.empty((int(sub_off[-1]), codes_dev.shape[1]), np.uint8)
    sub_ids = np.empty(int(sub_off[-1]), np.int64)
    for j, l in enumerate(lists):
        a, b = int(offsets_h[l]), int(offsets_h[l + 1])
        sub_codes[sub_off[j]:sub_off[j + 1]] = codes_dev[a:b].cpu().numpy()
        sub_ids[sub_off[j]:sub_off[j + 1]] = np.arange(a, b)
    remap = np.searchsorted(lists, pr).astype(np.int32)
    threads = orc.set_threads(0)
    t0 = time.perf_counter()
    od, oi = orc.ivf_quick_scan(q_h[:sample_q], coarse_h[lists], sub_off, sub_codes, sub_ids, cb_h, orc.CODES_U4_PACKED, remap, init,
                                kprime, topk)
    dt = time.perf_counter() - t0
    pairs = int(sizes[remap].sum())
    ok = bool(np.array_equal(gd[:sample_q], od) and np.array_equal(gi[:sample_q], oi))
    return {"value": pairs / dt / 1e9, "unit": "G codes/s", "cores": threads, "kind": "oracle",
            "sample": f"first {sample_q} of the 10000 queries on the lists the GPU probed ({pairs} code-query pairs, tables, qmax, 8-bit tables and rerank included), {dt:.1f} s wall",
            "queries_per_s": sample_q / dt, "gpu_matches_oracle_on_sample": ok}


if __name__ == "__main__":
    main()
