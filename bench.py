"""Benchmark of the GEMM lineage on one MI355X.

A step is one launch of the expert lineage state (K4, MFMA) on the headline workload: bf16
8192 x 8192 x 8192, A row-major, B column-major, fp32 accumulation, bf16 output, operands
resident in HBM before the timed region.  The timed region holds exactly --steps launches between
two device synchronisations; every launch is also bracketed by HIP events on the launch stream, and
the roofline figure uses the mean of those per-launch durations.  Operand sets are rotated over
three copies so that no launch finds its inputs in the Infinity Cache left by its predecessor.

The same JSON line carries, under "shapes", the expert state on the other four workloads (each
against its own roofline: HBM for the M=16 shape) and, under "lineage", every state K0..K4 on the
headline workload; under "conv2d" the paper's convolution layer on the same expert kernel and under
"topk" its selection workload; under "cpu_baseline" the CPU oracle timed on a slab of rows of the same product.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM-side bytes per launch of the headline kernel from the FETCH_SIZE / WRITE_SIZE counter runs
# summarised in profiles/gate_counters_all_states.md and profiles/k4_mfma_fast_bf16_C2.md (scaled by the copy probe's factor).  The figure
# belongs to one version of the kernel sources: when their digest differs it is reported as null.
TRAFFIC_C2 = {"bytes": 1.800e9, "sources_sha256": "3b29ea49c1f5bb715cdb578def3c2878910208a31aec4fabab03264613592bdd"}
KERNEL_SOURCES = ["csrc/common.hpp", "csrc/k4_kernels.hpp", "csrc/k4_mfma.hip"]


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2605_28213_amd", rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


PAPER_MM_8192_TFLOPS = 2.0 * 8192 ** 3 / 2.625e-3 / 1e12

PEAK = {"mfma_bf16": 2500.0, "mfma_f16": 2500.0, "mfma_fp8": 5000.0, "mfma_f32": 157.3, "hbm_GBs": 8000.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=25)
    ap.add_argument("--ramp-seconds", type=float, default=3.0,
                    help="untimed launches of the headline kernel for this long before the warm-up (clock ramp from idle)")
    ap.add_argument("--no-extras", action="store_true", help="headline workload only (used for profiling)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU; there is no multi-GPU path to measure (use --gpus 1)")

    import numpy as np
    import torch

    from paper_2605_28213_amd import build as gl_build
    from paper_2605_28213_amd import gemm
    from paper_2605_28213_amd import inputs as gen

    if not os.path.exists(gemm.LIB_PATH):
        gl_build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    NSETS = 3

    def device_sets(cfg, seed=0):
        inp = gen.make_inputs(cfg, seed)
        sets = []
        for _ in range(NSETS):
            A = torch.from_numpy(inp.A.view(np.uint8).reshape(-1)).cuda()
            B = torch.from_numpy(inp.B.view(np.uint8).reshape(-1)).cuda()
            C = torch.empty(max(1, cfg.batch * inp.stride_c) * 4, dtype=torch.uint8, device="cuda")
            sets.append((A, B, C))
        sa = torch.from_numpy(inp.scale_a).cuda() if inp.scale_a is not None else None
        sb = torch.from_numpy(inp.scale_b).cuda() if inp.scale_b is not None else None
        bias = torch.from_numpy(inp.bias).cuda() if inp.bias is not None else None
        d = gemm.make_desc(cfg.M, cfg.N, cfg.K, cfg.in_dtype, cfg.out_dtype, cfg.layout_a, cfg.layout_b,
                           lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=cfg.batch, stride_a=inp.stride_a,
                           stride_b=inp.stride_b, stride_c=inp.stride_c, scale_a=sa, scale_b=sb, bias=bias, stream=stream)
        # lend the scratch K4's packed path asks for (only the ragged fp16 workload needs any)
        need = gemm.gemm_query(gemm.GEMM_K4_MFMA, d, *sets[0]).workspace_bytes if cfg.in_dtype != gen.F32 else 0
        ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
        if ws is not None:
            d.workspace, d.workspace_bytes = ws.data_ptr(), need
        return inp, sets, d, (sa, sb, bias, ws)

    def timed(variant, sets, d, steps, warmup, ramp_s=0.0):
        """Returns (wall seconds for `steps` launches, list of per-launch ms from HIP events, launches of the
        clock-ramp phase).  The ramp phase (headline only) keeps the GPU busy with the same launches for
        `ramp_s` seconds before the warm-up: an idle MI355X sits at a few hundred MHz and takes some tenths
        of a second to reach the clock its power limit allows, far longer than a handful of warm-up launches."""
        ramp_n = 0
        t_ramp = time.perf_counter()
        while time.perf_counter() - t_ramp < ramp_s:
            for i in range(20):
                A, B, C = sets[i % NSETS]
                rc = gemm.gemm_run_ex(variant, d, A, B, C)
                assert rc == gemm.GEMM_OK, gemm.gemm_status_string(rc)
            stream.synchronize()
            ramp_n += 20
        for i in range(warmup):
            A, B, C = sets[i % NSETS]
            rc = gemm.gemm_run_ex(variant, d, A, B, C)
            assert rc == gemm.GEMM_OK, gemm.gemm_status_string(rc)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        rcs = [gemm.GEMM_OK] * steps
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            A, B, C = sets[i % NSETS]
            ev[i][0].record(stream)
            rcs[i] = gemm.gemm_run_ex(variant, d, A, B, C)
            ev[i][1].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        assert all(rc == gemm.GEMM_OK for rc in rcs), "a timed launch failed"
        return wall, [a.elapsed_time(b) for a, b in ev], ramp_n

    def stats(ms):
        s = sorted(ms)
        n = len(s)
        return {"median_us": 1e3 * s[n // 2], "mean_us": 1e3 * sum(s) / n, "min_us": 1e3 * s[0],
                "p10_us": 1e3 * s[n // 10], "p90_us": 1e3 * s[(9 * n) // 10]}

    def roofline_for(cfg, mean_us, bound):
        if bound == "hbm":
            ach = cfg.algorithmic_bytes / (mean_us * 1e-6) / 1e9
            return {"bound": "hbm", "achieved": ach, "peak": PEAK["hbm_GBs"], "unit": "GB/s",
                    "frac": ach / PEAK["hbm_GBs"], "traffic": None}
        peak = PEAK["mfma_fp8"] if cfg.in_dtype == gen.E4M3 else PEAK["mfma_f32"] if cfg.in_dtype == gen.F32 else PEAK["mfma_bf16"]
        ach = cfg.flops / (mean_us * 1e-6) / 1e12
        return {"bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak, "traffic": None}

    # ---- headline: K4 on C2 ------------------------------------------------------------------
    cfg = gen.CONFIGS["C2"]
    inp, sets, d, keep = device_sets(cfg)
    q = gemm.gemm_query(gemm.GEMM_K4_MFMA, d, *sets[0])
    from paper_2605_28213_amd import telemetry
    sampler = telemetry.Sampler(interval=0.01).start()
    t_phase = time.perf_counter()
    wall, ms, ramp_n = timed(gemm.GEMM_K4_MFMA, sets, d, args.steps, args.warmup, ramp_s=args.ramp_seconds)
    t_end = time.perf_counter() - t_phase
    samples = sampler.stop()
    st = stats(ms)
    value = cfg.flops * args.steps / wall / 1e12
    out = {
        "metric": "GEMM TFLOP/s of the expert lineage state (K4 MFMA) on bf16 8192^3; per-shape roofline fractions under 'shapes'",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * wall / args.steps, "higher_is_better": True, "scaling": "weak",
        # the paper's only figure for this shape and dtype: held-out MM 8192^3 bf16, 2.625 ms (TileLang +cfg)
        # on an RTX PRO 6000 Blackwell (App. D) = 418.9 TFLOP/s.  Another machine's number: context, not a target.
        "vs_baseline": value / PAPER_MM_8192_TFLOPS,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C2: bf16 GEMM M=N=K=8192, A row-major, B column-major, N(0,1)/sqrt(K), fp32 accumulate, bf16 out",
                   "variant": gemm.gemm_variant_name(gemm.GEMM_K4_MFMA), "path": q.path,
                   "tile": [q.bm, q.bn, q.bk], "threads": q.threads, "grid": q.grid,
                   "cache_state": f"operands rotated over {NSETS} buffer sets"},
        "launch_us": st,
        "roofline": roofline_for(cfg, st["mean_us"], "mfma"),
        "clock_ramp": {"seconds": args.ramp_seconds, "launches": ramp_n,
                       "what": "untimed launches of the same kernel before the warm-up, so that the timed steps do not run on a clock still rising from idle"},
    }
    # launch statistics of the timed steps (the first five apart: a clock still ramping would show there)
    out["roofline"]["launch_stats_us"] = {"min": st["min_us"], "median": st["median_us"], "p90": st["p90_us"], "mean": st["mean_us"],
                                          "first_five": [1e3 * x for x in ms[:5]]}
    # socket power and shader clock sampled over the timed steps and the last half second before them
    win = [x for x in samples if x[0] >= t_end - wall - 0.5]
    ps = telemetry.Sampler.summary(win)
    out["roofline"]["power"] = {"cap_w": sampler.power_cap_w(), "socket_w_mean": ps["power_w_mean"], "socket_w_max": ps["power_w_max"],
                                "sclk_mhz_mean": ps["sclk_mhz_mean"], "sclk_mhz_min": ps["sclk_mhz_min"], "samples": ps["samples"],
                                "source": "hwmon power1_input and pp_dpm_sclk, sampled every 10 ms"}
    if kernel_sources_digest() == TRAFFIC_C2["sources_sha256"]:
        out["roofline"]["traffic"] = TRAFFIC_C2["bytes"]

    if not args.no_extras:
        # ---- the lineage on the headline workload (few launches for the slow early states) ---------
        lineage = {}
        for v in range(gemm.gemm_variant_count()):
            n = 2 if v == 0 else 10
            _, vms, _ = timed(v, sets, d, n, 1)
            m = sorted(vms)[len(vms) // 2]
            lineage[gemm.gemm_variant_name(v)] = {"median_us": 1e3 * m, "TFLOP/s": cfg.flops / (m * 1e-3) / 1e12,
                                                  "path": gemm.gemm_query(v, d, *sets[0]).path, "launches": n}
        out["lineage"] = lineage
    if not args.no_extras:
        # ---- measured ceilings on this GPU, same session ------------------------------------------
        # matrix pipe: register-resident loop of the expert kernel's instruction on the headline
        # workload's own operand values (the clock the power limit allows depends on the data)
        def event_times(fn, n, warm):
            for _ in range(warm):
                fn()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            for a, b in ev:
                a.record(stream)
                fn()
                b.record(stream)
            torch.cuda.synchronize()
            return sorted(a.elapsed_time(b) for a, b in ev)

        wgs, iters = 1024, 400
        need = gemm.gemm_probe_mfma_operand_bytes(gemm.GEMM_BF16, wgs)
        sink = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
        A0 = sets[0][0]
        assert A0.numel() >= 2 * need
        flops_box = []

        def mfma_probe():
            rc, fl = gemm.gemm_probe_mfma(gemm.GEMM_BF16, A0, need, wgs, iters, sink, sink.numel() * 4, stream)
            assert rc == gemm.GEMM_OK
            flops_box.append(fl)
        tm = event_times(mfma_probe, 20, 10)
        mf32 = flops_box[-1] / (tm[len(tm) // 2] * 1e-3) / 1e12

        # the instruction the expert kernel uses on this workload (16x16x32), the same operand values
        def mfma16_probe():
            rc, fl = gemm.gemm_probe_mfma16(gemm.GEMM_BF16, A0, 2 * need, wgs, iters // 2, sink, sink.numel() * 4, stream)
            assert rc == gemm.GEMM_OK
            flops_box.append(fl)
        t16 = event_times(mfma16_probe, 20, 10)
        mf = flops_box[-1] / (t16[len(t16) // 2] * 1e-3) / 1e12
        # the same loop on all-zero operands: what the matrix pipe sustains when no operand bit toggles
        Z0 = torch.zeros(need, dtype=torch.uint8, device="cuda")

        def mfma_probe_zeros():
            rc, fl = gemm.gemm_probe_mfma(gemm.GEMM_BF16, Z0, need, wgs, iters, sink, sink.numel() * 4, stream)
            assert rc == gemm.GEMM_OK
            flops_box.append(fl)
        tz = event_times(mfma_probe_zeros, 20, 10)
        mz = flops_box[-1] / (tz[len(tz) // 2] * 1e-3) / 1e12
        big = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        s32 = torch.zeros(4, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        tr = event_times(lambda: gemm.gemm_probe_stream_read(big, big.numel(), s32, stream), 20, 5)
        tc = event_times(lambda: gemm.gemm_probe_copy(dst, big, dst.numel(), stream), 20, 5)
        rd = big.numel() / (tr[len(tr) // 2] * 1e-3) / 1e9
        cp = 2 * dst.numel() / (tc[len(tc) // 2] * 1e-3) / 1e9
        out["ceilings"] = {
            "mfma_bf16_on_headline_operands": {"TFLOP/s": mf, "frac_of_peak": mf / PEAK["mfma_bf16"],
                                               "what": f"{wgs} workgroups x 4 waves x {iters // 2} x 128 v_mfma_f32_16x16x32_bf16 (the expert kernel's instruction here), operands from A"},
            "mfma_bf16_32x32x16_on_headline_operands": {"TFLOP/s": mf32, "frac_of_peak": mf32 / PEAK["mfma_bf16"],
                                                        "what": f"{wgs} workgroups x 4 waves x {iters} x 32 v_mfma_f32_32x32x16_bf16, the same operands and flops"},
            "mfma_bf16_on_zeros": {"TFLOP/s": mz, "frac_of_peak": mz / PEAK["mfma_bf16"],
                                   "what": "the 32x32x16 loop on all-zero operands: the gap to the line above is the clock the chip gives up to data-dependent power"},
            "hbm_stream_read": {"GB/s": rd, "frac_of_peak": rd / PEAK["hbm_GBs"], "what": "512 MiB, 16-byte loads"},
            "hbm_copy": {"GB/s": cp, "frac_of_peak": cp / PEAK["hbm_GBs"], "what": "256 MiB read + 256 MiB written"},
        }
        out["roofline"]["frac_of_measured_mfma_ceiling"] = out["roofline"]["achieved"] / mf
        # The vendor's GEMM on the same operands in the same session, as the paper sets its kernels beside cuBLAS
        # (App. A): torch.mm reaches hipBLASLt / rocBLAS.  Context for the headline number, not part of the path.
        try:
            vs = [(A.view(torch.bfloat16).view(cfg.M, cfg.K), B.view(torch.bfloat16).view(cfg.N, cfg.K).t(),
                   torch.empty(cfg.M, cfg.N, dtype=torch.bfloat16, device="cuda")) for (A, B, _) in sets]
            box = [0]

            def vendor_mm():
                a_, b_, c_ = vs[box[0] % NSETS]
                box[0] += 1
                torch.mm(a_, b_, out=c_)
            with torch.cuda.stream(stream):
                tv = event_times(vendor_mm, 30, 60)
            vm = tv[len(tv) // 2]
            out["ceilings"]["vendor_library_bf16_8192"] = {
                "TFLOP/s": cfg.flops / (vm * 1e-3) / 1e12, "median_us": 1e3 * vm, "frac_of_peak": cfg.flops / (vm * 1e-3) / 1e12 / PEAK["mfma_bf16"],
                "what": "torch.mm (hipBLASLt / rocBLAS) on the headline workload's operands, A row-major, B column-major, rotated over the same 3 sets"}
            del vs
        except Exception as e:      # context only: a vendor library that refuses the call does not fail the bench
            out["ceilings"]["vendor_library_bf16_8192"] = {"error": str(e)[:200]}
        del big, dst, sink, Z0
    del sets, keep
    torch.cuda.empty_cache()

    if not args.no_extras:
        shapes = {}
        # the paper's own numbers for the shapes it shares with this bench (other hardware: context only)
        paper_ms = {"P4096": ("KLineage CUDA, H100 PCIe / RTX PRO 6000, App. A", (0.3130, 0.3681)),
                    "P2048": ("TileLang +cfg, RTX PRO 6000, App. D", (0.074,)),
                    "PBMM16": ("TileLang +cfg, RTX PRO 6000, App. D", (0.703,)),
                    "PBMM32": ("TileLang +cfg, RTX PRO 6000, App. D", (0.226,)),
                    "PADDMM": ("TileLang +cfg, RTX PRO 6000, App. D", (0.375,))}
        for name, bound in (("C1", "mfma"), ("C3", "mfma"), ("C4", "hbm"), ("C5", "mfma"), ("P4096", "mfma"),
                            ("P2048", "mfma"), ("PBMM16", "mfma"), ("PBMM32", "mfma"), ("PADDMM", "mfma"), ("D32", "hbm"), ("D64", "hbm"), ("D128", "hbm"), ("D16_e4m3", "hbm")):
            c = gen.CONFIGS[name]
            v = gemm.GEMM_K4_MFMA
            _, s2, d2, keep2 = device_sets(c)
            _, sms, _ = timed(v, s2, d2, 100, 25, ramp_s=0.3)     # (each shape gets a short clock ramp of its own)
            ss = stats(sms)
            rl = roofline_for(c, ss["mean_us"], bound)
            entry = {"variant": gemm.gemm_variant_name(v), "path": gemm.gemm_query(v, d2, *s2[0]).path,
                     "launch_us": ss, "TFLOP/s": c.flops / (ss["mean_us"] * 1e-6) / 1e12,
                     "GB/s": c.algorithmic_bytes / (ss["mean_us"] * 1e-6) / 1e9, "roofline": rl}
            if name == "C5":
                entry["roofline_hbm"] = roofline_for(c, ss["mean_us"], "hbm")
            if name in paper_ms:
                entry["paper_context"] = {"source": paper_ms[name][0], "latency_ms": list(paper_ms[name][1])}
            if name == "C4" and "ceilings" in out:
                rl["frac_of_measured_stream_read"] = rl["achieved"] / out["ceilings"]["hbm_stream_read"]["GB/s"]
            shapes[name] = entry
            del s2, keep2
            torch.cuda.empty_cache()
        out["shapes"] = shapes

        # ---- the paper's Conv2d layer (Sec. 4.1 workload table) on the lineage's expert state -----------
        from paper_2605_28213_amd import conv
        cc = gen.CONV_CONFIGS["CONV"]
        ci = gen.make_conv_inputs(cc, 0)
        to_dev = lambda a: torch.from_numpy(a.reshape(-1).view(np.uint8).copy()).cuda()
        xs = [to_dev(ci.x) for _ in range(NSETS)]
        wd = to_dev(ci.w)
        yd = torch.empty(cc.N * cc.P * cc.Q * cc.F * gen.ELEM_BYTES[cc.out_dtype], dtype=torch.uint8, device="cuda")
        layer = {}
        for v in (conv.CONV_C1_IM2COL_MFMA, conv.CONV_C2_IMPLICIT_MFMA):
            dd = conv.make_desc(cc.N, cc.H, cc.W, cc.C, cc.F, cc.R, cc.S, cc.in_dtype, cc.out_dtype, stride=cc.stride,
                                pad=cc.pad, stream=stream)
            need = conv.conv2d_query(v, dd, xs[0], wd, yd).workspace_bytes
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
            dd.workspace, dd.workspace_bytes = ws.data_ptr(), need
            k = [0]
            def launch():
                rc = conv.conv2d_run(v, dd, xs[k[0] % NSETS], wd, yd)
                k[0] += 1
                if rc != gemm.GEMM_OK:
                    raise RuntimeError(f"conv2d_run: {gemm.gemm_status_string(rc)}")
            ss = stats(event_times(launch, 100, 25))
            tf = cc.flops / (ss["mean_us"] * 1e-6) / 1e12
            layer[conv.conv2d_variant_name(v)] = {
                "path": conv.conv2d_query(v, dd, xs[0], wd, yd).path, "launch_us": ss,
                "TFLOP/s": tf, "GB/s": cc.algorithmic_bytes / (ss["mean_us"] * 1e-6) / 1e9,
                # 378 flop per algorithmic byte: above the ridge, so the matrix peak is the bound; one round of 196
                # workgroups of 9 K slabs each is latency, not throughput
                "roofline": {"bound": "mfma", "achieved": tf, "peak": PEAK["mfma_bf16"], "unit": "TFLOP/s",
                             "frac": tf / PEAK["mfma_bf16"], "traffic": None}}
            del ws
        layer["workload"] = "fp16 N=8 H=W=56 C=64 F=128 3x3 stride 1 pad 1, NHWC, 3.70 GFLOP, 9.78 MB"
        layer["paper_context"] = {"source": "KLineage CUDA / cuDNN, H100 PCIe and RTX PRO 6000, App. A",
                                  "latency_ms": {"H100 KLineage": 0.0157, "H100 cuDNN": 0.0272, "RTX PRO 6000 KLineage": 0.0235,
                                                 "RTX PRO 6000 cuDNN": 0.0253}}
        out["conv2d"] = layer
        del xs, wd, yd
        torch.cuda.empty_cache()

        # ---- the paper's Top-K shape (Sec. 4.1 workload table): batch 64, 4096 values, k = 512, fp32 ----
        from paper_2605_28213_amd import topk
        tc = gen.TOPK_CONFIGS["TOPK"]
        txs = [torch.from_numpy(gen.make_topk_inputs(tc, 0)).cuda() for _ in range(NSETS)]
        tidx = torch.empty(tc.batch * tc.k, dtype=torch.int32, device="cuda")
        tval = torch.empty(tc.batch * tc.k, dtype=torch.float32, device="cuda")
        td = topk.make_desc(tc.batch, tc.n, tc.k, stream=stream)
        sel = {}
        for v in (topk.TOPK_T1_RADIX_SELECT, topk.TOPK_T2_RESIDENT):
            k = [0]
            def launch_topk():
                rc = topk.topk_run(v, td, txs[k[0] % NSETS], tidx, tval)
                k[0] += 1
                if rc != gemm.GEMM_OK:
                    raise RuntimeError(f"topk_run: {gemm.gemm_status_string(rc)}")
            ss = stats(event_times(launch_topk, 100, 25))
            gbs = tc.algorithmic_bytes / (ss["mean_us"] * 1e-6) / 1e9
            # 1.3 MB in one round of 64 workgroups: far below any bandwidth bound, a chain of passes over a row
            sel[topk.topk_variant_name(v)] = {"path": topk.topk_query(v, td, txs[0]).path, "launch_us": ss, "GB/s": gbs,
                                              "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK["hbm_GBs"], "unit": "GB/s",
                                                           "frac": gbs / PEAK["hbm_GBs"], "traffic": None}}
        sel["workload"] = "fp32 batch 64 x 4096, k = 512, indices + values out, 1.31 MB"
        sel["paper_context"] = {"source": "KLineage CUDA / FlashInfer, H100 PCIe and RTX PRO 6000, App. A",
                                "latency_ms": {"H100 KLineage": 0.0143, "H100 FlashInfer": 0.0160, "RTX PRO 6000 KLineage": 0.0131,
                                               "RTX PRO 6000 FlashInfer": 0.0169}}
        out["topk"] = sel
        del txs, tidx, tval

    if not args.no_cpu:
        # ---- CPU oracle on a bounded sample of the headline workload ---------------------------------
        import oracle
        rows = 4096                      # half of the product: about ten seconds of host time
        t0 = time.perf_counter()
        oracle.gemm(cfg.in_dtype, cfg.layout_a, cfg.layout_b, rows, cfg.N, cfg.K, inp.A[: rows * inp.lda], inp.lda,
                    inp.B, inp.ldb)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * rows * cfg.N * cfg.K / dt / 1e12, "unit": "TFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"first {rows} rows of C of the same product ({rows}x8192x8192), {dt:.1f} s, "
                                         "fp64 triple loop incl. operand decode"}
        # ---- gate pass rate (the other half of the metric): correctness legs against the oracle -------
        # every state on the five reduced workloads at seeds 0..2 (whole product), and the expert state on
        # the five full-size workloads at seed 0 (sampled outputs: random points, first and last row and column)
        from paper_2605_28213_amd import gate
        entries = []

        def whole(c):
            return lambda i: gate.Reference(*oracle.gemm(c.in_dtype, c.layout_a, c.layout_b, c.M, c.N, c.K, i.A, i.lda, i.B, i.ldb,
                                                         batch=c.batch, stride_a=i.stride_a, stride_b=i.stride_b,
                                                         scale_a=i.scale_a, scale_b=i.scale_b, bias=i.bias))

        def sampled(c):
            def ref(i):
                rng = np.random.default_rng(7)
                n = 4000
                pb, pi, pj = rng.integers(0, c.batch, n), rng.integers(0, c.M, n), rng.integers(0, c.N, n)
                pi[:500], pi[500:1000], pj[1000:1500], pj[1500:2000] = 0, c.M - 1, 0, c.N - 1
                pts = (pb.astype(np.int64), pi.astype(np.int64), pj.astype(np.int64))
                C_ref, D = oracle.gemm_points(c.in_dtype, c.layout_a, c.layout_b, c.M, c.N, c.K, i.A, i.lda, i.B, i.ldb, *pts,
                                              batch=c.batch, stride_a=i.stride_a, stride_b=i.stride_b,
                                              scale_a=i.scale_a, scale_b=i.scale_b, bias=i.bias)
                return gate.Reference(C_ref, D, pts)
            return ref
        for name in ("C1", "C2_small", "C3_small", "C4_small", "C5_small"):
            c, cache = gen.CONFIGS[name], {}
            for v in range(gemm.gemm_variant_count()):
                entries.append(gate.run_gate(v, c, whole(c), inputs_cache=cache, reps=5, warmup=1))
        for name in ("C2", "C3", "C4", "C5"):
            c = gen.CONFIGS[name]
            entries.append(gate.run_gate(gemm.GEMM_K4_MFMA, c, sampled(c), seeds=(0,), reps=5, warmup=1))
        pr = gate.pass_rate(entries)
        out["gate"] = {"attempted": pr["attempted"], "passed": pr["passed"], "rate": pr["rate"], "refused": pr["refused"],
                       "what": "(state, workload, seed) correctness legs against the CPU oracle: K0..K4 on C1 and the reduced "
                               "C2..C5 at seeds 0..2 (all outputs), K4 on the full-size C2..C5 at seed 0 (4000 sampled outputs)",
                       "failed": [(e.get("variant_name"), e["workload"], e["verdict"]) for e in entries if e["verdict"] != "passed"]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
