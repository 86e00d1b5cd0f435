#!/usr/bin/env python3
"""Benchmark of the MI355X W4A8 MSQ linear path (one GPU).

A step is one pass of the whole hot path over one batch of the Qwen2-VL-7B
shaped prefill workload (T = 1280 tokens, 1024 visual in one span): the AIFS
mask remap and the standalone row permute of the [T, 3584] embeddings once,
then for each of the four decoder-layer linears (qkv, o, gate_up, down) the
block-Hadamard rotation + modality-specific static int8 quantization (with the
AIFS gather fused in) and the int4 x int8 GEMM with the fused dequant epilogue.
Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is prefill int8 TOPS = 2*T*sum(K*N) / step time.
`roofline` covers the dominant kernel (the MFMA GEMM), its duration measured
with HIP events in a second pass over the same steps (the event pairs themselves
cost idle time, so the pass that gives `value` runs without them).  `decode` reports the weight-streaming
GEMV (T in {1,4,16}) over 28 distinct layers of weights (3.1 GB, more than the
256 MB last-level cache) in GB/s.  `cpu_baseline` times the CPU oracle on a
bounded row sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "W4A8 linear throughput: prefill int8 TOPS (% MFMA peak); decode GB/s (% HBM)"
INT8_MFMA_PEAK_TOPS = 5000.0       # MI355X dense int8, published
HBM_PEAK_GBPS = 8000.0             # MI355X HBM3E, published
FP16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense fp16, published
# HBM-side bytes per GEMM launch (mean of the four launches of a step) from the two rocprofv3
# --pmc runs summarised in profiles/gemm_c1_prefill_hbm_traffic_pmc.md (FETCH_SIZE x 2.000,
# WRITE_SIZE x 1.000, factors from a plain 1 GiB copy; includes the split-K partials of down).  A counter run cannot happen inside
# this script; re-measure when the GEMM kernel or its tile order changes.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = 159.0e6


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--decode-layers", type=int, default=28)
    ap.add_argument("--decode-iters", type=int, default=10)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the attainable-peak probes")
    ap.add_argument("--no-attention", action="store_true", help="skip the attention / RoPE leg")
    ap.add_argument("--no-rms", action="store_true", help="skip the RMS split-path leg")
    ap.add_argument("--no-dynamic", action="store_true", help="skip the per-token dynamic baseline leg")
    ap.add_argument("--no-weight-only", action="store_true", help="skip the weight-only (W4 group 128) leg")
    ap.add_argument("--no-graphs", action="store_true",
                    help="time the decode loop with plain launches instead of one HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (3 launches) so that a counter run "
                         "has a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE with")
    ap.add_argument("--cpu-rows", type=int, default=512,
                    help="rows of the prefill workload the CPU oracle is timed on")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(rows and output channels are independent, so the path would shard along either without a collective)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    from paper_2502_00425_amd import build as hip_build
    hip_build.ensure_fresh()                             # load what is built unless its sources changed
    from paper_2502_00425_amd import binding as mq       # raises if libmquant.so is missing
    from paper_2502_00425_amd import probes
    from paper_2502_00425_amd import workloads as wl

    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------ prefill set-up
    w = wl.workload(1)
    T, B = w.T, w.had_block
    perm, inv, V = mq.aifs_build_perm(T, w.vis_spans)
    permd = dev(perm)
    mask = torch.tril(torch.ones((T, T), dtype=torch.uint8, device="cuda"))
    mask_u = torch.empty_like(mask)
    lin = {}
    for proj, (K, N) in w.projections.items():
        inp = wl.make_linear_inputs(w, proj)
        absmax = torch.zeros(2, dtype=torch.float32, device="cuda")
        mq.hadamard_absmax(dev(inp["calib_vis"]), B, absmax[0:1])
        mq.hadamard_absmax(dev(inp["calib_txt"]), B, absmax[1:2])
        a = absmax.cpu().numpy()
        lin[proj] = {
            "K": K, "N": N, "x": dev(inp["x"]),
            "wp": mq.w4_prepack(dev(inp["w_packed"])), "w_scale": dev(inp["w_scale"]),
            "s_vis": mq.static_scale_from_absmax(a[0], B),
            "s_txt": mq.static_scale_from_absmax(a[1], B),
            "xq": torch.empty((T, K), dtype=torch.int8, device="cuda"),
            "y": torch.empty((T, N), dtype=torch.float16, device="cuda"),
            "host": inp,
        }
        nws = mq.w4a8_workspace_bytes(T, N, K)
        lin[proj]["ws"] = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
    x_embed = lin["qkv"]["x"]
    x_u = torch.empty_like(x_embed)
    gemm_ops = sum(2.0 * T * l["K"] * l["N"] for l in lin.values())

    ev_pairs = []      # (kind, proj, start, end) around kernel launches of the instrumented steps

    def bracket(record, kind, proj, fn):
        if not record:
            fn()
            return
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        ev_pairs.append((kind, proj, e0, e1))

    def step(record: bool):
        mq.aifs_remap_mask(mask, permd, out=mask_u)
        mq.aifs_permute(x_embed, permd, out=x_u)
        for proj, l in lin.items():
            bracket(record, "quant", proj, lambda: mq.hadamard_quant_act(
                l["x"], V, l["s_vis"], l["s_txt"], B, perm_dev=permd, out=l["xq"]))
            bracket(record, "gemm", proj, lambda: mq.w4a8_gemm(
                l["xq"], l["wp"], l["w_scale"], l["N"], V, l["s_vis"], l["s_txt"],
                out=l["y"], workspace=l["ws"]))

    # Timed region 1: exactly `steps` steps, no instrumentation -> value.
    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    plain_ms_per_step = ms_per_step
    # The same steps as replays of one captured HIP graph (what a serving loop would do: the
    # step is a fixed sequence of ten launches on fixed buffers).  `value` is taken from
    # this loop; the plain-launch figure is reported next to it.
    if not args.no_graphs:
        g_step = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_step):
            step(False)
        for _ in range(args.warmup):
            g_step.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g_step.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / args.steps
    tops = gemm_ops / (ms_per_step * 1e-3) / 1e12

    # Timed region 2: the same `steps` steps again with a HIP event pair around every
    # rotate+quant and GEMM launch (an event pair costs about 5 us of idle time around the
    # kernel it brackets, which is why region 1 runs without them).
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()

    per_proj_ms = {p: 0.0 for p in lin}
    fe_ms = 0.0
    for kind, proj, e0, e1 in ev_pairs:
        if kind == "gemm":
            per_proj_ms[proj] += e0.elapsed_time(e1)
        else:
            fe_ms += e0.elapsed_time(e1)
    for p in per_proj_ms:
        per_proj_ms[p] /= args.steps
    fe_ms /= args.steps
    gemm_ms = sum(per_proj_ms.values())
    n_launch = len(lin)
    gemm_tops = gemm_ops / (gemm_ms * 1e-3) / 1e12
    breakdown = {p: {"gemm_us": round(per_proj_ms[p] * 1e3, 2),
                     "tops": round(2.0 * T * lin[p]["K"] * lin[p]["N"] / (per_proj_ms[p] * 1e-3) / 1e12, 1)}
                 for p in lin}
    fe_bytes = sum(3.0 * T * l["K"] for l in lin.values())
    # Front end on its own: the four rotate+quant launches back to back inside one HIP graph
    # (event pairs around 6-20 us kernels mostly measure the events).
    def fe_pass():
        for _ in range(10):
            for proj, l in lin.items():
                mq.hadamard_quant_act(l["x"], V, l["s_vis"], l["s_txt"], B, perm_dev=permd, out=l["xq"])
    fe_event_ms = fe_ms
    if not args.no_graphs:
        fe_pass()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fe_pass()
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            g.replay()
        torch.cuda.synchronize()
        fe_ms = (time.perf_counter() - t0) * 1e3 / 50

    result = {
        "metric": METRIC, "value": round(tops, 2), "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_plain_launches": round(plain_ms_per_step, 4),
        "launch": "plain" if args.no_graphs else "one HIP graph per step",
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8 x int4 -> int32 (fp16 in/out)", "data": "synthetic",
        "config": {"workload": "configs[1]: Qwen2-VL-7B-shaped prefill, T=1280 (1024 visual at 16), "
                               "qkv 3584x4608, o 3584x3584, gate_up 3584x37888, down 18944x3584, "
                               "block-Hadamard 512",
                   "T": T, "n_vis": V, "had_block": B},
        "roofline": {
            "bound": "mfma", "kernel": "w4a8_gemm_kernel",
            "achieved": round(gemm_tops, 1), "peak": INT8_MFMA_PEAK_TOPS,
            "unit": "TOP/s", "frac": round(gemm_tops / INT8_MFMA_PEAK_TOPS, 4),
            "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH,
            "algorithmic_bytes_per_launch": sum(l["K"] * l["N"] / 2 + T * l["K"] + 2 * T * l["N"] + 2 * l["N"]
                                                for l in lin.values()) / n_launch,
            "avg_launch_us": round(gemm_ms * 1e3 / n_launch, 2),
            "ops_per_launch_avg": gemm_ops / n_launch,
            "per_projection": breakdown,
        },
        "front_end": {"kernel": "hadamard_quant_kernel", "bound": "hbm",
                      "us_per_step": round(fe_ms * 1e3, 2),
                      "GBps": round(fe_bytes / (fe_ms * 1e-3) / 1e9, 1),
                      "frac": round(fe_bytes / (fe_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
    }

    # ------------------------------------------------- attainable peaks, measured live
    # What this machine reaches on the two bounding resources: an MFMA-only int8 loop on random
    # operands (the matrix clock drops under data-dependent power; zeros for comparison) and a
    # read-only stream over 2 GiB.  The published peaks stay the denominators of `frac`.
    if not args.no_probes:
        def timed_once(fn, reps=3):
            fn()
            torch.cuda.synchronize()
            best = float("inf")
            for _ in range(reps):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                e1.synchronize()
                best = min(best, e0.elapsed_time(e1))
            return best
        gen_p = torch.Generator(device="cuda")
        gen_p.manual_seed(5000)
        rnd = torch.randint(0, 256, (1 << 16,), dtype=torch.uint8, device="cuda", generator=gen_p)
        zer = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        iters = 20000
        ops = float(probes.mfma_i8(iters, rnd, sink))
        att = {"mfma_i8_random_operands_TOPS": round(ops / timed_once(lambda: probes.mfma_i8(iters, rnd, sink)) / 1e9, 1),
               "mfma_i8_zero_operands_TOPS": round(ops / timed_once(lambda: probes.mfma_i8(iters, zer, sink)) / 1e9, 1)}
        big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
        nbytes = float(probes.hbm_read(big, sink))
        att["hbm_read_GBps"] = round(nbytes / timed_once(lambda: probes.hbm_read(big, sink)) / 1e6, 1)
        del big
        torch.cuda.empty_cache()
        result["attainable"] = att
        result["roofline"]["frac_of_attainable"] = round(gemm_tops / att["mfma_i8_random_operands_TOPS"], 4)

    # ------------------------------------------- per-token dynamic baseline (context)
    # The scheme the paper's speed tables compare against: same rotation, same GEMM, but
    # one scale per token found at run time and applied per row in the epilogue.
    if not args.no_dynamic:
        row_scale = torch.empty((T,), dtype=torch.float32, device="cuda")

        def dyn_step():
            mq.aifs_remap_mask(mask, permd, out=mask_u)
            mq.aifs_permute(x_embed, permd, out=x_u)
            for proj, l in lin.items():
                mq.hadamard_dynquant_act(l["x"], B, perm_dev=permd, out=l["xq"], row_scale=row_scale)
                mq.w4a8_gemm_rowscale(l["xq"], l["wp"], l["w_scale"], row_scale, l["N"],
                                      out=l["y"], workspace=l["ws"])

        def dyn_fe_pass():
            for _ in range(10):
                for proj, l in lin.items():
                    mq.hadamard_dynquant_act(l["x"], B, perm_dev=permd, out=l["xq"], row_scale=row_scale)

        # The two schemes differ by a few percent, less than the clock drift between two
        # separately timed regions: time them in alternating blocks and compare block means.
        def timed(fn, n):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / n

        for _ in range(args.warmup):
            dyn_step()
        blocks, per_block = 6, max(args.steps // 5, 5)
        st_ms, dy_ms = [], []
        for _ in range(blocks):
            st_ms.append(timed(lambda: step(False), per_block))
            dy_ms.append(timed(dyn_step, per_block))
        dyn_ms, stat_ms = sum(dy_ms) / blocks, sum(st_ms) / blocks
        dyn = {"scheme": "A8 per-token dynamic, W4 per-channel static (same rotation and GEMM kernels)",
               "ms_per_step": round(dyn_ms, 4), "TOPS": round(gemm_ops / (dyn_ms * 1e-3) / 1e12, 2),
               "static_ms_per_step_interleaved": round(stat_ms, 4),
               "static_over_dynamic_speedup": round(dyn_ms / stat_ms, 4)}
        if not args.no_graphs:
            dyn_fe_pass()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                dyn_fe_pass()
            g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                g.replay()
            torch.cuda.synchronize()
            dyn_fe_ms = (time.perf_counter() - t0) * 1e3 / 50
            dyn["front_end_us_per_step"] = round(dyn_fe_ms * 1e3, 2)
            dyn["front_end_GBps"] = round((fe_bytes + 4.0 * T * len(lin)) / (dyn_fe_ms * 1e-3) / 1e9, 1)
        result["dynamic_baseline"] = dyn

    # --------------------------------------- RMS split path on the down projection (context)
    # Main GEMM plus the split GEMV of the flagged channels fused into its epilogue, for one
    # flagged channel (the paper's 1/18944 case) and for one per Hadamard block.
    if not args.no_rms:
        l = lin["down"]
        gen = torch.Generator(device="cuda")
        gen.manual_seed(77)

        def timed_launches(fn, n=20):
            # n launches inside one HIP graph: the Python side of the split call (array
            # marshalling) costs more than the kernels differ by
            fn()
            torch.cuda.synchronize()
            run, reps = fn, n
            if not args.no_graphs:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    for _ in range(n):
                        fn()
                run, reps = g.replay, 1
                run()
                torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                run()
            e1.record()
            e1.synchronize()
            return e0.elapsed_time(e1) * 1e3 / n

        rms = {"projection": "down 18944x3584, T=%d" % T}
        variants = {"plain_us": lambda: mq.w4a8_gemm(
            l["xq"], l["wp"], l["w_scale"], l["N"], V, l["s_vis"], l["s_txt"], out=l["y"],
            workspace=l["ws"])}
        for n_split in (1, l["K"] // B):
            idx = np.arange(n_split, dtype=np.int32) * B
            sw = torch.randint(-8, 8, (n_split, l["N"]), dtype=torch.int8, device="cuda", generator=gen)
            ss = np.linspace(0.05, 0.35, n_split, dtype=np.float32)
            variants["split_%d_us" % n_split] = (lambda idx=idx, sw=sw, ss=ss: mq.w4a8_gemm_rms(
                l["xq"], l["wp"], l["w_scale"], l["N"], V, l["s_vis"], l["s_txt"], idx, sw, ss,
                out=l["y"], workspace=l["ws"]))
        # alternate the variants and keep the best of three rounds each (clock drift between
        # separately timed blocks is of the order of the differences)
        best = {k: float("inf") for k in variants}
        for _ in range(3):
            for k, fn in variants.items():
                best[k] = min(best[k], timed_launches(fn))
        rms.update({k: round(v, 2) for k, v in best.items()})
        result["rms_split"] = rms

    # ----------------------------- AIFS attention + rotary embedding (context, next row 2)
    if not args.no_attention:
        result["attention"] = bench_attention(args, torch, mq, wl, np)

    # ------------------- weight-only W4 group-128 linears on the same shapes (context, next row 4)
    if not args.no_weight_only:
        result["weight_only_g128"] = bench_weight_only(args, torch, mq, lin, T, per_proj_ms)

    # ------------------------------------------------------------------ decode
    if not args.no_decode:
        result["decode"] = bench_decode(args, torch, mq, wl)

    # ------------------------------------------------------------ CPU baseline
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, np, w, lin, V)

    print(json.dumps(result), flush=True)


def bench_weight_only(args, torch, mq, lin, T, w4a8_gemm_ms):
    """The four projections of the prefill workload as weight-only linears: fp16 activations
    straight into an fp16 MFMA GEMM whose weight operand is dequantised (int4, one fp16 scale per
    128 input channels) in registers.  Random codes and scales; no rotation, no quantizer."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(6100)
    out = {"scheme": "W4 group 128, A fp16 (dequantise in registers, fp16 MFMA, fp32 accumulate)",
           "per_projection": {}}
    total_us, flops = 0.0, 0.0
    for proj, l in lin.items():
        K, N = l["K"], l["N"]
        wq = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda", generator=gen)
        sc = (torch.rand((N, K // 128), device="cuda", generator=gen) * 0.008 + 0.002).to(torch.float16)
        wp = mq.w4g128_prepack(wq, sc)
        del wq
        y = l["y"]
        fn = lambda: mq.w4g128_gemm(l["x"], wp, N, out=y)
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                fn()
            e1.record()
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1) * 100.0)      # us per launch
        fl = 2.0 * T * K * N
        out["per_projection"][proj] = {
            "us": round(best, 2), "TFLOPs": round(fl / best / 1e6, 1),
            "w4a8_gemm_us": round(w4a8_gemm_ms[proj] * 1e3, 2)}
        total_us += best
        flops += fl
        del wp
    out["us_per_step"] = round(total_us, 2)
    out["TFLOPs"] = round(flops / total_us / 1e6, 1)
    # decode shape: the same four weight matrices against one token (weight-streaming GEMV)
    dec, dec_us, dec_bytes = {}, 0.0, 0.0
    for proj, l in lin.items():
        K, N = l["K"], l["N"]
        wq = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda", generator=gen)
        sc = (torch.rand((N, K // 128), device="cuda", generator=gen) * 0.008 + 0.002).to(torch.float16)
        wp = mq.w4g128_prepack(wq, sc)
        del wq
        x1 = l["x"][:1]
        y1 = l["y"][:1]
        fn = lambda: mq.w4g128_gemm(x1, wp, N, out=y1)
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                fn()
            e1.record()
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1) * 50.0)
        nbytes = float(wp.numel()) + 2.0 * K + 2.0 * N
        dec[proj] = {"us": round(best, 2), "GBps": round(nbytes / best / 1e3, 1)}
        dec_us += best
        dec_bytes += nbytes
        del wp
    out["decode_T1"] = {"per_projection": dec, "us_per_layer": round(dec_us, 2),
                        "GBps": round(dec_bytes / dec_us / 1e3, 1),
                        "frac_of_hbm_peak": round(dec_bytes / dec_us / 1e3 / HBM_PEAK_GBPS, 4)}
    out["frac_of_fp16_mfma_peak"] = round(flops / total_us / 1e6 / FP16_MFMA_PEAK_TFLOPS, 4)
    out["w4a8_gemm_us_per_step"] = round(sum(w4a8_gemm_ms.values()) * 1e3, 2)
    return out


def bench_attention(args, torch, mq, wl, np):
    """Attention on AIFS-ordered tokens (28 query heads on 4 key/value heads of 128 channels,
    the 7B shapes) for the layouts of configs[1] and configs[2]; q, k, v are column slices of
    one [T, 4608] buffer as the qkv projection leaves them.  Algorithmic flops: 4*D per
    allowed (query, key) pair and query head; peak: dense fp16 MFMA 2.5 PFLOP/s."""
    out = {"unit": "TFLOP/s", "peak": 2500.0, "bound": "mfma (fp16)", "per_config": {}}
    Hq, Hkv, D = 28, 4, 128
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4000)
    for cfg in (1, 2):
        w = wl.workload(cfg)
        T = w.T
        perm, _, V = mq.aifs_build_perm(T, list(w.vis_spans))
        pos = torch.from_numpy(np.ascontiguousarray(perm)).cuda()
        qkv = (torch.randn((T, (Hq + 2 * Hkv) * D), device="cuda", generator=gen) * 0.5).half()
        q, k, v = qkv[:, :Hq * D], qkv[:, Hq * D:(Hq + Hkv) * D], qkv[:, (Hq + Hkv) * D:]
        ws = torch.empty(mq.aifs_attention_workspace_bytes(T, Hkv), dtype=torch.uint8, device="cuda")
        o = torch.empty((T, Hq * D), dtype=torch.float16, device="cuda")

        def timed(fn, n=10):
            fn()
            torch.cuda.synchronize()
            run, reps = fn, n
            if not args.no_graphs:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    for _ in range(n):
                        fn()
                run, reps = g.replay, 1
                run()
                torch.cuda.synchronize()
            best = float("inf")
            for _ in range(3):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    run()
                e1.record()
                e1.synchronize()
                best = min(best, e0.elapsed_time(e1) / n)
            return best

        ms = timed(lambda: mq.aifs_attention(q, k, v, pos, Hq, Hkv, out=o, workspace=ws))
        # the same kernel on tokens in their original order (positions 0..T-1: a plain causal
        # mask): what the reorder costs the attention (the paper's comparison of FlashAttention
        # with and without AIFS)
        pos_plain = torch.arange(T, dtype=torch.int32, device="cuda")
        ms_plain = timed(lambda: mq.aifs_attention(q, k, v, pos_plain, Hq, Hkv, out=o, workspace=ws))
        pairs = T * (T + 1) // 2                      # allowed pairs of a causal mask in any order
        flops = 4.0 * D * pairs * Hq
        ms_rope = timed(lambda: mq.rope_apply(qkv[:, :(Hq + Hkv) * D], pos, Hq + Hkv))
        rope_bytes = 4.0 * T * (Hq + Hkv) * D
        out["per_config"]["configs[%d] T=%d" % (cfg, T)] = {
            "attention_us": round(ms * 1e3, 1), "TFLOPs": round(flops / ms / 1e9, 1),
            "frac": round(flops / ms / 1e9 / 2500.0, 4),
            "plain_causal_order_us": round(ms_plain * 1e3, 1),
            "aifs_overhead": round(ms / ms_plain - 1.0, 4),
            "rope_us": round(ms_rope * 1e3, 2), "rope_GBps": round(rope_bytes / ms_rope / 1e6, 1)}
    return out


def bench_decode(args, torch, mq, wl):
    """GEMV over `decode_layers` distinct layers of 7B weights (uniform random
    int4 nibbles written directly in the streamed layout; the contents do not
    change the traffic) for T in {1, 4, 16}, text rows only."""
    out = {"unit": "GB/s", "peak": HBM_PEAK_GBPS, "layers": args.decode_layers,
           "launch": "plain" if args.no_graphs else "hipGraph", "per_T": {}}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3000)
    streams = [torch.cuda.Stream() for _ in range(4)]
    wd = wl.workload(3, 1)
    layers = []
    for _ in range(args.decode_layers):
        layer = {}
        for proj, (K, N) in wd.projections.items():
            nbytes = mq.w4_prepacked_bytes(N, K)
            wp = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=gen)
            ws = (torch.rand(N, device="cuda", generator=gen) * 0.015 + 0.005).half()
            layer[proj] = (K, N, wp, ws)
        layers.append(layer)
    # The same weights grouped as a decoder layer launches them when q/k/v and gate/up are
    # fused (as in the prefill configuration): qkv N=4608, o, gate_up N=37888, down.  In the
    # streamed layout concatenating along N is concatenating the buffers.
    fused_layers = []
    for layer in layers:
        f = {}
        f["qkv"] = (3584, 4608, torch.cat([layer[p][2] for p in ("q", "k", "v")]),
                    torch.cat([layer[p][3] for p in ("q", "k", "v")]))
        f["o"] = layer["o"]
        f["gate_up"] = (3584, 37888, torch.cat([layer[p][2] for p in ("gate", "up")]),
                        torch.cat([layer[p][3] for p in ("gate", "up")]))
        f["down"] = layer["down"]
        fused_layers.append(f)
    for T in (1, 4, 16):
        xs = {K: torch.randn((T, K), device="cuda", generator=gen).half() for K in (3584, 18944)}
        xq = {K: torch.empty((T, K), dtype=torch.int8, device="cuda") for K in xs}
        ys = {N: torch.empty((T, N), dtype=torch.float16, device="cuda")
              for N in (3584, 512, 18944, 4608, 37888)}
        ys_multi = [{N: torch.empty((T, N), dtype=torch.float16, device="cuda") for N in (3584, 512, 18944)}
                    for _ in range(8)]
        s_txt = 0.035

        def one_pass():
            for layer in layers:
                for proj, (K, N, wp, ws) in layer.items():
                    mq.hadamard_quant_act(xs[K], 0, s_txt, s_txt, 512, out=xq[K])
                    mq.w4a8_gemm(xq[K], wp, ws, N, 0, s_txt, s_txt, out=ys[N])

        def fused_linear_pass():
            # front end inside the GEMV launch (T <= 4): one launch per linear
            for layer in layers:
                for proj, (K, N, wp, ws) in layer.items():
                    mq.w4a8_linear_decode(xs[K], wp, ws, N, 0, s_txt, s_txt, 512, out=ys[N])

        def gemv_only_pass():
            for layer in layers:
                for proj, (K, N, wp, ws) in layer.items():
                    mq.w4a8_gemm(xq[K], wp, ws, N, 0, s_txt, s_txt, out=ys[N])

        def gemv_fused_pass():
            for layer in fused_layers:
                for proj, (K, N, wp, ws) in layer.items():
                    mq.w4a8_gemm(xq[K], wp, ws, N, 0, s_txt, s_txt, out=ys[N])

        def layer_pass():
            # a decoder layer as deployed: q/k/v and gate/up concatenated, one rotate+quant per
            # distinct input (four per layer), four GEMVs
            for layer in fused_layers:
                for proj, (K, N, wp, ws) in layer.items():
                    mq.hadamard_quant_act(xs[K], 0, s_txt, s_txt, 512, out=xq[K])
                    mq.w4a8_gemm(xq[K], wp, ws, N, 0, s_txt, s_txt, out=ys[N])

        def layer_one_launch_pass():
            for layer in fused_layers:
                for proj, (K, N, wp, ws) in layer.items():
                    mq.w4a8_linear_decode(xs[K], wp, ws, N, 0, s_txt, s_txt, 512, out=ys[N])

        def gemv_streams_pass():
            # Kernel throughput when launches overlap: the GEMVs here have no data dependence
            # on each other (own input and output buffers), so four independent stream chains
            # share the pass and join once at its end.  A real decode step is a dependent
            # chain; this leg only shows what the kernel streams when the launch gaps are hidden.
            main = torch.cuda.current_stream()
            for s_ in streams:
                s_.wait_stream(main)
            i = 0
            for layer in layers:
                for proj, (K, N, wp, ws) in layer.items():
                    with torch.cuda.stream(streams[i & 3]):
                        mq.w4a8_gemm(xq[K], wp, ws, N, 0, s_txt, s_txt, out=ys_multi[i % len(ys_multi)][N])
                    i += 1
            for s_ in streams:
                main.wait_stream(s_)

        bytes_layer = sum(K * N / 2 + 2 * N + T * K + 2 * T * N for (K, N) in wd.projections.values())
        res = {}
        legs = [("quant+gemv", one_pass), ("layer_4quant_4gemv", layer_pass)]
        if T <= 4:
            legs.append(("quant+gemv_one_launch", fused_linear_pass))
            legs.append(("layer_4_one_launch_linears", layer_one_launch_pass))
        for name, fn in legs + [("gemv_only", gemv_only_pass),
                         ("gemv_only_fused_qkv_gateup", gemv_fused_pass),
                         ("gemv_only_4streams", gemv_streams_pass)]:
            fn()
            torch.cuda.synchronize()
            if args.no_graphs:
                run = fn
            else:
                # one HIP graph holds the whole 28-layer pass: the Python launch path
                # (several microseconds per call) is otherwise the bound
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    fn()
                run = graph.replay
                run()
                torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.decode_iters):
                run()
            torch.cuda.synchronize()
            ms_layer = (time.perf_counter() - t0) * 1e3 / args.decode_iters / len(layers)
            gbps = bytes_layer / (ms_layer * 1e-3) / 1e9
            res[name] = {"us_per_layer": round(ms_layer * 1e3, 2), "GBps": round(gbps, 1),
                         "frac": round(gbps / HBM_PEAK_GBPS, 4)}
        res["bytes_per_layer"] = bytes_layer
        if T == 1:
            # per projection: the same projection of every layer back to back (distinct weights,
            # so nothing is served from the last-level cache), one HIP graph per projection
            per_proj = {}
            for proj, (K, N) in wd.projections.items():
                def proj_pass(proj=proj, K=K, N=N):
                    for layer in layers:
                        _, _, wp, ws = layer[proj]
                        mq.w4a8_gemm(xq[K], wp, ws, N, 0, s_txt, s_txt, out=ys[N])
                proj_pass()
                torch.cuda.synchronize()
                run = proj_pass
                if not args.no_graphs:
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph):
                        proj_pass()
                    run = graph.replay
                    run()
                    torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.decode_iters):
                    run()
                torch.cuda.synchronize()
                us = (time.perf_counter() - t0) * 1e6 / args.decode_iters / len(layers)
                nbytes = K * N / 2 + 2 * N + T * K + 2 * T * N
                per_proj[proj] = {"us": round(us, 2), "GBps": round(nbytes / us / 1e3, 1),
                                  "frac": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)}
            res["per_projection_gemv"] = per_proj
        out["per_T"][f"T{T}"] = res
    del layers, fused_layers
    out["large_shapes_T1"] = bench_decode_large(args, torch, mq, wl, gen)
    return out


def bench_decode_large(args, torch, mq, wl, gen):
    """The same GEMV on the 72B-class shapes of configs[4] at T=1 (context: on the 7B shapes a
    launch streams for 1-10 us and launch latency is a large share; here a launch streams 30-240
    MB).  Six distinct layers (2.6 GB) defeat the last-level cache; one HIP graph per pass."""
    w4 = wl.workload(4, 1)
    n_layers = 6
    layers = []
    for _ in range(n_layers):
        layer = {}
        for proj, (K, N) in w4.projections.items():
            nbytes = mq.w4_prepacked_bytes(N, K)
            wp = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda", generator=gen)
            ws = (torch.rand(N, device="cuda", generator=gen) * 0.015 + 0.005).half()
            layer[proj] = (K, N, wp, ws)
        layers.append(layer)
    Ks = sorted({K for (K, N) in w4.projections.values()})
    xq = {K: torch.randint(-128, 128, (1, K), dtype=torch.int8, device="cuda", generator=gen) for K in Ks}
    ys = {N: torch.empty((1, N), dtype=torch.float16, device="cuda") for (K, N) in w4.projections.values()}

    def one_pass():
        for layer in layers:
            for proj, (K, N, wp, ws) in layer.items():
                mq.w4a8_gemm(xq[K], wp, ws, N, 0, 0.035, 0.035, out=ys[N])

    one_pass()
    torch.cuda.synchronize()
    if args.no_graphs:
        run = one_pass
    else:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one_pass()
        run = graph.replay
        run()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.decode_iters):
        run()
    torch.cuda.synchronize()
    ms_layer = (time.perf_counter() - t0) * 1e3 / args.decode_iters / n_layers
    bytes_layer = sum(K * N / 2 + 2 * N + K + 2 * N for (K, N) in w4.projections.values())
    gbps = bytes_layer / (ms_layer * 1e-3) / 1e9
    return {"workload": "configs[4] projections (qkv 8192x10240, o 8192x8192, gate_up 8192x59136, "
                        "down 29568x8192), T=1, %d layers" % n_layers,
            "us_per_layer": round(ms_layer * 1e3, 2), "bytes_per_layer": bytes_layer,
            "GBps": round(gbps, 1), "frac": round(gbps / HBM_PEAK_GBPS, 4)}


def cpu_baseline(args, np, w, lin, V):
    """The oracle as it stands, on a row sample of the prefill workload: the
    first cpu_rows/2 visual rows and the first cpu_rows/2 text rows (AIFS
    order) through all four projections, all output channels."""
    from oracle import mquant_oracle as orc
    half = max(args.cpu_rows // 2, 1)
    rows = np.r_[np.arange(0, half), np.arange(V, V + half)]
    ops = 0.0
    t_total = 0.0
    stages = {"permute": 0.0, "rotate_quant": 0.0, "unpack": 0.0, "gemm": 0.0, "dequant": 0.0}
    for proj, l in lin.items():
        inp = l["host"]
        t = time.perf_counter()
        perm, _, V2 = orc.aifs_build_perm(inp["T"], inp["vis_spans"])
        x_u = orc.aifs_permute_rows(inp["x"], perm)[rows]
        stages["permute"] += time.perf_counter() - t
        t = time.perf_counter()
        xq = orc.msq_quantize(orc.hadamard_rotate(x_u, w.had_block), half, l["s_vis"], l["s_txt"], w.had_block)
        stages["rotate_quant"] += time.perf_counter() - t
        t = time.perf_counter()
        wq = orc.unpack_w4(inp["w_packed"])
        stages["unpack"] += time.perf_counter() - t
        t = time.perf_counter()
        acc = orc.gemm_i8_i4_i32(xq, wq)
        stages["gemm"] += time.perf_counter() - t
        t = time.perf_counter()
        orc.dequant(acc, half, l["s_vis"], l["s_txt"], inp["w_scale"])
        stages["dequant"] += time.perf_counter() - t
        ops += 2.0 * len(rows) * l["K"] * l["N"]
    t_total = sum(stages.values())
    return {"value": round(ops / t_total / 1e12, 5), "unit": "TOPS", "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": f"{len(rows)} of {w.T} rows ({half} visual + {half} text) x all channels of the "
                      f"four projections; {round(t_total, 2)} s wall",
            "seconds": round(t_total, 3),
            "stage_seconds": {k: round(v, 3) for k, v in stages.items()}}


if __name__ == "__main__":
    main()
