#!/usr/bin/env python3
"""Benchmark of the MI355X W4A8 MSQ linear path (one GPU).

A step is one pass of the whole hot path over one batch of a prefill workload: the AIFS
mask remap and the standalone row permute of the embeddings once, then for each of the four
decoder-layer linears (qkv, o, gate_up, down) the block-Hadamard rotation + modality-specific
static int8 quantization (with the AIFS gather fused in) and the int4 x int8 GEMM with the
fused dequant epilogue.  Inputs are resident in HBM before the timed region.

The headline (`value`, `roofline`) is on configs[4], the largest single-GPU configuration
(72B-class shapes, T = 16384, four visual spans); configs[1] and configs[2] (7B shapes,
T = 1280 and 4096) are reported under `prefill.per_config`, each with its own GEMM roofline.
Every timed figure is the median of `--repeats` (>= 5) timed blocks, with min and max beside
it; a block of the headline is exactly `--steps` steps.

Prints ONE JSON line.  `value` is prefill int8 TOPS = 2*T*sum(K*N) / step time.  `roofline`
covers the dominant kernel (the MFMA GEMM), its launches timed with HIP event pairs on the
launch stream in a second pass over the same steps (the event pairs themselves cost idle time,
so the pass that gives `value` runs without them).  `decode` reports the weight-streaming GEMV
(T in {1,4,16}) over 28 distinct layers of weights (3.1 GB, more than the 256 MB last-level
cache) in GB/s.  `cpu_baseline` times the CPU oracle on the whole of configs[1].
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "W4A8 linear throughput: prefill int8 TOPS (% MFMA peak); decode GB/s (% HBM)"
INT8_MFMA_PEAK_TOPS = 5000.0       # MI355X dense int8, published
HBM_PEAK_GBPS = 8000.0             # MI355X HBM3E, published
FP16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense fp16, published
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "gemm_hbm_traffic.json")

WORKLOAD_TEXT = {
    1: "configs[1]: Qwen2-VL-7B-shaped prefill, T=1280 (1024 visual at 16), qkv 3584x4608, o 3584x3584, "
       "gate_up 3584x37888, down 18944x3584, block-Hadamard 512",
    2: "configs[2]: 7B shapes at long prefill, T=4096 (3584 visual at 256), same four linears, "
       "block-Hadamard 512",
    4: "configs[4]: 72B-class shapes, T=16384 (4 visual spans of 3072 between 5 text spans), qkv 8192x10240, "
       "o 8192x8192, gate_up 8192x59136, down 29568x8192, block-Hadamard 128",
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--repeats", type=int, default=5, help="timed blocks per figure (median reported)")
    ap.add_argument("--headline", type=int, default=4, choices=(1, 2, 4),
                    help="configuration the headline value and roofline are taken on")
    ap.add_argument("--configs", type=str, default="1,2,4",
                    help="prefill configurations to run (the headline one is always run)")
    ap.add_argument("--decode-layers", type=int, default=28)
    ap.add_argument("--decode-iters", type=int, default=4)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the attainable-peak probes")
    ap.add_argument("--no-attention", action="store_true", help="skip the attention / RoPE leg")
    ap.add_argument("--no-rms", action="store_true", help="skip the RMS split-path leg")
    ap.add_argument("--no-dynamic", action="store_true", help="skip the per-token dynamic baseline leg")
    ap.add_argument("--no-weight-only", action="store_true", help="skip the weight-only (W4 group 128) leg")
    ap.add_argument("--no-graphs", action="store_true",
                    help="time with plain launches only (no HIP graph replay anywhere)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prefill-only", action="store_true",
                    help="only the prefill steps of --configs with plain launches: the run profiled "
                         "under rocprofv3 (kernel trace or one counter)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (3 launches) so that a counter run "
                         "has a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE with")
    return ap.parse_args()


def stats(xs, nd=4):
    return {"median": round(statistics.median(xs), nd), "min": round(min(xs), nd), "max": round(max(xs), nd)}


class Bench:
    def __init__(self, args, torch, np, mq, wl, probes):
        self.args, self.torch, self.np, self.mq, self.wl, self.probes = args, torch, np, mq, wl, probes
        self.dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    # ---------------------------------------------------------------- timing helpers
    def time_blocks(self, run, calls_per_block, repeats=None):
        """`repeats` timed blocks of exactly `calls_per_block` calls of run(), each bracketed by
        a device synchronisation; returns the per-call milliseconds of every block."""
        torch = self.torch
        out = []
        for _ in range(repeats or self.args.repeats):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(calls_per_block):
                run()
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t0) * 1e3 / calls_per_block)
        return out

    def graph_of(self, fn):
        """fn captured as one HIP graph (after one eager run); plain fn with --no-graphs."""
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        if self.args.no_graphs:
            return fn
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        g.replay()
        torch.cuda.synchronize()
        return g.replay

    def time_launch(self, fn, n=10, repeats=None):
        """Microseconds per call of fn: n calls inside one HIP graph, `repeats` replays timed with
        an event pair each (the Python launch path would otherwise be the bound)."""
        torch = self.torch

        def many():
            for _ in range(n):
                fn()
        run = self.graph_of(many)
        us = []
        for _ in range(repeats or self.args.repeats):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            run()
            e1.record()
            e1.synchronize()
            us.append(e0.elapsed_time(e1) * 1e3 / n)
        return us

    # ---------------------------------------------------------------- prefill
    def setup_prefill(self, cfg, host_inputs):
        torch, mq, wl = self.torch, self.mq, self.wl
        w = wl.workload(cfg)
        T, B = w.T, w.had_block
        perm, inv, V = mq.aifs_build_perm(T, w.vis_spans)
        st = {"cfg": cfg, "w": w, "T": T, "B": B, "V": V, "permd": self.dev(perm), "lin": {}}
        st["mask"] = torch.tril(torch.ones((T, T), dtype=torch.uint8, device="cuda"))
        st["mask_u"] = torch.empty_like(st["mask"])
        for proj, (K, N) in w.projections.items():
            if host_inputs:
                inp = wl.make_linear_inputs(w, proj)
                d = {k: self.dev(inp[k]) for k in ("x", "w_packed", "w_scale", "calib_vis", "calib_txt")}
            else:
                inp = None
                d = wl.device_linear_inputs(torch, w, proj)
            absmax = torch.zeros(2, dtype=torch.float32, device="cuda")
            mq.hadamard_absmax(d["calib_vis"], B, absmax[0:1])
            mq.hadamard_absmax(d["calib_txt"], B, absmax[1:2])
            a = absmax.cpu().numpy()
            l = {"K": K, "N": N, "x": d["x"], "wp": mq.w4_prepack(d["w_packed"]), "w_scale": d["w_scale"],
                 "s_vis": mq.static_scale_from_absmax(a[0], B), "s_txt": mq.static_scale_from_absmax(a[1], B),
                 "xq": torch.empty((T, K), dtype=torch.int8, device="cuda"),
                 "y": torch.empty((T, N), dtype=torch.float16, device="cuda"), "host": inp}
            nws = mq.w4a8_workspace_bytes(T, N, K)
            l["ws"] = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
            st["lin"][proj] = l
            del d
        first = next(iter(st["lin"].values()))
        st["x_embed"], st["x_u"] = first["x"], torch.empty_like(first["x"])
        st["gemm_ops"] = sum(2.0 * T * l["K"] * l["N"] for l in st["lin"].values())
        return st

    def prefill_step(self, st, record=None):
        mq, V, B, permd = self.mq, st["V"], st["B"], st["permd"]
        torch = self.torch

        def bracket(kind, proj, fn):
            if record is None:
                fn()
                return
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            record.append((kind, proj, e0, e1))

        mq.aifs_remap_mask(st["mask"], permd, out=st["mask_u"])
        mq.aifs_permute(st["x_embed"], permd, out=st["x_u"])
        for proj, l in st["lin"].items():
            bracket("quant", proj, lambda: mq.hadamard_quant_act(
                l["x"], V, l["s_vis"], l["s_txt"], B, perm_dev=permd, out=l["xq"]))
            bracket("gemm", proj, lambda: mq.w4a8_gemm(
                l["xq"], l["wp"], l["w_scale"], l["N"], V, l["s_vis"], l["s_txt"],
                out=l["y"], workspace=l["ws"]))

    def run_prefill(self, st, steps, warmup, traffic):
        """Times the step of one configuration; returns its report."""
        torch, args = self.torch, self.args
        T, lin = st["T"], st["lin"]
        step = lambda: self.prefill_step(st)
        for _ in range(warmup):
            step()
        plain = self.time_blocks(step, steps)
        if args.no_graphs:
            timed, launch = plain, "plain launches"
        else:
            # The same steps as replays of one captured HIP graph (what a serving loop would do:
            # the step is a fixed sequence of ten launches on fixed buffers).
            replay = self.graph_of(step)
            for _ in range(warmup):
                replay()
            timed, launch = self.time_blocks(replay, steps), "one HIP graph per step"
        ms = statistics.median(timed)
        tops = st["gemm_ops"] / (ms * 1e-3) / 1e12

        # Second pass over the same steps with a HIP event pair (torch's current stream, which is
        # the stream every launch goes to) around each rotate+quant and GEMM launch.
        rec = []
        n_inst = max(steps, args.repeats)
        for _ in range(n_inst):
            self.prefill_step(st, rec)
        torch.cuda.synchronize()
        per_proj = {p: [] for p in lin}
        fe_event = {p: [] for p in lin}
        for kind, proj, e0, e1 in rec:
            (per_proj if kind == "gemm" else fe_event)[proj].append(e0.elapsed_time(e1) * 1e3)
        gemm_us = {p: statistics.median(v) for p, v in per_proj.items()}
        gemm_total_us = sum(gemm_us.values())
        gemm_tops = st["gemm_ops"] / gemm_total_us / 1e6
        n_launch = len(lin)
        breakdown = {}
        for p, l in lin.items():
            ops = 2.0 * T * l["K"] * l["N"]
            breakdown[p] = {"gemm_us": stats(per_proj[p], 2), "tops": round(ops / gemm_us[p] / 1e6, 1),
                            "frac": round(ops / gemm_us[p] / 1e6 / INT8_MFMA_PEAK_TOPS, 4)}
        alg_bytes = sum(l["K"] * l["N"] / 2 + T * l["K"] + 2 * T * l["N"] + 2 * l["N"] for l in lin.values())
        roof = {"bound": "mfma", "kernel": "w4a8_gemm_kernel", "achieved": round(gemm_tops, 1),
                "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": round(gemm_tops / INT8_MFMA_PEAK_TOPS, 4),
                "traffic": None, "algorithmic_bytes_per_launch": alg_bytes / n_launch,
                "avg_launch_us": round(gemm_total_us / n_launch, 2),
                "ops_per_launch_avg": st["gemm_ops"] / n_launch,
                "timing": f"HIP event pair per launch, median of {n_inst} instrumented steps",
                "per_projection": breakdown}
        tr = traffic.get(f"c{st['cfg']}") if traffic else None
        if tr is not None:
            roof["traffic"] = tr["bytes_per_gemm_launch"]
            roof["traffic_over_algorithmic"] = round(tr["bytes_per_gemm_launch"] / (alg_bytes / n_launch), 3)
        elif traffic is not None:
            roof["traffic_note"] = "no counter run of this configuration on this build"
        # front end on its own: the four rotate+quant launches back to back inside one HIP graph
        fe_bytes = sum(3.0 * T * l["K"] for l in lin.values())
        n_rep = 2 if st["cfg"] == 4 else 10

        def fe_pass():
            for proj, l in lin.items():
                self.mq.hadamard_quant_act(l["x"], st["V"], l["s_vis"], l["s_txt"], st["B"],
                                           perm_dev=st["permd"], out=l["xq"])
        fe_us = self.time_launch(fe_pass, n=n_rep)
        fe_med = statistics.median(fe_us)
        per_k = {}
        for p, l in lin.items():
            k = f"K={l['K']}"
            if k not in per_k:
                us = statistics.median(self.time_launch(lambda l=l: self.mq.hadamard_quant_act(
                    l["x"], st["V"], l["s_vis"], l["s_txt"], st["B"], perm_dev=st["permd"], out=l["xq"]),
                    n=n_rep))
                per_k[k] = {"us": round(us, 2), "GBps": round(3.0 * T * l["K"] / us / 1e3, 1),
                            "frac": round(3.0 * T * l["K"] / us / 1e3 / HBM_PEAK_GBPS, 4)}
        return {
            "workload": WORKLOAD_TEXT[st["cfg"]], "T": T, "n_vis": st["V"], "had_block": st["B"],
            "steps_per_block": steps, "blocks": args.repeats, "launch": launch,
            "ms_per_step": stats(timed), "ms_per_step_plain_launches": stats(plain),
            "TOPS": round(tops, 2), "frac_of_int8_peak_whole_step": round(tops / INT8_MFMA_PEAK_TOPS, 4),
            "gemm": roof,
            "front_end": {"kernel": "hadamard_quant_kernel", "bound": "hbm", "us_per_step": stats(fe_us, 2),
                          "GBps": round(fe_bytes / fe_med / 1e3, 1),
                          "frac": round(fe_bytes / fe_med / 1e3 / HBM_PEAK_GBPS, 4), "per_K": per_k},
        }


def load_traffic(mq):
    """HBM-side bytes per GEMM launch from the counter runs summarised in profiles/ (a counter
    run cannot happen inside this script).  Only figures measured on the library build that is
    loaded now are used: the file carries the build id of the kernels it was measured on."""
    if not os.path.exists(TRAFFIC_JSON):
        return None, "profiles/gemm_hbm_traffic.json is missing"
    with open(TRAFFIC_JSON) as f:
        tr = json.load(f)
    if tr.get("build_id") != mq.build_id():
        return None, (f"counter summary was measured on build {tr.get('build_id')}, the library loaded now is "
                      f"{mq.build_id()}: not reported")
    return tr.get("configs", {}), None


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(rows and output channels are independent, so the path would shard along either without a collective)", file=sys.stderr)
        sys.exit(2)
    args.repeats = max(args.repeats, 1)

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

    b = Bench(args, torch, np, mq, wl, probes)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cfgs = sorted({int(c) for c in args.configs.split(",") if c} | {args.headline})
    if args.prefill_only:
        # the run that is profiled: plain launches of the prefill steps, nothing else
        for cfg in cfgs:
            st = b.setup_prefill(cfg, host_inputs=False)
            for _ in range(args.warmup + args.steps):
                b.prefill_step(st)
            torch.cuda.synchronize()
            del st
            torch.cuda.empty_cache()
        print(json.dumps({"prefill_only": cfgs, "steps": args.warmup + args.steps, "build_id": mq.build_id()}), flush=True)
        return

    traffic, traffic_note = load_traffic(mq)
    per_config = {}
    c1_state = None
    for cfg in cfgs:
        st = b.setup_prefill(cfg, host_inputs=(cfg == 1))
        # blocks of `steps` steps for the headline; the smaller configurations get as many steps
        # as make a block comparable in length (their step is 5 to 30 times shorter)
        steps = args.steps if cfg == args.headline else args.steps * (10 if cfg == 1 else 3)
        per_config[cfg] = b.run_prefill(st, steps, args.warmup, traffic)
        if cfg == 1:
            c1_state = st
        else:
            del st
            torch.cuda.empty_cache()

    head = per_config[args.headline]
    result = {
        "metric": METRIC, "value": head["TOPS"], "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "repeats": args.repeats,
        "ms_per_step": head["ms_per_step"]["median"],
        "ms_per_step_min": head["ms_per_step"]["min"], "ms_per_step_max": head["ms_per_step"]["max"],
        "ms_per_step_plain_launches": head["ms_per_step_plain_launches"]["median"],
        "timing": f"median of {args.repeats} timed blocks of exactly {args.steps} steps each",
        "launch": head["launch"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8 x int4 -> int32 (fp16 in/out)", "data": "synthetic",
        "config": {"workload": head["workload"], "T": head["T"], "n_vis": head["n_vis"],
                   "had_block": head["had_block"]},
        "roofline": head["gemm"],
        "front_end": head["front_end"],
        "prefill": {"per_config": {f"configs[{c}]": r for c, r in per_config.items()}},
        "build_id": mq.build_id(),
    }
    if traffic_note:
        result["roofline"]["traffic_note"] = traffic_note

    # ------------------------------------------------- attainable peaks, measured live
    # What this machine reaches on the bounding resources: an MFMA-only int8 loop (the matrix clock
    # drops under data-dependent power: operands like the path's -- quantizer codes against
    # 16 x int4 weights --, uniform random bytes, and zeros for comparison), a read-only stream
    # over 2 GiB, and the launch-to-launch floor of an empty kernel.  The published peaks stay
    # the denominators of every `frac`.
    if not args.no_probes:
        gen_p = torch.Generator(device="cuda")
        gen_p.manual_seed(5000)
        rnd = torch.randint(0, 256, (1 << 16,), dtype=torch.uint8, device="cuda", generator=gen_p)
        zer = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        iters = 20000
        ops = float(probes.mfma_i8(iters, rnd, sink))
        t_r = statistics.median(b.time_launch(lambda: probes.mfma_i8(iters, rnd, sink), n=1))
        t_z = statistics.median(b.time_launch(lambda: probes.mfma_i8(iters, zer, sink), n=1))
        # first half of the buffer feeds one operand, second half the other
        codes = (torch.randn(1 << 16, device="cuda", generator=gen_p) * 32.0).round().clamp(-128, 127).to(torch.int8)
        w16 = (torch.randint(-8, 8, (1 << 16,), device="cuda", generator=gen_p) * 16).to(torch.int8)
        like = torch.cat([codes, w16]).view(torch.uint8)
        t_l = statistics.median(b.time_launch(lambda: probes.mfma_i8(iters, like, sink), n=1))
        att = {"mfma_i8_path_like_operands_TOPS": round(ops / t_l / 1e6, 1),
               "mfma_i8_random_operands_TOPS": round(ops / t_r / 1e6, 1),
               "mfma_i8_zero_operands_TOPS": round(ops / t_z / 1e6, 1)}
        big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
        nbytes = float(probes.hbm_read(big, sink))
        att["hbm_read_GBps"] = round(nbytes / statistics.median(b.time_launch(lambda: probes.hbm_read(big, sink), n=1)) / 1e3, 1)
        del big
        torch.cuda.empty_cache()
        att["empty_kernel_back_to_back_us"] = round(statistics.median(b.time_launch(lambda: probes.empty(256, 512), n=50)), 2)
        result["attainable"] = att
        for r in per_config.values():
            r["gemm"]["frac_of_attainable"] = round(r["gemm"]["achieved"] / att["mfma_i8_path_like_operands_TOPS"], 4)

    if c1_state is not None:
        st = c1_state
        if not args.no_dynamic:
            result["dynamic_baseline"] = bench_dynamic(b, st)
        if not args.no_rms:
            result["rms_split"] = bench_rms(b, st)
        if not args.no_weight_only:
            w4a8_us = {p: v["gemm_us"]["median"] for p, v in per_config[1]["gemm"]["per_projection"].items()}
            result["weight_only_g128"] = bench_weight_only(b, st, w4a8_us)
    if not args.no_attention:
        result["attention"] = bench_attention(b)
    if not args.no_decode:
        result["decode"] = bench_decode(b)
    if not args.no_cpu_baseline and c1_state is not None:
        result["cpu_baseline"] = cpu_baseline(np, c1_state)

    print(json.dumps(result), flush=True)


def bench_dynamic(b, st):
    """The scheme the paper's speed tables compare against, on configs[1]: same rotation, same
    GEMM, but one scale per token found at run time and applied per row in the epilogue.  The two
    schemes differ by a few percent, less than the clock drift between separately timed regions:
    they are timed in alternating blocks."""
    torch, mq, args = b.torch, b.mq, b.args
    T, V, B, permd, lin = st["T"], st["V"], st["B"], st["permd"], st["lin"]
    row_scale = torch.empty((T,), dtype=torch.float32, device="cuda")

    def dyn_step():
        mq.aifs_remap_mask(st["mask"], permd, out=st["mask_u"])
        mq.aifs_permute(st["x_embed"], permd, out=st["x_u"])
        for proj, l in lin.items():
            mq.hadamard_dynquant_act(l["x"], B, perm_dev=permd, out=l["xq"], row_scale=row_scale)
            mq.w4a8_gemm_rowscale(l["xq"], l["wp"], l["w_scale"], row_scale, l["N"], out=l["y"], workspace=l["ws"])

    run_s = b.graph_of(lambda: b.prefill_step(st))
    run_d = b.graph_of(dyn_step)
    st_ms, dy_ms = [], []
    per_block = max(args.steps * 5, 20)
    for _ in range(max(args.repeats, 5)):
        st_ms += b.time_blocks(run_s, per_block, 1)
        dy_ms += b.time_blocks(run_d, per_block, 1)
    dyn_med, stat_med = statistics.median(dy_ms), statistics.median(st_ms)
    fe_bytes = sum(3.0 * T * l["K"] for l in lin.values())

    def dyn_fe():
        for proj, l in lin.items():
            mq.hadamard_dynquant_act(l["x"], B, perm_dev=permd, out=l["xq"], row_scale=row_scale)
    fe_us = b.time_launch(dyn_fe, n=10)
    return {"scheme": "A8 per-token dynamic, W4 per-channel static (same rotation and GEMM kernels), configs[1]",
            "ms_per_step": stats(dy_ms), "TOPS": round(st["gemm_ops"] / (dyn_med * 1e-3) / 1e12, 2),
            "static_ms_per_step_interleaved": stats(st_ms),
            "static_over_dynamic_speedup": round(dyn_med / stat_med, 4),
            "front_end_us_per_step": stats(fe_us, 2),
            "front_end_GBps": round((fe_bytes + 4.0 * T * len(lin)) / statistics.median(fe_us) / 1e3, 1)}


def bench_rms(b, st):
    """RMS split path on the down projection of configs[1]: main GEMM plus the split GEMV of the
    flagged channels fused into its epilogue, for one flagged channel (the paper's 1/18944 case)
    and for one per Hadamard block; variants alternate, median of the repeats each."""
    torch, mq, np = b.torch, b.mq, b.np
    l, V, B, T = st["lin"]["down"], st["V"], st["B"], st["T"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    variants = {"plain_us": lambda: mq.w4a8_gemm(l["xq"], l["wp"], l["w_scale"], l["N"], V, l["s_vis"], l["s_txt"],
                                                 out=l["y"], workspace=l["ws"])}
    for n_split in (1, l["K"] // B):
        idx = np.arange(n_split, dtype=np.int32) * B
        sw = torch.randint(-8, 8, (n_split, l["N"]), dtype=torch.int8, device="cuda", generator=gen)
        ss = np.linspace(0.05, 0.35, n_split, dtype=np.float32)
        variants["split_%d_us" % n_split] = (lambda idx=idx, sw=sw, ss=ss: mq.w4a8_gemm_rms(
            l["xq"], l["wp"], l["w_scale"], l["N"], V, l["s_vis"], l["s_txt"], idx, sw, ss,
            out=l["y"], workspace=l["ws"]))
    out = {"projection": "down 18944x3584, T=%d" % T}
    samples = {k: [] for k in variants}
    for _ in range(max(b.args.repeats, 5)):
        for k, fn in variants.items():
            samples[k] += b.time_launch(fn, n=20, repeats=1)
    out.update({k: stats(v, 2) for k, v in samples.items()})
    return out


def bench_weight_only(b, st, w4a8_gemm_us):
    """The four projections of configs[1] as weight-only linears: fp16 activations straight into
    an fp16 MFMA GEMM whose weight operand is dequantised (int4, one fp16 scale per 128 input
    channels) in registers.  Random codes and scales; no rotation, no quantizer."""
    torch, mq = b.torch, b.mq
    lin, T = st["lin"], st["T"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(6100)
    out = {"scheme": "W4 group 128, A fp16 (dequantise in registers, fp16 MFMA, fp32 accumulate), configs[1]",
           "per_projection": {}}
    total_us, flops = 0.0, 0.0
    dec, dec_us, dec_bytes = {}, 0.0, 0.0
    for proj, l in lin.items():
        K, N = l["K"], l["N"]
        wq = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, device="cuda", generator=gen)
        sc = (torch.rand((N, K // 128), device="cuda", generator=gen) * 0.008 + 0.002).to(torch.float16)
        wp = mq.w4g128_prepack(wq, sc)
        del wq
        us = b.time_launch(lambda: mq.w4g128_gemm(l["x"], wp, N, out=l["y"]), n=10)
        med = statistics.median(us)
        fl = 2.0 * T * K * N
        out["per_projection"][proj] = {"us": stats(us, 2), "TFLOPs": round(fl / med / 1e6, 1),
                                       "w4a8_gemm_us": round(w4a8_gemm_us[proj], 2)}
        total_us += med
        flops += fl
        # decode shape: the same weight matrix against one token (weight-streaming GEMV)
        x1, y1 = l["x"][:1], l["y"][:1]
        us1 = b.time_launch(lambda: mq.w4g128_gemm(x1, wp, N, out=y1), n=20)
        med1 = statistics.median(us1)
        nbytes = float(wp.numel()) + 2.0 * K + 2.0 * N
        dec[proj] = {"us": stats(us1, 2), "GBps": round(nbytes / med1 / 1e3, 1)}
        dec_us += med1
        dec_bytes += nbytes
        del wp
    out["us_per_step"] = round(total_us, 2)
    out["TFLOPs"] = round(flops / total_us / 1e6, 1)
    out["frac_of_fp16_mfma_peak"] = round(flops / total_us / 1e6 / FP16_MFMA_PEAK_TFLOPS, 4)
    out["w4a8_gemm_us_per_step"] = round(sum(w4a8_gemm_us.values()), 2)
    out["decode_T1"] = {"per_projection": dec, "us_per_layer": round(dec_us, 2),
                        "GBps": round(dec_bytes / dec_us / 1e3, 1),
                        "frac_of_hbm_peak": round(dec_bytes / dec_us / 1e3 / HBM_PEAK_GBPS, 4),
                        "note": "the same weights every launch (they fit the 256 MB last-level cache)"}
    return out


def bench_attention(b):
    """Attention on AIFS-ordered tokens (28 query heads on 4 key/value heads of 128 channels,
    the 7B shapes) for the layouts of configs[1] and configs[2]; q, k, v are column slices of
    one [T, 4608] buffer as the qkv projection leaves them.  Algorithmic flops: 4*D per
    allowed (query, key) pair and query head; peak: dense fp16 MFMA 2.5 PFLOP/s."""
    torch, mq, wl, np = b.torch, b.mq, b.wl, b.np
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
        us = b.time_launch(lambda: mq.aifs_attention(q, k, v, pos, Hq, Hkv, out=o, workspace=ws), n=10)
        # the same kernel on tokens in their original order (positions 0..T-1: a plain causal
        # mask): what the reorder costs the attention (the paper's comparison of FlashAttention
        # with and without AIFS)
        pos_plain = torch.arange(T, dtype=torch.int32, device="cuda")
        us_plain = b.time_launch(lambda: mq.aifs_attention(q, k, v, pos_plain, Hq, Hkv, out=o, workspace=ws), n=10)
        pairs = T * (T + 1) // 2                      # allowed pairs of a causal mask in any order
        flops = 4.0 * D * pairs * Hq
        us_rope = b.time_launch(lambda: mq.rope_apply(qkv[:, :(Hq + Hkv) * D], pos, Hq + Hkv), n=10)
        rope_bytes = 4.0 * T * (Hq + Hkv) * D
        med, med_p, med_r = statistics.median(us), statistics.median(us_plain), statistics.median(us_rope)
        out["per_config"]["configs[%d] T=%d" % (cfg, T)] = {
            "attention_us": stats(us, 1), "TFLOPs": round(flops / med / 1e6, 1),
            "frac": round(flops / med / 1e6 / 2500.0, 4),
            "plain_causal_order_us": stats(us_plain, 1),
            "aifs_overhead": round(med / med_p - 1.0, 4),
            "rope_us": stats(us_rope, 2), "rope_GBps": round(rope_bytes / med_r / 1e3, 1)}
    return out


def bench_decode(b):
    """GEMV over `decode_layers` distinct layers of 7B weights (uniform random int4 nibbles written
    directly in the streamed layout; the contents do not change the traffic) for T in {1, 4, 16},
    text rows only.  Every leg is one HIP graph of a whole 28-layer pass (the Python launch path,
    several microseconds per call, is otherwise the bound), replayed `decode_iters` times per timed
    block; median of the blocks."""
    torch, mq, wl, args = b.torch, b.mq, b.wl, b.args
    out = {"unit": "GB/s", "peak": HBM_PEAK_GBPS, "layers": args.decode_layers,
           "launch": "plain" if args.no_graphs else "hipGraph", "per_T": {}}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3000)
    streams = [torch.cuda.Stream() for _ in range(4)]
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
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

        def gemv_grouped_pass():
            # four launches per layer through the grouped entry: q/k/v and gate/up keep their own
            # weight buffers and outputs (nothing is concatenated), o and down are groups of one
            for layer in layers:
                mq.w4a8_gemv_grouped(xq[3584], [(layer[p][2], layer[p][3], layer[p][1], ys_multi[i][layer[p][1]])
                                                for i, p in enumerate(("q", "k", "v"))], 0, s_txt, s_txt)
                mq.w4a8_gemv_grouped(xq[3584], [(layer["o"][2], layer["o"][3], 3584, ys[3584])], 0, s_txt, s_txt)
                mq.w4a8_gemv_grouped(xq[3584], [(layer[p][2], layer[p][3], layer[p][1], ys_multi[i][layer[p][1]])
                                                for i, p in enumerate(("gate", "up"))], 0, s_txt, s_txt)
                mq.w4a8_gemv_grouped(xq[18944], [(layer["down"][2], layer["down"][3], 3584, ys[3584])], 0, s_txt, s_txt)

        def layer_grouped_pass():
            # a decoder layer as deployed with the grouped entry: one rotate+quant per distinct
            # input (four per layer: attention input, attention output, MLP input, MLP hidden)
            for layer in layers:
                mq.hadamard_quant_act(xs[3584], 0, s_txt, s_txt, 512, out=xq[3584])
                mq.w4a8_gemv_grouped(xq[3584], [(layer[p][2], layer[p][3], layer[p][1], ys_multi[i][layer[p][1]])
                                                for i, p in enumerate(("q", "k", "v"))], 0, s_txt, s_txt)
                mq.hadamard_quant_act(xs[3584], 0, s_txt, s_txt, 512, out=xq[3584])
                mq.w4a8_gemv_grouped(xq[3584], [(layer["o"][2], layer["o"][3], 3584, ys[3584])], 0, s_txt, s_txt)
                mq.hadamard_quant_act(xs[3584], 0, s_txt, s_txt, 512, out=xq[3584])
                mq.w4a8_gemv_grouped(xq[3584], [(layer[p][2], layer[p][3], layer[p][1], ys_multi[i][layer[p][1]])
                                                for i, p in enumerate(("gate", "up"))], 0, s_txt, s_txt)
                mq.hadamard_quant_act(xs[18944], 0, s_txt, s_txt, 512, out=xq[18944])
                mq.w4a8_gemv_grouped(xq[18944], [(layer["down"][2], layer["down"][3], 3584, ys[3584])], 0, s_txt, s_txt)

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

        def layer_one_launch_grouped_pass():
            # the same four launches per layer without concatenated weights: q/k/v and gate/up
            # keep their own buffers and outputs and share the rotate+quant of their launch
            for layer in layers:
                mq.w4a8_linear_decode_grouped(xs[3584], [(layer[p][2], layer[p][3], layer[p][1], ys_multi[i][layer[p][1]])
                                                         for i, p in enumerate(("q", "k", "v"))], 0, s_txt, s_txt, 512)
                mq.w4a8_linear_decode_grouped(xs[3584], [(layer["o"][2], layer["o"][3], 3584, ys[3584])], 0, s_txt, s_txt, 512)
                mq.w4a8_linear_decode_grouped(xs[3584], [(layer[p][2], layer[p][3], layer[p][1], ys_multi[i][layer[p][1]])
                                                         for i, p in enumerate(("gate", "up"))], 0, s_txt, s_txt, 512)
                mq.w4a8_linear_decode_grouped(xs[18944], [(layer["down"][2], layer["down"][3], 3584, ys[3584])], 0, s_txt, s_txt, 512)

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
        legs = [("quant+gemv", one_pass), ("layer_4quant_4gemv", layer_pass),
                ("layer_4quant_4grouped_gemv", layer_grouped_pass)]
        if T <= 4:
            legs.append(("quant+gemv_one_launch", fused_linear_pass))
            legs.append(("layer_4_one_launch_linears", layer_one_launch_pass))
            legs.append(("layer_4_one_launch_grouped", layer_one_launch_grouped_pass))
        for name, fn in legs + [("gemv_only", gemv_only_pass),
                                ("gemv_only_fused_qkv_gateup", gemv_fused_pass),
                                ("gemv_only_grouped_4_launches", gemv_grouped_pass),
                                ("gemv_only_4streams", gemv_streams_pass)]:
            run = b.graph_of(fn)
            ms = [m / len(layers) for m in b.time_blocks(run, args.decode_iters)]
            med = statistics.median(ms)
            gbps = bytes_layer / (med * 1e-3) / 1e9
            res[name] = {"us_per_layer": stats([m * 1e3 for m in ms], 2), "GBps": round(gbps, 1),
                         "frac": round(gbps / HBM_PEAK_GBPS, 4)}
        res["bytes_per_layer"] = bytes_layer
        # per projection: the same projection of every layer back to back (distinct weights,
        # so nothing is served from the last-level cache), one HIP graph per projection
        per_proj = {}
        groups = dict(wd.projections)
        groups.update({"qkv (one launch)": (3584, 4608), "gate_up (one launch)": (3584, 37888)})
        for proj, (K, N) in groups.items():
            src = fused_layers if "one launch" in proj else layers
            key = proj.split(" ")[0]

            def proj_pass(src=src, key=key, K=K, N=N):
                for layer in src:
                    _, _, wp, ws = layer[key]
                    mq.w4a8_gemm(xq[K], wp, ws, N, 0, s_txt, s_txt, out=ys[N])
            run = b.graph_of(proj_pass)
            us = [m * 1e3 / len(layers) for m in b.time_blocks(run, args.decode_iters)]
            med = statistics.median(us)
            nbytes = K * N / 2 + 2 * N + T * K + 2 * T * N
            per_proj[proj] = {"us": stats(us, 2), "GBps": round(nbytes / med / 1e3, 1),
                              "frac": round(nbytes / med / 1e3 / HBM_PEAK_GBPS, 4)}
            if T == 1 and not args.no_probes:
                # the floor of this launch pattern: a kernel that only reads the same weight
                # buffers (the probe library's read stream), one launch per layer, same graph form
                def read_pass(src=src, key=key):
                    for layer in src:
                        b.probes.hbm_read(layer[key][2], sink)
                us_r = [m * 1e3 / len(layers) for m in b.time_blocks(b.graph_of(read_pass), args.decode_iters)]
                per_proj[proj]["read_only_kernel_us"] = round(statistics.median(us_r), 2)
                per_proj[proj]["read_only_kernel_over_gemv"] = round(statistics.median(us_r) / med, 3)
        res["per_projection_gemv"] = per_proj
        out["per_T"][f"T{T}"] = res
    del layers, fused_layers
    torch.cuda.empty_cache()
    out["large_shapes"] = bench_decode_large(b, gen)
    return out


def bench_decode_large(b, gen):
    """The same GEMV on the 72B-class shapes of configs[4] (a launch streams 30-240 MB, against
    1-34 MB on the 7B shapes, so launch latency is a small share).  Six distinct layers (2.6 GB)
    defeat the last-level cache; one HIP graph per pass."""
    torch, mq, wl, args = b.torch, b.mq, b.wl, b.args
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
    res = {"workload": "configs[4] projections (qkv 8192x10240, o 8192x8192, gate_up 8192x59136, "
                       "down 29568x8192), %d layers" % n_layers}
    for T in (1, 4, 16):
        xq = {K: torch.randint(-128, 128, (T, K), dtype=torch.int8, device="cuda", generator=gen) for K in Ks}
        ys = {N: torch.empty((T, N), dtype=torch.float16, device="cuda") for (K, N) in w4.projections.values()}

        def one_pass():
            for layer in layers:
                for proj, (K, N, wp, ws) in layer.items():
                    mq.w4a8_gemm(xq[K], wp, ws, N, 0, 0.035, 0.035, out=ys[N])

        run = b.graph_of(one_pass)
        us = [m * 1e3 / n_layers for m in b.time_blocks(run, args.decode_iters)]
        med = statistics.median(us)
        bytes_layer = sum(K * N / 2 + 2 * N + T * K + 2 * T * N for (K, N) in w4.projections.values())
        gbps = bytes_layer / med / 1e3
        res[f"T{T}"] = {"us_per_layer": stats(us, 2), "bytes_per_layer": bytes_layer,
                        "GBps": round(gbps, 1), "frac": round(gbps / HBM_PEAK_GBPS, 4)}
    return res


def cpu_baseline(np, st):
    """The oracle as it stands on the WHOLE of configs[1] (all 1280 rows, all channels of the four
    projections), every stage timed, all host threads."""
    from oracle import mquant_oracle as orc
    w, lin, V = st["w"], st["lin"], st["V"]
    ops = 0.0
    stages = {"permute": 0.0, "rotate_quant": 0.0, "unpack": 0.0, "gemm": 0.0, "dequant": 0.0}
    for proj, l in lin.items():
        inp = l["host"]
        t = time.perf_counter()
        perm, _, V2 = orc.aifs_build_perm(inp["T"], inp["vis_spans"])
        x_u = orc.aifs_permute_rows(inp["x"], perm)
        stages["permute"] += time.perf_counter() - t
        t = time.perf_counter()
        xq = orc.msq_quantize(orc.hadamard_rotate(x_u, w.had_block), V, l["s_vis"], l["s_txt"], w.had_block)
        stages["rotate_quant"] += time.perf_counter() - t
        t = time.perf_counter()
        wq = orc.unpack_w4(inp["w_packed"])
        stages["unpack"] += time.perf_counter() - t
        t = time.perf_counter()
        acc = orc.gemm_i8_i4_i32(xq, wq)
        stages["gemm"] += time.perf_counter() - t
        t = time.perf_counter()
        orc.dequant(acc, V, l["s_vis"], l["s_txt"], inp["w_scale"])
        stages["dequant"] += time.perf_counter() - t
        ops += 2.0 * inp["T"] * l["K"] * l["N"]
    t_total = sum(stages.values())
    return {"value": round(ops / t_total / 1e12, 5), "unit": "TOPS", "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": f"all of configs[1]: {w.T} rows x all channels of the four projections "
                      f"({ops / 1e9:.1f} GOP); {round(t_total, 2)} s wall",
            "seconds": round(t_total, 3),
            "stage_seconds": {k: round(v, 3) for k, v in stages.items()}}


if __name__ == "__main__":
    main()
