#!/usr/bin/env python3
"""Benchmark of the micro-rotated FP4 linear-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
    python bench.py --summarize-db <rocprofv3 *_results.db> [--pmc]      (no GPU: prints the tables kept under profiles/)

A "step" is one pass of the whole hot path -- fused Hadamard rotation + MXFP4 quantization of the bf16
activations, then the W4A4 FP4 GEMM against weights that were rotated and quantized ahead of time -- over the
four linear layers of a Llama-3-8B-shaped block at M = 4096 tokens (the compute-bound prefill regime).  All
inputs are synthetic, seeded, and resident in HBM before the timed region.  One JSON line is printed.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP4_TFLOPS = 10100.0     # MI355X dense FP4/FP6 MFMA
PEAK_F16_TFLOPS = 2500.0      # dense fp16 / bf16 MFMA
PEAK_HBM_GBS = 8000.0
RQ_BYTES_PER_ELEM_MX = 2.0 + 0.5 + 1.0 / 32.0   # bf16 in, 4-bit code out, one scale byte per 32
MIN_EVENT_SAMPLES = 8          # per kernel of the step, whatever --steps is
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic__llama3_8b_prefill_m4096_and_rq_16384x8192__pmc.txt")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=192)
    ap.add_argument("--warmup", type=int, default=24)
    ap.add_argument("--tokens", type=int, default=4096, help="M of the prefill workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip every side measurement (baselines, ceilings, other configurations)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for HBM-traffic counters under a profiler)")
    ap.add_argument("--summarize-db", metavar="DB", help="print the per-kernel table of a rocprofv3 results database and exit")
    ap.add_argument("--pmc", action="store_true", help="with --summarize-db: the database holds --pmc counters, not a kernel trace")
    return ap.parse_args()


# --------------------------------------------------------------------------------------------------------------
# profiles/: the tables kept there are these group-bys over rocprofv3's own SQLite output
def summarize_db(path, pmc):
    import sqlite3
    c = sqlite3.connect(path)
    clean = lambda n: (n or "").replace("fp4mr::(anonymous namespace)::", "").replace("void ", "")
    if not pmc:
        rows = c.execute("select name, count(*), sum(duration), avg(duration), min(duration), max(duration), grid_x, workgroup_x, "
                         "lds_size, vgpr_count, accum_vgpr_count from kernels group by name, grid_x order by sum(duration) desc").fetchall()
        tot = sum(r[2] for r in rows) or 1
        print(f"{'kernel':<78} {'calls':>5} {'total_us':>10} {'avg_us':>9} {'min_us':>9} {'max_us':>9} {'pct':>6} {'grid':>8} {'wg':>4} {'lds':>7} {'vgpr':>4} {'agpr':>4}")
        for r in rows:
            print(f"{clean(r[0])[:76]:<78} {r[1]:>5} {r[2] / 1e3:>10.1f} {r[3] / 1e3:>9.2f} {r[4] / 1e3:>9.2f} {r[5] / 1e3:>9.2f} "
                  f"{100 * r[2] / tot:>6.2f} {r[6]:>8} {r[7]:>4} {r[8]:>7} {r[9]:>4} {r[10]:>4}")
        return
    rows = c.execute("select kernel_name, counter_name, grid_size_x, count(*), avg(value), min(value), max(value) from counters_collection "
                     "group by kernel_name, counter_name, grid_size_x order by sum(value) desc").fetchall()
    print(f"{'kernel':<70} {'counter':<11} {'grid':>9} {'calls':>5} {'avg_KiB':>12} {'min_KiB':>12} {'max_KiB':>12}")
    for r in rows:
        print(f"{clean(r[0])[:68]:<70} {r[1]:<11} {r[2]:>9} {r[3]:>5} {r[4]:>12.1f} {r[5]:>12.1f} {r[6]:>12.1f}")


def committed_traffic():
    """HBM-side bytes per launch from the committed counter summary (two rocprofv3 --pmc runs of this script, scaled by
    what the same counters read for a plain copy of known size): its last line is a JSON object."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in reversed(f.read().splitlines()):
                if line.startswith("TRAFFIC_JSON "):
                    return json.loads(line[len("TRAFFIC_JSON "):])
    except (OSError, ValueError):
        pass
    return {}


def to_dev_bf16(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def cpu_baseline(recipe, layer, M_sample, N_sample, threads=None):
    """The oracle as it stands, on a bounded sample of the same workload: rotate+quantize of M_sample tokens and
    the fp64 product against N_sample pre-quantized weight rows (weight preparation is offline for both sides)."""
    from oracle import reference as R
    K = layer.K
    all_threads = R.max_threads()
    xb = recipe.x(M_sample, K)
    wb = recipe.w(N_sample, K)
    wc, wsc, wT, _ = R.rotate_quantize(wb, recipe.had_block, R.MXFP4)
    W = R.dequantize(wc, wsc, R.MXFP4, wT)
    if threads:
        R.set_threads(threads)
    try:
        t0 = time.perf_counter()
        ac, asc, aT, _ = R.rotate_quantize(xb, recipe.had_block, R.MXFP4)
        A = R.dequantize(ac, asc, R.MXFP4, aT)
        R.matmul(A, W, want_abs=False)
        dt = time.perf_counter() - t0
    finally:
        if threads:
            R.set_threads(all_threads)
    flops = 2.0 * M_sample * N_sample * K
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": threads or all_threads, "kind": "oracle",
            "sample": f"{layer.name} layer, {M_sample} of the tokens x {N_sample} of the {layer.N} output features, K={K}: "
                      f"rotate+quantize X, dequantize, fp64 product ({dt:.1f} s)"}


def main():
    args = parse()
    if args.summarize_db:
        summarize_db(args.summarize_db, args.pmc)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives exist in the path); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2509_23202_amd import binding as fp4
    from paper_2509_23202_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    recipe = inputs.RECIPES[3]
    layers = inputs.LLAMA3_8B_LAYERS
    M = args.tokens
    b = recipe.had_block
    GL = fp4.LAYOUT_GEMM
    gflags = fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM
    ev_pair = lambda: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))

    # ---- inputs resident in HBM; weights rotated + quantized ahead of time (not timed)
    state = []
    for i, L in enumerate(layers):
        x = to_dev_bf16(recipe.x(M, L.K, salt=i))
        w = to_dev_bf16(recipe.w(L.N, L.K, salt=i))
        wc, ws, _ = fp4.fp4_quantize_weights(w, b, fp4.MXFP4, flags=GL)
        cb, sb = fp4.packed_bytes(M, L.K, fp4.MXFP4, GL)
        state.append(dict(L=L, x=x, w=w, wc=wc, ws=ws,
                          ac=torch.empty(cb, dtype=torch.uint8, device="cuda"), asc=torch.empty(sb, dtype=torch.uint8, device="cuda"),
                          out=torch.empty((M, L.N), dtype=torch.bfloat16, device="cuda")))
    torch.cuda.synchronize()

    # One pass of the hot path.  To time individual kernels inside the timed region without perturbing it, each step
    # brackets exactly ONE of its 2*len(layers) launches with a pair of HIP events on the launch stream (launch
    # `probe` of the step); over the K steps every kernel gets K / (2*len(layers)) samples.
    n_kern = 2 * len(state)

    def step(probe=-1, ev=None):
        for li, s in enumerate(state):
            L = s["L"]
            if probe == 2 * li:
                e0, e1 = ev_pair(); e0.record()
            fp4.fp4_rotate_quantize(s["x"], b, fp4.MXFP4, flags=GL, codes=s["ac"], scales=s["asc"])
            if probe == 2 * li:
                e1.record(); ev.append((L.name, "rq", e0, e1))
            if probe == 2 * li + 1:
                e0, e1 = ev_pair(); e0.record()
            fp4.fp4_gemm(s["ac"], s["asc"], None, s["wc"], s["ws"], None, M, L.N, L.K, fp4.MXFP4, flags=gflags, out=s["out"])
            if probe == 2 * li + 1:
                e1.record(); ev.append((L.name, "gemm", e0, e1))

    for _ in range(args.warmup):
        step()
    # Clock pre-warm, stated in the JSON line: a GPU that was idle (input preparation above) comes back at a low clock and
    # climbs for roughly 60 ms of continuous load; a short timed region (--steps 20 is 10 ms) would otherwise measure the
    # climb rather than the throughput of a busy GPU.  These are further untimed passes of the same step.
    N_PRE = max(0, 128 - args.warmup)
    for _ in range(N_PRE):
        step()

    ev = []
    # (nothing between this synchronize and the timed loop: a GPU left idle for even a millisecond comes back at a lower
    # clock and needs some twenty steps to recover, which a short timed region would be charged for)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i % n_kern, ev)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # Every kernel of the step gets at least MIN_EVENT_SAMPLES event samples: what the timed steps did not supply comes
    # from further passes of the same step, right behind the timed region (untimed, GPU still busy and warm)
    n_timed_samples = len(ev)
    extra_passes = 0
    count = lambda: {(n_, k_): sum(1 for a_, b_, _, _ in ev if (a_, b_) == (n_, k_)) for n_ in [s["L"].name for s in state] for k_ in ("rq", "gemm")}
    while min(count().values()) < MIN_EVENT_SAMPLES and extra_passes < 64 * n_kern:
        step(extra_passes % n_kern, ev)
        extra_passes += 1
    torch.cuda.synchronize()
    # An event pair around a launch also times the dispatch hand-off on both sides of it (a few microseconds that
    # back-to-back launches hide).  Calibrate that bracket overhead on a launch that does almost no work (a 16 x 128
    # quantize, ~2 KB) and subtract it, so that the per-kernel figures line up with a kernel trace.  This runs BEHIND the
    # timed region: twenty near-empty launches in front of it leave the GPU at a lower clock for the next ~20 steps.
    N_CAL = 20
    tiny_x = torch.zeros((16, 128), dtype=torch.bfloat16, device="cuda")
    tiny_c = torch.empty(fp4.packed_bytes(16, 128, fp4.MXFP4, GL)[0], dtype=torch.uint8, device="cuda")
    tiny_s = torch.empty(fp4.packed_bytes(16, 128, fp4.MXFP4, GL)[1], dtype=torch.uint8, device="cuda")
    cal = []
    for _ in range(N_CAL):
        step()  # keep the queue in the same state as in the timed loop
        e0, e1 = ev_pair()
        e0.record()
        fp4.fp4_rotate_quantize(tiny_x, b, fp4.MXFP4, flags=GL, codes=tiny_c, scales=tiny_s)
        e1.record()
        cal.append((e0, e1))
    torch.cuda.synchronize()
    TINY_KERNEL_MS = 0.0035  # the calibration launch itself (one wave, one fragment; 3.4-4.1 us in a kernel trace)
    bracket_ms = max(0.0, float(np.median([a.elapsed_time(b_) for a, b_ in cal])) - TINY_KERNEL_MS)
    ms_per_step = dt * 1e3 / args.steps
    flops_step = sum(2.0 * M * s["L"].N * s["L"].K for s in state)
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel durations from the events
    per_layer = {}
    for name, kind, e0, e1 in ev:
        per_layer.setdefault(name, {"rq": [], "gemm": []})[kind].append(e0.elapsed_time(e1))
    layers_out = {}
    gemm_ms_total = 0.0
    for s in state:
        L = s["L"]
        d = per_layer.get(L.name, {"rq": [], "gemm": []})
        rq = float(np.mean(d["rq"])) - bracket_ms if d["rq"] else float("nan")
        gm = float(np.mean(d["gemm"])) - bracket_ms if d["gemm"] else float("nan")
        gemm_ms_total += gm
        fl = 2.0 * M * L.N * L.K
        layers_out[L.name] = {"K": L.K, "N": L.N, "rq_us": round(rq * 1e3, 2), "gemm_us": round(gm * 1e3, 2),
                              "gemm_tflops": round(fl / (gm * 1e-3) / 1e12, 1),
                              "gemm_frac_of_fp4_peak": round(fl / (gm * 1e-3) / 1e12 / PEAK_FP4_TFLOPS, 4),
                              "rq_gbs": round(M * L.K * RQ_BYTES_PER_ELEM_MX / (rq * 1e-3) / 1e9, 1),
                              "actual_tflops": round(fl / ((rq + gm) * 1e-3) / 1e12, 1),
                              "event_samples": [len(d["rq"]), len(d["gemm"])]}
    n_launch = len(state)
    avg_gemm_ms = gemm_ms_total / n_launch
    achieved = flops_step / (gemm_ms_total * 1e-3) / 1e12
    traffic = committed_traffic()
    roofline = {"bound": "mfma", "kernel": "gemm_mx_kernel (v_mfma_scale_f32_16x16x128_f8f6f4, E2M1 x E2M1)",
                "achieved": round(achieved, 1), "peak": PEAK_FP4_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP4_TFLOPS, 4),
                "avg_launch_us": round(avg_gemm_ms * 1e3, 2), "launches_per_step": n_launch,
                "traffic": traffic.get("gemm_mean_bytes_per_launch") if M == 4096 else None,
                "traffic_source": os.path.relpath(TRAFFIC_FILE, ROOT) if traffic else None,
                "timing": "HIP events around one launch per step on the launch stream, minus the event-bracket overhead "
                          f"({bracket_ms * 1e3:.1f} us, calibrated on a 2 KB launch); {n_timed_samples} samples inside the timed region + "
                          f"{len(ev) - n_timed_samples} from {extra_passes} further untimed passes of the same step right behind it "
                          f"(at least {MIN_EVENT_SAMPLES} per kernel)"}

    result = {"metric": "MXFP4 rotate+quant+GEMM TFLOP/s (% FP4 MFMA peak) and speedup vs bf16 GEMM", "value": round(value, 2),
              "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp4_e2m1(e8m0 scales), fp32 accumulate",
              "data": "synthetic",
              "config": {"workload": f"llama3-8b-shaped prefill, MXFP4 W4A4, Hadamard block {b}, M={M}: qkv/o_proj/gate_up/down "
                                     "(BASELINE configs[2])", "M": M, "had_block": b, "format": "mxfp4",
                         "layers": [[L.name, L.K, L.N] for L in layers]},
              "prewarm": f"{args.warmup} warm-up steps, then {N_PRE} further untimed steps (clock pre-warm: 128 untimed steps in all), then the "
                         f"timed region with no idle gap; the event-bracket calibration ({N_CAL} untimed steps) runs behind it",
              "pct_of_fp4_peak": round(100.0 * value / PEAK_FP4_TFLOPS, 2), "layers": layers_out, "roofline": roofline}

    if not args.no_extras:
        # Each section below is a side measurement: a failure in one is recorded and must not cost the headline line.
        extras_errors = {}

        def time_us(fn, n=12, warm=4):
            for _ in range(warm):
                fn()
            torch.cuda.synchronize()
            e0, e1 = ev_pair()
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n * 1e3

        def graph_us(fn, out_t, n=20, reps=5):
            """A few-microsecond kernel cannot be timed through Python-issued launches (the host needs ~8 us per call): n
            calls fn(0) .. fn(n - 1) are captured into a HIP graph on a side stream and the graph is replayed; every
            replayed result is compared with the eager one (the library records kernels only, no memsets).  The index lets
            a call pick one of several identical copies of its weights (cold_copies below)."""
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                for i in range(3):
                    fn(i)
                st.synchronize()
                eager = out_t.clone()
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr, stream=st):
                    for i in range(n):
                        fn(i)
            torch.cuda.synchronize()
            gr.replay()
            torch.cuda.synchronize()
            assert torch.equal(out_t, eager), "graph replay differs from the eager result"
            a0, a1 = ev_pair()
            a0.record()
            for _ in range(reps):
                gr.replay()
            a1.record()
            torch.cuda.synchronize()
            assert torch.equal(out_t, eager), "graph replay differs from the eager result"
            return a0.elapsed_time(a1) / (reps * n) * 1e3

        # Weight streaming is timed with COLD weights: back-to-back calls on one weight tensor would find it in the 256 MB
        # last-level cache (an FP4 layer is 9-62 MB), which no decoding step does -- a model's layers pass through between
        # two uses of the same weights.  Each timed call therefore takes the next of several identical copies, at least
        # COLD_BYTES of them in all, and a graph holds at least as many calls as there are copies.  The bf16 baseline is
        # treated the same way.
        COLD_BYTES = 640e6

        def cold_copies(tensors, nbytes):
            n = max(2, min(80, int(COLD_BYTES / nbytes) + 1))
            return [tuple(tensors)] + [tuple(t.clone() for t in tensors) for _ in range(n - 1)]

        try:
            # ---- measured ceilings (small kernels of the library itself): what the matrix pipes and HBM deliver on this machine
            # when nothing else is in the way.  Run right behind the step loop.
            cus = torch.cuda.get_device_properties(0).multi_processor_count
            rec = torch.zeros(3 * cus, dtype=torch.int64, device="cuda")
            ceil = {"compute_units": cus}
            for name, which, flop_per_mfma, iters, peak in (("fp4_mfma_scaled_16x16x128", fp4.PROBE_MFMA_FP4, 65536.0, 40000, PEAK_FP4_TFLOPS),
                                                            ("f16_mfma_16x16x32", fp4.PROBE_MFMA_F16, 16384.0, 40000, PEAK_F16_TFLOPS)):
                for _ in range(2):
                    step()               # come from the same thermal / clock state as the GEMMs
                us = time_us(lambda: fp4.fp4_probe(which, rec, iters), n=4, warm=1)
                tf = cus * 8 * iters * 32 * flop_per_mfma / us / 1e6
                # time between two MFMAs of one SIMD (two waves share it), from the event-timed launch alone: the
                # datasheet rate is one per 16 clocks of 2.4 GHz = 6.67 ns.  (The kernel also records the shader's own
                # cycle and reference counters; on this machine neither ticks at a documented rate, so they are not used.)
                ceil[name] = {"tflops": round(tf, 1), "frac_of_datasheet": round(tf / peak, 4),
                              "ns_per_mfma_per_simd": round(us * 1e3 / (2 * iters * 32), 2), "datasheet_ns_per_mfma_per_simd": 6.67,
                              "launch_us": round(us, 1)}
            buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            buf.fill_(1)
            us = time_us(lambda: fp4.fp4_probe(fp4.PROBE_COPY, buf), n=10, warm=3)
            ceil["hbm_stream_copy_gbs"] = round(buf.numel() / us / 1e3, 1)
            us = time_us(lambda: fp4.fp4_probe(fp4.PROBE_READ, buf), n=10, warm=3)
            ceil["hbm_stream_read_gbs"] = round(buf.numel() / 2 / us / 1e3, 1)
            del buf
            # the same copy at the size of one rotate+quantize call of the timed step (bf16 [4096, 4096] in, codes and
            # scales out: 42.5 MB of traffic): start-up and drain are a visible share of a kernel this short, so this is
            # the ceiling for the per-layer rq_gbs figures.  Cold operands: 24 buffers cycled (about 1 GB).
            small_n = 42_500_000 // 32 * 32
            smalls = [torch.ones(small_n, dtype=torch.uint8, device="cuda") for _ in range(24)]
            for b_ in smalls[:4]:
                fp4.fp4_probe(fp4.PROBE_COPY, b_)
            torch.cuda.synchronize()
            e0, e1 = ev_pair()
            e0.record()
            for b_ in smalls:
                fp4.fp4_probe(fp4.PROBE_COPY, b_)
            e1.record()
            torch.cuda.synchronize()
            ceil["hbm_stream_copy_gbs_at_42mb"] = round(small_n / (e0.elapsed_time(e1) / len(smalls) * 1e3) / 1e3, 1)
            del smalls
            for name_, l_ in result.get("layers", {}).items():
                if isinstance(l_, dict) and "rq_gbs" in l_ and name_ != "down":
                    l_["rq_frac_of_copy_at_size"] = round(l_["rq_gbs"] / ceil["hbm_stream_copy_gbs_at_42mb"], 3)
            # the cost of a launch that does (almost) nothing, as a kernel duration: the floor under every small call
            ceil["event_bracket_overhead_us"] = round(bracket_ms * 1e3, 2)
            ceil["note"] = ("issue loops: one 8-wave workgroup per compute unit, 16 independent accumulators per wave, operands in "
                            "registers, timed with events; copy/read: 1 GiB buffer, 16 B per lane, non-temporal")
            result["measured_ceilings"] = ceil
            m_fp4 = ceil["fp4_mfma_scaled_16x16x128"]["tflops"]
            roofline["measured_ceiling"] = m_fp4
            roofline["frac_of_measured"] = round(achieved / m_fp4, 4)
        except Exception as exc:  # noqa: BLE001 - reported in the JSON line
            extras_errors["measured_ceilings"] = repr(exc)

        try:
            # ---- bf16 GEMM baseline on the same shapes (library GEMM through torch.matmul), unquantized X and W
            # the four GEMMs run as one step, like the FP4 path above, warmed up and timed over the same number of steps
            # with no idle gap (a GPU that has idled runs its first milliseconds at a lower clock, which would flatter
            # the speedup); per-layer times come from event pairs placed like the probes of the timed loop
            wts = [s["w"].t() for s in state]
            outs = [torch.empty((M, s["L"].N), dtype=torch.bfloat16, device="cuda") for s in state]
            n_base = max(8 * len(state), min(args.steps, 64))
            bev = []

            def base_step(probe=-1):
                for li, s in enumerate(state):
                    if probe == li:
                        b0_, b1_ = ev_pair()
                        b0_.record()
                    torch.matmul(s["x"], wts[li], out=outs[li])
                    if probe == li:
                        b1_.record()
                        bev.append((li, b0_, b1_))

            for _ in range(max(4, min(args.warmup, 16))):
                base_step()
            torch.cuda.synchronize()
            tb0 = time.perf_counter()
            for it in range(n_base):
                base_step(it % len(state))
            torch.cuda.synchronize()
            base_ms = (time.perf_counter() - tb0) * 1e3 / n_base
            for li, s in enumerate(state):
                ms = float(np.mean([e0_.elapsed_time(e1_) for l_, e0_, e1_ in bev if l_ == li])) - bracket_ms
                layers_out[s["L"].name]["bf16_gemm_us"] = round(ms * 1e3, 2)
                layers_out[s["L"].name]["speedup_vs_bf16"] = round(ms / (layers_out[s["L"].name]["rq_us"] * 1e-3 + layers_out[s["L"].name]["gemm_us"] * 1e-3), 3)
            del outs
            result["bf16_gemm_tflops"] = round(flops_step / (base_ms * 1e-3) / 1e12, 1)
            result["speedup_vs_bf16_gemm"] = round(base_ms / ms_per_step, 3)
        except Exception as exc:  # noqa: BLE001 - reported in the JSON line
            extras_errors["bf16_gemm"] = repr(exc)

        try:
            # ---- standalone rotate+quantize on [16384, 8192] Laplace inputs with outlier channels (HBM roofline).
            # Three distinct input buffers are cycled so that no call finds its input in the 256 MB last-level cache.
            r6 = inputs.RECIPES[6]
            Mr, Kr = 16384, 8192
            xs = [to_dev_bf16(r6.x(Mr, Kr, salt=j)) for j in range(3)]
            cb, sb = fp4.packed_bytes(Mr, Kr, fp4.MXFP4, GL)
            oc = torch.empty(cb, dtype=torch.uint8, device="cuda")
            osc = torch.empty(sb, dtype=torch.uint8, device="cuda")
            n_rq = 30

            def time_rq(fn):
                for j in range(3):
                    fn(xs[j])
                torch.cuda.synchronize()
                a0, a1 = ev_pair()
                a0.record()
                for it in range(n_rq):
                    fn(xs[it % 3])
                a1.record()
                torch.cuda.synchronize()
                t = a0.elapsed_time(a1) / n_rq
                return {"avg_launch_us": round(t * 1e3, 2), "achieved_gbs": round(Mr * Kr * RQ_BYTES_PER_ELEM_MX / (t * 1e-3) / 1e9, 1)}

            t_main = time_rq(lambda x_: fp4.fp4_rotate_quantize(x_, 32, fp4.MXFP4, flags=GL, codes=oc, scales=osc))
            gbs = t_main["achieved_gbs"]
            rq_roof = {"bound": "hbm", "kernel": "rq_frag_kernel<32, MXFP4> (GEMM layout)",
                       "workload": "X bf16 [16384, 8192], Laplace(0,1), 1% outlier channels x100, block 32",
                       "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                       "avg_launch_us": t_main["avg_launch_us"], "traffic": traffic.get("rq_16384x8192_bytes_per_launch")}
            copy_gbs = result.get("measured_ceilings", {}).get("hbm_stream_copy_gbs")
            if copy_gbs:
                rq_roof["measured_ceiling"] = copy_gbs
                rq_roof["frac_of_measured"] = round(gbs / copy_gbs, 4)
            result["roofline_rotate_quantize"] = rq_roof

            # ---- the same tensor through a caller-supplied dense rotation (orthonormal DCT-II block rounded to bf16)
            dense = {}
            for bd in (32, 128):
                n_ = np.arange(bd)[:, None]
                k_ = np.arange(bd)[None, :]
                R = np.cos(np.pi * (2 * n_ + 1) * k_ / (2 * bd)) * np.sqrt(2.0 / bd)
                R[:, 0] = 1.0 / np.sqrt(bd)
                Rd = to_dev_bf16(inputs.f32_to_bf16_bits(R.astype(np.float32)))
                dense[f"dct{bd}"] = time_rq(lambda x_: fp4.fp4_rotate_quantize_dense(x_, Rd, fp4.MXFP4, flags=GL, codes=oc, scales=osc))
                dense[f"hadamard{bd}"] = time_rq(lambda x_: fp4.fp4_rotate_quantize(x_, bd, fp4.MXFP4, flags=GL, codes=oc, scales=osc))
            dense["hadamard32_mse_scales"] = time_rq(lambda x_: fp4.fp4_rotate_quantize(x_, 32, fp4.MXFP4, flags=GL | fp4.SCALE_MSE, codes=oc, scales=osc))
            dense["hadamard32_round43_scales"] = time_rq(lambda x_: fp4.fp4_rotate_quantize(x_, 32, fp4.MXFP4, flags=GL | fp4.SCALE_ROUND43, codes=oc, scales=osc))
            # scale byte fitted to the tensor's range of scales (appendix on MXFP scale fitting): a range pre-pass, then the quantize pass
            dense["hadamard32_fit_range_scales"] = time_rq(lambda x_: fp4.fp4_rotate_quantize(x_, 32, fp4.MXFP4, flags=GL | fp4.SCALE_FIT_RANGE, codes=oc, scales=osc))
            # the decoding side (fp4_dequantize): the codes just written, GEMM layout, back to bf16 [16384, 8192]
            fp4.fp4_rotate_quantize(xs[0], 32, fp4.MXFP4, flags=GL, codes=oc, scales=osc)
            dq_out = torch.empty((Mr, Kr), dtype=torch.bfloat16, device="cuda")
            t_dq = time_us(lambda: fp4.fp4_dequantize(oc, osc, None, Mr, Kr, fp4.MXFP4, flags=GL, out=dq_out), n=n_rq, warm=3)
            dense["dequantize_to_bf16"] = {"avg_launch_us": round(t_dq, 2), "achieved_gbs": round(Mr * Kr * (0.5 + 1.0 / 32 + 2.0) / t_dq / 1e3, 1)}
            del dq_out
            result["rotate_quantize_variants"] = dense
            del xs, oc, osc
        except Exception as exc:  # noqa: BLE001 - reported in the JSON line
            extras_errors["rotate_quantize"] = repr(exc)

        try:
            # ---- BASELINE configs[0]: one layer, M = 64, K = N = 4096 (weight streaming: time and GB/s of W)
            r1 = inputs.RECIPES[1]
            M1, K1, N1 = 64, 4096, 4096
            x1, w1 = to_dev_bf16(r1.x(M1, K1)), to_dev_bf16(r1.w(N1, K1))
            q1 = fp4.fp4_quantize_weights(w1, 32, fp4.MXFP4, flags=GL)
            cb, sb = fp4.packed_bytes(M1, K1, fp4.MXFP4, GL)
            c1, s1 = torch.zeros(cb, dtype=torch.uint8, device="cuda"), torch.zeros(sb, dtype=torch.uint8, device="cuda")
            o1, ob1 = torch.empty((M1, N1), dtype=torch.bfloat16, device="cuda"), torch.empty((M1, N1), dtype=torch.bfloat16, device="cuda")
            wbytes = N1 * K1 * (0.5 + 1.0 / 32)
            q1c = cold_copies((q1[0], q1[1]), wbytes)
            w1c = cold_copies((w1,), N1 * K1 * 2.0)
            t_rq = graph_us(lambda i: fp4.fp4_rotate_quantize(x1, 32, fp4.MXFP4, flags=GL, codes=c1, scales=s1), c1)
            t_g = graph_us(lambda i: fp4.fp4_gemm(c1, s1, None, q1c[i % len(q1c)][0], q1c[i % len(q1c)][1], None, M1, N1, K1, fp4.MXFP4,
                                                 flags=gflags, out=o1), o1, n=max(20, len(q1c)))
            t_b = graph_us(lambda i: torch.matmul(x1, w1c[i % len(w1c)][0].t(), out=ob1), ob1, n=max(20, len(w1c)))
            result["config0_m64"] = {"workload": "BASELINE configs[0]: M=64, K=N=4096, MXFP4, block 32; weights cold (copies cycled)", "rq_us": round(t_rq, 2), "gemm_us": round(t_g, 2),
                                     "w_gbs": round(wbytes / t_g / 1e3, 1), "actual_tflops": round(2.0 * M1 * N1 * K1 / (t_rq + t_g) / 1e6, 1),
                                     "bf16_gemm_us": round(t_b, 2), "speedup_vs_bf16": round(t_b / (t_rq + t_g), 2)}
            del x1, w1, q1, q1c, w1c
        except Exception as exc:  # noqa: BLE001 - reported in the JSON line
            extras_errors["config0_m64"] = repr(exc)

        try:
            # ---- BASELINE configs[4], first half: Hadamard block sweep as full rotate+quantize+GEMM, M = 2048, K = N = 8192:
            # "ideal" = the GEMM alone, "actual" = quantization + GEMM (the two curves of Section 5 item 4)
            r5 = inputs.RECIPES[5]
            M5, K5, N5 = 2048, 8192, 8192
            x5, w5 = to_dev_bf16(r5.x(M5, K5)), to_dev_bf16(r5.w(N5, K5))
            cb, sb = fp4.packed_bytes(M5, K5, fp4.MXFP4, GL)
            c5, s5 = torch.empty(cb, dtype=torch.uint8, device="cuda"), torch.empty(sb, dtype=torch.uint8, device="cuda")
            o5 = torch.empty((M5, N5), dtype=torch.bfloat16, device="cuda")
            w5t = w5.t()
            t_b = time_us(lambda: torch.matmul(x5, w5t, out=o5), n=20)
            sweep = {}
            fl5 = 2.0 * M5 * N5 * K5
            for bb in (16, 32, 64, 128):
                q5 = fp4.fp4_quantize_weights(w5, bb, fp4.MXFP4, flags=GL)
                t_rq = time_us(lambda: fp4.fp4_rotate_quantize(x5, bb, fp4.MXFP4, flags=GL, codes=c5, scales=s5), n=30)
                t_g = time_us(lambda: fp4.fp4_gemm(c5, s5, None, q5[0], q5[1], None, M5, N5, K5, fp4.MXFP4, flags=gflags, out=o5), n=30)

                def both():
                    fp4.fp4_rotate_quantize(x5, bb, fp4.MXFP4, flags=GL, codes=c5, scales=s5)
                    fp4.fp4_gemm(c5, s5, None, q5[0], q5[1], None, M5, N5, K5, fp4.MXFP4, flags=gflags, out=o5)
                t_a = time_us(both, n=30)
                sweep[f"b={bb}"] = {"rq_us": round(t_rq, 2), "gemm_us": round(t_g, 2), "ideal_tflops": round(fl5 / t_g / 1e6, 1),
                                    "actual_us": round(t_a, 2), "actual_tflops": round(fl5 / t_a / 1e6, 1),
                                    "speedup_vs_bf16": round(t_b / t_a, 3)}
                del q5
            sweep["bf16_gemm_us"] = round(t_b, 2)
            sweep["workload"] = "BASELINE configs[4]: M=2048, K=N=8192, MXFP4, rotate+quantize+GEMM per Hadamard block size"
            result["block_sweep_2048_8192"] = sweep
            del x5, w5, c5, s5, o5
        except Exception as exc:  # noqa: BLE001 - reported in the JSON line
            extras_errors["block_sweep"] = repr(exc)

        try:
            # ---- the decode configuration (BASELINE configs[1]: M in {1, 16}, same four layers): weight streaming, so the
            # figure of merit is time and GB/s of W, not TFLOP/s (HIP-graph replays, see graph_us)
            decode = {}
            for Md in (1, 16):
                per = {}
                for s_ in state:
                    L = s_["L"]
                    xd = s_["x"][:Md].contiguous()
                    cbd, sbd = fp4.packed_bytes(Md, L.K, fp4.MXFP4, GL)
                    acd = torch.zeros(cbd, dtype=torch.uint8, device="cuda")
                    ascd = torch.zeros(sbd, dtype=torch.uint8, device="cuda")
                    outd = torch.empty((Md, L.N), dtype=torch.bfloat16, device="cuda")
                    outb = torch.empty((Md, L.N), dtype=torch.bfloat16, device="cuda")
                    wbytes = L.N * L.K * (0.5 + 1.0 / 32)
                    wq = cold_copies((s_["wc"], s_["ws"]), wbytes)
                    wb = cold_copies((s_["w"],), L.N * L.K * 2.0)
                    nq, nb_ = len(wq), len(wb)
                    t_rq = graph_us(lambda i: fp4.fp4_rotate_quantize(xd, b, fp4.MXFP4, flags=GL, codes=acd, scales=ascd), acd)
                    t_g = graph_us(lambda i: fp4.fp4_gemm(acd, ascd, None, wq[i % nq][0], wq[i % nq][1], None, Md, L.N, L.K, fp4.MXFP4,
                                                         flags=gflags, out=outd), outd, n=max(20, nq))
                    t_b = graph_us(lambda i: torch.matmul(xd, wb[i % nb_][0].t(), out=outb), outb, n=max(20, nb_))
                    per[L.name] = {"rq_us": round(t_rq, 2), "gemm_us": round(t_g, 2), "w_gbs": round(wbytes / t_g / 1e3, 1),
                                   "bf16_gemm_us": round(t_b, 2), "speedup_vs_bf16": round(t_b / (t_rq + t_g), 2)}
                    if Md <= 4:
                        # one launch: rotation and quantization inside the GEMM (bit-identical result; up to four tokens)
                        outf = torch.empty((Md, L.N), dtype=torch.bfloat16, device="cuda")
                        t_f = graph_us(lambda i: fp4.fp4_fused_linear(xd, b, wq[i % nq][0], wq[i % nq][1], L.N, fp4.MXFP4, out=outf), outf,
                                       n=max(20, nq))
                        assert torch.equal(outf, outd), "one-launch path differs from the two-launch path"
                        per[L.name].update({"fused_us": round(t_f, 2), "fused_w_gbs": round(wbytes / t_f / 1e3, 1),
                                            "fused_speedup_vs_bf16": round(t_b / t_f, 2)})
                    # weight-only variant: rotated activations stay bf16
                    outw = torch.empty((Md, L.N), dtype=torch.bfloat16, device="cuda")
                    t_w = graph_us(lambda i: fp4.fp4_w4a16_linear(xd, b, wq[i % nq][0], wq[i % nq][1], L.N, fp4.MXFP4, out=outw), outw,
                                   n=max(20, nq))
                    per[L.name]["w4a16_us"] = round(t_w, 2)
                    del wq, wb
                decode[f"M={Md}"] = per
            decode["weights"] = "cold: every call of a replayed graph takes the next of several identical weight copies (>= 640 MB in all), for the bf16 baseline too"
            result["decode_configs1"] = decode
            # ---- batched decoding, M = 128 on the same four layers (not a BASELINE config: the regime between the few-token
            # kernels and prefill, where narrow layers leave most of the chip without a tile and fp4_gemm splits K when it is
            # given the FP4MR_OP_GEMM_SPLIT_K workspace)
            mid = {}
            Mm = 128
            for s_ in state:
                L = s_["L"]
                xd = s_["x"][:Mm].contiguous()
                cbd, sbd = fp4.packed_bytes(Mm, L.K, fp4.MXFP4, GL)
                acd = torch.zeros(cbd, dtype=torch.uint8, device="cuda")
                ascd = torch.zeros(sbd, dtype=torch.uint8, device="cuda")
                outd = torch.empty((Mm, L.N), dtype=torch.bfloat16, device="cuda")
                outb = torch.empty((Mm, L.N), dtype=torch.bfloat16, device="cuda")
                wbytes = L.N * L.K * (0.5 + 1.0 / 32)
                wq = cold_copies((s_["wc"], s_["ws"]), wbytes)
                wb = cold_copies((s_["w"],), L.N * L.K * 2.0)
                nq, nb_ = len(wq), len(wb)
                need_s = fp4.workspace_bytes(fp4.OP_GEMM_SPLIT_K, Mm, L.N, L.K, fp4.MXFP4, gflags)
                wss = torch.empty(max(need_s, 16), dtype=torch.uint8, device="cuda")
                ws0 = torch.empty(16, dtype=torch.uint8, device="cuda")
                fp4.fp4_rotate_quantize(xd, b, fp4.MXFP4, flags=GL, codes=acd, scales=ascd)
                t_rq = graph_us(lambda i: fp4.fp4_rotate_quantize(xd, b, fp4.MXFP4, flags=GL, codes=acd, scales=ascd), acd)
                t_g = graph_us(lambda i: fp4.fp4_gemm(acd, ascd, None, wq[i % nq][0], wq[i % nq][1], None, Mm, L.N, L.K, fp4.MXFP4,
                                                     flags=gflags, out=outd, workspace=wss), outd, n=max(20, nq))
                t_g0 = graph_us(lambda i: fp4.fp4_gemm(acd, ascd, None, wq[i % nq][0], wq[i % nq][1], None, Mm, L.N, L.K, fp4.MXFP4,
                                                      flags=gflags, out=outd, workspace=ws0), outd, n=max(20, nq))
                t_b = graph_us(lambda i: torch.matmul(xd, wb[i % nb_][0].t(), out=outb), outb, n=max(20, nb_))
                mid[L.name] = {"rq_us": round(t_rq, 2), "gemm_us": round(t_g, 2), "gemm_unsplit_us": round(t_g0, 2),
                               "split_k_parts": int(need_s // (Mm * L.N * 4)), "bf16_gemm_us": round(t_b, 2),
                               "speedup_vs_bf16": round(t_b / (t_rq + t_g), 2)}
                del wq, wb
            mid["weights"] = "cold (copies cycled), bf16 baseline too"
            result["batched_decode_m128"] = mid
        except Exception as exc:  # noqa: BLE001 - reported in the JSON line
            extras_errors["decode"] = repr(exc)

        try:
            # ---- offline MR-GPTQ sweep of one [4096, 4096] layer (not part of the step; fp32 vector arithmetic): the
            # factor is a random upper-triangular matrix with a positive diagonal (timing does not depend on its values)
            Ng, Kg = 4096, 4096
            wg = (torch.randn(Ng, Kg, device="cuda") * 0.02).to(torch.bfloat16)
            xg = (torch.randn(2 * Kg, Kg, device="cuda") * (1.0 + 9.0 * (torch.rand(Kg, device="cuda") < 0.01))).to(torch.bfloat16)  # a few loud channels
            wsh = torch.empty(fp4.workspace_bytes(fp4.OP_GPTQ_HESSIAN, 2 * Kg, 0, Kg, fp4.MXFP4, 0), dtype=torch.uint8, device="cuda")
            Hg = fp4.fp4_gptq_accumulate_hessian(xg, b, workspace=wsh)     # Hessian of 8192 synthetic calibration rows
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fp4.fp4_gptq_accumulate_hessian(xg, b, Hg, workspace=wsh)
            torch.cuda.synchronize()
            th = time.perf_counter() - t0
            Hg = fp4.fp4_gptq_accumulate_hessian(xg, b, workspace=wsh)
            del xg, wsh
            wsp = torch.empty(fp4.workspace_bytes(fp4.OP_GPTQ_PREPARE, 0, 0, Kg, fp4.MXFP4, 0), dtype=torch.uint8, device="cuda")
            pg, Ug = fp4.fp4_gptq_prepare(Hg, 1e-2, True, workspace=wsp)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(2):
                fp4.fp4_gptq_prepare(Hg, 1e-2, True, workspace=wsp)
            torch.cuda.synchronize()
            tp = (time.perf_counter() - t0) / 2
            del wsp
            wsg = torch.empty(fp4.workspace_bytes(fp4.OP_GPTQ, Ng, 0, Kg, fp4.MXFP4, 0), dtype=torch.uint8, device="cuda")
            fp4.fp4_gptq_quantize_weights(wg, b, fp4.MXFP4, Ug, pg, workspace=wsg)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(3):
                fp4.fp4_gptq_quantize_weights(wg, b, fp4.MXFP4, Ug, pg, workspace=wsg)
            torch.cuda.synchronize()
            tg = (time.perf_counter() - t0) / 3
            fl = float(Ng) * Kg * Kg      # N K^2 / 2 multiply-adds
            flp = 2.0 * float(Kg) ** 3 / 3.0    # K^3/3 flops for the factorization plus K^3/3 for the triangular inverse
            result["gptq_offline"] = {"workload": f"W [{Ng}, {Kg}] bf16, MXFP4, Hadamard block {b}, Hessian of 8192 synthetic rows, act-order",
                                      "sweep_ms": round(tg * 1e3, 3), "bound": "alu", "achieved": round(fl / tg / 1e12, 2),
                                      "peak": 157.3, "unit": "TFLOP/s", "frac": round(fl / tg / 1e12 / 157.3, 4),
                                      "prepare_ms": round(tp * 1e3, 3), "prepare_tflops": round(flp / tp / 1e12, 2),
                                      "hessian_ms": round(th * 1e3, 3), "hessian_tflops": round(2.0 * 2 * Kg * Kg * Kg / th / 1e12, 2)}
            del wg, Ug, pg, wsg, Hg
        except Exception as exc:  # noqa: BLE001 - reported in the JSON line
            extras_errors["gptq_offline"] = repr(exc)

        try:
            # ---- BASELINE configs[3]: NVFP4 on Llama-3-70B-shaped layers.  M = 4096: the fp16-MFMA kernel (its roofline is
            # the fp16 MFMA peak, not the FP4 one: E4M3 group scales cannot go through the block-scaled MFMA) against the
            # bf16 library GEMM; M = 16: weight streaming, GB/s of W (HIP-graph replays)
            nv, nv16 = {}, {}
            m_f16 = result.get("measured_ceilings", {}).get("f16_mfma_16x16x32", {}).get("tflops")
            for name, Kn, Nn in (("qkv", 8192, 10240), ("gate_up", 8192, 57344), ("down", 28672, 8192)):
                xn = torch.randn(M, Kn, device="cuda").to(torch.bfloat16)
                wn = (torch.randn(Nn, Kn, device="cuda") * 0.02).to(torch.bfloat16)
                qa = fp4.fp4_rotate_quantize(xn, 16, fp4.NVFP4, flags=GL)
                qw = fp4.fp4_quantize_weights(wn, 16, fp4.NVFP4, flags=GL)
                on = torch.empty((M, Nn), dtype=torch.bfloat16, device="cuda")
                wsn = fp4.workspace_bytes(fp4.OP_GEMM, M, Nn, Kn, fp4.NVFP4, gflags)
                wsn_t = torch.empty(max(wsn, 16), dtype=torch.uint8, device="cuda")
                wnt = wn.t()
                t_rq = time_us(lambda: fp4.fp4_rotate_quantize(xn, 16, fp4.NVFP4, flags=GL, codes=qa[0], scales=qa[1]), n=8, warm=2)
                tn = time_us(lambda: fp4.fp4_gemm(qa[0], qa[1], qa[2], qw[0], qw[1], qw[2], M, Nn, Kn, fp4.NVFP4, flags=gflags, out=on, workspace=wsn_t))
                tb = time_us(lambda: torch.matmul(xn, wnt, out=on))
                fl = 2.0 * M * Nn * Kn
                nv[name] = {"K": Kn, "N": Nn, "rq_us": round(t_rq, 1), "gemm_us": round(tn, 1), "gemm_tflops": round(fl / tn / 1e6, 1),
                            "frac_of_f16_mfma_peak": round(fl / tn / 1e6 / PEAK_F16_TFLOPS, 4),
                            "frac_of_fp4_mfma_peak": round(fl / tn / 1e6 / PEAK_FP4_TFLOPS, 4),
                            "bf16_gemm_us": round(tb, 1), "speedup_vs_bf16": round(tb / tn, 3),
                            "actual_speedup_vs_bf16": round(tb / (tn + t_rq), 3)}
                if m_f16:
                    nv[name]["frac_of_measured_f16_ceiling"] = round(fl / tn / 1e6 / m_f16, 4)
                # M = 16 on the same weights
                Md = 16
                xd = xn[:Md].contiguous()
                cbd, sbd = fp4.packed_bytes(Md, Kn, fp4.NVFP4, GL)
                acd, ascd = torch.zeros(cbd, dtype=torch.uint8, device="cuda"), torch.zeros(sbd, dtype=torch.uint8, device="cuda")
                tsd = torch.zeros(1, dtype=torch.float32, device="cuda")
                wsd = torch.empty(fp4.workspace_bytes(fp4.OP_ROTATE_QUANTIZE, Md, 0, Kn, fp4.NVFP4, GL), dtype=torch.uint8, device="cuda")
                outd, outb = torch.empty((Md, Nn), dtype=torch.bfloat16, device="cuda"), torch.empty((Md, Nn), dtype=torch.bfloat16, device="cuda")

                def rq_small(i):
                    st_ = fp4.lib.fp4_rotate_quantize(xd.data_ptr(), Md, Kn, 16, fp4.NVFP4, acd.data_ptr(), ascd.data_ptr(), tsd.data_ptr(),
                                                      wsd.data_ptr(), wsd.numel(), GL, torch.cuda.current_stream().cuda_stream)
                    assert st_ == 0
                t_rq16 = graph_us(rq_small, acd)
                wbytes = Nn * Kn * (0.5 + 1.0 / 16)
                qwc = cold_copies((qw[0], qw[1]), wbytes)
                wnc = cold_copies((wn,), Nn * Kn * 2.0)
                nq, nb_ = len(qwc), len(wnc)
                t_g16 = graph_us(lambda i: fp4.fp4_gemm(acd, ascd, tsd, qwc[i % nq][0], qwc[i % nq][1], qw[2], Md, Nn, Kn, fp4.NVFP4, flags=gflags,
                                                       out=outd), outd, n=max(20, nq))
                t_b16 = graph_us(lambda i: torch.matmul(xd, wnc[i % nb_][0].t(), out=outb), outb, n=max(20, nb_))
                del qwc, wnc
                nv16[name] = {"K": Kn, "N": Nn, "rq_us": round(t_rq16, 2), "gemm_us": round(t_g16, 2), "w_gbs": round(wbytes / t_g16 / 1e3, 1),
                              "frac_of_hbm_peak": round(wbytes / t_g16 / 1e3 / PEAK_HBM_GBS, 4),
                              "bf16_gemm_us": round(t_b16, 2), "speedup_vs_bf16": round(t_b16 / (t_rq16 + t_g16), 2)}
                del xn, wn, qa, qw, on, wsn_t, wnt
            nv["path"] = "NVFP4 codes dequantized to fp16 (exact) and multiplied on v_mfma_f32_16x16x32_f16: bound by the fp16 MFMA peak"
            result["nvfp4_prefill_70b_shapes"] = nv
            nv16["weights"] = "cold: copies cycled (>= 640 MB in all), for the bf16 baseline too"
            result["nvfp4_m16_70b_shapes"] = nv16
        except Exception as exc:  # noqa: BLE001 - reported in the JSON line
            extras_errors["nvfp4"] = repr(exc)

        try:
            # ---- offline NVFP4 weight preparation under the three scale policies (Section 4.1 Ingredient 1): abs-max, the
            # per-group squared-error search, and the search alternated with a least-squares tensor scale
            Nw, Kw = 8192, 8192
            ww = (torch.randn(Nw, Kw, device="cuda") * 0.015).to(torch.bfloat16)
            cbw, sbw = fp4.packed_bytes(Nw, Kw, fp4.NVFP4, GL)
            ocw = torch.empty(cbw, dtype=torch.uint8, device="cuda")
            osw = torch.empty(sbw, dtype=torch.uint8, device="cuda")
            prep = {"workload": f"W [{Nw}, {Kw}] bf16 -> NVFP4, Hadamard block 16, GEMM layout"}
            for key, fl_ in (("absmax", 0), ("mse", fp4.SCALE_MSE), ("mse_fit_tensor", fp4.SCALE_MSE | fp4.SCALE_FIT_TENSOR)):
                wsw = torch.empty(max(256, fp4.workspace_bytes(fp4.OP_QUANTIZE_WEIGHTS, Nw, 0, Kw, fp4.NVFP4, GL | fl_)), dtype=torch.uint8, device="cuda")
                prep[key + "_us"] = round(time_us(lambda: fp4.fp4_quantize_weights(ww, 16, fp4.NVFP4, flags=GL | fl_, codes=ocw, scales=osw,
                                                                                    workspace=wsw), n=6, warm=2), 1)
            result["nvfp4_weight_prep_8192x8192"] = prep
            del ww, ocw, osw
        except Exception as exc:  # noqa: BLE001 - reported in the JSON line
            extras_errors["nvfp4_weight_prep"] = repr(exc)

        if extras_errors:
            result["extras_errors"] = extras_errors

    if args.copy_calibration:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(recipe, layers[2], min(M, 4096), 16384)
        # the same oracle on one thread, on a sixteenth of the tokens
        result["cpu_baseline_single_thread"] = cpu_baseline(recipe, layers[2], min(M, 256), 16384, threads=1)

    print(json.dumps(result))


if __name__ == "__main__":
    main()
