#!/usr/bin/env python3
"""Benchmark of the LUT-GEMM hot path on one MI355X.

A step is one pass over the four linear layers of an OPT-175B-shaped decoder block
(QKV 36864x12288, out-proj 12288x12288, FC1 49152x12288, FC2 12288x49152) as batch-1
GEMVs with BCQ weights q = 3, g = 128, enqueued back to back on one stream: table build,
lookup/accumulate, scale epilogue and cross-tile reduction for every layer.  Weights are
synthetic (W ~ N(0, 0.02) fp16 from a fixed seed, greedy BCQ on the host), activations
x ~ N(0, 1) fp16; everything is resident in HBM before the timed region.  Every layer has
enough device copies of its weights that a pass over all of them streams at least 1 GB, and
successive launches rotate through them, so no launch finds its weights in the 256 MB
last-level cache.

Order of a run: (1) a declared, untimed ramp phase of `--ramp` steps that brings the device to
its clocks after the host-side packing; (2) `--warmup` untimed steps; (3) `--regions` timed
regions of exactly `--steps` steps each, every one bracketed by a synchronisation on both
sides and by a HIP event pair on the launch stream.  `value` is the median region (the first
region and the 10th / 90th percentiles are reported beside it).  After that, outside the timed
regions: every layer alone, the same with one weight copy, a read-only bandwidth probe, the
small-batch sweep on FC1, and the fp64 oracle on the host cores, whose outputs are also what
the run's own y is checked against (relative L2 and largest absolute error per layer).

Prints ONE JSON line.
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

HBM_PEAK_GBS = 8000.0
Q, G, MU = 3, 128, 8
LAYERS = ["qkv", "out", "fc1", "fc2"]
ROTATE_BYTES = 1 << 30     # every layer rotates through at least this many bytes of weight copies
# Paper table 1 (A100-80GB, FFN-1 of OPT-175B, 3-bit, g = 128): 0.2250 ms.  Other hardware:
# context only, never used for vs_baseline.
PAPER_A100_FC1_MS = 0.2250

# HBM bytes per launch of the dominant kernel (average over the four layer shapes of a
# step), measured offline with two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE), each
# scaled by what the counter reads for a 256 MiB copy kernel in the same run: summary in
# profiles/lutgemm_gemv_kernel_opt175b_q3_g128_hbm_traffic.md.
MEASURED_TRAFFIC_BYTES = 193.3e6


def algorithmic_bytes(m, n, q, g, batch=1, with_z=False):
    """Section 3.4 eq. 4 in bytes, plus offsets, activations and outputs (fp16)."""
    ng = n // g
    return m * n * q // 8 + 2 * m * ng * q + (2 * m * ng if with_z else 0) + 2 * batch * n + 2 * batch * m


def percentiles(values):
    v = np.asarray(values, dtype=np.float64)
    return {"p10": round(float(np.percentile(v, 10)), 3), "p50": round(float(np.percentile(v, 50)), 3),
            "p90": round(float(np.percentile(v, 90)), 3)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="steps per timed region")
    ap.add_argument("--warmup", type=int, default=5, help="untimed steps right before the timed regions")
    ap.add_argument("--ramp", type=int, default=400,
                    help="untimed steps before the warm-up: the device needs about 100 steps (15 ms) after the "
                         "host-side packing to reach its clocks")
    ap.add_argument("--regions", type=int, default=25, help="timed regions of --steps steps each")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing and parity leg")
    ap.add_argument("--no-batch-sweep", action="store_true", help="skip the FC1 small-batch pass")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three plain 256 MiB device copies before the timed regions (the known-size "
                         "reference that scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives are part of this library).", file=sys.stderr)
        return 2

    import torch

    import paper_2206_09557_amd as L
    from paper_2206_09557_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    L.lib()   # raises if the HIP library is not built: there is no fallback path

    t_setup = time.time()
    layers = []
    for li, name in enumerate(LAYERS):
        m, n = synth.OPT_175B[name]
        W = synth.weights_fp16(m, n, seed=3000 + li)
        bits, alpha, _ = L.lutgemm_pack_bcq(W, Q, G)
        del W
        x = synth.activations_fp16(n, seed=3500 + li)
        wsb = L.lutgemm_workspace_bytes(m, n, Q, G)
        copies = max(2, -(-ROTATE_BYTES // (bits.nbytes + alpha.nbytes)))
        ent = {
            "name": name, "m": m, "n": n, "bytes": algorithmic_bytes(m, n, Q, G), "copies": copies,
            "host": (bits, alpha, x),
            "bits": [torch.from_numpy(bits).cuda() for _ in range(copies)],
            "alpha": [torch.from_numpy(alpha.view(np.int16)).cuda() for _ in range(copies)],
            "x": torch.from_numpy(x.view(np.int16)).cuda(),
            "y": torch.empty(m, dtype=torch.float16, device="cuda"),
            "ws": torch.empty(wsb, dtype=torch.uint8, device="cuda"), "wsb": wsb,
            "grid": L.lutgemm_plan_grid(m, n, Q, G, 1),
        }
        L.lutgemm_workspace_init(ent["ws"], wsb, torch.cuda.current_stream().cuda_stream)
        layers.append(ent)
        print(f"[bench] {name} {m}x{n} packed, {copies} copies uploaded ({time.time() - t_setup:.1f}s)",
              file=sys.stderr, flush=True)

    stream = torch.cuda.current_stream()
    sptr = stream.cuda_stream

    def launch(ent, step, flags=L.LUTGEMM_Y_F16, y=None):
        c = step % ent["copies"]
        L.lutgemm_gemv(ent["x"], ent["bits"][c], ent["alpha"][c], None, ent["y"] if y is None else y, Q, G, MU,
                       ent["m"], ent["n"], flags, ent["ws"], ent["wsb"], sptr)

    if args.copy_probe:
        ref_src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        ref_dst = torch.empty_like(ref_src)
        for _ in range(3):
            ref_dst.copy_(ref_src)
        torch.cuda.synchronize()

    # ---- (1) ramp: untimed, declared in the output ----
    step_no = 0
    t0 = time.perf_counter()
    for _ in range(args.ramp):
        for ent in layers:
            launch(ent, step_no)
        step_no += 1
    torch.cuda.synchronize()
    ramp_ms = (time.perf_counter() - t0) * 1e3

    # ---- (2) warm-up ----
    for _ in range(args.warmup):
        for ent in layers:
            launch(ent, step_no)
        step_no += 1
    torch.cuda.synchronize()

    # ---- (3) timed regions: exactly `steps` steps each; a synchronisation on both sides and
    # one HIP event pair on the launch stream around each ----
    nL = len(layers)
    wall_ms, event_ms = [], []
    for _ in range(args.regions):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(stream)
        for _ in range(args.steps):
            for ent in layers:
                launch(ent, step_no)
            step_no += 1
        ev1.record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        wall_ms.append((t1 - t0) * 1e3 / args.steps)
        event_ms.append(ev0.elapsed_time(ev1) / args.steps)
    y_timed = [ent["y"].cpu().numpy().copy() for ent in layers]   # what the timed launches wrote

    wall_ms_per_step = float(np.median(wall_ms))
    event_ms_per_step = float(np.median(event_ms))
    total_bytes = sum(e["bytes"] for e in layers)
    us_per_gemv = wall_ms_per_step * 1e3 / nL
    step_gbs = total_bytes / (wall_ms_per_step * 1e-3) / 1e9

    # dominant kernel: lutgemm_gemv_kernel, ONE launch per GEMV (table build, lookups, scale
    # epilogue and the split-K reduction are all in it).  Per-launch figures are averages
    # over the four layer shapes of a step, which is what a per-name profiler average is.
    avg_launch_us = event_ms_per_step * 1e3 / nL
    avg_launch_bytes = total_bytes / nL
    achieved = avg_launch_bytes / (avg_launch_us * 1e-6) / 1e9

    # ---- per-layer breakdown, outside the timed regions: each shape alone, back to back,
    # rotating through its copies; then the same with ONE weight copy (whatever the last-level
    # cache keeps of it stays there between launches: "hot", not a figure a decoder sees,
    # where every layer has weights of its own) ----
    def time_alone(ent, rotate, regions=9, reps=20):
        us = []
        for s in range(60):     # (the copies between the passes leave the device idle for a moment)
            launch(ent, s if rotate else 0)
        for r in range(regions):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record(stream)
            for s in range(reps):
                launch(ent, (r * reps + s) if rotate else 0)
            b.record(stream)
            torch.cuda.synchronize()
            us.append(a.elapsed_time(b) * 1e3 / reps)
        return us

    alone = [time_alone(ent, True) for ent in layers]
    for li, ent in enumerate(layers):      # a second round in the same order: 18 regions per layer
        alone[li] += time_alone(ent, True)
    hot = [time_alone(ent, False) for ent in layers]

    # ---- the same step as ONE grouped launch (lutgemm_gemv_group): the four products are
    # independent here (each has its own input), so the workgroups of one layer may follow
    # those of the previous one onto the device without a kernel boundary in between ----
    ms, ns = [e["m"] for e in layers], [e["n"] for e in layers]
    gwsb = L.lutgemm_group_workspace_bytes(ms, ns, Q, G)
    gws = torch.empty(gwsb, dtype=torch.uint8, device="cuda")
    L.lutgemm_workspace_init(gws, gwsb, sptr)
    yg = [torch.empty(e["m"], dtype=torch.float16, device="cuda") for e in layers]
    group_args = []
    for c in range(max(e["copies"] for e in layers)):
        group_args.append(([e["x"] for e in layers], [e["bits"][c % e["copies"]] for e in layers],
                           [e["alpha"][c % e["copies"]] for e in layers]))

    def launch_group(step):
        xs, bs, als = group_args[step % len(group_args)]
        L.lutgemm_gemv_group(xs, bs, als, None, yg, ms, ns, Q, G, MU, L.LUTGEMM_Y_F16, gws, gwsb, sptr)

    for s in range(args.warmup + 3):
        launch_group(s)
    torch.cuda.synchronize()
    group_ms = []
    for r in range(args.regions):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record(stream)
        for s in range(args.steps):
            launch_group(r * args.steps + s)
        ev1.record(stream)
        torch.cuda.synchronize()
        group_ms.append(ev0.elapsed_time(ev1) / args.steps)
    group_equal = all(bool(torch.equal(a, e["y"])) for a, e in zip(yg, layers))
    group_us = float(np.median(group_ms)) * 1e3

    # fp32 output of every layer, once, for the parity report
    y32 = []
    for ent in layers:
        d = torch.empty(ent["m"], dtype=torch.float32, device="cuda")
        launch(ent, 0, L.LUTGEMM_Y_F32, d)
        torch.cuda.synchronize()
        y32.append(d.cpu().numpy())

    # ---- yardstick: what a kernel that only reads gets out of this device's memory, in the
    # access shape of the weight stream, over 1 GiB (far beyond the last-level cache) ----
    probe_bytes = 1 << 30
    probe_src = torch.empty(probe_bytes, dtype=torch.uint8, device="cuda").random_(0, 256)
    probe_sink = torch.empty(8192, dtype=torch.int32, device="cuda")
    for _ in range(3):
        L.lutgemm_stream_read(probe_src, probe_bytes, probe_sink, 32768, sptr)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(10):
        L.lutgemm_stream_read(probe_src, probe_bytes, probe_sink, 32768, sptr)
    b.record(stream)
    torch.cuda.synchronize()
    stream_read_gbs = probe_bytes / (a.elapsed_time(b) * 1e-3 / 10) / 1e9
    del probe_src

    per_layer = []
    for li, ent in enumerate(layers):
        med = float(np.median(alone[li]))
        gbs = ent["bytes"] / (med * 1e-6) / 1e9
        kg, tpg, rs = ent["grid"]
        per_layer.append({"layer": ent["name"], "m": ent["m"], "n": ent["n"], "bytes": ent["bytes"],
                          "us_alone_back_to_back": round(med, 2), "us_alone": percentiles(alone[li]),
                          "gbs": round(gbs, 1), "frac_of_8TBs": round(gbs / HBM_PEAK_GBS, 4),
                          "frac_of_stream_read": round(gbs / stream_read_gbs, 4),
                          "us_same_weight_copy": round(float(np.median(hot[li])), 2),
                          "weight_copies_rotated": ent["copies"],
                          "grid": {"k_groups": kg, "tiles_per_k_group": tpg, "row_ranges": rs}})

    # ---- small batch on the FC1 shape (section 6 of the paper), outside the timed regions:
    # the lookup path (lutgemm_gemm), the plane-wise matrix-core path (lutgemm_gemm_mfma), the
    # dequantise-to-fp16-then-multiply comparison kernel (lutgemm_gemm_dequant_mfma) and
    # lutgemm_gemm left to choose between the first two, side by side ----
    fc1 = layers[2]
    batch_sweep = []
    for bsz in (() if args.no_batch_sweep else (1, 2, 4, 8, 16, 32)):
        xb = torch.randn(bsz, fc1["n"], device="cuda", generator=torch.Generator(device="cuda").manual_seed(77)).half()
        yb = torch.empty(bsz, fc1["m"], dtype=torch.float16, device="cuda")
        wsb = L.lutgemm_workspace_bytes(fc1["m"], fc1["n"], Q, G, batch=bsz)
        wsg = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        L.lutgemm_workspace_init(wsg, wsb, sptr)

        def timed(fn, flags):
            def call(step):
                c = step % fc1["copies"]
                fn(xb, fc1["bits"][c], fc1["alpha"][c], None, yb, Q, G, MU, fc1["m"], fc1["n"], bsz, flags, wsg, wsb, sptr)
            for s in range(3):
                call(s)
            a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for s in range(20):
                call(s)
            e.record(stream)
            torch.cuda.synchronize()
            return a.elapsed_time(e) * 1e3 / 20

        us = timed(L.lutgemm_gemm, L.LUTGEMM_Y_F16)
        us_mfma = timed(L.lutgemm_gemm_mfma, L.LUTGEMM_Y_F16)
        us_dequant = timed(L.lutgemm_gemm_dequant_mfma, L.LUTGEMM_Y_F16)
        us_auto = timed(L.lutgemm_gemm, L.LUTGEMM_Y_F16 | L.LUTGEMM_PATH_AUTO)
        batch_sweep.append({"batch": bsz, "lut_us": round(us, 2), "lut_us_per_vector": round(us / bsz, 2),
                            "mfma_us": round(us_mfma, 2), "mfma_us_per_vector": round(us_mfma / bsz, 2),
                            "dequant_mfma_us": round(us_dequant, 2), "auto_us": round(us_auto, 2)})
        del xb, yb, wsg

    us_regions = [w * 1e3 / nL for w in wall_ms]
    out = {
        "metric": "us/GEMV + achieved HBM GB/s (% roofline), OPT-175B-shape q=3 g=128 batch 1",
        "value": round(us_per_gemv, 3), "unit": "us/GEMV",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms_per_step, 5), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "OPT-175B-shaped decoder layer GEMVs (qkv,out,fc1,fc2), hidden 12288, "
                               "greedy BCQ q=3 g=128, x fp16, batch 1, fp32 accumulate, fp16 out",
                   "gemvs_per_step": nL, "weight_copies_rotated": {e["name"]: e["copies"] for e in layers}},
        "timing": {"ramp_steps": args.ramp, "ramp_ms": round(ramp_ms, 1), "regions": args.regions,
                   "steps_per_region": args.steps, "value_is": "median region",
                   "us_per_gemv": percentiles(us_regions), "us_per_gemv_first_region": round(us_regions[0], 3),
                   "us_per_gemv_min": round(min(us_regions), 3), "us_per_gemv_max": round(max(us_regions), 3)},
        "effective_gbs": round(step_gbs, 1), "frac_of_hbm_peak": round(step_gbs / HBM_PEAK_GBS, 4),
        "stream_read_probe": {"gbs": round(stream_read_gbs, 1), "bytes": probe_bytes,
                              "kernel": "lutgemm_stream_read_kernel (read-only, 16 B per lane)"},
        "frac_of_stream_read": round(step_gbs / stream_read_gbs, 4),
        "decoder_block": {"layers": LAYERS, "us_four_launches": round(event_ms_per_step * 1e3, 2),
                          "us_one_grouped_launch": round(group_us, 2),
                          "us_one_grouped_launch_p10_p90": [round(float(np.percentile(group_ms, 10)) * 1e3, 2),
                                                            round(float(np.percentile(group_ms, 90)) * 1e3, 2)],
                          "grouped_gbs": round(total_bytes / (group_us * 1e-6) / 1e9, 1),
                          "grouped_frac_of_8TBs": round(total_bytes / (group_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                          "grouped_outputs_equal_separate_launches_bitwise": group_equal,
                          "note": "lutgemm_gemv_group: one launch for four independent products; `value` is NOT "
                                  "this figure but the four separate launches a dependent chain needs"},
        "per_layer": per_layer,
        "fc1_batch_sweep": batch_sweep,
        "paper_context": {"fc1_ms": PAPER_A100_FC1_MS, "hardware": "A100-80GB (paper table 1)"},
        "roofline": {"bound": "hbm", "kernel": "lutgemm_gemv_kernel<3,false,0,0>",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES,
                     "bytes_per_launch": avg_launch_bytes, "avg_launch_us": round(avg_launch_us, 3)},
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["parity_vs_oracle"] = cpu_baseline(layers, y_timed, y32)
    print(json.dumps(out), flush=True)
    return 0


def cpu_baseline(layers, y_timed, y32):
    """The fp64 C oracle, as it stands, on the host cores: the whole FC1 GEMV, repeated for
    about ten seconds (a row sample scaled to the whole if one run takes longer); then one
    whole GEMV of every layer of the step, whose outputs are the reference the run's own
    outputs (fp16 from the timed launches, fp32 from one extra launch) are compared with."""
    from oracle import bcq_oracle as O
    from oracle import c_oracle
    ent = layers[2]
    bits, alpha, x = ent["host"]
    m, n = ent["m"], ent["n"]
    rng = np.random.default_rng(99)

    def timed(nrows):
        rows = np.sort(rng.choice(m, size=nrows, replace=False))
        t0 = time.perf_counter()
        _, used = c_oracle.gemv_packed(bits, alpha, None, x, m, n, Q, G, rows=rows)
        return time.perf_counter() - t0, used

    t_probe, used = timed(256)
    nrows = int(min(m, max(256, 256 * 10.0 / max(t_probe, 1e-4))))
    t, used = timed(nrows)
    reps = 1
    while t < 10.0 and nrows == m and reps < 64:   # the whole GEMV takes under ten seconds: repeat it
        dt, used = timed(nrows)
        t += dt
        reps += 1
    t /= reps
    us_full = t * (m / nrows) * 1e6
    # the smallest workload (one 1024 x 1024 GEMV) on a single thread, whole
    from paper_2206_09557_amd import synth
    import paper_2206_09557_amd as L
    Ws = synth.weights_fp16(1024, 1024, seed=1000)
    bs, als, _ = L.lutgemm_pack_bcq(Ws, Q, G)
    xs = synth.activations_fp16(1024, seed=1500)
    c_oracle.gemv_packed(bs, als, None, xs, 1024, 1024, Q, G, nthreads=1)
    t0 = time.perf_counter()
    for _ in range(5):
        c_oracle.gemv_packed(bs, als, None, xs, 1024, 1024, Q, G, nthreads=1)
    small_us = (time.perf_counter() - t0) / 5 * 1e6

    per_layer, parity = {}, []
    for li, e in enumerate(layers):
        b_, a_, x_ = e["host"]
        t0 = time.perf_counter()
        # (the one-thread run above left the thread count at one)
        y_ref, _ = c_oracle.gemv_packed(b_, a_, None, x_, e["m"], e["n"], Q, G, nthreads=int(used))
        per_layer[e["name"]] = round((time.perf_counter() - t0) * 1e6, 1)
        xinf = float(np.abs(x_.astype(np.float64)).max())
        a_dec = np.abs(O.decode_alpha(a_, e["m"], e["n"] // G, Q).astype(np.float64)).sum(axis=0)   # [m][NG]
        strict = 1e-2 * xinf * a_dec.max(axis=1)
        row_l1 = 1e-2 * xinf * G * a_dec.sum(axis=1)
        norm = float(np.linalg.norm(y_ref))
        e16 = np.abs(y_timed[li].astype(np.float64) - y_ref)
        e32 = np.abs(y32[li].astype(np.float64) - y_ref)
        parity.append({
            "layer": e["name"], "rows_compared": int(e["m"]),
            "fp16_out": {"rel_l2": float(f"{np.linalg.norm(y_timed[li].astype(np.float64) - y_ref) / norm:.3e}"),
                         "max_abs": float(f"{e16.max():.3e}"), "limit_rel_l2": 1e-3,
                         "rows_over_1e-2_xinf_row_l1": int((e16 > row_l1).sum())},
            "fp32_out": {"rel_l2": float(f"{np.linalg.norm(y32[li].astype(np.float64) - y_ref) / norm:.3e}"),
                         "max_abs": float(f"{e32.max():.3e}"), "limit_rel_l2": 1e-5,
                         "smallest_strict_bound": float(f"{strict.min():.3e}"),
                         "rows_over_1e-2_xinf_max_group_sum_alpha": int((e32 > strict).sum())},
        })
    baseline = {"value": round(us_full, 1), "unit": "us/GEMV", "cores": int(used), "kind": "oracle",
                "per_layer_us": per_layer,
                "sample": f"fp64 C oracle on {nrows} of {m} rows of the FC1 49152x12288 GEMV "
                          f"({t:.2f} s each, mean of {reps} runs), scaled by m/rows",
                "gemv_1024x1024_one_thread_us": round(small_us, 1)}
    return baseline, parity


if __name__ == "__main__":
    sys.exit(main())
