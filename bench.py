#!/usr/bin/env python3
"""Throughput of the CMPQ quantization path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload block70b]

A step is one pass of the whole path over one decoder block (or layer) of synthetic
input already resident in HBM: activation statistics for every distinct input, then for
each linear layer the orientation copy, O_act, Algorithm 1, preliminary k-means, O_q,
final k-means, packing and the reconstruction error.  Prints ONE JSON line:
Mparams/s, the roofline figures of the dominant kernel (k-means) and of the
memory-bound kernels - each kernel bracketed by events right around its launch, on its
launch stream, in steps that run on one stream so that no other launch shares the GPU,
and again inside the timed steps - and the CPU oracle timed on a bounded sample of the
same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X's published fp32 vector peak: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz x 2 (a
# fused multiply-add counts as two) x 2 (two packed pairs per lane) = 157.3 TFLOP/s.  The
# k-means figure is quoted against it.  Compares, adds and selects are neither fused nor packed:
# one result per lane and clock, 256 x 64 x 2.4e9 = 39.3 T results/s, is the rate at which vector
# instructions can issue at all (the clock is the data sheet's, not measured).
FP32_PEAK_TFLOPS = 157.3
ISSUE_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12
HBM_PEAK_GBS = 8000.0
# Constants taken from the kept rocprofv3 --pmc summaries (bench.py cannot collect counters):
# mean HBM bytes per k-means launch (FETCH_SIZE + WRITE_SIZE scaled by a plain copy of known
# size) and mean vector-ALU instructions per k-means launch (SQ_INSTS_VALU, per wavefront).
KMEANS_TRAFFIC_BYTES = {"block70b": 583.6e6}
KMEANS_VALU_WAVE_INSTS_PER_STEP = {"block70b": 1.85e9}     # 14 launches
KMEANS_COUNTERS_FILE = "profiles/kmeans_bucket_block70b_counters.txt"


def measured_shader_clock(B, dev):
    """GHz of the shader clock while the vector ALUs of all compute units are busy."""
    import torch
    n_wg = 4 * torch.cuda.get_device_properties(dev).multi_processor_count
    ticks = torch.zeros((n_wg, 2), dtype=torch.int64, device=dev)
    B.shader_clock_probe(200, ticks)           # warm-up: clocks ramp
    khz = B.shader_clock_probe(2000, ticks)
    torch.cuda.synchronize()
    t = ticks.cpu().double()
    if not bool((t[:, 1] > 0).all()):
        return None
    return float((t[:, 0] / t[:, 1]).mean() * khz * 1e3 / 1e9)


def credited_kmeans_flops(result, iters, coded=True):
    """Per weight and Lloyd round: K-1 nearest-level compares and 2 accumulations; the
    final coding (where the pass writes codes) K-1 compares.  Summed over the channels that
    are quantized."""
    total = 0
    for b, c in zip(result.bit_set, result.counts):
        K = 1 << b
        total += c * result.d_out * (iters * (K + 1) + (K - 1 if coded else 0))
    return total


def cpu_baseline(wl, weights, acts):
    """The oracle, as it stands, on a bounded sample of the workload: the first layer cut to a
    few thousand input channels, and for a block also a slice of its widest layer (the longest
    channels, which hold most of the block's weights), 2048 calibration tokens each; sized to
    keep the run to roughly 10-30 s."""
    import oracle
    oracle.build()
    picks = [(wl.layers[0], 16_800_000)]
    if len(wl.layers) > 1:
        widest = max(wl.layers, key=lambda l: l.d_out)
        if widest is not wl.layers[0]:
            picks.append((widest, 34_000_000))
    total, dt, what = 0, 0.0, []
    for layer, target in picks:
        ch = max(8, min(layer.d_in, target // layer.d_out))
        tok = min(2048, wl.x_shapes[layer.x_key][0])
        W = weights[layer.name][:, :ch].t().contiguous().cpu().numpy()          # [ch, d_out]
        X = acts[layer.x_key][:tok, :ch].contiguous().cpu().numpy()
        t0 = time.perf_counter()
        oracle.quantize_layer(W, X, wl.bit_set, wl.avg_bits, wl.rho_act_ppm, wl.rho_q_ppm, wl.iters)
        dt += time.perf_counter() - t0
        total += ch * layer.d_out
        what.append(f"{layer.name} cut to its first {ch} of {layer.d_in} input channels ({ch}x{layer.d_out} "
                    f"weights, {tok} of {wl.x_shapes[layer.x_key][0]} tokens)")
    return {"value": total / dt / 1e6, "unit": "Mparams/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": "; ".join(what) + "; whole path incl. both k-means passes"}


def deployed_matvec(P, B, torch, out, layers, wl, acts, reps):
    """The consumer of the stored format: one token through the 7 products of the block just
    quantized (Sec. 6 / Fig. 4).  HBM bound: the packed codes are read once per token."""
    dev = next(iter(out.values())).codes.device
    ws = B.Workspace(dev)
    deps = {name: P.prepare_deployment(out[name], ws) for name, _ in layers}
    xs = {name: acts[x_key][:1].to(torch.float16).contiguous() for name, x_key in layers}
    algo_bytes = 0
    for name, _ in layers:
        d = deps[name]
        algo_bytes += sum(t.numel() * t.element_size() for t in d.packed + d.lut + d.chan_idx if t is not None)
        algo_bytes += d.W_act.numel() * 2 + d.row_idx.numel() * 8 + d.colptr.numel() * 4 + d.d_in * 2 + d.d_out * 4
    ys = {name: torch.empty((1, deps[name].d_out), dtype=torch.float32, device=dev) for name, _ in layers}

    def per_layer():
        for name, _ in layers:
            deps[name].matvec_into(xs[name], ys[name], ws)

    # products that read the same input can run side by side (query/key/value; gate/up)
    by_input = {}
    for name, x_key in layers:
        by_input.setdefault(x_key, []).append(name)
    groups = [(P.group_products([deps[n] for n in names]), [xs[n] for n in names], [ys[n] for n in names])
              for names in by_input.values()]
    whole = (P.group_products([deps[n] for n, _ in layers]), [xs[n] for n, _ in layers], [ys[n] for n, _ in layers])

    def grouped():
        for call, gx, gy in groups:
            call(gx, gy, ws)

    def one_group():
        whole[0](whole[1], whole[2], ws)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    dt_layer, dt, dt_whole = timed(per_layer), timed(grouped), timed(one_group)
    # the variant that adds the packed rows up in FP16, same grouping (its own outputs)
    ys_h = {name: torch.empty_like(ys[name]) for name, _ in layers}
    groups_h = [(P.group_products([deps[n] for n in names], fp16acc=True), [xs[n] for n in names],
                 [ys_h[n] for n in names]) for names in by_input.values()]
    whole_h = (P.group_products([deps[n] for n, _ in layers], fp16acc=True), [xs[n] for n, _ in layers],
               [ys_h[n] for n, _ in layers])

    def grouped_h():
        for call, gx, gy in groups_h:
            call(gx, gy, ws)

    dt_h, dt_whole_h = timed(grouped_h), timed(lambda: whole_h[0](whole_h[1], whole_h[2], ws))
    torch.cuda.synchronize()
    num = sum(float((ys_h[n].double() - ys[n].double()).pow(2).sum()) for n, _ in layers)
    den = sum(float(ys[n].double().pow(2).sum()) for n, _ in layers)
    graph = P.capture_products(groups, ws)      # the same launches as `grouped`, submitted as one HIP graph
    dt_graph = timed(graph.replay)
    return {"what": "Y = x W_hat for one token through all layers of the block, from the stored format; "
                    "products that read the same input are launched together",
            "launch_groups": [names for names in by_input.values()],
            "ms_per_token": dt * 1e3, "Gweights_per_s": wl.params / dt / 1e9,
            "ms_per_token_launches_in_a_hip_graph": dt_graph * 1e3,
            "ms_per_token_one_call_per_layer": dt_layer * 1e3,
            "ms_per_token_all_products_in_one_group": dt_whole * 1e3,
            "roofline": {"bound": "hbm", "achieved": algo_bytes / dt / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": algo_bytes / dt / 1e9 / HBM_PEAK_GBS,
                         "algorithmic_bytes_per_token": algo_bytes},
            "fp16_sums": {"what": "the same products with the packed rows added up in FP16 "
                                  "(cmpq_lut_matvec_group_fp16acc), same grouping",
                          "ms_per_token": dt_h * 1e3, "ms_per_token_all_products_in_one_group": dt_whole_h * 1e3,
                          "hbm_frac": algo_bytes / dt_h / 1e9 / HBM_PEAK_GBS,
                          "relative_rms_difference_from_fp32_sums": (num / den) ** 0.5 if den > 0 else None}}


def rtn_variant(P, B, torch, out, layers, wl, reps):
    """CMPQ with the uniform quantizer (App. A.2): O_act at 0.5 %, Algorithm 1 and round-to-nearest
    in groups of 128 for every layer of the block, on the d_in x d_out copies already in HBM.
    HBM bound: a weight is read once (2 bytes) and its code written once (1 byte)."""
    dev = next(iter(out.values())).codes.device
    ws = B.Workspace(dev)

    def block():
        for name, _ in layers:
            r = out[name]
            P.quantize_layer_rtn(r.W_t, r.sumsq, wl.bit_set, wl.avg_bits, 5000, 128, ws, with_error=True,
                                 transposed=True)

    block()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        block()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    algo = sum(out[n].d_in * out[n].d_out * (out[n].W_t.element_size() + 1)
               + out[n].d_in * -(-out[n].d_out // 128) * 8 for n, _ in layers)
    return {"what": "uniform round-to-nearest in groups of 128 with the widths of Algorithm 1, all layers, "
                    "with the reconstruction error",
            "ms_per_block": dt * 1e3, "Mparams_per_s": wl.params / dt / 1e6,
            "roofline": {"bound": "hbm", "achieved": algo / dt / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": algo / dt / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes_per_block": algo}}


def retarget(P, B, torch, out, layers, wl, reps):
    """Other average widths for the block just quantized, from one kept K-means run per width
    (the cost the paper's closing section names): the first pass becomes a row-wise choice."""
    dev = next(iter(out.values())).codes.device
    ws = B.Workspace(dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    caches = {n: P.build_width_cache(out[n].W_t, wl.bit_set, wl.iters, ws, transposed=True) for n, _ in layers}
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t0) * 1e3
    lo, hi = min(wl.bit_set), max(wl.bit_set)
    budgets = [lo + (hi - lo) * f for f in (0.2, 0.5, 0.8)]

    def block(avg):
        for n, _ in layers:
            P.quantize_layer_from_cache(caches[n], out[n].sumsq, avg, wl.rho_act_ppm, wl.rho_q_ppm, ws,
                                        with_error=True)

    block(budgets[0])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        for avg in budgets:
            block(avg)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / (reps * len(budgets))
    return {"what": "the block at another average width from kept per-width runs (one stream; without "
                    "statistics, orientation and the first K-means pass)",
            "budgets": [round(b, 3) for b in budgets], "build_ms": build_ms,
            "ms_per_budget": dt * 1e3, "Mparams_per_s": wl.params / dt / 1e6}


def lut4_variant(P, B, torch, out, layers, wl, reps):
    """The tables of the block just quantized held in 4 bits per entry (Sec. 5.1 / Tab. 7): codes
    into one 16-level table per layer found by K-means over the layer's centres, the stored format
    written again, and the reconstruction error with them; the uniform 16-level grid beside it."""
    dev = next(iter(out.values())).codes.device
    ws = B.Workspace(dev)

    def block(mode):
        return [P.tables_in_4_bits(out[n], ws, with_error=True, mode=mode, iters=wl.iters)[2] for n, _ in layers]

    block(B.LUT4_CODEBOOK)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        qs = block(B.LUT4_CODEBOOK)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    e16 = sum(float(out[n].err_total[0]) for n, _ in layers)
    e4 = sum(float(q.err_total[0]) for q in qs)
    e4u = sum(float(q.err_total[0]) for q in block(B.LUT4_UNIFORM))
    return {"what": "look-up tables in 4 bits (codes into one 16-level table per layer, K-means over the layer's "
                    "centres): tables, stored format and error of all layers", "ms_per_block": dt * 1e3,
            "weighted_error_vs_fp16_tables": e4 / e16 if e16 > 0 else None,
            "weighted_error_vs_fp16_tables_uniform_grid": e4u / e16 if e16 > 0 else None}


def continued_final_pass(P, torch, step_variant, out, layers, wl, rounds, reps, n_streams, dev):
    """The block with the final K-means of every layer continued from the preliminary levels for
    `rounds` rounds instead of started again from the quantiles (a variant; the paper names no
    start): time per block in the launch configuration of the headline figure, and the weighted
    reconstruction error against that of the default."""
    res = {}
    e_default = sum(float(out[n].err_total[0]) for n, _ in layers)
    for r in rounds:
        o = step_variant(r)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            o = step_variant(r)
        if n_streams > 1:
            P.join_streams(dev, n_streams)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        e = sum(float(o[n].err_total[0]) for n, _ in layers)
        res[str(r)] = {"ms_per_block": dt * 1e3, "Mparams_per_s": wl.params / dt / 1e6,
                       "weighted_error_vs_default": e / e_default if e_default > 0 else None}
        del o
    return {"what": "final K-means continued from the preliminary levels for r rounds (not the default: both "
                    "passes start from the quantiles); keyed by r", "rounds": res}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="block70b",
                    help="block70b (default, the headline target), block13b, block7b, q7b, tiny")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--joined-steps", type=int, default=None,
                    help="steps of the extra run that joins the streams after every step (default: --steps; 0: none)")
    ap.add_argument("--continued-reps", type=int, default=3,
                    help="repetitions of the variant whose final K-means continues from the preliminary "
                         "levels; 0: skip")
    ap.add_argument("--streams", type=int, default=3,
                    help="streams the independent layers of a block are shared out over (default 3)")
    ap.add_argument("--serial-steps", type=int, default=2,
                    help="extra untimed steps on one stream for the per-stage and per-kernel figures "
                         "that overlap would blur (at least 1)")
    ap.add_argument("--deploy-reps", type=int, default=20,
                    help="repetitions of the one-token product with the deployed block (Fig. 4), reported "
                         "beside the headline figure; 0: skip")
    ap.add_argument("--retarget-reps", type=int, default=2,
                    help="repetitions of three other average widths from kept per-width runs; 0: skip")
    ap.add_argument("--lut4-reps", type=int, default=3,
                    help="repetitions of the block's tables put into 4 bits (Sec. 5.1, Tab. 7); 0: skip")
    ap.add_argument("--rtn-reps", type=int, default=5,
                    help="repetitions of the block through the uniform-quantizer variant (App. A.2), reported "
                         "beside the headline figure; 0: skip")
    ap.add_argument("--two-calls", action="store_true",
                    help="final K-means and stored format + error as two calls (cmpq_kmeans_quantize, then "
                         "cmpq_pack_with_error) instead of the one call whose coding pass writes them")
    ap.add_argument("--no-shared-tables", dest="shared_tables", action="store_false",
                    help="the final K-means builds its per-channel tables again instead of starting from "
                         "the ones the preliminary K-means kept (same results; sharing is the default)")
    ap.add_argument("--prelim-codes", action="store_true",
                    help="the preliminary K-means writes its codes and O_q reads them, instead of ranking the "
                         "distance to the nearest level (same results; not the default)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (outside the timed region): under "
                         "rocprofv3 --pmc it gives the HBM counters a kernel of known traffic to scale by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; every box here has one, and the path needs no "
              "collective (layers are independent).  Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2410_13056_amd import binding as B, pipeline as P, synth
    B.lib()                                       # no library, no benchmark
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = synth.workload(args.workload)
    weights, acts = synth.materialize(wl, dev)
    layers = [(l.name, l.x_key) for l in wl.layers]
    ws = B.Workspace(dev) if args.streams <= 1 else [B.Workspace(dev) for _ in range(args.streams)]
    status = torch.zeros(1, dtype=torch.int32, device=dev)

    def step(timer=None, join=True):
        return P.quantize_block(weights, acts, layers, wl.bit_set, wl.avg_bits, wl.rho_act_ppm,
                                wl.rho_q_ppm, wl.iters, ws, with_error=True, status=status, timer=timer,
                                streams=args.streams, join=join, fused=not args.two_calls,
                                share_tables=args.shared_tables, prelim_codes=args.prelim_codes)

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                            # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        out = step()
        del out
    torch.cuda.synchronize()
    # The timed region: K steps enqueued one after the other, as when a model is quantized block
    # after block; with several streams the queues of one step run on into the next and the
    # streams are joined once, before the closing synchronisation.
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = step(join=False)
    if args.streams > 1:
        P.join_streams(dev, args.streams)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # The same K steps once more with a pair of events around every entry point, on its stream:
    # how long each stage takes while the other streams' launches share the GPU.  (Kept out of
    # the timed steps: 70 event records a step on three streams cost a few per cent.)
    timer = P.StageTimer()
    t_ev = time.perf_counter()
    for _ in range(args.steps):
        o_ev = step(timer, join=False)
    if args.streams > 1:
        P.join_streams(dev, args.streams)
    torch.cuda.synchronize()
    dt_ev = time.perf_counter() - t_ev
    del o_ev
    joined = None
    n_joined = args.steps if args.joined_steps is None else args.joined_steps
    if args.streams > 1 and n_joined > 0:
        # the same steps with every stream joined after every step: no step starts before the
        # one before it has drained
        t1 = time.perf_counter()
        for _ in range(n_joined):
            o2 = step(join=True)
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t1
        del o2
        joined = {"note": "the same steps with the streams joined after every step instead of once at the end",
                  "steps": n_joined, "ms_per_step": dt2 / n_joined * 1e3,
                  "Mparams_per_s": wl.params * n_joined / dt2 / 1e6}
    assert status.item() == 0, "non-finite input flagged"

    stages = timer.totals()
    # One stream: no other launch shares the GPU.  These steps give the per-kernel durations the
    # roofline figures are quoted on (they are what a one-stream kernel trace shows).
    ws1 = ws[0] if args.streams > 1 else ws
    t1 = P.StageTimer(kernels=True)
    n_serial = max(1, args.serial_steps)
    for _ in range(n_serial):
        o1 = P.quantize_block(weights, acts, layers, wl.bit_set, wl.avg_bits, wl.rho_act_ppm,
                              wl.rho_q_ppm, wl.iters, ws1, with_error=True, status=status, timer=t1,
                              fused=not args.two_calls, share_tables=args.shared_tables, prelim_codes=args.prelim_codes)
        del o1
    serial = t1.totals()
    kern = t1.kernel_totals()

    def per_step(table, name, steps):
        n, ms = table.get(name, (0, 0.0))
        return n // steps, ms / steps

    # ---- k-means: the dominant kernel
    # two passes per layer; the preliminary one codes only on the route that hands codes to O_q
    flops = sum(credited_kmeans_flops(r, wl.iters) + credited_kmeans_flops(r, wl.iters, coded=args.prelim_codes)
                for r in out.values())
    n_km = per_step(kern, "kmeans_prelim", n_serial)[0] + per_step(kern, "kmeans_final", n_serial)[0]
    ms_km = per_step(kern, "kmeans_prelim", n_serial)[1] + per_step(kern, "kmeans_final", n_serial)[1]
    avg_launch_s = ms_km / 1e3 / max(n_km, 1)
    achieved = flops / max(n_km, 1) / avg_launch_s / 1e12
    ms_km_timed = per_step(stages, "kmeans_prelim", args.steps)[1] + per_step(stages, "kmeans_final", args.steps)[1]
    roofline = {"kernel": "kmeans_bucket_kernel", "bound": "alu", "achieved": achieved, "peak": FP32_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / FP32_PEAK_TFLOPS,
                "traffic": KMEANS_TRAFFIC_BYTES.get(wl.name),
                "what": "credited work (per weight and round K-1 compares + 2 accumulations, K-1 for the coding "
                        "of the final pass: what a brute-force Lloyd executes) / mean duration of the kernel on one stream, "
                        "against the published fp32 vector peak; the kernel reaches the same bits with fewer "
                        "operations, see `executed`",
                "launches_per_step": n_km, "avg_launch_ms": avg_launch_s * 1e3,
                "credited_flop_per_launch": flops / max(n_km, 1),
                "traffic_from": "constant: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under profiles/",
                "avg_entry_point_ms_in_timed_region": ms_km_timed / max(n_km, 1),
                "timed_region_note": "events around the entry point on its stream in a repeat of the timed steps; with "
                                     "several streams the launches share the GPU, so this is longer than a launch alone"}
    valu = KMEANS_VALU_WAVE_INSTS_PER_STEP.get(wl.name)
    if valu is not None:
        lane_ops = valu * 64
        roofline["executed"] = {
            "what": "vector-ALU instructions the kernel issues (SQ_INSTS_VALU x 64 lanes, a constant from the "
                    "kept counter summary) / the same duration, against one instruction per lane and clock",
            "lane_ops_per_step": lane_ops, "achieved_Tops": lane_ops / (ms_km / 1e3) / 1e12,
            "issue_peak_Tops": ISSUE_PEAK_TOPS, "frac_of_issue_peak": lane_ops / (ms_km / 1e3) / 1e12 / ISSUE_PEAK_TOPS,
            "clock_assumed_GHz": 2.4, "from": KMEANS_COUNTERS_FILE,
            "executed_over_credited": lane_ops / flops}
        clock = measured_shader_clock(B, dev)
        if clock is not None:
            roofline["executed"]["clock_measured_GHz"] = clock
            roofline["executed"]["frac_of_issue_peak_at_measured_clock"] = (
                roofline["executed"]["frac_of_issue_peak"] * 2.4 / clock)
            roofline["executed"]["clock_note"] = ("shader-clock counter against the constant-rate counter inside a "
                                                  "kernel that keeps every compute unit on dependent FMAs for ~1 ms "
                                                  "(mean over workgroups); the peaks above stay the published ones")

    # ---- the memory-bound kernels: algorithmic bytes / kernel duration on one stream
    x_bytes = sum(acts[k].numel() * acts[k].element_size() for k in acts)
    esz = 2 if wl.dtype == "f16" else 4
    live = sum(sum(r.counts) * r.d_out for r in out.values())                       # weights outside O_act
    pe_bytes = sum(r.d_in * r.d_out * (esz + 1) + sum(c * ((r.d_out * b + 31) // 32) * 4 for b, c in zip(r.bit_set, r.counts))
                   for r in out.values())
    hbm = {}
    for kernel, stage, nbytes, what in (
            ("act_stats_vec_kernel", "act_stats", x_bytes, "X read once"),
            ("transpose16_vec_kernel", "transpose", 2 * esz * wl.params, "W read and written once"),
            ("wsel_stage_kernel", "outlier_weights", live * (esz + (1 if args.prelim_codes else 0)),
             "weight and code of every candidate read once" if args.prelim_codes else "weight of every candidate read once"),
            ("pack_error_kernel", "pack_with_error", pe_bytes, "weight and code read once, packed words written")):
        n_k, ms_k = per_step(kern, stage, n_serial)
        if n_k == 0 or ms_k <= 0:
            continue
        gbs = nbytes / (ms_k / 1e3) / 1e9
        hbm[kernel] = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                       "algorithmic_bytes_per_step": nbytes, "what": what, "launches_per_step": n_k,
                       "ms_per_step": ms_k, "entry_point_ms_per_step": per_step(serial, stage, n_serial)[1],
                       "entry_point_ms_per_step_in_timed_region": per_step(stages, stage, args.steps)[1]}
    line = {
        "metric": "Mparams/s quantized (whole CMPQ path, both k-means passes) at the target average bits",
        "value": wl.params * args.steps / dt / 1e6,
        "unit": "Mparams/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int64 (exact sums over 16-bit keys, one f64 divide per level)" if wl.dtype == "f16"
                 else "f32 compares, f64 sums (f32 weights)",
        "data": "synthetic",
        "config": {"workload": wl.name, "params": wl.params, "layers": len(wl.layers),
                   "weights": wl.dtype, "bit_set": list(wl.bit_set), "avg_bits": wl.avg_bits,
                   "rho_act_ppm": wl.rho_act_ppm, "rho_q_ppm": wl.rho_q_ppm, "iters": wl.iters,
                   "tokens": {k: v[0] for k, v in wl.x_shapes.items()}},
        "roofline": roofline,
        "hbm_kernels": hbm,
        "stages_ms_per_step": {k: round(v[1] / args.steps, 4) for k, v in sorted(stages.items())},
        "stages_note": "entry-point durations from events on the launch streams, in a repeat of the timed steps "
                       "(%.3f ms per step with the events in place)" % (dt_ev / args.steps * 1e3),
        "streams": args.streams,
        "preliminary_pass": ("levels and codes; O_q reads the codes" if args.prelim_codes else
                             "levels only; O_q ranks the distance to the nearest level") +
                            ("; per-channel tables kept for the final pass" if args.shared_tables else ""),
        "final_pass": "two calls: cmpq_kmeans_quantize, cmpq_pack_with_error" if args.two_calls else
                      "one call: cmpq_kmeans_quantize_job writes the stored format and the error from its coding pass",
        "serial": {
            "note": "same step on one stream, run after the timed region: launches do not overlap; the "
                    "per-kernel figures above come from these steps",
            "steps": n_serial,
            "ms_per_step": round(sum(v[1] for v in serial.values()) / n_serial, 4),
            "stages_ms_per_step": {k: round(v[1] / n_serial, 4) for k, v in sorted(serial.items())},
            "kernels_ms_per_step": {k: round(v[1] / n_serial, 4) for k, v in sorted(kern.items())}},
    }
    if joined is not None:
        line["steps_joined_one_by_one"] = joined
    if args.deploy_reps > 0:
        line["deployed_matvec"] = deployed_matvec(P, B, torch, out, layers, wl, acts, args.deploy_reps)
    if args.retarget_reps > 0:
        line["retarget"] = retarget(P, B, torch, out, layers, wl, args.retarget_reps)
    if args.lut4_reps > 0:
        line["lut4_variant"] = lut4_variant(P, B, torch, out, layers, wl, args.lut4_reps)
    if args.continued_reps > 0:
        def step_variant(r):
            return P.quantize_block(weights, acts, layers, wl.bit_set, wl.avg_bits, wl.rho_act_ppm,
                                    wl.rho_q_ppm, wl.iters, ws, with_error=True, status=status,
                                    streams=args.streams, join=False, iters_final_from_prelim=r,
                                    fused=not args.two_calls, share_tables=args.shared_tables, prelim_codes=args.prelim_codes)
        line["final_pass_continued_from_prelim"] = continued_final_pass(
            P, torch, step_variant, out, layers, wl, (5, wl.iters), args.continued_reps, args.streams, dev)
    if args.rtn_reps > 0:
        line["rtn_variant"] = rtn_variant(P, B, torch, out, layers, wl, args.rtn_reps)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, weights, acts)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
