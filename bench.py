#!/usr/bin/env python3
"""Benchmark of the NEZHA draft + verify step on one MI355X.

One "step" is one full decode of a batch: L calls of nezha_draft_step (beam expansion at every
level, hash-set verification and pruning at the last) on synthetic inputs that are already
resident in device memory.  The metric is verified candidate items per second: the B*K*K
level-L candidates submitted to the verifier per decode, divided by the decode time.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|serving|wide|recall|tiny|
                    paper_yelp|paper_beauty|paper_games|stress|user_gemm] [--eager]
                    [--no-cpu-baseline] [--no-serving-leg]

The default workload is the largest configuration that runs on one GPU (Large: B = 4096, d = 2048,
T_l = 4096, K = 100, 5 * 10^7 items).  Since the metric also names the p50 latency of a step, the
same line carries a short second leg under `serving_latency`: the Serving configuration's decode
latency percentiles (its own set-up, 20 warm-up and 200 timed decodes; never part of `value`).

Prints ONE JSON line.  `roofline` describes the kernel that took the most time, timed with HIP
events by the library itself; `cpu_baseline` is the CPU oracle timed on the host cores."""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth  # noqa: E402
import paper_2511_18793_amd as nz  # noqa: E402

# MI355X peaks used for the roofline fractions.
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
# plain (unpacked, non-FMA) fp32 vector issue rate: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz
PEAK_ALU_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# issue slots the fused expansion needs per logit: add of the user part (folded into the MFMA
# accumulator, not counted), scale (1), exponential (quarter rate: 4), sum (1), running max (1),
# threshold compare (1)
EXPAND_SLOTS_PER_LOGIT = 8
BUCKET_BYTES = 64
# Which kernels of a profiler trace belong to a kernel kind of the library's own event timing.
TRACE_NAMES = {
    "expand_kernel": ("expand_small_kernel", "expand_chunked_kernel", "expand_kernel"),
    "expand_request_kernel": ("expand_request_kernel",),
    "user_gemm_kernel": ("user_gemm_",),
    "merge_kernel": ("merge_kernel",),
    "decode_small_kernel": ("decode_small_kernel",),
    "level_small_kernel": ("level_small_kernel",),
    "wide_logits_kernel": ("wide_fused_bf16_kernel", "wide_logits_"),
    "wide_rows_kernel": ("wide_rows_kernel",),
    "wide_select_kernel": ("wide_collect_kernel", "wide_finish_kernel", "wide_select_kernel",
                           "wide_bound_kernel"),
    "verify_probe_kernel": ("verify_probe_kernel",),
}


def traffic_from_profile(workload, kind):
    """HBM bytes per launch of a kernel kind, read from the counter table of the rocprofv3 summary
    profiles/<kind's kernel>__<workload>.md (FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each
    times the scale factor its plain-copy calibration gave; the dispatch-weighted mean over the
    kernel's template variants).  Nothing is pasted here: the figure is whatever the committed
    summary holds, and `source` names the file and the commit it was measured at.  (None, reason)
    when no summary covers the kernel."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*__%s.md" % workload))):
        text = open(path).read()
        m = re.search(r"FETCH_SIZE x ([0-9]+(?:\.[0-9]+)?), WRITE_SIZE x ([0-9]+(?:\.[0-9]+)?)", text)
        if not m:
            continue
        ff, wf = float(m.group(1)), float(m.group(2))
        total = n = 0.0
        in_counters = False
        for line in text.splitlines():
            if line.startswith("## "):
                in_counters = "traffic counters" in line
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if not in_counters or len(cells) != 4 or not cells[0].startswith(TRACE_NAMES.get(kind, (kind,))):
                continue
            try:
                f, w, k = float(cells[1]), float(cells[2]), float(cells[3])
            except ValueError:
                continue
            total += (f * ff + w * wf) * 1024.0 * k
            n += k
        if n:
            c = re.search(r"[Mm]easured at commit[: ]+([0-9a-f]{7,40})", text)
            return total / n, "%s (measured at commit %s)" % (
                os.path.relpath(path, ROOT), c.group(1) if c else "not recorded")
    return None, "no rocprofv3 counter summary for this kernel and workload under profiles/"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--seed", type=int, default=42)
    ap.add_argument("--launch", choices=("auto", "direct", "graph"), default="auto",
                    help="how a step reaches the GPU: 'direct' = one call of the C ABI per step "
                         "(nezha_decode where it applies), 'graph' = replay of a HIP graph that "
                         "holds the step; 'auto' = direct where one call per step applies (bf16, "
                         "weights packed at set-up), else graph")
    ap.add_argument("--eager", action="store_true", help="same as --launch direct")
    ap.add_argument("--two-streams", action="store_true",
                    help="also time the same decodes issued alternately on two streams (reported "
                         "as two_stream_ms_per_step, never as value)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-serving-leg", action="store_true",
                    help="skip the Serving latency leg that the default (Large) run appends")
    ap.add_argument("--pack-per-call", action="store_true",
                    help="rearrange the weights inside every step instead of once at set-up")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain elementwise copy of 256 MiB (torch.mul by 1) three "
                         "times, so that hardware counters of a profiler run can be scaled")
    ap.add_argument("--transition", choices=("add", "rnn"), default="add",
                    help="Transition of Eq. 3: additive (the measured path) or the recurrent cell "
                         "c' = tanh(U c + e_l) (variant; U and the embeddings are synthetic)")
    ap.add_argument("--head", choices=("nezha", "nezha1", "nezha2", "mtp"), default="nezha",
                    help="comparison heads of the ablation (Sec. 4.3), same kernels with a term "
                         "removed: nezha1 = no autoregressive state; nezha2 = no placeholder "
                         "hidden states (one hidden vector for all levels, state kept); mtp = "
                         "parallel heads on one hidden state, no state")
    ap.add_argument("--prefix-sets", action="store_true",
                    help="variant: also verify each level below L against the set of the "
                         "catalog's prefixes of that length")
    ap.add_argument("--gemm-shape", default="4096x2048x4096",
                    help="--workload user_gemm: B x d x T_l of the projection")
    ap.add_argument("--batch", type=int, default=0, help="override B (debugging)")
    ap.add_argument("--catalog", type=int, default=0, help="override N (debugging)")
    return ap.parse_args()


def percentile(xs, q):
    return float(np.percentile(np.asarray(xs, dtype=np.float64), q))


def kernel_models(cfg):
    """Algorithmic work of one launch of each kernel at each level: (bound, unit, amount)."""
    B, K, V, d, e, L = cfg.B, cfg.K, cfg.V, cfg.d, cfg.e, cfg.L
    esz = 2 if cfg.dtype == "bf16" else 4
    per_level = []
    # all levels in one launch (nezha_draft_levels) when every level fits the single-launch kernel
    one_launch = (cfg.dtype == "bf16" and K <= 32 and V <= 512 and e in (32, 64, 128, 256))
    for level in range(1, L + 1):
        K_in = 1 if level == 1 else K
        rows = B * K_in
        probes = rows * K if level == L else 0
        # which kernel takes the expansion (the library's own rule, from the shape alone)
        fused = (cfg.dtype == "bf16" and K <= 32 and K_in <= 32 and V <= 512
                 and e in (32, 64, 128, 256))
        per_request = (cfg.dtype == "bf16" and K_in >= 16 and e in (32, 64, 128, 256)
                       and not fused and not (V <= 1024 and K <= 64))
        slots = float(EXPAND_SLOTS_PER_LOGIT) * rows * V
        # beams wider than 128: the level's logits go through HBM (three kernels per level)
        wide = K > 128 or K_in > 128
        if wide:
            fused = per_request = False
            slots = 0.0
        wide_probes = rows * min(K, V) if level == L else 0
        per_level.append({
            "wide_logits_kernel": ("hbm", (4.0 * rows * V + rows * e * esz + 4.0 * B * V) if wide else 0.0),
            "wide_rows_kernel": ("hbm", (8.0 * rows * V + wide_probes * BUCKET_BYTES) if wide else 0.0),
            "wide_select_kernel": ("hbm", (4.0 * rows * V + B * K * (24.0 + (2 * e * esz if level < L else 0)))
                                   if wide else 0.0),
            "pack_weights_kernel": ("hbm", 2.0 * (d + e) * V * esz),
            "user_gemm_kernel": ("mfma", 2.0 * B * d * V),
            "expand_kernel": ("alu", 0.0 if per_request else slots),
            "expand_request_kernel": ("alu", slots if per_request else 0.0),
            "merge_kernel": ("hbm", 0.0 if wide else rows * K * 8.0 + probes * BUCKET_BYTES
                             + B * K * (24.0 + (2 * e * esz if level < L else 0))),
            # expansion, merge, verification and Transition of one level in one launch
            "level_small_kernel": ("alu", 0.0 if one_launch else slots),
            "decode_small_kernel": ("alu", slots if one_launch else 0.0),
        })
    return per_level


class DraftSetup:
    """Inputs, catalog, item set, packed weights and the step function of one draft workload."""


def setup_draft(args, cfg):
    st = DraftSetup()
    dev = torch.device("cuda:0")
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    t0 = time.time()
    x = synth.draft_inputs(cfg, args.seed)
    if args.head in ("nezha2", "mtp"):
        # nezha2: the variant without the placeholder hidden states h_l (one hidden vector, the
        # first, serves every level; the autoregressive state is kept); mtp: parallel heads on
        # that one hidden vector with no state between the levels
        x["H"] = np.repeat(x["H"][:, :1], cfg.L, axis=1).copy()
    H = torch.from_numpy(x["H"]).to(dev).to(dt)
    W = [torch.from_numpy(w).to(dev).to(dt) for w in x["W"]]
    E = [torch.from_numpy(w).to(dev).to(dt) for w in x["E"]]
    bufs = nz.DraftBuffers(cfg.B, cfg.L, cfg.K, cfg.d, cfg.e, cfg.radices, dt, dev)
    U = Unp = None
    if args.transition == "rnn":
        # variant: recurrent cell.  U_l ~ N(0, 1/e); embeddings scaled so that tanh is not linear
        rng = np.random.default_rng(args.seed + 1000)
        Unp = [(rng.standard_normal((cfg.e, cfg.e)) / np.sqrt(cfg.e)).astype(np.float32)
               for _ in range(cfg.L - 1)]
        if cfg.dtype == "bf16":
            Unp = [synth.round_to_bf16(u) for u in Unp]
            x["E"] = [synth.round_to_bf16(em * 25.0) for em in x["E"]]
        else:
            x["E"] = [(em * 25.0).astype(np.float32) for em in x["E"]]
        E = [torch.from_numpy(w).to(dev).to(dt) for w in x["E"]]
        U = [torch.from_numpy(u).to(dev).to(dt) for u in Unp]
    use_state = args.head not in ("mtp", "nezha1")

    # Catalog: Zipf / uniform background, with about 70 % of the unverified top-K beams planted
    # so that about 30 % of them are hallucinations (this pass runs without a verifier).
    free = nz.decode(H, W, E, cfg.radices, cfg.K, None, buffers=bufs, U=U, use_state=use_state)
    torch.cuda.synchronize()
    beams = nz.unpack_keys(free[-1]["key"].cpu().numpy().ravel(), cfg.radices)
    if cfg.catalog == "uniform":
        background = synth.uniform_catalog(cfg.radices, cfg.N, args.seed)[0]
    else:
        background = synth.zipf_catalog(cfg.radices, cfg.N, args.seed, cfg.zipf_s,
                                        depth=2 if cfg.catalog == "zipf12" else 1)
    keep = synth.plant_mask(beams, cfg.radices, args.seed)
    catalog = synth.planted_catalog(cfg.radices, background, beams[keep], beams[~keep], args.seed)
    del background
    itemset = nz.build_itemset(catalog, cfg.radices, cfg.load_factor)
    prefix_sets = None
    if args.prefix_sets:
        prefix_sets = [nz.build_itemset(np.unique(catalog[:, :l], axis=0), cfg.radices[:l],
                                        cfg.load_factor) for l in range(1, cfg.L)]
    st.setup_s = time.time() - t0

    # The head's weights are static in serving: their operand-order form is made once, here,
    # outside the timed region (bf16 only; --pack-per-call keeps the packing inside every step).
    Wrun = W
    if cfg.dtype == "bf16" and not args.pack_per_call:
        Wrun = [nz.pack_weights(l + 1, cfg.L, cfg.radices, W[l], cfg.d) for l in range(cfg.L)]

    plan = None
    if cfg.dtype == "bf16" and not args.pack_per_call and use_state:
        # everything a decode needs, marshalled once: a step is one call of nezha_decode
        plan = nz.DecodePlan(H, Wrun, E, cfg.radices, cfg.K, itemset, buffers=bufs, U=U,
                             prefix_sets=prefix_sets)

    def step():
        if plan is not None:
            plan.run()
        else:
            nz.decode(H, Wrun, E, cfg.radices, cfg.K, itemset, buffers=bufs, U=U,
                      prefix_sets=prefix_sets, use_state=use_state)

    st.dev, st.dt, st.x, st.H, st.E, st.U, st.Unp, st.Wrun = dev, dt, x, H, E, U, Unp, Wrun
    st.bufs, st.catalog, st.itemset, st.prefix_sets, st.keep = bufs, catalog, itemset, prefix_sets, keep
    st.plan, st.step, st.use_state = plan, step, use_state
    return st


def serving_latency_leg(args):
    """p50 / p90 / p99 latency of one decode of the Serving configuration (the shape a latency
    figure belongs to): 20 warm-up and 200 timed decodes, one after the other on one stream, one
    nezha_decode call each.  Reported under `serving_latency`; never part of `value`."""
    cfg = synth.get_config("serving")
    st = setup_draft(args, cfg)
    steps, warmup = 200, 20
    for _ in range(warmup):
        st.step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        st.step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    cands = cfg.B * cfg.K * cfg.K
    ms = ev[0].elapsed_time(ev[-1]) / steps
    return {"workload": "serving", "B": cfg.B, "d": cfg.d, "e": cfg.e, "L": cfg.L, "V": cfg.V,
            "K": cfg.K, "catalog_items": int(st.catalog.shape[0]), "steps": steps, "warmup": warmup,
            "ms_per_step": ms, "p50_step_ms": percentile(per, 50),
            "p90_step_ms": percentile(per, 90), "p99_step_ms": percentile(per, 99),
            "items_per_s": cands / (ms * 1e-3),
            "accepted_per_step": int(st.bufs.outs[-1]["count"].sum().item())}


def bench_draft(args, cfg):
    st = setup_draft(args, cfg)
    dev, dt, x, H, E, U, Unp, Wrun = st.dev, st.dt, st.x, st.H, st.E, st.U, st.Unp, st.Wrun
    bufs, catalog, itemset, prefix_sets, keep = st.bufs, st.catalog, st.itemset, st.prefix_sets, st.keep
    plan, step, setup_s, use_state = st.plan, st.step, st.setup_s, st.use_state

    launch = "direct" if args.eager else args.launch
    if launch == "auto":
        # one host call per step keeps the GPU busy without a graph (replaying a two-kernel graph
        # costs about 8 us between replays on this stack); the Python level loop does not
        launch = "direct" if plan is not None else "graph"
    graph = None
    if launch == "graph":
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay
    else:
        run = step

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t_wall = time.perf_counter()
    ev[0].record()
    for i in range(args.steps):
        run()
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall) * 1e3
    total_ms = ev[0].elapsed_time(ev[-1])
    per_step = [ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)]
    accepted = int(bufs.outs[-1]["count"].sum().item())
    hallucinated = 1.0 - float(keep.mean())

    # Extra figure (never `value`): the same K decodes issued alternately on two streams, each
    # with buffers of its own, as a server would overlap consecutive, independent batches: the
    # projections of one batch run beside the level kernel of the batch before.
    two_stream_ms = None
    if plan is not None and args.two_streams:
        bufs2 = nz.DraftBuffers(cfg.B, cfg.L, cfg.K, cfg.d, cfg.e, cfg.radices, dt, dev)
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        plans = [nz.DecodePlan(H, Wrun, E, cfg.radices, cfg.K, itemset, buffers=b_, U=U,
                               prefix_sets=prefix_sets, stream=s_)
                 for b_, s_ in zip((bufs, bufs2), streams)]
        torch.cuda.synchronize()
        for i in range(args.warmup):
            plans[i & 1].run()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for i in range(args.steps):
            plans[i & 1].run()
        torch.cuda.synchronize()
        two_stream_ms = (time.perf_counter() - t2) * 1e3 / args.steps
        assert torch.equal(bufs.outs[-1]["key"], bufs2.outs[-1]["key"])

    # Per-level latency: the same steps eager, events around each level's nezha_draft_step.
    lev_steps = min(args.steps, 50)
    lev_ev = [[[torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)]
               for _ in range(cfg.L + 1)] for _ in range(lev_steps)]
    for i in range(lev_steps):
        nz.decode(H, Wrun, E, cfg.radices, cfg.K, itemset, buffers=bufs, U=U,
                  prefix_sets=prefix_sets, level_events=lev_ev[i], use_state=use_state)
    torch.cuda.synchronize()
    level_ms = [[lev_ev[i][l][0].elapsed_time(lev_ev[i][l][1]) for i in range(lev_steps)]
                for l in range(cfg.L + 1)]

    # Per-kernel durations: the same steps again, eager, with the library's event timing on.
    nz.profile_reset()
    nz.profile_enable(True)
    prof_steps = min(args.steps, 50)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = nz.profile_read()
    nz.profile_enable(False)
    nz.profile_reset()
    event_overhead_us = nz.profile_event_overhead(200)

    models = kernel_models(cfg)
    kernels = {}
    for name, (launches, ms) in prof.items():
        if name not in models[0]:
            continue
        bound = models[0][name][0]
        work = sum(m[name][1] for m in models) * prof_steps        # all levels, all steps
        kernels[name] = {"bound": bound, "launches": launches, "avg_us": 1e3 * ms / launches,
                         "total_ms": ms, "work": work}
    dom = max(kernels, key=lambda k: kernels[k]["total_ms"])
    kd = kernels[dom]
    if kd["bound"] == "mfma":
        unit, peak = "TFLOP/s", PEAK_MFMA_TFLOPS[cfg.dtype]
        achieved = kd["work"] / (kd["total_ms"] * 1e-3) / 1e12
    elif kd["bound"] == "alu":
        unit, peak = "Tops/s", PEAK_ALU_TOPS
        achieved = kd["work"] / (kd["total_ms"] * 1e-3) / 1e12
    else:
        unit, peak = "GB/s", PEAK_HBM_GBS
        achieved = kd["work"] / (kd["total_ms"] * 1e-3) / 1e9
    roofline = {"kernel": dom, "bound": kd["bound"], "achieved": achieved, "peak": peak,
                "unit": unit, "frac": achieved / peak,
                "traffic": traffic_from_profile(cfg.name, dom)[0],
                "traffic_source": traffic_from_profile(cfg.name, dom)[1],
                "avg_launch_us": kd["avg_us"],
                "timing": "HIP events by the library around each launch, eager pass of %d steps"
                          % prof_steps,
                # what the same bracket reports for an empty kernel: dispatch latency that
                # avg_launch_us contains and a profiler's kernel trace does not
                "event_overhead_us": event_overhead_us}
    if dom in ("expand_kernel", "expand_request_kernel", "level_small_kernel",
               "decode_small_kernel"):
        flops = sum(2.0 * cfg.B * (1 if l == 0 else cfg.K) * cfg.e * cfg.V * (0 if l == 0 else 1)
                    for l in range(cfg.L)) * prof_steps
        roofline["mfma_tflops"] = flops / (kd["total_ms"] * 1e-3) / 1e12
    if dom == "expand_request_kernel" and cfg.e == 128:
        # The kernel's two sweeps issue one "tile step" (16 beams x 16 codes: four MFMAs and the
        # vector work on four logits per lane) per wave, tile and sweep.  Matrix and vector
        # instructions of a SIMD overlap only in part, so the peak of neither unit bounds that
        # loop; the library's microbenchmark times the same instruction mix without any memory
        # access at the kernel's occupancy (four waves per SIMD), and the kernel's own rate of
        # tile steps per SIMD is set against it.
        props = torch.cuda.get_device_properties(0)
        simds = 4 * props.multi_processor_count
        waves = (cfg.K + 15) // 16
        steps_per_launch = 2.0 * (cfg.V // 16) * waves * cfg.B      # levels 2 .. L: one launch each
        kernel_rate = steps_per_launch / simds / (kd["avg_us"] * 1e-6)
        both, clk = nz.bench_tile_step(2)
        mat, _ = nz.bench_tile_step(0)
        vec, _ = nz.bench_tile_step(1)
        roofline["tile_steps"] = {
            "unit": "tile steps/s per SIMD", "kernel": kernel_rate,
            "instruction_mix_bound": both, "frac_of_bound": kernel_rate / both,
            "matrix_only": mat, "vector_only": vec, "clock_mhz": clk,
            "note": "bound: nezha_bench_tile_step mode 2 (sweep 1's instructions, no memory "
                    "access, 4 waves per SIMD); the kernel's figure includes both sweeps' LDS "
                    "traffic, list appends, per-beam selection and output"}
    breakdown = {k: {"avg_us": round(v["avg_us"], 3), "launches": v["launches"]}
                 for k, v in kernels.items()}

    cands = cfg.B * cfg.K * cfg.K if cfg.L > 1 else cfg.B * cfg.K
    ms_per_step = total_ms / args.steps
    result = {
        "metric": "verified candidate items/sec (level-L candidates submitted to the hash-set "
                  "verifier per full L-level decode / decode time), 1 MI355X",
        "value": cands / (ms_per_step * 1e-3),
        "unit": "items/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "p50_step_ms": percentile(per_step, 50), "p90_step_ms": percentile(per_step, 90),
        "p99_step_ms": percentile(per_step, 99),
        "wall_ms_per_step": wall_ms / args.steps,
        # eager launches, events around each call: [projections ahead of the loop, level 1..L]
        "level_call_ms": {"p50": [round(percentile(v, 50), 5) for v in level_ms],
                          "p90": [round(percentile(v, 90), 5) for v in level_ms],
                          "p99": [round(percentile(v, 99), 5) for v in level_ms]},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "d": cfg.d, "e": cfg.e, "L": cfg.L,
                   "V": cfg.V, "K": cfg.K, "catalog_items": int(catalog.shape[0]),
                   "load_factor": cfg.load_factor, "candidates_per_step": cands,
                   "accepted_per_step": accepted, "hallucinated_topk_frac": round(hallucinated, 3),
                   "launch": ("direct: one nezha_decode call per step" if plan is not None
                              else "direct: one nezha_draft_step call per level")
                   if launch == "direct" else "hip_graph_replay",
                   "weights": "packed per call" if (args.pack_per_call or cfg.dtype != "bf16")
                   else "packed once at set-up",
                   "transition": args.transition, "prefix_sets": bool(args.prefix_sets),
                   "head": args.head,
                   "setup_s": round(setup_s, 1)},
        "accepted_items_per_s": accepted / (ms_per_step * 1e-3),
        "roofline": roofline,
        "kernels": breakdown,
    }
    if two_stream_ms is not None:
        result["two_stream_ms_per_step"] = two_stream_ms
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline_draft(cfg, x, catalog, cands, Unp, args.prefix_sets,
                                                    use_state)
    return result


def cpu_baseline_draft(cfg, x, catalog, cands, U=None, prefix_sets=False, use_state=True):
    """The CPU oracle, as it stands, on the host cores: a bounded sample of requests of the same
    workload, scaled to the batch."""
    from oracle import oracle as orc
    threads = os.cpu_count() or 1
    oset = orc.ItemSet(catalog, cfg.radices)
    opre = None
    if prefix_sets:
        opre = [orc.ItemSet(np.unique(catalog[:, :l], axis=0), cfg.radices[:l])
                for l in range(1, cfg.L)]
    # about 2.2 * B*K*(d+e)*V multiply-adds per decode; keep the sample near 10 s of CPU work
    macs_per_req = (1 + (cfg.L - 1) * cfg.K) * (cfg.d + cfg.e) * cfg.V
    budget = 4e9 * threads
    n = int(max(1, min(cfg.B, budget // max(1, macs_per_req))))
    Hs = x["H"][:n]
    # the sample is decoded again and again until about 10 s of CPU time have gone by (a single
    # pass over a small workload takes a fraction of a second, too short to time well)
    reps, dt = 0, 0.0
    while reps == 0 or (dt < 10.0 and reps < 2000):
        t = time.perf_counter()
        orc.decode(Hs, x["W"], x["E"], cfg.radices, cfg.K, oset,
                   round_state_bf16=cfg.dtype == "bf16", threads=threads, U=U, prefix_sets=opre,
                   use_state=use_state)
        dt += time.perf_counter() - t
        reps += 1
    return {"value": cands * (n / cfg.B) * reps / dt, "unit": "items/s", "cores": min(threads, n),
            "kind": "oracle", "seconds": round(dt, 3),
            "sample": "%d of %d requests, full decode incl. set lookups, %d passes, scaled by "
                      "request count" % (n, cfg.B, reps)}


def bench_stress(args, cfg):
    """Stand-alone verifier: probes per second and bytes per second over the hash table."""
    dev = torch.device("cuda:0")
    N = args.catalog or cfg.N
    t0 = time.time()
    cat, pi = synth.uniform_catalog(cfg.radices, N, args.seed)
    itemset = nz.build_itemset(cat, cfg.radices, cfg.load_factor)
    q, present = synth.stress_queries(cfg.radices, N, pi, args.seed, cfg.queries)
    setup_s = time.time() - t0
    qd = torch.from_numpy(q).to(dev)
    n = qd.shape[0]
    mask = torch.empty(n, dtype=torch.uint8, device=dev)
    idx = torch.empty(n, dtype=torch.int64, device=dev)
    cnt = torch.empty(1, dtype=torch.int64, device=dev)
    ws = torch.empty(nz.verify_workspace(n), dtype=torch.uint8, device=dev)

    def step():
        nz.verify_tuples(itemset, qd, mask, idx, cnt, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    ev[0].record()
    for i in range(args.steps):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    total_ms = ev[0].elapsed_time(ev[-1])
    per_step = [ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)]
    accepted = int(cnt.item())
    assert accepted == int(present.sum())

    nz.profile_reset()
    nz.profile_enable(True)
    prof_steps = min(args.steps, 50)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = nz.profile_read()
    nz.profile_enable(False)
    nz.profile_reset()
    launches, ms = prof["verify_probe_kernel"]
    # the same kernel on queries whose present keys are drawn uniformly (no help from caches)
    qu, _ = synth.stress_queries(cfg.radices, N, pi, args.seed + 1, cfg.queries, zipf=False)
    qud = torch.from_numpy(qu).to(dev)
    nz.profile_enable(True)
    for _ in range(3):
        nz.verify_tuples(itemset, qud, mask, idx, cnt, ws)
    torch.cuda.synchronize()
    nz.profile_reset()
    for _ in range(prof_steps):
        nz.verify_tuples(itemset, qud, mask, idx, cnt, ws)
    torch.cuda.synchronize()
    uni_launches, uni_ms = nz.profile_read()["verify_probe_kernel"]
    nz.profile_reset()
    # What the memory system delivers for independent random line reads over a buffer of the
    # table's size: the denominator of "fraction of achievable random-access bandwidth".  Every
    # form of the gather kernel is tried (1 to 16 lines in flight per lane, a lane per line or
    # eight lanes per line) and the BEST one is the denominator, so that it does not mirror the
    # verifier's own launch shape.
    table_bytes = itemset.info()["n_slots"] * 8
    scratch = torch.zeros(table_bytes // 8, dtype=torch.int64, device=dev)
    sink = torch.zeros(1, dtype=torch.int64, device=dev)
    gather = {}
    forms = [(64, dp, 1) for dp in (1, 2, 4, 8, 16)] + [(64, dp, 8) for dp in (1, 2, 4, 8, 16)] + \
            [(128, dp, 1) for dp in (1, 2, 4, 8)]
    for line, depth, lanes in forms:
        for _ in range(3):
            nz.bench_random_gather(scratch, n, line, depth=depth, lanes_per_line=lanes, sink=sink)
        torch.cuda.synchronize()
        nz.profile_reset()
        reps = min(prof_steps, 20)
        for _ in range(reps):
            nz.bench_random_gather(scratch, n, line, depth=depth, lanes_per_line=lanes, sink=sink)
        torch.cuda.synchronize()
        gl, gms = nz.profile_read()["random_gather_kernel"]
        gather["%dB_depth%d_%s" % (line, depth, "lane_per_line" if lanes == 1 else "8_lanes_per_line")] = {
            "lines_per_s": n * gl / (gms * 1e-3), "GBps": n * line * gl / (gms * 1e-3) / 1e9,
            "avg_us": 1e3 * gms / gl}
    nz.profile_reset()
    nz.profile_enable(False)
    del scratch
    best64 = max((k for k in gather if k.startswith("64B")), key=lambda k: gather[k]["lines_per_s"])
    best128 = max((k for k in gather if k.startswith("128B")), key=lambda k: gather[k]["lines_per_s"])
    bytes_per_probe = 4 * cfg.L + BUCKET_BYTES + 1
    achieved = n * bytes_per_probe * launches / (ms * 1e-3) / 1e9
    ms_per_step = total_ms / args.steps
    result = {
        "metric": "verified candidate items/sec (stand-alone hash-set verifier: tuples probed "
                  "per second, mask + ordered index list written), 1 MI355X",
        "value": n / (ms_per_step * 1e-3), "unit": "items/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "p50_step_ms": percentile(per_step, 50), "p99_step_ms": percentile(per_step, 99),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64",
        "data": "synthetic",
        "config": {"workload": cfg.name, "catalog_items": N, "L": cfg.L, "V": cfg.V,
                   "load_factor": cfg.load_factor, "queries": n, "accepted": accepted,
                   "table_bytes": itemset.info()["n_slots"] * 8, "setup_s": round(setup_s, 1)},
        "roofline": {"kernel": "verify_probe_kernel", "bound": "hbm", "achieved": achieved,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                     "traffic": traffic_from_profile(cfg.name, "verify_probe_kernel")[0],
                     "traffic_source": traffic_from_profile(cfg.name, "verify_probe_kernel")[1],
                     "avg_launch_us": 1e3 * ms / launches,
                     "bytes_per_probe": bytes_per_probe,
                     "probes_per_s": n * launches / (ms * 1e-3),
                     "uniform_present_probes_per_s": n * uni_launches / (uni_ms * 1e-3),
                     "random_gather_sweep": gather,
                     "random_gather_best_64B": dict(gather[best64], form=best64),
                     "random_gather_best_128B": dict(gather[best128], form=best128),
                     "frac_of_achievable_random_access":
                         (n * uni_launches / (uni_ms * 1e-3)) / gather[best64]["lines_per_s"]},
        "kernels": {k: {"avg_us": round(1e3 * v[1] / v[0], 3), "launches": v[0]}
                    for k, v in prof.items()},
    }
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        m = min(N, 5_000_000)                      # a 10^8-element std::unordered_set is too slow
        oset = orc.ItemSet(cat[:m], cfg.radices)
        qs = q[:1_000_000]
        reps, dt = 0, 0.0
        while dt < 10.0 and reps < 1000:             # about 10 s of CPU work
            t = time.perf_counter()
            oset.verify_tuples(qs)
            dt += time.perf_counter() - t
            reps += 1
        result["cpu_baseline"] = {"value": len(qs) * reps / dt, "unit": "items/s", "cores": 1,
                                  "kind": "oracle", "seconds": round(dt, 3),
                                  "sample": "10^6 of the queries against a set of the first %d "
                                            "catalog items, %d passes (single thread)" % (m, reps)}
    return result


def bench_user_gemm(args):
    """Row a1 on its own: A = H W_l[0:d] (bf16 in, float32 accumulation and output) through
    nezha_user_projection with packed weights, at the Large workload's shape (B x d x T_l = 4096 x
    2048 x 4096) or the shape given by --gemm-shape.  A step is one projection; the roofline is
    the bf16 MFMA peak on 2 B d T_l flops."""
    dev = torch.device("cuda:0")
    B, d, V = (int(v) for v in args.gemm_shape.lower().split("x"))
    e = 32
    rng = np.random.default_rng(args.seed)
    H = torch.from_numpy(synth.round_to_bf16(rng.standard_normal((B, d)).astype(np.float32))).to(dev).to(torch.bfloat16)
    W = torch.from_numpy(synth.round_to_bf16((rng.standard_normal((d + e, V)) * 0.02).astype(np.float32))).to(dev).to(torch.bfloat16)
    Wp = nz.pack_weights(1, 1, [V], W, d)
    A = torch.empty((B, V), dtype=torch.float32, device=dev)
    ws = torch.empty(256, dtype=torch.uint8, device=dev)

    def step():
        nz.user_projection(1, 1, [V], H, Wp, out=A, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    ev[0].record()
    for i in range(args.steps):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    total_ms = ev[0].elapsed_time(ev[-1])
    per_step = [ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)]
    # check of a sample of the outputs against a float64 product of the same bf16 values
    rows = rng.integers(0, B, 64)
    cols = rng.integers(0, V, 64)
    want = (H[rows].double().cpu().numpy() @ W[:d].double().cpu().numpy()[:, cols])
    err = float(np.abs(A[rows][:, cols].cpu().numpy() - want).max())
    nz.profile_reset()
    nz.profile_enable(True)
    prof_steps = min(args.steps, 50)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    launches, ms = nz.profile_read()["user_gemm_kernel"]
    nz.profile_enable(False)
    nz.profile_reset()
    overhead = nz.profile_event_overhead(200)
    # what the matrix units sustain on these operand values with nothing else to do (the chip
    # lowers its clock under matrix load, by an amount that depends on the values)
    sus_h, clk_h = nz.bench_mfma_rate(H)
    sus_w, clk_w = nz.bench_mfma_rate(W)
    sus_0, clk_0 = nz.bench_mfma_rate(torch.zeros(4096, dtype=torch.bfloat16, device=dev))
    flops = 2.0 * B * d * V
    ms_per_step = total_ms / args.steps
    achieved = flops * launches / (ms * 1e-3) / 1e12
    return {
        "metric": "user-part projection of the draft head (Eq. 2, beam-independent part), "
                  "request rows per second, 1 MI355X",
        "value": B / (ms_per_step * 1e-3), "unit": "rows/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step,
        "p50_step_ms": percentile(per_step, 50), "p99_step_ms": percentile(per_step, 99),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "user_gemm", "B": B, "d": d, "V": V, "output": "float32",
                   "max_abs_error_vs_float64_on_a_sample": err},
        "roofline": {"kernel": "user_gemm_kernel", "bound": "mfma", "achieved": achieved,
                     "peak": PEAK_MFMA_TFLOPS["bf16"], "unit": "TFLOP/s",
                     "frac": achieved / PEAK_MFMA_TFLOPS["bf16"],
                     "traffic": traffic_from_profile("user_gemm", "user_gemm_kernel")[0],
                     "traffic_source": traffic_from_profile("user_gemm", "user_gemm_kernel")[1],
                     "avg_launch_us": 1e3 * ms / launches, "event_overhead_us": overhead,
                     "frac_from_back_to_back_steps": flops / (ms_per_step * 1e-3) / 1e12
                                                     / PEAK_MFMA_TFLOPS["bf16"],
                     "algorithmic_bytes": 2.0 * B * d + 2.0 * d * V + 4.0 * B * V,
                     "sustained_mfma": {
                         "what": "loop of independent 32x32x16 bf16 MFMAs alone, one wave per SIMD "
                                 "on all CUs, operand values from the workload; clock from the "
                                 "core-clock and 100 MHz counters read inside the kernel",
                         "hidden_state_values": {"TFLOP/s": sus_h, "clock_MHz": clk_h},
                         "weight_values": {"TFLOP/s": sus_w, "clock_MHz": clk_w},
                         "zero_values": {"TFLOP/s": sus_0, "clock_MHz": clk_0}},
                     "frac_of_sustained_mfma": achieved / min(sus_h, sus_w)},
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: every request is independent and this build runs on "
              "a single MI355X; --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if args.calibrate:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    if args.workload == "user_gemm":
        print(json.dumps(bench_user_gemm(args)))
        return
    cfg = synth.get_config(args.workload)
    if args.batch:
        cfg = cfg.scaled(B=args.batch)
    if args.catalog and cfg.B:
        cfg = cfg.scaled(N=args.catalog)
    result = bench_stress(args, cfg) if cfg.B == 0 else bench_draft(args, cfg)
    if cfg.name == "large" and not args.no_serving_leg and not args.batch:
        result["serving_latency"] = serving_latency_leg(args)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
