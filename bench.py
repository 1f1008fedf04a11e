#!/usr/bin/env python3
"""Benchmark of the D-PSGD hot path on one MI355X.

A "step" is one synchronous iteration of Algorithm 1 over all n simulated workers: the minibatch
gradient of every worker at its own iterate (step 3), the neighbourhood average and the update
(steps 4-5) and the consensus distance.  Bf16 MLP workloads on the ring run it as dpsgd_step (the
weight gradient of the large layers is formed inside the mix kernel); everything else, or
--two-call, runs dpsgd_grad followed by dpsgd_mix_step.  Inputs (replicas, a pool of pre-generated
minibatches) are resident in HBM before the timed region; drawing the minibatches (step 2) is not
timed.

Prints ONE JSON line: worker-iterations/s, plus the roofline of the dominant kernel measured with
HIP events inside the timed region, on the stream the kernels run on - the fused weight-gradient +
mix kernel (8 bytes per (worker, weight): X read once, X written once) on the dpsgd_step path, the
mix+step kernel (12 bytes per (worker, parameter)) on the two-call path - and the CPU oracle timed
on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PROFILES = os.path.join(ROOT, "profiles")


def traffic_from_profile(workload, path, kernel, ld):
    """HBM bytes per launch of the dominant kernel as a rocprofv3 --pmc run of this very command counted them
    (FETCH_SIZE and WRITE_SIZE, scaled by what the same counters read for a plain copy of known size).  A counter
    run cannot happen inside a timed run, so the figure comes from the committed summary under profiles/ that
    carries a machine-readable line

        bench-traffic: {"workload": ..., "path": ..., "kernel": ..., "ld": ..., "bytes_per_launch": ...}

    and is used only if workload, path, kernel name and row stride all match what this run launched; otherwise
    None.  Returns (bytes or None, file name or None)."""
    try:
        names = sorted(os.listdir(PROFILES))
    except OSError:
        return None, None
    for name in names:
        if not name.endswith((".md", ".txt")):
            continue
        try:
            with open(os.path.join(PROFILES, name)) as f:
                for line in f:
                    if "bench-traffic:" not in line:
                        continue
                    rec = json.loads(line.split("bench-traffic:", 1)[1].strip().rstrip("->").strip())
                    if (rec.get("workload") == workload and rec.get("path") == path and rec.get("ld") == ld
                            and rec.get("kernel") and rec["kernel"] in kernel):
                        return float(rec["bytes_per_launch"]), name
        except (OSError, ValueError):
            continue
    return None, None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed iterations (0 = the workload's K)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="mlp3_ring64",
                    help="lsq_ring8 | softmax_ring16 | mlp2_ring32 | mlp3_ring64 | mlp3_torus8x8 | resnet20_ring112")
    ap.add_argument("--pool", type=int, default=4, help="distinct minibatches kept in HBM and cycled through")
    ap.add_argument("--batch", type=int, default=0,
                    help="override the per-worker minibatch (a kernel check at a large batch; NOT a benchmark "
                         "configuration, and flagged as such in the output)")
    ap.add_argument("--workers", type=int, default=0, help="override n (same caveat as --batch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-consensus", action="store_true")
    ap.add_argument("--two-call", action="store_true", help="dpsgd_grad + dpsgd_mix_step even where dpsgd_step fuses")
    ap.add_argument("--momentum", type=float, default=0.0,
                    help="run the heavy-ball variant dpsgd_mix_step_momentum with this mu (two-call path; a variant "
                         "of the benchmark, flagged in the output)")
    ap.add_argument("--topology", default="", choices=["", "ring_chord"],
                    help="override the workload's W: ring_chord = the supplement's ring with a link to the farthest "
                         "node (its 16-machine runs); a variant, flagged as such in the output")
    ap.add_argument("--overlap", action="store_true",
                    help="variant for comparison: the averaging W X runs on a second stream beside dpsgd_grad, then "
                         "X = (W X) - gamma G is formed by a third pass (three existing entry points, 8 + 12 bytes per "
                         "(worker, parameter) instead of the mix kernel's 12); not the benchmark's path")
    ap.add_argument("--ld-multiple", type=int, default=0,
                    help="row stride of X: d rounded up to a multiple of this many floats (0 = the stride the library "
                         "recommends for the topology, dpsgd_recommended_ld)")
    ap.add_argument("--ring-rows", type=int, default=-1,
                    help="set the library's ring_rows option (see include/dpsgd.h); -1 leaves the default")
    ap.add_argument("--shadow", action="store_true",
                    help="dpsgd_step with the bf16_shadow option: the fused kernel leaves the bf16 rounding of the new "
                         "hidden-layer weights for the next iteration's forward and data gradient (same results; the "
                         "caller must not touch X between iterations, which this loop does not)")
    ap.add_argument("--graph", action="store_true",
                    help="after the eager pass, record the K iterations into one HIP graph and report the timed "
                         "replay of it as the value (pays where the iteration is launch-bound: the small workloads)")
    ap.add_argument("--option", action="append", default=[], metavar="KEY=VALUE",
                    help="set a launch-shape option of the library (dpsgd_set_option, see include/dpsgd.h); may be repeated; "
                         "the run is flagged as a variant")
    ap.add_argument("--repeats", type=int, default=5,
                    help="the timed region (exactly --steps iterations) is run this many times; the median repeat is reported")
    ap.add_argument("--no-others", action="store_true",
                    help="the default run also times every other workload of the benchmark definition in short runs after "
                         "the headline (the `others` array of the JSON line); this leaves them out")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB device-to-device copy (reference for the FETCH_SIZE / WRITE_SIZE "
                         "counters under rocprofv3 --pmc) and exit")
    return ap.parse_args()


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, seconds_budget=20.0):
    """The oracle as it stands, on this machine's host cores, on a bounded sample of the workload:
    the gradient of `m` workers (OpenMP over workers) and the mix+step on a column sample, scaled to
    one full iteration of all n workers."""
    import numpy as np

    import oracle
    from paper_1705_09056_amd import synth

    threads = oracle.num_threads()
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    # per-worker gradient cost estimate (fp64 scalar flops) to size the sample
    flops_per_worker = {0: 4.0 * cfg.batch * d, 1: 4.0 * cfg.batch * d, 2: 6.0 * cfg.batch * d,
                        3: 6.0 * 40.6e6 * cfg.batch}[cfg.model_kind]
    est_rate = 0.8e9  # scalar fp64 flop/s per core of the plain loops, order of magnitude
    all_workers_s = flops_per_worker * cfg.n / max(1, min(threads, cfg.n)) / est_rate
    m = cfg.n if all_workers_s <= seconds_budget else min(cfg.n, threads)
    workers = list(range(m))
    x0 = synth.make_x0(cfg).astype(np.float64)
    X = np.tile(x0, (m, 1))
    inp, tgt = synth.make_batch(cfg, 0, workers)
    t0 = time.perf_counter()
    oracle.grad_all(cfg.model_kind, cfg.widths, X, inp, tgt)
    t_grad = time.perf_counter() - t0
    # mix + step on a column sample of all n rows
    dcols = int(min(d, max(1, 4_000_000 // cfg.n)))
    rng = np.random.default_rng(0)
    Xs = rng.standard_normal((cfg.n, dcols))
    Gs = rng.standard_normal((cfg.n, dcols))
    topo = oracle.ring(cfg.n) if cfg.topology == "ring" else oracle.ring_chord(cfg.n) if cfg.topology == "ring_chord" \
        else oracle.torus(*cfg.torus_dims)
    t0 = time.perf_counter()
    oracle.mix_step(topo, Xs, Gs, cfg.gamma)
    t_mix = (time.perf_counter() - t0) * (d / dcols)
    # m workers ran on min(m, threads) cores at once; all n workers need n/m such rounds
    t_iter = t_grad * (cfg.n / m) + t_mix
    # one core, measured: one worker's gradient through the single-worker entry of the oracle (no OpenMP inside a
    # worker), scaled by n; the mix sample above already ran on one thread
    t0 = time.perf_counter()
    oracle.loss_grad(cfg.model_kind, cfg.widths, X[0], inp[0], tgt[0])
    t_one = time.perf_counter() - t0
    t_iter_1 = t_one * cfg.n + t_mix
    return {
        "value": cfg.n / t_iter, "unit": "worker-iters/s", "cores": int(min(threads, m)), "kind": "oracle",
        "cpu_model": _cpu_model(),
        "sample": f"gradient of {m} of {cfg.n} workers (one minibatch each, OpenMP over workers, {t_grad:.2f} s) "
                  f"scaled by n/{m}; mix+step on {dcols} of {d} columns (single thread, scaled to d)",
        "single_thread": {"value": cfg.n / t_iter_1, "unit": "worker-iters/s", "cores": 1,
                          "sample": f"gradient of 1 of {cfg.n} workers on one core ({t_one:.2f} s, measured) scaled by n; "
                                    f"the same mix+step sample"},
    }


MFMA_PEAK_TFLOPS = 2500.0   # dense bf16


def gradient_roofline(cfg, d, step_ms):
    """Arithmetic of the gradient (Algorithm 1 step 3) per iteration against the bf16 MFMA peak and against the
    ceiling its arithmetic intensity allows: a GEMM M x K . K x N counts 2MKN; forward + weight gradient for a first
    layer, + data gradient for the others.  Minimum HBM bytes: every worker has its own weights, so an MLP weight is
    read (4 B) for the forward, again for the data gradient (not the first layer) and its fp32 gradient or update is
    written (4 B), and the minibatch is read twice; the CNN streams each conv's bf16 input and output once per pass (forward, data and weight
    gradient).  The rate is taken over the whole iteration (gradient + mix), not over the gradient kernels alone."""
    from paper_1705_09056_amd.configs import MODEL_LSQ, MODEL_RESNET20
    n, Bw = cfg.n, cfg.batch
    if cfg.model_kind == MODEL_LSQ:
        flop, byts = 4.0 * Bw * d * n, 4.0 * Bw * d * n
    elif cfg.model_kind == MODEL_RESNET20:
        in_ch, H, Wd, base, blocks, classes = cfg.widths
        convs = [(in_ch, base, H * Wd, H * Wd)]
        c, px = base, H * Wd
        for stage in range(3):
            for blk in range(blocks):
                if stage > 0 and blk == 0:
                    convs.append((c, 2 * c, px, px // 4))
                    c, px = 2 * c, px // 4
                else:
                    convs.append((c, c, px, px))
                convs.append((c, c, px, px))
        mac = sum(9 * ci * co * po for ci, co, _, po in convs) + c * classes
        first = 9 * convs[0][0] * convs[0][1] * convs[0][3]
        flop = 2.0 * (3 * mac - first) * Bw * n
        byts = 3.0 * 2.0 * sum(ci * pi + co * po for ci, co, pi, po in convs) * Bw * n
    else:
        flop = 0.0
        byts = 2.0 * (2.0 if cfg.bf16 else 4.0) * Bw * cfg.widths[0] * n   # minibatch: forward and first weight gradient
        for l in range(len(cfg.widths) - 1):
            w = cfg.widths[l] * cfg.widths[l + 1]
            flop += (4.0 if l == 0 else 6.0) * Bw * w * n
            byts += (8.0 if l == 0 else 12.0) * w * n
    peak = MFMA_PEAK_TFLOPS if cfg.bf16 else 157.3
    achieved = flop / (step_ms * 1e-3) / 1e12
    ceiling = min(1.0, (flop / byts) / (peak * 1e12 / (HBM_PEAK_GBS * 1e9)))
    return {"flop_per_step": flop, "min_hbm_bytes_per_step": byts, "achieved_tflops": achieved,
            "peak_tflops": peak, "peak_kind": "bf16 MFMA" if cfg.bf16 else "fp32 vector",
            "frac_of_peak": achieved / peak, "intensity_ceiling_frac": ceiling,
            "frac_of_ceiling": achieved / peak / ceiling, "timed_over": "whole iteration (gradient + mix)"}


def run_one(args, with_cpu_baseline):
    """Times one workload as the flags in `args` say and returns its record (the fields of the JSON line)."""
    import numpy as np
    import torch

    from paper_1705_09056_amd import binding as B
    from paper_1705_09056_amd import synth
    from paper_1705_09056_amd.configs import MODEL_MLP, MODEL_SOFTMAX, by_name

    cfg = by_name(args.workload)
    variant = None
    if args.batch or args.workers:
        import dataclasses
        cfg = dataclasses.replace(cfg, batch=args.batch or cfg.batch, n=args.workers or cfg.n)
        variant = f"batch={cfg.batch}, n={cfg.n}: kernel check, not a benchmark configuration"
    if args.topology:
        import dataclasses
        cfg = dataclasses.replace(cfg, topology=args.topology)
        variant = (variant + "; " if variant else "") + f"W = {args.topology}: not a benchmark configuration"
    K = args.steps or cfg.iters
    W = args.warmup
    R = max(1, args.repeats)
    d = synth.model_dim(cfg.model_kind, cfg.widths)
    topo = B.Topology.ring() if cfg.topology == "ring" else B.Topology.ring_chord() if cfg.topology == "ring_chord" \
        else B.Topology.torus(*cfg.torus_dims)
    ld = synth.padded_stride(d, args.ld_multiple) if args.ld_multiple else B.recommended_ld(d, topo)
    model = B.Model(cfg.model_kind, cfg.widths, compute_bf16=cfg.bf16)

    # replicas: n copies of x_0 (Algorithm 1, Require)
    x0 = torch.from_numpy(synth.make_x0(cfg)).cuda()
    X = torch.zeros(cfg.n, ld, device="cuda")
    X[:, :d] = x0
    G = torch.zeros_like(X)
    loss = torch.zeros(cfg.n, device="cuda")
    cons = None if args.no_consensus else torch.zeros(1, device="cuda")
    pool = []
    for k in range(max(1, args.pool)):
        inp, tgt = synth.make_batch(cfg, k)
        if cfg.bf16:
            inp_d = torch.from_numpy(synth.bf16_bits(inp).astype(np.int16)).view(torch.bfloat16).cuda()
        else:
            inp_d = torch.from_numpy(inp).cuda()
        pool.append((inp_d, torch.from_numpy(tgt).cuda()))

    ctx = B.Dpsgd(cfg.n, d, topo, cfg.gamma, ld=ld)
    if args.shadow:
        ctx.set_option("bf16_shadow", 1)
    if args.ring_rows >= 0:
        ctx.set_option("ring_rows", args.ring_rows)
        variant = (variant + "; " if variant else "") + f"ring_rows={args.ring_rows}"
    for kv in args.option:
        key, _, val = kv.partition("=")
        ctx.set_option(key, int(val))
        variant = (variant + "; " if variant else "") + kv
    # layers whose weight gradient dpsgd_step forms inside the mix kernel (same rule as the library)
    fused_weights = 0
    rows_kernel = []     # per fused ring layer: does the [16 rows][1 KB] kernel take it (same rule as the library)
    shadow_weights = 0   # of those, the hidden-layer weights whose bf16 copy the fused kernel also writes (--shadow)
    ring_ok = cfg.topology == "ring" and cfg.n >= 3
    torus_ok = cfg.topology == "torus" and 3 <= cfg.torus_dims[1] <= 16 and cfg.torus_dims[0] >= 3
    # any other W of at most 64 workers: the kernel that holds every worker's tile in LDS
    slab_ok = not ring_ok and not torus_ok and cfg.n <= 64 and "fused_slab=0" not in args.option
    if cfg.bf16 and cfg.model_kind in (MODEL_MLP, MODEL_SOFTMAX) and (ring_ok or torus_ok or slab_ok):
        for l in range(len(cfg.widths) - 1):
            w_in, w_out = cfg.widths[l], cfg.widths[l + 1]
            if w_in % (128 if ring_ok else 32) == 0 and w_out % 32 == 0 and w_in * w_out >= (1 << 20):
                fused_weights += w_in * w_out
                rows_kernel.append(ring_ok and cfg.batch <= 32 and w_in % 256 == 0 and ld % 4 == 0 and args.ring_rows != 0)
                if args.shadow and ring_ok and l >= 1:
                    shadow_weights += w_in * w_out
    fused = fused_weights > 0 and not args.two_call and not args.momentum and not args.overlap
    Vel = torch.zeros_like(X) if args.momentum else None
    if args.momentum:
        variant = (variant + "; " if variant else "") + f"heavy-ball momentum {args.momentum} (not the benchmark's update)"

    if args.overlap:
        # Algorithm 1 steps 3 and 4 do not depend on each other: W X on a side stream while the gradient runs, then
        # the update X = (W X) - gamma G as a mix with the identity for W.  The averaging context has gamma = 0 and
        # is handed X itself as its "gradient", so that pass reads nothing beyond X (the second read of a row hits
        # in cache).
        variant = (variant + "; " if variant else "") + \
            "gradient and averaging on two streams, update as a third pass (comparison only)"
        main_stream, side_stream = torch.cuda.current_stream(), torch.cuda.Stream()
        Xavg = torch.zeros_like(X)
        ctx_avg = B.Dpsgd(cfg.n, d, topo, 0.0, ld=ld, stream=side_stream)
        ident = B.Topology.csr(np.arange(cfg.n + 1, dtype=np.int32), np.arange(cfg.n, dtype=np.int32),
                               np.ones(cfg.n, dtype=np.float32))
        ctx_upd = B.Dpsgd(cfg.n, d, ident, cfg.gamma, ld=ld)

    def step(k, ev=None):
        inp_d, tgt_d = pool[k % len(pool)]
        if fused:
            ctx.step(model, X, inp_d, tgt_d, cfg.batch, G, loss, cons, input_is_bf16=cfg.bf16)
            return
        if args.overlap:
            side_stream.wait_stream(main_stream)
            with torch.cuda.stream(side_stream):
                ctx_avg.mix_step(X, X, Xavg, None)
            ctx.grad(model, X, inp_d, tgt_d, cfg.batch, G, loss, input_is_bf16=cfg.bf16)
            main_stream.wait_stream(side_stream)
            if ev is not None:
                ev[0].record()
            ctx_upd.mix_step(Xavg, G, X, cons)
            if ev is not None:
                ev[1].record()
            return
        ctx.grad(model, X, inp_d, tgt_d, cfg.batch, G, loss, input_is_bf16=cfg.bf16)
        if ev is not None:
            ev[0].record()
        if Vel is not None:
            ctx.mix_step_momentum(X, G, Vel, args.momentum, X, cons)
        else:
            ctx.mix_step(X, G, X, cons)
        if ev is not None:
            ev[1].record()

    for k in range(W):
        step(k)
    torch.cuda.synchronize()
    if fused:
        ctx.set_option("time_fused", 1)
    # R repeats of the timed region; each is EXACTLY K iterations between two HIP events on the stream the library
    # launches on (torch's current stream was handed to dpsgd_create).  The repeat with the median time is reported.
    repeats = []
    wall0 = time.perf_counter()
    for r in range(R):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
        t_begin, t_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t_begin.record()
        for k in range(K):
            step(W + r * K + k, evs[k])
        t_end.record()
        torch.cuda.synchronize()
        rec = {"total_ms": t_begin.elapsed_time(t_end)}
        if fused:
            rec["kernel_ms"], rec["launches"] = ctx.read_timing()
        else:
            rec["kernel_ms"], rec["launches"] = sum(a.elapsed_time(b) for a, b in evs), K
        repeats.append(rec)
    wall = time.perf_counter() - wall0
    med = sorted(repeats, key=lambda q: q["total_ms"])[len(repeats) // 2]
    total_ms = med["total_ms"]
    launch_ms = med["kernel_ms"] / med["launches"]
    mix_ms = med["kernel_ms"] / K
    if fused:
        # minibatches of more than 32 rows (padded to a multiple of 32): operands through LDS unless switched off
        tiles_name = "mlp_fused_ring_lds_kernel" if (cfg.batch > 32 and not args.shadow and "fused_lds=0" not in args.option) \
            else "mlp_fused_ring_kernel"
        ring_name = "mlp_fused_ring_rows_kernel" if all(rows_kernel) else tiles_name if not any(rows_kernel) \
            else "mlp_fused_ring_rows_kernel / " + tiles_name
        kernel_name = (ring_name if ring_ok else "mlp_fused_torus_cols_kernel" if torus_ok else "mlp_fused_slab_kernel") + \
            " (weight gradient + Algorithm 1 steps 4-5, in place)"
        launch_bytes = (8.0 * fused_weights + 2.0 * shadow_weights) * cfg.n * K / med["launches"]
    else:
        mix_kernel = ("mix_ring_fat_kernel" if d >= 64 * 131072 else "mix_ring_kernel") if ring_ok else \
            ("mix_csr_slab_wide_kernel" if d >= 16 * 32768 else "mix_csr_slab_kernel")
        kernel_name = "update pass X = (W X) - gamma G (identity as W)" if args.overlap else \
            f"dpsgd_mix_step: {mix_kernel} (Algorithm 1 steps 4-5 fused) + consensus reduction"
        launch_bytes = (20.0 if Vel is not None else 12.0) * cfg.n * d
    graph_ms = None
    if args.graph:
        if fused:
            ctx.set_option("time_fused", 0)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.current_stream()):
            for k in range(K):
                step(W + k)
        graph.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        graph.replay()
        g1.record()
        torch.cuda.synchronize()
        graph_ms = g0.elapsed_time(g1)
    # Algorithm 1 step 7 (run once after the K iterations): the node average, read-only, 4 n d bytes
    xbar = torch.empty(d, device="cuda")
    m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ctx.mean(X, xbar)
    m0.record()
    for _ in range(3):
        ctx.mean(X, xbar)
    m1.record()
    torch.cuda.synchronize()
    mean_ms = m0.elapsed_time(m1) / 3
    final_loss = float(loss.mean().item())
    final_cons = None if cons is None else float(cons.item())
    ctx.close()
    if args.overlap:
        ctx_avg.close()
        ctx_upd.close()

    achieved = launch_bytes / (launch_ms * 1e-3) / 1e9
    eager_ms = total_ms
    if graph_ms is not None:
        total_ms = graph_ms
    path = "fused" if fused else "two-call"
    traffic, traffic_file = (None, None) if (variant or args.shadow or args.no_consensus) else \
        traffic_from_profile(cfg.name, path, kernel_name, ld)
    out = {
        "metric": "worker-iters/sec (grad+mix) at n workers",
        "value": cfg.n * K / (total_ms * 1e-3),
        "unit": "worker-iters/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": total_ms / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": cfg.name, "model_kind": int(cfg.model_kind), "widths": list(cfg.widths), "n": cfg.n,
                   "topology": cfg.topology, "batch_per_worker": cfg.batch, "d": d, "ld": ld, "gamma": cfg.gamma,
                   "minibatch_pool": len(pool), "consensus": cons is not None,
                   "path": "dpsgd_step" if fused else "dpsgd_grad beside dpsgd_mix_step, then dpsgd_mix_step" if args.overlap
                   else ("dpsgd_grad + dpsgd_mix_step_momentum" if Vel is not None
                                                           else "dpsgd_grad + dpsgd_mix_step"),
                   **({"launch": f"one HIP graph of {K} iterations, one replay timed",
                       "eager_ms_per_step": eager_ms / K} if graph_ms is not None else {}),
                   **({"bf16_shadow": True} if args.shadow else {}),
                   **({"variant": variant} if variant else {})},
        "timing": {"repeats": R, "reported": "the repeat with the median time; each repeat is exactly `steps` iterations",
                   "ms_per_step_of_each_repeat": [q["total_ms"] / K for q in repeats]},
        "roofline": {"kernel": kernel_name, "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_file and f"profiles/{traffic_file}",
                     "algorithmic_bytes_per_launch": launch_bytes, "avg_launch_ms": launch_ms},
        "gradient": gradient_roofline(cfg, d, total_ms / K),
        "mean": {"kernel": "dpsgd_mean (Algorithm 1 step 7)", "ms": mean_ms, "algorithmic_bytes": 4.0 * cfg.n * d,
                 "achieved": 4.0 * cfg.n * d / (mean_ms * 1e-3) / 1e9, "unit": "GB/s",
                 "frac": 4.0 * cfg.n * d / (mean_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "mix_fraction_of_step": mix_ms / (eager_ms / K),
        "wall_s": wall,
        "final_mean_loss": final_loss, "final_consensus": final_cons,
    }
    if with_cpu_baseline and not variant:
        out["cpu_baseline"] = cpu_baseline(cfg)
    del X, G, pool, Vel, xbar
    torch.cuda.empty_cache()
    return out


# The other workloads of the benchmark definition, each as a short run after the headline's timed region, so that one
# invocation witnesses every configuration: (workload, extra flags).  The two-call run of the default workload is the
# one whose dominant kernel is dpsgd_mix_step itself (12 bytes per worker and parameter).
OTHERS = (("mlp3_ring64", {"two_call": True}), ("mlp3_torus8x8", {}), ("mlp3_torus8x8", {"two_call": True}),
          ("mlp2_ring32", {}), ("resnet20_ring112", {}), ("softmax_ring16", {}), ("lsq_ring8", {}))


def short_record(rec):
    """What the `others` array keeps of a run."""
    g = rec["gradient"]
    return {"workload": rec["config"]["workload"], "path": rec["config"]["path"], "steps": rec["steps"],
            "warmup": rec["warmup"], "repeats": rec["timing"]["repeats"], "ms_per_step": rec["ms_per_step"],
            "value": rec["value"], "unit": rec["unit"], "dtype": rec["dtype"],
            "dominant_kernel": rec["roofline"]["kernel"], "bound": "hbm", "achieved": rec["roofline"]["achieved"],
            "frac": rec["roofline"]["frac"], "avg_launch_ms": rec["roofline"]["avg_launch_ms"],
            "traffic": rec["roofline"]["traffic"], "traffic_source": rec["roofline"]["traffic_source"],
            "algorithmic_bytes_per_launch": rec["roofline"]["algorithmic_bytes_per_launch"],
            "gradient_tflops": g["achieved_tflops"], "gradient_frac_of_peak": g["frac_of_peak"],
            "gradient_frac_of_intensity_ceiling": g["frac_of_ceiling"], "gradient_peak_kind": g["peak_kind"]}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding across GPUs); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    if args.calibrate_copy:
        torch.cuda.set_device(0)
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")    # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "calibrate_copy_bytes_written": src.numel() * 4}))
        return

    torch.cuda.set_device(0)
    if args.graph:   # capture needs a stream other than the default one; the library launches on torch's current stream
        torch.cuda.set_stream(torch.cuda.Stream())
    out = run_one(args, not args.no_cpu_baseline)
    plain = not (args.batch or args.workers or args.two_call or args.momentum or args.overlap or args.shadow or
                 args.graph or args.ld_multiple or args.ring_rows >= 0 or args.no_consensus or args.option)
    if plain and args.workload == "mlp3_ring64" and not args.no_others:
        others = []
        for name, extra in OTHERS:
            # short runs: 10 iterations of the multi-millisecond workloads, 100 of those whose iteration is a fraction
            # of a millisecond (ten of them are over before the clocks and caches have settled)
            quick = name in ("mlp2_ring32", "softmax_ring16", "lsq_ring8")
            a = argparse.Namespace(**{**vars(args), "workload": name, "steps": 100 if quick else 10,
                                      "warmup": 10 if quick else 3, "repeats": 3, **extra})
            others.append(short_record(run_one(a, False)))
        out["others"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
