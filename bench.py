#!/usr/bin/env python3
"""Throughput of the ASI hot path on one MI355X.

One "step" = the whole path (asi_compress -> asi_core_project -> asi_weight_grad_*)
for every layer of a workload on one batch of synthetic activations that are
already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N] [--no-cpu-baseline]

Without --config the headline (`value`, `ms_per_step`, `roofline`, `cpu_baseline`) is the largest
fp32 workload, config 4, and `per_config` carries the same figures for every workload (1-5: the headline set, 6: the language-model shape).
With --config N only that workload is measured.
"""
from __future__ import annotations

import argparse
import hashlib
import itertools
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HEADLINE_CONFIG = 4
HBM_PEAK_GBS = 8000.0
# published dense peaks of the units each kernel uses (TFLOP/s); "mfma_f32+f64" is the harmonic
# mean for a kernel whose flops are half fp32 MFMA (V = A_m^T U) and half fp64 MFMA (P = A_m V)
PEAK_TFLOPS = {"mfma_f32": 157.3, "mfma_f64": 78.6, "mfma_bf16": 2500.0, "valu_f32": 157.3, "valu_f64": 78.6,
               "mfma_f32+f64": 2.0 / (1.0 / 157.3 + 1.0 / 78.6), "valu_f32+f64": 2.0 / (1.0 / 157.3 + 1.0 / 78.6),
               "mfma_bf16+f64": 2.0 / (1.0 / 2500.0 + 1.0 / 78.6)}
# which arithmetic unit each kernel symbol runs its contraction on; a symbol that is not listed is an error
KERNEL_UNIT = {"k_subspace_small": "mfma_f32+f64", "k_subspace_tiny": "valu_f32+f64", "k_subspace_long": "mfma_f32+f64", "k_subspace_planes": "mfma_f32+f64",
               "k_subspace_gram": "mfma_f64", "k_gauss_fill": "valu_f64",
               "k_ttm_mfma": "mfma_f32", "k_ttm_ksplit": "mfma_f32", "k_ttm_stream": "mfma_f32", "k_ttm_stream_short": "mfma_f32", "k_ttm_expand": "valu_f32", "k_ttm_duo": "mfma_f32", "k_ttm_thin": "valu_f32",
               "k_gemm_bf16": "mfma_bf16", "k_split_bf16": "valu_f32", "k_pair": "mfma_f64",
               "k_corr_mfma": "mfma_f32", "k_corr": "valu_f32",
               "k_orth_gram0": "mfma_f64", "k_orth_apply": "mfma_f64",
               "k_orthw_gram": "mfma_f64", "k_orthw_apply": "mfma_f64", "k_orthw_chol": "valu_f64",
               "k_orth_big": "valu_f64", "k_orth_presum": "valu_f64", "k_orthw_gsum": "valu_f64", "k_sum_partials": "valu_f64",
               "k_expand_grouped": "valu_f32", "k_dw_fold": "mfma_f32", "k_z_planes": "mfma_f32", "k_core_planes": "mfma_f32", "k_init_ctrl": "valu_f32"}


def unit_of(symbol: str) -> str:
    base = symbol.split("<")[0]
    if base not in KERNEL_UNIT:
        raise KeyError(f"bench.py: kernel {symbol!r} has no entry in KERNEL_UNIT")
    return KERNEL_UNIT[base]


def source_digest() -> str:
    """Digest of the kernel sources: a stored counter summary belongs to one build."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2505_05086_amd", "csrc")
    for fn in sorted(os.listdir(d)):
        if fn.endswith((".hip", ".h")):
            h.update(fn.encode())
            with open(os.path.join(d, fn), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def stored_traffic(cfg_index: int):
    """The committed rocprofv3 --pmc summary of this workload (FETCH_SIZE / WRITE_SIZE per launch), or None.
    Returns (kernels, meta): meta says which build the counters were read on and whether that is this one."""
    path = os.path.join(ROOT, "profiles", f"config{cfg_index}_hbm_traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None, None
    built = rec.get("csrc_digest")
    meta = {"profile": os.path.relpath(path, ROOT), "profile_csrc_digest": built, "this_csrc_digest": source_digest()}
    meta["same_build"] = built is not None and built == meta["this_csrc_digest"]
    return rec.get("kernels", {}), meta


# ---- the cost model of the method (multiply-accumulates) and the two whole-step bounds ---------------
def layer_model(lay) -> dict:
    """Per layer-step: the paper's MAC counts (O_ASI without the r^3 terms, the cheapest chain of mode
    products for the core, C_ASI resp. its linear analogue), the pack size M_i (Eq. 5) and the bytes
    the step must move: the activation twice (subspace step, then projection once the factors exist),
    grad_out once, dW once, the pack once."""
    dims, ranks = list(lay.dims), list(lay.ranks)
    numel = 1
    for n in dims:
        numel *= n
    o_asi = sum(2 * numel * r for r in ranks)
    best = None
    for perm in itertools.permutations(range(len(dims))):
        cur, macs = list(dims), 0
        for m in perm:
            tot = 1
            for n in cur:
                tot *= n
            macs += tot * ranks[m]
            cur[m] = ranks[m]
        best = macs if best is None else min(best, macs)
    if lay.kind == "conv2d":
        B, C, H, W = dims
        r1, r2, r3, r4 = ranks
        Ho, Wo = lay.out_hw
        D2 = lay.k * lay.k
        c_asi = (r1 * B * lay.cout * Ho * Wo + r1 * r2 * r3 * r4 * H + r1 * r2 * r4 * H * W
                 + r1 * r2 * lay.cout * Ho * Wo * D2 + r2 * lay.cout * (C // lay.groups) * D2)
    else:
        B, N, D = dims
        r1, r2, r3 = ranks
        c_asi = r1 * B * N * lay.cout + r1 * r2 * N * lay.cout + r1 * r2 * r3 * lay.cout + r3 * lay.cout * D
    pack = 1
    for r in ranks:
        pack *= r
    pack += sum(n * r for n, r in zip(dims, ranks))
    dy = 1
    for n in lay.grad_out_shape:
        dy *= n
    dw = 1
    for n in lay.dw_shape:
        dw *= n
    nbytes = 2 * numel * lay.itemsize + dy * lay.itemsize + 4 * dw + 4 * pack
    return {"macs_subspace": o_asi, "macs_core_chain": best, "macs_dw": c_asi, "pack_elements": pack,
            "flops": 2 * (o_asi + best + c_asi), "bytes": nbytes}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=0,
                    help="measure only this workload (1-6); default: headline = config 4 plus per_config for every workload")
    ap.add_argument("--distinct", type=int, default=8, help="distinct input steps kept in HBM and cycled")
    ap.add_argument("--streams", type=int, default=0, help="HIP streams the layers are spread over (0 = one per layer)")
    ap.add_argument("--batch", type=int, default=0,
                    help="layers per batched call (every launch serves that many layers), 1 = all layers in one batch "
                         "up to the library's limit; batches run on their own streams; 0: one call chain per layer, "
                         "spread over --streams")
    ap.add_argument("--graph", type=int, default=2,
                    help="2: one captured HIP graph per layer, replayed on that layer's stream; 1: one graph per step "
                         "whose layers fork from and join the main stream; 0: eager launches")
    ap.add_argument("--copy-calib-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB ten times (calibrates rocprofv3 byte counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="oracle time budget for the headline workload")
    ap.add_argument("--cpu-seconds-other", type=float, default=3.0,
                    help="oracle time budget for each further workload of per_config (at least one layer-step is timed)")
    return ap.parse_args()


def cpu_baseline(cfg, streams, budget_s, extras=False):
    """The float64 oracle, as it stands, on the host cores: whole path per layer-step."""
    import numpy as np
    from oracle import asi_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    done_bytes, t_used, n_ls = 0, 0.0, 0
    U = [[u.astype(np.float64) for u in st.u_prev0()] for st in streams]
    step = 0
    while t_used < budget_s and step < cfg.steps:
        for li, (lay, st) in enumerate(zip(cfg.layers, streams)):
            if t_used >= budget_s and n_ls > 0:
                break
            A = st.activation(step).astype(np.float64)
            dY = st.grad_out(step).astype(np.float64)
            t0 = time.perf_counter()
            Un = O.compress(A, U[li])
            S = O.core_project(A, Un)
            if lay.kind == "conv2d":
                cs = O.Conv2dSpec(lay.cout, lay.k, lay.k, (lay.stride,) * 2, (lay.pad,) * 2, (lay.dil,) * 2, lay.groups)
                O.conv2d_weight_grad_lowrank(S, Un, dY, cs)
            else:
                O.linear_weight_grad_lowrank(S, Un, dY)
            t_used += time.perf_counter() - t0
            U[li] = Un
            done_bytes += lay.act_bytes
            n_ls += 1
        step += 1
    out = {"value": done_bytes / t_used / 1e9, "unit": "GB/s", "cores": int(cores), "kind": "oracle",
           "sample": f"{n_ls} layer-step(s) of config {cfg.index} in layer order from step 0 "
                     f"({t_used:.1f} s of float64 NumPy oracle time, input generation excluded)"}
    if extras:
        out["variants"] = cpu_variants(cfg, streams)
    return out


def cpu_variants(cfg, streams):
    """Two more host figures on the first layer of the workload (step 0): the same oracle layer-step with the
    BLAS pool limited to one thread, and the dense weight gradient (Eq. 1 on the activation itself, what
    a trainer without compression computes) on all cores."""
    import numpy as np
    from oracle import asi_oracle as O
    lay, st = cfg.layers[0], streams[0]
    A = st.activation(0).astype(np.float64)
    dY = st.grad_out(0).astype(np.float64)
    U0 = [u.astype(np.float64) for u in st.u_prev0()]
    cs = None
    if lay.kind == "conv2d":
        cs = O.Conv2dSpec(lay.cout, lay.k, lay.k, (lay.stride,) * 2, (lay.pad,) * 2, (lay.dil,) * 2, lay.groups)

    def layer_step():
        Un = O.compress(A, U0)
        S = O.core_project(A, Un)
        if cs is not None:
            O.conv2d_weight_grad_lowrank(S, Un, dY, cs)
        else:
            O.linear_weight_grad_lowrank(S, Un, dY)

    res = {}
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            layer_step()
            t1 = time.perf_counter() - t0
        res["oracle_one_thread"] = {"value": lay.act_bytes / t1 / 1e9, "unit": "GB/s", "cores": 1,
                                    "sample": f"one layer-step of layer {lay.name} ({t1:.1f} s)"}
    except ImportError:
        pass
    t0 = time.perf_counter()
    if cs is not None:
        O.conv2d_weight_grad_dense(A, dY, cs)
    else:
        O.linear_weight_grad_dense(A, dY)
    t2 = time.perf_counter() - t0
    res["dense_weight_grad_only"] = {"value": lay.act_bytes / t2 / 1e9, "unit": "GB/s",
                                     "sample": f"Eq. 1 on the uncompressed activation of layer {lay.name}, float64 NumPy, all cores ({t2:.1f} s)"}
    return res


def measure(cfg, args, cpu_seconds):
    """Times `args.steps` steps of one workload and prices its kernels.  Returns the fields of a bench line."""
    import torch

    import paper_2505_05086_amd as asi
    from asi_inputs import LayerStream
    from paper_2505_05086_amd.runner import BatchRunner, LayerRunner

    streams = [LayerStream(cfg.index, li, lay, cfg.theta) for li, lay in enumerate(cfg.layers)]
    batches = None
    if args.batch:
        mb = asi.binding.MAX_BATCH if args.batch == 1 else min(args.batch, asi.binding.MAX_BATCH)
        batches = [BatchRunner(cfg.layers[i:i + mb]) for i in range(0, len(cfg.layers), mb)]
        runners = [r for b in batches for r in b.runs]
    else:
        runners = [LayerRunner(lay) for lay in cfg.layers]
    ndist = max(1, args.distinct)
    if cfg.steps > 1:
        ndist = min(ndist, cfg.steps)
    if args.graph and ndist > 1:
        ndist -= ndist % 2          # the captured steps alternate the two factor buffers

    # inputs resident in HBM before any timing: `ndist` consecutive steps of the drifting sequence
    # (a single-step workload is generated once and held in `ndist` separate copies)
    A_dev, dY_dev = [], []
    for t in range(ndist):
        if cfg.steps > 1 or t == 0:
            A_dev.append([r.upload(st.activation(t)) for r, st in zip(runners, streams)])
            dY_dev.append([r.upload(st.grad_out(t)) for r, st in zip(runners, streams)])
        else:
            A_dev.append([x.clone() for x in A_dev[0]])
            dY_dev.append([x.clone() for x in dY_dev[0]])
    for r, st in zip(runners, streams):
        r.set_factors(st.u_prev0())
    act_bytes = sum(lay.act_bytes for lay in cfg.layers)

    # The layers of one step are independent jobs: each gets its own workspace and they are
    # spread over side streams (default priority) that fork from / join the main stream.
    nstreams = len(runners) if args.streams <= 0 else min(args.streams, len(runners))
    if batches is not None:
        nstreams = len(batches)
    main_stream = torch.cuda.current_stream()
    side = [torch.cuda.Stream() for _ in range(nstreams)] if nstreams > 1 else [None]

    def batched_step(a, g, concurrent=True):
        cur = torch.cuda.current_stream()
        multi = concurrent and len(batches) > 1
        if multi:
            for s in side:
                s.wait_stream(cur)
        i = 0
        for bi, b in enumerate(batches):
            n = len(b.runs)
            with torch.cuda.stream(side[bi] if multi else cur):
                b.step(a[i:i + n], g[i:i + n])
            i += n
        if multi:
            for s in side:
                cur.wait_stream(s)

    def one_step(k):
        a, g = A_dev[k % ndist], dY_dev[k % ndist]
        if batches is not None:
            batched_step(a, g)
            return
        cur = torch.cuda.current_stream()
        if nstreams > 1:
            for s in side:
                s.wait_stream(cur)
        for li, (r, at, gt) in enumerate(zip(runners, a, g)):
            with torch.cuda.stream(side[li % nstreams] if nstreams > 1 else cur):
                r.step(at, gt)
        if nstreams > 1:
            for s in side:
                cur.wait_stream(s)

    # optional: one captured HIP graph per distinct input step, replayed in the timed loop
    graphs = None
    if args.graph == 1 or (args.graph and (batches is not None or nstreams == 1)):
        one_step(0)
        torch.cuda.synchronize()
        graphs = []
        cap = torch.cuda.Stream()
        for k in range(ndist):
            g_ = torch.cuda.CUDAGraph()
            with torch.cuda.stream(cap):
                g_.capture_begin()
                one_step(k)
                g_.capture_end()
            graphs.append(g_)
        torch.cuda.synchronize()

    # --graph 2: one linear graph per layer and input step, replayed on that layer's own stream.
    # Layers are independent jobs and a layer's step k+1 depends only on its own step k (the warm
    # start), which stream order provides; the streams fork from the main stream before the timed
    # steps and join it after them, not once per step.
    layer_graphs = None
    queue_probe = None
    if args.graph == 2 and batches is None and nstreams > 1:
        graphs = None
        layer_graphs = []
        capture_only = torch.cuda.Stream()
        one_step(0)
        torch.cuda.synchronize()
        for li, r in enumerate(runners):
            per = []
            for k in range(ndist):
                g_ = torch.cuda.CUDAGraph()
                with torch.cuda.stream(capture_only):
                    g_.capture_begin()
                    r.step(A_dev[k][li], dY_dev[k][li])
                    g_.capture_end()
                per.append(g_)
            layer_graphs.append(per)
        torch.cuda.synchronize()

        # HIP maps streams onto a few hardware queues (4 per process here) and two streams on one
        # queue run one after the other.  Which streams share is not visible from the API, so it
        # is measured: two different layers' graphs replayed on a pair of streams take about the
        # time of the longer one if the queues differ and the sum if they are the same.
        def probe_us(jobs, reps=6):
            """Time per round of replaying the given (graph, stream) jobs side by side."""
            t0_, t1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            used = {s_ for _, s_ in jobs if s_ is not main_stream}
            torch.cuda.synchronize()
            t0_.record(main_stream)
            for s_ in used:
                s_.wait_stream(main_stream)
            for _ in range(reps):
                for g_, s_ in jobs:
                    with torch.cuda.stream(s_):
                        g_.replay()
            for s_ in used:
                main_stream.wait_stream(s_)
            t1_.record(main_stream)
            torch.cuda.synchronize()
            return t0_.elapsed_time(t1_) * 1e3 / reps

        ga, gb = layer_graphs[0][0], layer_graphs[1][0]
        probe_us([(ga, main_stream), (gb, main_stream)], 2)
        ta, tb = probe_us([(ga, main_stream)]), probe_us([(gb, main_stream)])
        # On one queue two chains take the sum of their times; side by side, between the longer one
        # (small layers, which only wait on launch and memory latency) and ~80 % of the sum (large
        # layers that compete for the CUs).
        shared_above = 0.9 * (ta + tb)
        candidates = [main_stream] + [torch.cuda.Stream() for _ in range(11)]
        chosen, tested = [main_stream], 0
        for cand in candidates[1:]:
            if len(chosen) >= nstreams:
                break
            apart = True
            for c in chosen:
                tested += 1
                if probe_us([(ga, c), (gb, cand)]) > shared_above:
                    apart = False
                    break
            if apart:
                chosen.append(cand)
        queue_probe = {"streams_on_distinct_queues": len(chosen), "pairs_timed": tested,
                       "chain_us": [ta, tb], "same_queue_above_us": shared_above}
        side = [chosen[i % len(chosen)] for i in range(nstreams)]

    def fork():
        if layer_graphs is not None:
            for s in side:
                if s is not main_stream:
                    s.wait_stream(main_stream)

    def join():
        if layer_graphs is not None:
            for s in side:
                if s is not main_stream:
                    main_stream.wait_stream(s)

    def run_step(k):
        if layer_graphs is not None:
            for li, per in enumerate(layer_graphs):
                with torch.cuda.stream(side[li % nstreams]):
                    per[k % ndist].replay()
        elif graphs is not None:
            graphs[k % ndist].replay()
        else:
            one_step(k)

    if args.copy_calib_mib > 0:
        src = torch.empty(args.copy_calib_mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    fork()
    for k in range(args.warmup):
        run_step(k)
    join()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    fork()
    for k in range(args.steps):
        run_step(args.warmup + k)
    join()
    e1.record()
    enqueue_ms = (time.perf_counter() - t0) * 1e3      # host time to hand the steps over, GPU still running
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    ms_per_step = max(wall_ms, gpu_ms) / args.steps
    for r in runners:
        assert int(r.info.item()) == 0, "numeric breakdown during the benchmark"
    value = act_bytes / (ms_per_step * 1e-3) / 1e9

    # per-kernel pass: same steps with every launch bracketed by HIP events on its stream
    # (eager, one stream, so that no two kernels overlap and each duration is its own)
    asi.asi_profile_enable(True)
    nprof = min(args.steps, 10)
    for k in range(nprof):
        a_, g_ = A_dev[k % ndist], dY_dev[k % ndist]
        if batches is not None:
            batched_step(a_, g_, concurrent=False)
        else:
            for r, at, gt in zip(runners, a_, g_):
                r.step(at, gt)
    torch.cuda.synchronize()
    rep = asi.asi_profile_report()
    asi.asi_profile_enable(False)

    # a launch site is "phase|instantiation[:role]"
    def split_site(site):
        phase, _, rest = site.partition("|")
        cut = rest.rfind(":")             # the instantiation itself may hold "::"
        if cut > 0 and rest[cut - 1] != ":" and ">" not in rest[cut:]:
            return phase, rest[:cut], rest[cut + 1:]
        return phase, rest, ""

    per_kernel, per_phase = {}, {}
    for site, v in rep.items():
        phase, sym, _role = split_site(site)
        a = per_kernel.setdefault(sym, {"launches": 0, "ms": 0.0, "bytes": 0.0, "flops": 0.0, "workgroups": 0.0})
        for key in a:
            a[key] += v[key]
        ph = per_phase.setdefault(phase, {"launches": 0, "ms": 0.0})
        ph["launches"] += v["launches"]
        ph["ms"] += v["ms"]

    def price(sym, launches, ms, nbytes, flops):
        """Roofline of one kernel (or launch site): bound by whichever of its algorithmic bytes at the HBM
        peak and its algorithmic flops at its unit's peak takes longer."""
        avg_s = ms * 1e-3 / launches
        bpl, fpl = nbytes / launches, flops / launches
        unit = unit_of(sym)
        t_mem, t_alu = bpl / (HBM_PEAK_GBS * 1e9), fpl / (PEAK_TFLOPS[unit] * 1e12)
        if t_mem >= t_alu:
            out = {"bound": "hbm", "achieved": bpl / avg_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        else:
            out = {"bound": "mfma" if unit.startswith("mfma") else "alu", "achieved": fpl / avg_s / 1e12,
                   "peak": PEAK_TFLOPS[unit], "unit": "TFLOP/s"}
        out["frac"] = out["achieved"] / out["peak"]
        out["avg_launch_us"] = avg_s * 1e6
        out["arith_unit"] = unit
        out["hbm_frac"] = bpl / avg_s / 1e9 / HBM_PEAK_GBS
        out["unit_frac"] = fpl / avg_s / 1e12 / PEAK_TFLOPS[unit]
        return out

    dom = max(per_kernel, key=lambda s_: per_kernel[s_]["ms"])
    d = per_kernel[dom]
    roof = price(dom, d["launches"], d["ms"], d["bytes"], d["flops"])
    kernels, meta = stored_traffic(cfg.index)
    roof["traffic"] = None
    if kernels is not None and meta["same_build"]:
        rec = kernels.get(dom) or kernels.get(dom.replace("asi::", ""))
        if rec is not None:
            roof["traffic"] = float(rec["fetch_bytes_per_launch"]) + float(rec["write_bytes_per_launch"])
    roof["traffic_source"] = meta
    roof["kernel"] = dom
    roof["launches_per_step"] = d["launches"] / nprof
    tot_ms = sum(v["ms"] for v in per_kernel.values())
    roof["kernel_time_share"] = d["ms"] / tot_ms

    # whole step against the two models of what the method must move / compute
    models = [layer_model(lay) for lay in cfg.layers]
    alg_bytes = sum(m["bytes"] for m in models)
    alg_flops = sum(m["flops"] for m in models)
    in_unit = "mfma_f32" if cfg.layers[0].dtype == "f32" else "mfma_bf16"
    t_step = ms_per_step * 1e-3
    whole = {"algorithmic_bytes_per_step": alg_bytes, "bytes_model": "sum over layers of 2|A| + |dY| + |dW| + 4 M_i",
             "hbm_us_at_peak": alg_bytes / (HBM_PEAK_GBS * 1e9) * 1e6, "hbm_frac": alg_bytes / t_step / 1e9 / HBM_PEAK_GBS,
             "algorithmic_flops_per_step": alg_flops, "flop_model": "2 (O_ASI + cheapest core chain + C_ASI) in MACs of the paper's formulas",
             "flop_peak_unit": in_unit, "flop_us_at_peak": alg_flops / (PEAK_TFLOPS[in_unit] * 1e12) * 1e6,
             "flop_frac": alg_flops / t_step / 1e12 / PEAK_TFLOPS[in_unit]}
    whole["counter_traffic_bytes_per_step"] = None
    whole["counter_traffic_over_algorithmic"] = None
    if kernels is not None and meta["same_build"]:
        tot = 0.0
        ok = True
        for sym, v in per_kernel.items():
            rec = kernels.get(sym) or kernels.get(sym.replace("asi::", ""))
            if rec is None:
                ok = False
                break
            tot += (float(rec["fetch_bytes_per_launch"]) + float(rec["write_bytes_per_launch"])) * v["launches"] / nprof
        if ok:
            whole["counter_traffic_bytes_per_step"] = tot
            whole["counter_traffic_over_algorithmic"] = tot / alg_bytes
    roof["whole_step"] = whole

    breakdown = {}
    for site, v in sorted(rep.items(), key=lambda kv: -kv[1]["ms"]):
        if v["ms"] <= 0:
            continue
        phase, sym, role = split_site(site)
        pr = price(sym, v["launches"], v["ms"], v["bytes"], v["flops"])
        breakdown[site] = {"us_per_step": v["ms"] * 1e3 / nprof, "launches_per_step": v["launches"] / nprof,
                           "avg_launch_us": pr["avg_launch_us"], "bound": pr["bound"], "frac": pr["frac"],
                           "GBps": v["bytes"] / (v["ms"] * 1e-3) / 1e9, "TFLOPs": v["flops"] / (v["ms"] * 1e-3) / 1e12,
                           "hbm_frac": pr["hbm_frac"], "unit_frac": pr["unit_frac"], "arith_unit": pr["arith_unit"],
                           "workgroups_per_launch": v["workgroups"] / v["launches"]}
    phases = {ph: {"us_per_step": v["ms"] * 1e3 / nprof, "launches_per_step": v["launches"] / nprof}
              for ph, v in per_phase.items()}

    out = {
        "value": value, "unit": "GB/s", "ms_per_step": ms_per_step,
        "host_enqueue_ms_per_step": enqueue_ms / args.steps,
        "dtype": "f32" if cfg.layers[0].dtype == "f32" else "bf16",
        "config": {"workload": f"config {cfg.index} ({cfg.name}): " + ", ".join(
            f"{'x'.join(map(str, l.dims))} r{'/'.join(map(str, l.ranks))}" for l in cfg.layers),
            "layers": len(cfg.layers), "raw_activation_bytes_per_step": act_bytes,
            "distinct_input_steps_in_hbm": ndist, "phases": "compress+core_project+weight_grad",
            "batched_launches": bool(args.batch), "streams": nstreams, "hip_graph": bool(args.graph),
            "graph_mode": {0: "eager", 1: "one graph per step, layers fork/join",
                           2: "one graph per layer on its own stream"}[
                args.graph if (args.graph != 2 or layer_graphs is not None) else 1],
            "queue_probe": queue_probe},
        "roofline": roof,
        "phases_eager_single_stream": phases,
        "kernel_breakdown": breakdown,
        "gpu_ms_per_step_events": gpu_ms / args.steps,
    }
    if cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, streams, cpu_seconds, extras=cpu_seconds >= 10)
    del A_dev, dY_dev, runners, batches, graphs, layer_graphs
    torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch

    from asi_inputs import CONFIGS

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    head_index = args.config if args.config else HEADLINE_CONFIG
    cpu_s = 0.0 if args.no_cpu_baseline else args.cpu_seconds
    head = measure(CONFIGS[head_index], args, cpu_s)
    out = {"metric": "ASI compress+dW throughput (GB/s raw activation), % of HBM/MFMA roofline",
           "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": head["dtype"], "data": "synthetic"}
    for key in ("config", "roofline", "cpu_baseline", "host_enqueue_ms_per_step", "phases_eager_single_stream",
                "kernel_breakdown", "gpu_ms_per_step_events"):
        if key in head:
            out[key] = head[key]
    if not args.config:
        # the same figures for every workload (the headline one is not measured twice)
        cpu_o = 0.0 if args.no_cpu_baseline else args.cpu_seconds_other
        per = []
        for ci in sorted(CONFIGS):
            m = head if ci == head_index else measure(CONFIGS[ci], args, cpu_o)
            r = m["roofline"]
            per.append({"config": ci, "workload": m["config"]["workload"], "dtype": m["dtype"],
                        "value": m["value"], "unit": "GB/s", "ms_per_step": m["ms_per_step"],
                        "steps": args.steps, "warmup": args.warmup,
                        "host_enqueue_ms_per_step": m["host_enqueue_ms_per_step"],
                        "dominant_kernel": r["kernel"], "roofline": r,
                        "phases_eager_single_stream": m["phases_eager_single_stream"],
                        "passes": m["kernel_breakdown"],
                        "cpu_baseline": m.get("cpu_baseline")})
        out["per_config"] = per
    print(json.dumps(out))


if __name__ == "__main__":
    main()
