#!/usr/bin/env python3
"""Benchmark of the LGC per-node compression hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic gradients of the
ResNet50-sized workload (4 simulated nodes x 25.6 M fp32 elements, k = 25 600 per node):
fused accumulate + exact top-k (all nodes in one call), encoder, decoder, scatter/average.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
ALGO_BYTES_PER_ELEM = 20       # read g,u,v + write u,v, fp32: what accumulate+select must move


def measured_traffic(cfg, ratio_index, selection, pattern):
    """HBM bytes per launch of the streaming kernel as counted by rocprofv3 (FETCH_SIZE and WRITE_SIZE passes, each
    scaled by a plain copy of known size), from profiles/hbm_traffic.json.  The file names the sources the counted
    kernel was built from (their sha256); the figure is reported only while those sources are unchanged: None
    (printed as null) means "not counted for this workload, or the kernel changed since it was counted"."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(path))
        digest = hashlib.sha256()
        for rel in table["kernel_sources"]:
            digest.update(open(os.path.join(ROOT, rel), "rb").read())
        if digest.hexdigest() != table["kernel_sources_sha256"]:
            return None, "the streaming kernel's sources changed since the counters were read"
        for e in table["entries"]:
            if (e["workload"], e["ratio_index"], e["selection"], e["pattern"]) == (cfg, ratio_index, selection, pattern):
                return e["bytes_per_launch"], f"{e['source']} (counted at commit {table['commit']})"
    except (OSError, KeyError, ValueError):
        pass
    return None, "not counted for this workload"


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=50)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--workload", type=int, default=2, help="1..5 (default 2: ResNet50-sized)")
    p.add_argument("--no-plain-kernels", action="store_true",
                   help="do not run the stand-alone program that measures plain streaming kernels (use under a profiler)")
    p.add_argument("--ratio-index", type=int, default=-1, help="which of the workload's ratios")
    p.add_argument("--grad-sets", type=int, default=0, help="distinct gradient sets kept in HBM (0 = workload's)")
    p.add_argument("--pattern", choices=["ps", "rar", "ps-innovation"], default="ps",
                   help="ps: every node selects (default, the headline); rar: ring-allreduce pattern, one "
                        "rotating node selects and the others take the values at its positions (Alg. 2); "
                        "ps-innovation: Alg. 1 in full, every node also forms its innovation component (top 10 %% "
                        "of each layer's selected values) and the decoder takes it as one more channel")
    p.add_argument("--selection", choices=["flat", "layers"], default=None,
                   help="flat: one top-k over the whole vector (default, the headline); layers: per-layer "
                        "top-k over the workload's layers, mu_l = max(1, floor(ratio n_l)) (Sec. V-A; the default "
                        "of --pattern ps-innovation on workloads 2-4, Alg. 1 being written per layer)")
    p.add_argument("--ae", choices=["config", "paper"], default="config",
                   help="config: the workload's two-layer autoencoder (default); paper: Table I / Table II layer "
                        "shapes (1-64-128-256-64-4 / 4-4-32-64-128-32-1, leaky slope 0.01), deep layers on the matrix cores")
    p.add_argument("--state-iters", type=int, default=40,
                   help="iterations of the step run before the warm-up, untimed, to bring the residuals u, v from zero "
                        "to those of a run in progress (0: start the warm-up from zero residuals)")
    p.add_argument("--graph", action="store_true",
                   help="record two steps into a HIP graph and time its replays (steps must be even)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-kernel-events", action="store_true",
                   help="do not bracket the streaming kernel with HIP events (roofline.achieved = null)")
    return p.parse_args()


def cpu_baseline(w, k, enc, dec, host_w, g_host, momentum, plan=None, inv_plan=None):
    """The oracle, as it stands, on one iteration of the same workload: accumulate + top-k +
    encode + decode + scatter for every node, nodes on separate threads (the only parallelism
    that cannot change its results)."""
    import numpy as np
    from oracle import lgc_oracle as oracle
    K, n = g_host.shape
    threads = min(K, os.cpu_count() or 1)
    ew, eb, dw, db = host_w

    def node(b):
        u = np.zeros(n, np.float32)
        v = np.zeros(n, np.float32)
        oracle.accumulate(g_host[b], u, v, momentum)
        vals, idx = oracle.topk(v, u, k) if plan is None else oracle.topk_segmented(v, u, plan[0], plan[1])
        lat = oracle.encode(vals, enc, ew, eb)
        if inv_plan is None:
            rec = oracle.decode(lat, k, enc, dec, dw, db)
        else:
            rec = oracle.decode_with_innovation(lat, oracle.innovation(vals, inv_plan[0], inv_plan[1]), k, enc, dec, dw, db)
        return rec, idx

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        outs = list(ex.map(node, range(K)))
    dense = np.zeros(n, np.float32)
    for rec, idx in outs:
        oracle.scatter(rec, idx, 1.0 / K, dense)
    dt = time.perf_counter() - t0
    return {"value": K * n / dt, "unit": "elements/s", "cores": threads, "kind": "oracle",
            "sample": f"1 iteration of all {K} nodes x {n} elements (zero initial state), "
                      f"{dt:.2f} s wall on {threads} threads"}


def ae_report(enc, dec, k, dec_batch, enc_batch, stages, which):
    """Multiply-adds of the encoder / decoder stacks at this k and the rate they ran at (their own
    entry-point timings): the roofline of a contraction is the fp32 MFMA peak."""
    lens = [k]
    for (_, _, ks, st) in enc:
        lens.append(lens[-1] if st == 1 else (lens[-1] + 1) // 2)
    enc_mac = sum(ci * co * ks * lens[i + 1] for i, (ci, co, ks, st) in enumerate(enc))
    consumed = [lens[i] for i, l in enumerate(enc) if l[3] == 2]
    cur, dec_mac = lens[-1], 0
    for (ci, co, ks, st) in dec:
        if st == 2:
            nxt = consumed.pop()
            dec_mac += ci * co * ks * cur          # every input position meets every tap once (edges aside)
            cur = nxt
        else:
            dec_mac += ci * co * ks * cur
    peak = 157.3
    enc_tf = 2.0 * enc_mac * enc_batch / (stages["a3_encode"] * 1e-3) / 1e12
    dec_tf = 2.0 * dec_mac * dec_batch / (stages["a4_decode"] * 1e-3) / 1e12
    return {"shape": which, "encode_mac_per_node": enc_mac, "decode_mac_per_node": dec_mac,
            "encode_TFLOPs": enc_tf, "decode_TFLOPs": dec_tf, "bound": "mfma", "peak": peak, "unit": "TFLOP/s",
            "encode_frac": enc_tf / peak, "decode_frac": dec_tf / peak,
            "note": "fp32 in, fp32 accumulate: the roofline is the fp32 MFMA peak"}


def plain_kernel_rates():
    """Runs the stand-alone program built from hbm_rates.hip beside this file: the rates of a
    plain read, a plain copy and a plain 3-reads-2-writes kernel on arrays of the ResNet50-sized
    workload, and of the runtime's device-to-device copy.  None if it is not built or fails."""
    import subprocess
    exe = os.path.join(ROOT, "hbm_rates")
    if not os.path.exists(exe):
        return None
    try:
        r = subprocess.run([exe, "--json"], capture_output=True, text=True, timeout=120)
        if r.returncode != 0:
            return None
        d = json.loads(r.stdout.strip().splitlines()[-1])
    except Exception:
        return None
    d["note"] = ("one 256-thread block per 4096 elements; 3r2w reads g, u, v and writes u, v like the fused kernel, "
                 "without any selection work; _nt = non-temporal loads and stores")
    return d


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the method shards by "
              "node, one simulated node set per GPU); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2103_08870_amd import binding as B
    from paper_2103_08870_amd import synth

    if not os.path.exists(B.LIB_PATH):
        from paper_2103_08870_amd import build
        build.build()
    # what kernels with no selection work reach on this GPU: measured by a child process, which is
    # started before this process makes its first GPU call
    plain = None if args.no_plain_kernels else plain_kernel_rates()
    B.lib()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    w = synth.workload(args.workload)
    if args.selection is None:
        args.selection = "layers" if args.pattern == "ps-innovation" and w.kind == "laplace_segments" else "flat"
    K, n = w.nodes, w.n
    k = w.ks[args.ratio_index]
    seg = None
    if args.selection == "layers":
        assert w.kind == "laplace_segments" and args.pattern != "rar", "--selection layers: workloads 2-4, not with rar"
        seg_off, seg_ks = synth.layer_plan(w, w.ratios[args.ratio_index])
        seg = B.Segments(seg_off, seg_ks)
        k = seg.total_k
    sets = args.grad_sets or w.iters
    inv_seg = inv_plan = None
    if args.pattern == "ps-innovation":
        # Alg. 1: per layer of the selected values (one layer when the selection is flat) the top 10 % are
        # the innovation component
        assert args.ae == "config", "ps-innovation: the workload's autoencoder with the innovation channel"
        ks_out = seg_ks if seg is not None else [k]
        out_off = [0]
        for k_l in ks_out:
            out_off.append(out_off[-1] + k_l)
        inv_plan = (out_off, [max(1, k_l // 10) for k_l in ks_out])
        inv_seg = B.Segments(*inv_plan)
    if args.pattern == "ps-innovation":
        enc, dec = synth.innovation_ae(w.ae_channels)
    else:
        enc, dec = synth.mirrored_ae(w.ae_channels) if args.ae == "config" else synth.paper_ae()
    slope = 0.0 if args.ae == "config" else 0.01
    ew, eb, dw, db = synth.ae_weights(enc, dec, device="cuda")
    ae = B.Autoencoder(enc, dec, ew, eb, dw, db, slope=slope)
    ctx = B.Context(n, k, K)
    B.lgc_reserve(ctx, ae, k, K, seg)     # all the scratch the step needs exists before the first call

    grads = [synth.gradients(w, t, device="cuda", k_for_ties=(k,)) for t in range(sets)]
    u = torch.zeros((K, n), device="cuda")
    v = torch.zeros((K, n), device="cuda")
    vals = torch.zeros((K, k), device="cuda")
    idx = torch.zeros((K, k), device="cuda", dtype=torch.int32)
    lat = torch.zeros((K, B.lgc_latent_len(ae, k)), device="cuda")
    rec = torch.zeros((K, k), device="cuda")
    dense = torch.zeros(n, device="cuda")

    def select(t):
        if seg is None:
            B.lgc_accumulate_topk(ctx, grads[t % sets], u, v, w.momentum, k, vals, idx)
        else:
            B.lgc_accumulate_topk_segmented(ctx, seg, grads[t % sets], u, v, w.momentum, vals, idx)

    def step_ps(t):
        select(t)
        B.lgc_encode(ctx, ae, vals, lat)
        B.lgc_decode(ctx, ae, lat, rec)
        B.lgc_scatter(ctx, rec, idx, 1.0 / K, dense)

    innov = torch.zeros((K, k), device="cuda") if inv_seg is not None else None

    def step_ps_innovation(t):
        select(t)
        B.lgc_innovation(ctx, inv_seg, vals, innov)
        B.lgc_encode(ctx, ae, vals, lat)
        B.lgc_decode_innovation(ctx, ae, lat, innov, rec)
        B.lgc_scatter(ctx, rec, idx, 1.0 / K, dense)

    lat_avg = torch.zeros((1, lat.shape[1]), device="cuda")

    def step_rar(t):
        g, L = grads[t % sets], t % K                 # node L selects in this iteration
        B.lgc_accumulate_topk(ctx, g[L], u[L], v[L], w.momentum, k, vals[L], idx[0])
        for lo, hi in ((0, L), (L + 1, K)):
            if hi > lo:
                B.lgc_accumulate_gather(ctx, g[lo:hi], u[lo:hi], v[lo:hi], w.momentum, idx[0], vals[lo:hi])
        B.lgc_encode(ctx, ae, vals, lat)
        B.lgc_average(ctx, lat, 1.0 / K, lat_avg[0])
        B.lgc_decode(ctx, ae, lat_avg, rec[:1])
        B.lgc_scatter(ctx, rec[:1], idx[:1], 1.0, dense)

    step = {"ps": step_ps, "rar": step_rar, "ps-innovation": step_ps_innovation}[args.pattern]

    # The residuals u, v are inputs of a step as much as the gradients are.  They start at zero, and from zero the
    # k-th largest magnitude grows by tens of per cent per iteration for the first iterations, which no training run
    # does for more than its first moments: the timed steps work on the residuals of a run in progress, produced
    # here by the path itself on the same gradient sets.
    t_first = args.state_iters
    for t in range(t_first):
        step(t)
    for t in range(args.warmup):
        step(t_first + t)
    t_first += args.warmup
    torch.cuda.synchronize()
    B.lgc_stats(ctx)
    B.lgc_stats_carried(ctx)
    dense.zero_()
    graph = None
    if args.graph:
        # two consecutive steps per graph (the selection scratch alternates between two state sets);
        # replays then cycle through two of the resident gradient sets only
        assert args.steps % 2 == 0 and args.pattern == "ps", "--graph: even --steps, pattern ps"
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(0)
            step(1)
        torch.cuda.synchronize()
    elif not args.no_kernel_events:
        B.lgc_set_option(ctx, B.LGC_OPT_PROFILE, 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        for t in range(args.steps // 2):
            graph.replay()
    else:
        for t in range(args.steps):
            step(t_first + t)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    B.lgc_set_option(ctx, B.LGC_OPT_PROFILE, 0)
    kern_ms, kern_launches = B.lgc_profile_read(ctx)
    fast, fallback, errors = B.lgc_stats(ctx)
    carried = B.lgc_stats_carried(ctx)
    assert errors == 0, "device-side failure during the timed region"

    ms_per_step = dt * 1e3 / args.steps
    value = K * n * args.steps / dt

    # outside the timed region: every entry point on its own, same buffers, all nodes per call
    def timed_n(fn, count):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for t in range(count):
            fn(t)
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / count

    def timed(fn):
        # one untimed call first: these sequences are not iterations of the method (fifty accumulations in a row,
        # then fifty selections), and the first selection after such a break may fall back to the exact path
        fn(0)
        return timed_n(fn, args.steps)

    fused_ms = timed(select)
    # spread of the fused call: five more repeats of a fifth of the steps each
    reps = sorted(timed_n(select, max(2, args.steps // 5)) for _ in range(5))
    stages = {
        "a1_accumulate": timed(lambda t: B.lgc_accumulate(ctx, grads[t % sets], u, v, w.momentum)),
        "a2_topk": timed((lambda t: B.lgc_topk(ctx, v, u, k, vals, idx)) if seg is None else
                         (lambda t: B.lgc_topk_segmented(ctx, seg, v, u, vals, idx))),
        "a1a2_fused": fused_ms,
        "a3_encode": timed(lambda t: B.lgc_encode(ctx, ae, vals, lat)),
        "a4_decode": timed((lambda t: B.lgc_decode(ctx, ae, lat, rec)) if inv_seg is None else
                           (lambda t: B.lgc_decode_innovation(ctx, ae, lat, innov, rec))),
        "a5_scatter": timed(lambda t: B.lgc_scatter(ctx, rec, idx, 1.0 / K, dense)),
    }
    if inv_seg is not None:
        stages["innovation"] = timed(lambda t: B.lgc_innovation(ctx, inv_seg, vals, innov))
    B.lgc_stats(ctx)
    torch.cuda.synchronize()
    ratio_index = args.ratio_index % len(w.ks)
    traffic, traffic_source = measured_traffic(w.cfg, ratio_index, args.selection, args.pattern)
    roofline = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
                "traffic": traffic, "traffic_source": traffic_source, "kernel": f"lgc::k_candidates<true, true, {'false' if seg is None else 'true'}> (fused accumulate + candidate bitmap, all nodes in one launch)",
                "algorithmic_bytes_per_launch": ALGO_BYTES_PER_ELEM * K * n}
    if kern_launches:
        # ps: one streaming launch per step covers all K nodes; rar: the selecting node's launch and
        # the other nodes' launches together cover them, so the bytes are counted per step
        per_step_ms = kern_ms / args.steps
        ach = ALGO_BYTES_PER_ELEM * K * n / (per_step_ms * 1e-3) / 1e9
        # large workloads stream in several launches per step (shares of about 2 GB): bytes are per launch
        roofline.update(achieved=ach, frac=ach / HBM_PEAK_GBS, kernel_avg_ms=kern_ms / kern_launches,
                        launches=kern_launches,
                        algorithmic_bytes_per_launch=ALGO_BYTES_PER_ELEM * K * n * args.steps // kern_launches)
        if args.pattern == "rar":
            roofline.update(kernel="lgc::k_candidates<true, true, false> (selecting node) + lgc::k_accumulate<true> "
                                   "(other nodes): the streaming launches of one step")

    if plain is not None:
        roofline["plain_kernels"] = plain

    out = {
        "metric": "gradient elements/sec compressed (accumulate+top-k+AE encode); % of HBM peak",
        "value": value, "unit": "elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {w.cfg} ({w.name}-sized): {K} nodes x {n} fp32 elements, k={k}/node, "
                               f"momentum {w.momentum}, autoencoder "
                               f"{'->'.join(map(str, w.ae_channels)) if args.ae == 'config' else 'Table I / Table II shapes'}, "
                               f"{sets} gradient sets resident in HBM",
                   "state": (f"residuals u, v of a run in progress: {args.state_iters} iterations of the same step from zero "
                             "residuals, untimed, before the warm-up" if args.state_iters else
                             "residuals u, v zero at the start of the warm-up"),
                   "step": ("accumulate+top-k (fused, all nodes in one call) + encode + decode + scatter"
                            if seg is None else
                            f"accumulate + per-layer top-k over {len(seg_ks)} layers (fused, all nodes in one call) "
                            "+ encode + decode + scatter")
                           if args.pattern == "ps" else
                           (f"Alg. 1 in full: accumulate + {'per-layer ' if seg is not None else ''}top-k (fused, all nodes "
                            f"in one call) + innovation component ({sum(inv_plan[1])} of {k} values per node, top 10 % per "
                            "layer) + encode + decode with the innovation channel + scatter")
                           if args.pattern == "ps-innovation" else
                           "ring-allreduce pattern: accumulate+top-k on the selecting node, accumulate+gather at "
                           "its positions on the others, encode (all), average, decode (once), scatter (once)"},
        "whole_step_hbm_frac": ALGO_BYTES_PER_ELEM * value / (HBM_PEAK_GBS * 1e9),
        "whole_step_algorithmic_GBps": ALGO_BYTES_PER_ELEM * value / 1e9,
        # per node and step: served by the fast path / fell back to the exact path on the device; `carried`: of the
        # fast ones, those whose candidate threshold came from the trend of the previous steps' thresholds, not a sample
        "select_path": {"fast": fast, "fallback": fallback, "carried": carried},
        "hip_graph": bool(args.graph),
        "accumulate_topk_call": {"ms": fused_ms, "algorithmic_GBps": ALGO_BYTES_PER_ELEM * K * n / fused_ms / 1e6,
                                 "hbm_frac": ALGO_BYTES_PER_ELEM * K * n / fused_ms / 1e6 / HBM_PEAK_GBS,
                                 "ms_median_of_5": reps[2], "ms_min_of_5": reps[0],
                                 "note": "same buffers, measured after the timed region"},
        "stages_ms": {name: round(ms, 5) for name, ms in stages.items()},
        "roofline": roofline,
    }
    if args.ae == "paper":   # only the Table I / II shapes are contractions worth a matrix-core roofline
        out["autoencoder"] = ae_report(enc, dec, k, 1 if args.pattern == "rar" else K, K, stages, args.ae)

    if not args.no_cpu_baseline:
        host_w = [[t.cpu().numpy() for t in xs] for xs in (ew, eb, dw, db)]
        out["cpu_baseline"] = cpu_baseline(w, k, enc, dec, host_w, grads[0].cpu().numpy(), w.momentum,
                                           None if seg is None else (seg_off, seg_ks), inv_plan)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
