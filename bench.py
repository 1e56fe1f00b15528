#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One step = K-layer normalized propagation forward plus backward (2K neighbour-sum passes) on the
resident graph of the 50 M-edge power-law workload (bf16, F=128, K=3).  Graph construction
(e2eg_build_csr + e2eg_normalize) happens once per graph and is timed separately.
Prints ONE JSON line on stdout (progress goes to stderr).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def recorded_traffic(config: int, scale: float):
    """HBM bytes per launch of the neighbour-sum kernel from the committed rocprofv3 counter
    summary, or None when it does not describe the kernel as it is now (sources changed) or
    this workload.  The summary ends with two lines `traffic_bytes_per_launch: N` and
    `source_sha1: H` (sha1 over propagate.hip, normalize.hip, common.h)."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", "spmm_rows_config3.txt")
    if config != 3 or scale != 1.0 or not os.path.exists(path):
        return None
    text = open(path).read()
    traffic = re.search(r"^traffic_bytes_per_launch: (\d+)$", text, re.M)
    sha = re.search(r"^source_sha1: ([0-9a-f]{40})$", text, re.M)
    if not traffic or not sha:
        return None
    h = hashlib.sha1()
    for f in ("propagate.hip", "normalize.hip", "common.h"):
        h.update(open(os.path.join(ROOT, "paper_2511_20564_amd", "csrc", f), "rb").read())
    return int(traffic.group(1)) if sha.group(1) == h.hexdigest() else None


def log(*a):
    print(*a, file=sys.stderr, flush=True)



def event_ms(fn, reps=5):
    """Mean duration of fn() in ms over `reps` back-to-back calls, by events on torch's current stream
    (the stream every call here is enqueued on)."""
    import torch
    fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def replay_ms(torch, fn, reps=20, inner=1):
    """The same calls replayed from a HIP graph: their duration without the host's launch work.
    `inner` calls are captured into one graph and the time is per call: the start of a graph costs
    some 15 us on the device's time line, which would swamp a single kernel of that length."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    hip_graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        fn()
        torch.cuda.synchronize()
        with torch.cuda.graph(hip_graph, stream=side):
            for _ in range(inner):
                fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    return event_ms(hip_graph.replay, reps=reps) / inner


def bench_transform(dev, torch, _event_ms=None):
    """The dense per-layer update on the matrix cores: forward, and backward (dP and dW), at the
    mini-batch shape (200 k sampled nodes, 128 x 128 weights) and at 4 M rows (2 GB of rows, beyond
    the last-level cache).  Calls go through the C ABI on preallocated buffers; `*_graph_ms` is the time
    per call of several calls replayed back to back from one HIP graph, which leaves the host's launch
    work out.  Flops and bytes are algorithmic."""
    from paper_2511_20564_amd import binding as B
    Ft = 128
    out = {"Fin": Ft, "Fout": Ft, "mfma_bf16_peak_TFLOPs": 2500.0, "hbm_peak_GBs": HBM_PEAK_GBS}
    Wt = (torch.randn(Ft, Ft, device="cuda") / Ft ** 0.5).to(torch.bfloat16)
    for tag, nt, reps in (("", 200_000, 20), ("_large", 4_000_000, 5)):
        Pt = torch.randn(nt, Ft, device="cuda").to(torch.bfloat16)
        gt = torch.randn(nt, Ft, device="cuda").to(torch.bfloat16)
        Ht, gP = torch.empty_like(Pt), torch.empty_like(Pt)
        gW = torch.empty(Ft, Ft, device="cuda", dtype=torch.float32)
        ws = torch.empty(max(B.e2eg_layer_transform_workspace_bytes(B.E2EG_TRANSFORM_BWD, nt, Ft, Ft, B.E2EG_BF16), 256),
                         dtype=torch.uint8, device="cuda")

        def fwd():
            B.e2eg_layer_transform(B.E2EG_TRANSFORM_FWD, nt, Ft, Ft, B.E2EG_BF16, 1, Pt, Wt, Ht, None, None, None, ws,
                                   None, torch.cuda.current_stream().cuda_stream)

        def bwd():
            B.e2eg_layer_transform(B.E2EG_TRANSFORM_BWD, nt, Ft, Ft, B.E2EG_BF16, 1, Pt, Wt, Ht, gt, gP, gW, ws,
                                   None, torch.cuda.current_stream().cuda_stream)

        # a plain copy of known size on the same stream: the scale for the profiler's byte counters
        B.e2eg_profile_copy(gP, Pt, Pt.numel() * Pt.element_size(), torch.cuda.current_stream().cuda_stream)
        tf_ms, tb_ms = event_ms(fwd, reps), event_ms(bwd, reps)
        inner = 10 if nt <= 1_000_000 else 2
        gf_ms, gb_ms = replay_ms(torch, fwd, reps, inner), replay_ms(torch, bwd, reps, inner)
        flop_f = 2.0 * nt * Ft * Ft
        bytes_f, bytes_b = 2 * nt * Ft * 2 + Ft * Ft * 2, 4 * nt * Ft * 2 + Ft * Ft * 6
        out.update({
            "rows" + tag: nt,
            "fwd" + tag + "_ms": round(tf_ms, 4), "fwd" + tag + "_graph_ms": round(gf_ms, 4),
            "fwd" + tag + "_TFLOPs": round(flop_f / gf_ms / 1e9, 1), "fwd" + tag + "_GBs": round(bytes_f / gf_ms / 1e6, 1),
            "bwd" + tag + "_ms": round(tb_ms, 4), "bwd" + tag + "_graph_ms": round(gb_ms, 4),
            "bwd" + tag + "_TFLOPs": round(2 * flop_f / gb_ms / 1e9, 1), "bwd" + tag + "_GBs": round(bytes_b / gb_ms / 1e6, 1),
        })
        del Pt, gt, Ht, gP, ws
    out["rates_from"] = "graph replay"
    return out


def time_propagation(dev, B, torch, g, X0, gY, K, F, esz, steps, warmup=2):
    """Forward + backward of K layers on a resident graph: wall time per step, the neighbour-sum
    kernel's mean duration, and the rates that follow (algorithmic and zero-reuse gather bytes)."""
    import numpy as np
    out_f, out_b = torch.empty_like(X0), torch.empty_like(X0)
    ws = dev.propagate_workspace(g, X0.dtype, F, K)

    def step():
        dev.propagate_fwd(g, X0, K, out=out_f, ws=ws)
        dev.propagate_bwd(g, gY, K, out=out_b, ws=ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    B.e2eg_profile_begin(2 * K * steps)
    t1 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t1) / steps * 1e3
    kernel_ms = B.e2eg_profile_end(2 * K * steps)
    n, nnz = g.n, g.nnz
    alg = 4 * nnz + 4 * (n + 1) + 4 * n + 2 * n * F * esz
    gather = alg - n * F * esz + nnz * F * esz + 4 * nnz
    return {
        "ms_per_step": round(ms, 4), "GTEPS": round(nnz * K * 2 / (ms * 1e-3) / 1e9, 3),
        "GTEPS_edges_only": round((nnz - n) * K * 2 / (ms * 1e-3) / 1e9, 3),
        "alg_GBs": round(alg * 2 * K / (ms * 1e-3) / 1e9, 1), "gather_GBs": round(gather * 2 * K / (ms * 1e-3) / 1e9, 1),
        "spmm_rows_avg_ms": round(float(np.mean(kernel_ms)), 4) if kernel_ms else None,
        "alg_bytes_per_launch": alg, "steps": steps,
    }


def bench_other_config(idx, dev, B, torch, steps):
    """Workloads 1, 2 and 5 (5: the largest that fits one GPU): graph construction and the K-layer
    forward + backward step, features made on the device."""
    from workloads import make_config
    t0 = time.time()
    c = make_config(idx, features=False)
    K, F, dt = c["K"], c["F"], c["dtype"]
    esz = 2 if dt == "bf16" else 4
    users, items = torch.from_numpy(c["users"]).cuda(), torch.from_numpy(c["items"]).cuda()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    g = dev.build_graph(c["n_users"], c["n_items"], users, items)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t1) * 1e3
    t1 = time.perf_counter()
    dev.normalize(g.n, g.nnz, g.row_ptr, g.col_idx)
    torch.cuda.synchronize()
    normalize_ms = (time.perf_counter() - t1) * 1e3
    del users, items
    gen = torch.Generator(device="cuda").manual_seed(c["seed"] + 1000)
    tdt = torch.bfloat16 if dt == "bf16" else torch.float32
    X0 = (torch.randn(g.n, F, device="cuda", generator=gen) * 0.1).to(tdt)
    gY = torch.randn(g.n, F, device="cuda", generator=gen).to(tdt)
    r = time_propagation(dev, B, torch, g, X0, gY, K, F, esz, steps)
    r.update({"workload": f"config {idx} ({c['name']}): {c['n_users']} users + {c['n_items']} items, {c['n_edges']} edges, "
                          f"{dt} F={F}, K={K} fwd+bwd", "n": g.n, "nnz": g.nnz, "max_degree": int(g.deg.max().item()),
              "build_csr_ms": round(build_ms - normalize_ms, 3), "normalize_ms": round(normalize_ms, 3)})
    log(f"[bench] config {idx}: {r['ms_per_step']} ms/step, {r['GTEPS']} GTEPS ({time.time() - t0:.0f}s incl. generation)")
    return r


def bench_minibatch(dev, B, torch, np, parent, X_parent, n_users_parent, seed0):
    """The mini-batch workload end to end, every step on a fresh subgraph: uniform two-hop sampling
    (4096 seed users, fan-outs 25 and 10) from the resident 50 M-edge graph, CSR + schedule of the
    sampled pairs, feature rows looked up, then K = 2 layers of propagate -> dense update (ReLU
    between the layers), forward and backward (dP, dW, transposed propagate)."""
    Fm, Km, fan, n_seeds = X_parent.shape[1], 2, [25, 10], 4096
    ones = torch.ones(parent.nnz, dtype=torch.float32, device="cuda")
    table = dev.sampler_table(parent, p=ones)                 # uniform: every neighbour the same weight
    del ones
    sws = torch.empty(B.e2eg_sample_subgraph_workspace_bytes(parent.n, n_seeds, fan), dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(seed0)
    seeds = torch.from_numpy(np.sort(rng.choice(n_users_parent, size=n_seeds, replace=False)).astype(np.int32)).cuda()
    gen = torch.Generator(device="cuda").manual_seed(seed0)
    W = [(torch.randn(Fm, Fm, device="cuda", generator=gen) / Fm ** 0.5).to(torch.bfloat16) for _ in range(Km)]
    cap_nodes = min(parent.n, n_seeds + B.e2eg_sample_capacity(parent.n, n_seeds, fan))
    g_up = torch.randn(cap_nodes, Fm, device="cuda", generator=gen).to(torch.bfloat16)

    def sample(seed):
        return dev.sample_subgraph(parent, table, seeds, fan, seed, with_weights=False, ws=sws)

    def graph_of(sub):
        return dev.build_graph(sub["n_users"], sub["n_items"], sub["users"], sub["items"])

    def compute(gs, H0, gH):
        P, H = [], [H0]
        for l in range(Km):
            P.append(dev.propagate_fwd(gs, H[l], 1))
            H.append(dev.layer_transform_fwd(P[l], W[l], relu=(l < Km - 1)))
        for l in range(Km - 1, -1, -1):
            gP, gW = dev.layer_transform_bwd(P[l], W[l], H[l + 1], gH, relu=(l < Km - 1))
            gH = dev.propagate_bwd(gs, gP, 1)
        return gH

    def whole(seed):
        sub = sample(seed)
        gs = graph_of(sub)
        H0 = X_parent.index_select(0, sub["nodes"].long())
        return compute(gs, H0, g_up[:gs.n])

    whole(1)
    torch.cuda.synchronize()
    reps = 20
    t1 = time.perf_counter()
    for r in range(reps):
        whole(2 + r)
    torch.cuda.synchronize()
    e2e_ms = (time.perf_counter() - t1) / reps * 1e3
    # the same steps with the next subgraph prepared (sampled, CSR + schedule, feature rows) on a second
    # stream while the current one is computed: the host waits only in the preparation's two read-backs
    main, prep = torch.cuda.current_stream(), torch.cuda.Stream()

    def prepare(seed):
        with torch.cuda.stream(prep):
            sub = sample(seed)
            gs = graph_of(sub)
            H0 = X_parent.index_select(0, sub["nodes"].long())
        for t in (gs.row_ptr, gs.col_idx, gs.deg, gs.dinv_sqrt, gs.sched, H0):
            t.record_stream(main)      # allocated on `prep`, read by kernels on `main`
        return gs, H0

    prep.wait_stream(main)
    ready = prepare(1)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for r in range(reps):
        main.wait_stream(prep)
        gs, H0 = ready
        compute(gs, H0, g_up[:gs.n])
        ready = prepare(2 + r)
    torch.cuda.synchronize()
    pipelined_ms = (time.perf_counter() - t1) / reps * 1e3
    del ready, gs, H0
    # the parts, on one subgraph
    sub = sample(2)
    t1 = time.perf_counter()
    for r in range(reps):
        sample(2 + r)
    sample_ms = (time.perf_counter() - t1) / reps * 1e3
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for r in range(reps):
        gs = graph_of(sub)
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t1) / reps * 1e3
    H0 = X_parent.index_select(0, sub["nodes"].long())
    gH = g_up[:gs.n]
    compute_ms = event_ms(lambda: compute(gs, H0, gH), reps=reps)
    compute_graph_ms = replay_ms(torch, lambda: compute(gs, H0, gH), reps=reps, inner=4)
    flop = 3 * 2.0 * gs.n * Fm * Fm * Km          # forward product, dP and dW per layer
    return {
        "workload": f"config 4 (minibatch): {n_seeds} seed users, uniform fan-out {fan} from the 50 M-edge graph -> "
                    f"{sub['n_users']} users + {sub['n_items']} items, {int(sub['users'].numel())} picks, nnz {gs.nnz}; "
                    f"bf16 F={Fm}, K={Km}, W {Fm}x{Fm}",
        "end_to_end_eager_ms": round(e2e_ms, 4), "end_to_end_two_streams_ms": round(pipelined_ms, 4),
        "sample_ms": round(sample_ms, 4),
        "csr_and_schedule_ms": round(graph_ms, 4), "compute_eager_ms": round(compute_ms, 4),
        "compute_hip_graph_ms": round(compute_graph_ms, 4),
        "compute_GTEPS_hip_graph": round(gs.nnz * Km * 2 / (compute_graph_ms * 1e-3) / 1e9, 2),
        "dense_TFLOPs_hip_graph": round(flop / compute_graph_ms / 1e9, 2),
        "sampler_table_once_per_graph": True,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="workload index (3 = headline)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (experiments only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="headline workload only (profiling runs)")
    ap.add_argument("--only", choices=["transform", "minibatch"], default=None,
                    help="profiling runs: the dense update alone, or the mini-batch step alone; prints that section")
    ap.add_argument("--no-config5", action="store_true", help="skip the 500 M-edge workload (80 s of generation)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library is single-GPU (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    os.environ.setdefault("E2EG_WORKLOAD_CACHE", "/tmp/e2eg_workload_cache")
    import numpy as np
    import torch

    import paper_2511_20564_amd.device as dev
    from paper_2511_20564_amd import binding as B
    from workloads import make_config

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    B.load_library()

    if args.only == "transform":
        print(json.dumps({"layer_transform": bench_transform(dev, torch)}), flush=True)
        return

    t0 = time.time()
    c = make_config(args.config, scale=args.scale)
    log(f"[bench] workload {c['name']} generated in {time.time() - t0:.1f}s: n={c['n']} E={c['n_edges']}")
    K, F, dt = c["K"], c["F"], c["dtype"]
    esz = 2 if dt == "bf16" else 4

    def dev_features(a):
        if dt == "bf16":
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    users = torch.from_numpy(c["users"]).cuda()
    items = torch.from_numpy(c["items"]).cuda()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    g = dev.build_graph(c["n_users"], c["n_items"], users, items)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t1) * 1e3
    t1 = time.perf_counter()
    g.deg, g.dinv_sqrt, g.sched = dev.normalize(g.n, g.nnz, g.row_ptr, g.col_idx)
    torch.cuda.synchronize()
    normalize_ms = (time.perf_counter() - t1) * 1e3
    del users, items
    n, nnz = g.n, g.nnz
    log(f"[bench] graph on device: nnz={nnz}, build_csr+normalize {build_ms:.1f} ms, normalize alone {normalize_ms:.2f} ms")

    X0 = dev_features(c["X0"])
    if args.only == "minibatch":
        print(json.dumps({"minibatch_end_to_end": bench_minibatch(dev, B, torch, np, g, X0, c["n_users"], c["seed"] + 7)}),
              flush=True)
        return
    gY = dev_features(c["gY"])
    out_f = torch.empty_like(X0)
    out_b = torch.empty_like(X0)
    ws = dev.propagate_workspace(g, X0.dtype, F, K)

    def step():
        dev.propagate_fwd(g, X0, K, out=out_f, ws=ws)
        dev.propagate_bwd(g, gY, K, out=out_b, ws=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.e2eg_profile_begin(2 * K * args.steps)
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    kernel_ms = B.e2eg_profile_end(2 * K * args.steps)
    ms_per_step = elapsed / args.steps * 1e3
    gteps = nnz * K * 2 / (ms_per_step * 1e-3) / 1e9
    log(f"[bench] {ms_per_step:.3f} ms/step, {gteps:.2f} GTEPS")

    # a plain copy of known size: the scale for the profiler's HBM byte counters (not timed)
    B.e2eg_profile_copy(out_b, X0, X0.numel() * X0.element_size(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()

    # forward and backward alone (information only)
    def timed(fn, reps=5):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / reps * 1e3

    fwd_ms = timed(lambda: dev.propagate_fwd(g, X0, K, out=out_f, ws=ws))
    bwd_ms = timed(lambda: dev.propagate_bwd(g, gY, K, out=out_b, ws=ws))

    # extras, each timed with events on the stream it runs on; bytes are the algorithmic ones
    gfae = weighted = sampler = transform = small = minibatch = others = None
    if not args.no_extras:
        H_all = dev.propagate_fwd(g, X0, K, all_layers=True)
        Y = dev.readout_mean(X0, H_all)
        readout_ms = event_ms(lambda: dev.readout_mean(X0, H_all))
        loss_ms = event_ms(lambda: dev.gfae_loss(X0, Y, grad_scale=1.0 / (K + 1)))
        readout_bytes = (K + 2) * n * F * esz
        loss_bytes = 3 * n * F * esz
        gfae = {
            "readout_mean_ms": round(readout_ms, 4), "readout_mean_GBs": round(readout_bytes / readout_ms / 1e6, 1),
            "gfae_loss_ms": round(loss_ms, 4), "gfae_loss_GBs": round(loss_bytes / loss_ms / 1e6, 1),
            "hbm_peak_GBs": HBM_PEAK_GBS,
        }
        del H_all, Y
        # two upstream gradients (one per task, as GradNorm needs them) through the K layers: two passes
        # of F columns against one pass of 2F columns
        g2 = torch.cat([gY, X0], dim=1).contiguous()
        ws2 = dev.propagate_workspace(g, g2.dtype, 2 * F, K)
        out2 = torch.empty_like(g2)
        two_ms = event_ms(lambda: (dev.propagate_bwd(g, gY, K, out=out_b, ws=ws), dev.propagate_bwd(g, X0, K, out=out_b, ws=ws)), reps=3)
        one_ms = event_ms(lambda: dev.propagate_bwd(g, g2, K, out=out2, ws=ws2), reps=3)
        gfae["two_backward_passes_ms"] = round(two_ms, 4)
        gfae["one_stacked_backward_pass_ms"] = round(one_ms, 4)
        del g2, ws2, out2

        # the same step on the weighted graph (A_ij = edge strength): one more float per stored entry
        from workloads import make_edge_weights
        uw, iw = torch.from_numpy(c["users"]).cuda(), torch.from_numpy(c["items"]).cuda()
        ww = torch.from_numpy(make_edge_weights(c["n_edges"], seed=c["seed"] + 4000)).cuda()
        gw = dev.build_weighted_graph(c["n_users"], c["n_items"], uw, iw, ww)
        del uw, iw, ww
        w_ms = event_ms(lambda: (dev.propagate_fwd(gw, X0, K, out=out_f, ws=ws), dev.propagate_bwd(gw, gY, K, out=out_b, ws=ws)), reps=3)
        weighted = {"ms_per_step": round(w_ms, 4), "GTEPS": round(nnz * K * 2 / (w_ms * 1e-3) / 1e9, 2),
                    "unweighted_ms_per_step": round(ms_per_step, 4)}

        # importance sampling on that graph (the step before the path): the table once per graph, then one
        # two-hop subgraph per call for 4096 seed users, fan-outs (25, 10), p ~ w^1.5; wall time per call
        # (the call waits for its counts)
        t1 = time.perf_counter()
        table = dev.sampler_table(gw, beta=1.5)
        torch.cuda.synchronize()
        table_ms = (time.perf_counter() - t1) * 1e3
        seeds_t = torch.from_numpy(np.sort(np.random.default_rng(c["seed"]).choice(c["n_users"], size=4096, replace=False)).astype(np.int32)).cuda()
        fan = [25, 10]
        sws = torch.empty(B.e2eg_sample_subgraph_workspace_bytes(n, 4096, fan), dtype=torch.uint8, device="cuda")
        sub = dev.sample_subgraph(gw, table, seeds_t, fan, 1, ws=sws)
        t1 = time.perf_counter()
        for r in range(10):
            sub = dev.sample_subgraph(gw, table, seeds_t, fan, 2 + r, ws=sws)
        sample_ms = (time.perf_counter() - t1) / 10 * 1e3
        # ... and what the sampled pairs need before the path can run on them: CSR, weighted degrees, schedule
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for r in range(10):
            gs = dev.build_weighted_graph(sub["n_users"], sub["n_items"], sub["users"], sub["items"], sub["weights"])
        torch.cuda.synchronize()
        subgraph_ms = (time.perf_counter() - t1) / 10 * 1e3
        sampler = {"table_ms": round(table_ms, 3), "sample_ms": round(sample_ms, 4), "seeds": 4096, "fanout": fan,
                   "picks": int(sub["users"].numel()), "nodes": int(sub["n_users"] + sub["n_items"]),
                   "Mpicks_per_s": round(sub["users"].numel() / sample_ms / 1e3, 2),
                   "subgraph_csr_and_schedule_ms": round(subgraph_ms, 4), "subgraph_nnz": int(gs.nnz)}
        del gw, table, sws, sub, gs

        transform = bench_transform(dev, torch)

        # small workloads are bound by kernel launches, not bytes: the same forward+backward step on the
        # sampled mini-batch graph, launched eagerly and replayed from a HIP graph of the same calls
        cm = make_config(4)
        gm = dev.build_graph(cm["n_users"], cm["n_items"], torch.from_numpy(cm["users"]).cuda(),
                             torch.from_numpy(cm["items"]).cuda())
        Xm, gm_up = dev_features(cm["X0"]), dev_features(cm["gY"])
        Km = cm["K"]
        wsm = dev.propagate_workspace(gm, Xm.dtype, cm["F"], Km)
        om_f, om_b = torch.empty_like(Xm), torch.empty_like(Xm)

        def small_step():
            dev.propagate_fwd(gm, Xm, Km, out=om_f, ws=wsm)
            dev.propagate_bwd(gm, gm_up, Km, out=om_b, ws=wsm)

        eager_ms = event_ms(small_step, reps=20)
        graph_ms = replay_ms(torch, small_step, reps=20, inner=4)
        small = {
            "workload": f"config 4 (minibatch): {cm['n_users']} users + {cm['n_items']} items, {cm['n_edges']} edges, "
                        f"bf16 F={cm['F']}, K={Km} fwd+bwd, propagation only",
            "eager_ms_per_step": round(eager_ms, 4), "hip_graph_ms_per_step": round(graph_ms, 4),
            "GTEPS_hip_graph": round(gm.nnz * Km * 2 / (graph_ms * 1e-3) / 1e9, 2),
        }
        del gm, Xm, gm_up, wsm, om_f, om_b


        # the mini-batch workload end to end on the resident graph
        minibatch = bench_minibatch(dev, B, torch, np, g, X0, c["n_users"], c["seed"] + 7)
        log(f"[bench] mini-batch end to end {minibatch['end_to_end_eager_ms']} ms, compute {minibatch['compute_eager_ms']} ms "
            f"eager / {minibatch['compute_hip_graph_ms']} ms from a HIP graph")

        # the other workloads of the list
        others = {}
        for idx in (1, 2) + (() if args.no_config5 else (5,)):
            if idx != args.config:
                others[f"config{idx}"] = bench_other_config(idx, dev, B, torch, steps={1: 50, 2: 30, 5: 5}[idx])

    # roofline of the neighbour-sum kernel: algorithmic bytes of one layer over its mean duration
    alg_bytes = 4 * nnz + 4 * (n + 1) + 4 * n + 2 * n * F * esz
    gather_bytes = alg_bytes - n * F * esz + nnz * F * esz + 4 * nnz
    avg_kernel_ms = float(np.mean(kernel_ms)) if kernel_ms else float("nan")
    achieved = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9
    roofline = {
        "bound": "hbm", "kernel": "spmm_rows", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": recorded_traffic(args.config, args.scale),
        "alg_bytes_per_launch": alg_bytes, "avg_kernel_ms": round(avg_kernel_ms, 4),
        "launches_timed": len(kernel_ms),
        "gather_GBs": round(gather_bytes / (avg_kernel_ms * 1e-3) / 1e9, 1),
    }
    if roofline["traffic"] is not None:   # what the kernel really moves through the fabric, as a rate
        roofline["traffic_GBs"] = round(roofline["traffic"] / (avg_kernel_ms * 1e-3) / 1e9, 1)
        roofline["traffic_frac_of_peak"] = round(roofline["traffic_GBs"] / HBM_PEAK_GBS, 4)
        roofline["traffic_over_algorithmic"] = round(roofline["traffic"] / alg_bytes, 2)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t1 = time.time()
        row_ptr, col = oracle.build_csr(c["n_users"], c["n_items"], c["users"], c["items"])
        log(f"[bench] oracle CSR built in {time.time() - t1:.1f}s")
        Xd = oracle.as_f64(c["X0"])
        t1 = time.perf_counter()
        Y = oracle.propagate_layer(row_ptr, col, Xd)
        t_f = time.perf_counter() - t1
        t1 = time.perf_counter()
        oracle.propagate_layer_transposed(row_ptr, col, Y)
        t_b = time.perf_counter() - t1
        cpu = {
            "value": round(2 * col.size / (t_f + t_b) / 1e9, 4), "unit": "GTEPS", "cores": oracle.max_threads(),
            "kind": "oracle",
            "sample": f"one forward layer ({t_f:.1f}s) + one transposed layer ({t_b:.1f}s) of the same graph, "
                      f"fp64, all F={F} columns",
        }
        log(f"[bench] oracle: {cpu['value']} GTEPS on {cpu['cores']} threads")

    line = {
        "metric": "normalized-SpMM GTEPS (edges*layers/s) fwd+bwd", "value": round(gteps, 3), "unit": "GTEPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dt, "data": "synthetic",
        "config": {
            "workload": f"config {args.config} ({c['name']}): {c['n_users']} users + {c['n_items']} items, "
                        f"{c['n_edges']} edges, power-law, symmetrized + self-loops, {dt} F={F}, K={K} fwd+bwd",
            "scale": args.scale, "seed": c["seed"], "n": n, "nnz": nnz, "max_degree": int(g.deg.max().item()),
            "F": F, "K": K,
        },
        "fwd_ms": round(fwd_ms, 4), "bwd_ms": round(bwd_ms, 4),
        "build_csr_ms": round(build_ms - normalize_ms, 3), "normalize_ms": round(normalize_ms, 3),
        "alg_GBs": round(alg_bytes * 2 * K / (ms_per_step * 1e-3) / 1e9, 1),
        "GTEPS_edges_only": round((nnz - n) * K * 2 / (ms_per_step * 1e-3) / 1e9, 3),
        "roofline": roofline, "cpu_baseline": cpu, "gfae_branch": gfae, "weighted_edges": weighted,
        "importance_sampler": sampler, "layer_transform": transform, "launch_bound_case": small,
        "minibatch_end_to_end": minibatch, "other_workloads": others,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
