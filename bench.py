#!/usr/bin/env python3
"""Benchmark of the SLO-NN hot path on one MI355X.

A step is one pass of the whole path (FreeHash projection, key + bucket lookup + merge,
gathered-row forward, for every layer) over one batch of synthetic queries that already
sit in HBM.  Workload: the 784-1024-1024-10 fp32 MLP, K=8, L=16 on both hidden layers,
batch 256, keep fraction 0.25 (the other keep fractions of that workload, and the dense
MFMA baseline, are timed briefly and reported beside it).  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--keep", type=float, default=0.25)
    ap.add_argument("--config", default="C2")
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--path", default="auto", choices=["auto", "layers", "fused"])
    ap.add_argument("--hash-nodes-always-active", action="store_true",
                    help="Section 3.4 variant: hash nodes always computed, never selected (default off)")
    ap.add_argument("--aclo", action="store_true",
                    help="also time the pass with k chosen per query inside it (ACLO, Confidence LSH tables)")
    ap.add_argument("--build-inputs", type=int, default=0, help="size of the table-training set (default: the config's)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy, for scaling rocprofv3 byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the path is data-parallel over queries with nothing "
                 "exchanged between GPUs, and this build has no multi-GPU leg (run with --gpus 1)")

    import numpy as np
    import torch
    from paper_2204_08400_amd import runtime, slonn, workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    slonn.load()
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.config]
    B = args.batch or cfg.batches[-1]
    K, W = args.steps, args.warmup

    # ---- synthetic workload (seeds: weights 0, build set 1, queries 2, hash nodes 3) ----
    t0 = time.time()
    layers = wl.make_mlp(cfg.dims, seed=0, w_dtype=cfg.w_dtype, last_act=cfg.last_act)
    X_build = wl.make_inputs(cfg, args.build_inputs or cfg.n_inputs, seed=1)
    X_query = wl.make_inputs(cfg, cfg.n_inputs, seed=2)
    log(f"generated {args.config} in {time.time() - t0:.1f}s")

    # hash nodes: variance of the full network's activations on the build set (device dense pass)
    ell = cfg.input_kind == "ell"
    if ell:     # wide sparse-input model: first layer stored input-major on the device
        layers[0].W = np.ascontiguousarray(layers[0].W.T)

    def to_dev(X):
        if ell:
            return tuple(torch.from_numpy(np.ascontiguousarray(a)).to(dev) for a in X)
        return torch.from_numpy(X).to(dev)

    plain = runtime.Network(layers, first_layer_rows_are_inputs=ell)
    xb = to_dev(X_build)
    dn = plain.dense_forward(xb, layer_outs=True)
    for l in cfg.hashed_layers:
        layers[l].K, layers[l].L = cfg.K, cfg.L
        # lists never need more entries than the largest budget below d_out that will be asked for
        top = max([k for k in cfg.keeps if k < 1.0] + ([cfg.keep_range[1]] if cfg.keep_range else []) + [args.keep])
        layers[l].list_cap = min(layers[l].d_out, int(np.ceil(top * layers[l].d_out)) + 1)
        layers[l].hash_nodes = runtime.hash_nodes_by_variance(dn["layers"][l], cfg.K, cfg.L,
                                                              wl.hash_node_draws(cfg.K, cfg.L, seed=3 + l))
    del plain, dn
    net = runtime.Network(layers, first_layer_rows_are_inputs=ell)
    t0 = time.time()
    net.build_tables(xb)
    net.set_path(args.path)
    net.set_hash_nodes_always_active(args.hash_nodes_always_active)
    log(f"built tables on the device in {time.time() - t0:.2f}s")

    xq = to_dev(X_query)
    nq = (xq[0] if ell else xq).shape[0]
    n_batches = nq // B
    if ell:
        batches = [slonn.make_input(idx=xq[0][i * B:(i + 1) * B], val=xq[1][i * B:(i + 1) * B],
                                    nnz=xq[2][i * B:(i + 1) * B]) for i in range(n_batches)]
    else:
        batches = [slonn.make_input(x=xq[i * B:(i + 1) * B]) for i in range(n_batches)]
    n_last = cfg.dims[-1]
    out_arg = torch.empty(B, dtype=torch.int32, device=dev)
    if layers[-1].K > 0:      # activated output layer: compact (id, value) output, no dense row
        cap = layers[-1].list_cap
        out_idx = torch.empty((B, n_last), dtype=torch.int32, device=dev)
        out_val = torch.empty((B, n_last), dtype=torch.float32, device=dev)
        out_cnt = torch.empty(B, dtype=torch.int32, device=dev)
        out = slonn.make_output(idx=out_idx, val=out_val, cnt=out_cnt, stride=n_last, argmax=out_arg)
    else:
        out_dense = torch.empty((B, n_last), dtype=torch.float32, device=dev)
        out = slonn.make_output(dense=out_dense, argmax=out_arg)
    ws = net.workspace(B)
    stream = torch.cuda.current_stream()

    def run(keep_t, steps, first=0):
        for i in range(steps):
            b = (first + i) % n_batches
            if mixed is not None:      # one keep fraction per query (mixed SLOs in one batch)
                slonn.slonn_sparse_forward(net.model, net.tables, batches[b], B, mixed[b * B:(b + 1) * B],
                                           1, 0, out, None, ws, stream)
            else:
                slonn.slonn_sparse_forward(net.model, net.tables, batches[b], B, keep_t, 0, 0, out, None,
                                           ws, stream)

    mixed = None
    if cfg.keep_range:
        mixed = torch.from_numpy(wl.keep_uniform(nq, cfg.keep_range[0], cfg.keep_range[1], seed=6)).to(dev)

    def timed(keep, steps, warm):
        keep_t = torch.full((1,), keep, dtype=torch.float32, device=dev)
        run(keep_t, warm)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        run(keep_t, steps, warm)
        e1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return e0.elapsed_time(e1) / 1e3, wall

    def mean_budget(keep, n):
        """mean node budget of a layer of n nodes (nearest whole node, at least one)"""
        k = mixed.cpu().numpy().astype(np.float64) if (mixed is not None and keep is None) else \
            np.asarray([np.float32(keep)], np.float64)
        return float(np.clip(np.floor(k * n + 0.5), 1, n).mean())

    def gathered_bytes_per_query(keep, activated_only=True):
        tot = 0.0
        for lay in layers:
            esz = 4 if lay.w_dtype == wl.W_F32 else 2
            if lay.K > 0:
                tot += mean_budget(keep, lay.d_out) * lay.d_in * esz
            elif not activated_only:
                if ell and lay is layers[0]:      # sparse input: one weight row per non-zero
                    tot += cfg.ell_nnz * lay.d_out * esz
                else:
                    tot += lay.d_out * lay.d_in * esz
        return tot

    head_keep = None if mixed is not None else args.keep
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)            # plain copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ---- what a plain device copy reaches on this GPU (256 MiB read + 256 MiB written) ----
    src = torch.empty(1 << 26, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbps = 20 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    log(f"plain device copy: {copy_gbps:,.0f} GB/s (read + write)")

    # ---- headline: K steps at the chosen keep fraction ----
    dev_s, wall_s = timed(args.keep, K, W)
    secs = max(dev_s, wall_s)             # the host loop must keep up: report the slower clock
    qps = K * B / secs
    eff_gbps = qps * gathered_bytes_per_query(head_keep) / 1e9
    log(f"keep {args.keep}: {qps:,.0f} q/s, {secs / K * 1e6:.1f} us/step, effective {eff_gbps:,.0f} GB/s")

    # ---- per-kernel durations over the same steps (HIP events on the launch stream) ----
    keep_t = torch.full((1,), args.keep, dtype=torch.float32, device=dev)
    slonn.slonn_profile_begin(K * (4 * len(layers) + 4))
    run(keep_t, K, W)
    prof = slonn.slonn_profile_end()
    split_us = {k: (v[0] * 1e3 / max(v[1], 1)) for k, v in prof.items() if v[1]}
    per_step_us = {k: v[0] * 1e3 / K for k, v in prof.items() if v[1]}
    # dominant kernel: the one holding most of the step.  Its algorithmic bytes per launch are
    # the weight rows the method must read: budget x row bytes for each activated layer, the whole
    # matrix per query for a layer computed in full, summed over the layers that launch covers.
    bytes_per_step = B * gathered_bytes_per_query(head_keep, activated_only=False)
    dom = "fused" if prof["fused"][1] else "gather"
    g_ms, g_n = prof[dom]
    launches_per_step = g_n / K
    avg_launch_s = g_ms / 1e3 / g_n
    if dom == "fused" and launches_per_step == 1:
        # one kernel per step: the event pair around the K back-to-back launches of the timed
        # region times that kernel without the per-launch cost of the bracketing events
        avg_launch_s = min(avg_launch_s, dev_s / K)
    achieved = (bytes_per_step / launches_per_step) / avg_launch_s / 1e9
    roofline = {"bound": "hbm", "kernel": ("fused_wide_kernel" if ell else "fused_forward_kernel") if dom == "fused" else "gather_forward_kernel",
                "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": None, "avg_launch_us": round(avg_launch_s * 1e6, 2),
                "algorithmic_bytes_per_launch": int(bytes_per_step / launches_per_step),
                "note": "algorithmic bytes = the weight rows the method must evaluate (budget x row bytes per "
                        "activated layer, whole matrix per query for layers computed in full); a fraction above 1 "
                        "means rows were served to several queries from L2 (traffic = bytes that reached HBM)"}
    if dom == "gather" and prof["tiles"][1] and prof["tiles"][0] > prof["gather"][0]:
        # large batches: most of the step is the masked tiles on the bf16 matrix cores, a dense
        # contraction.  Flops per launch = every (query, node) pair of the layer, 2 d flops each,
        # times the bf16 products per fp32 product (6 with fp32 weights in three parts, 3 with bf16
        # weights); the selected pairs are the part of them that is written.
        t_ms, t_n = prof["tiles"]
        tile_flops = sum(2.0 * B * lay.d_in * lay.d_out * (3 if lay.w_dtype == wl.W_BF16 else 6)
                         for lay in layers if lay.K > 0)
        per_launch = tile_flops / max(1, sum(1 for lay in layers if lay.K > 0))
        avg_s = t_ms / 1e3 / t_n
        peak = 2500.0
        roofline = {"bound": "mfma", "kernel": "masked_tiles_kernel", "achieved": round(per_launch / avg_s / 1e12, 1),
                    "peak": peak, "unit": "TFLOP/s", "frac": round(per_launch / avg_s / 1e12 / peak, 4),
                    "traffic": None, "avg_launch_us": round(avg_s * 1e6, 2),
                    "flops_per_launch": int(per_launch),
                    "note": "bf16 MFMA flops issued per launch (all pairs of a 128-query tile, fp32 operands as "
                            "three bf16 parts) over the mean launch duration of the masked tiles; the gathered-bytes "
                            "figure of the whole step is effective_GBps"}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            roofline["traffic"] = json.load(open(tpath)).get(f"{args.config}_keep{args.keep}_B{B}")
        except Exception:
            pass

    extra = {"effective_GBps": round(eff_gbps, 1), "frac_of_hbm_peak": round(eff_gbps / HBM_PEAK_GBPS, 4),
             "measured_copy_GBps": round(copy_gbps, 1), "frac_of_measured_copy": round(eff_gbps / copy_gbps, 4),
             "per_step_us_with_event_overhead": {k: round(v, 2) for k, v in per_step_us.items()},
             "avg_launch_us_with_event_overhead": {k: round(v, 2) for k, v in split_us.items()}}

    # ---- the other keep fractions and the dense baseline, briefly ----
    if not args.no_sweep:
        sweep = {}
        for keep in (cfg.keeps if mixed is None else ()):
            d_s, w_s = timed(keep, 120, 20)
            s = max(d_s, w_s)
            q = 120 * B / s
            sweep[str(keep)] = {"qps": round(q), "effective_GBps": round(q * gathered_bytes_per_query(keep) / 1e9, 1)}
        extra["sweep"] = sweep
        yd = torch.empty((B, n_last), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        for i in range(20):
            slonn.slonn_dense_forward(net.model, batches[i % n_batches], B, yd, out_arg, None, ws, stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(120):
            slonn.slonn_dense_forward(net.model, batches[i % n_batches], B, yd, out_arg, None, ws, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        dsec = e0.elapsed_time(e1) / 1e3
        extra["dense_baseline_qps"] = round(120 * B / dsec)
        dflops = 2.0 * sum(lay.d_in * lay.d_out for lay in layers if not (ell and lay is layers[0]))
        extra["dense_baseline_tflops"] = round(dflops * 120 * B / dsec / 1e12, 2)
        extra["dense_baseline_frac_of_fp32_mfma_peak"] = round(dflops * 120 * B / dsec / 157.3e12, 4)

    # ---- small batches are launch-bound: the same step recorded once and replayed as a HIP graph ----
    if B <= 64 and mixed is None:
        keep_g = torch.full((1,), args.keep, dtype=torch.float32, device=dev)
        graph = slonn.slonn_forward_graph_create(net.model, net.tables, batches[0], B, keep_g, 0, 0, out, ws)
        for _ in range(20):
            graph.launch(stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(200):
            graph.launch(stream)
        e1.record(stream)
        torch.cuda.synchronize()
        g_s = max(e0.elapsed_time(e1) / 1e3, time.perf_counter() - t0)
        # latency of one step seen from the host: launch, then wait for the result
        lat = {}
        for name, fn in (("eager", lambda: run(keep_g, 1)), ("graph", lambda: graph.launch(stream))):
            ts = []
            for _ in range(60):
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                fn()
                torch.cuda.synchronize()
                ts.append(time.perf_counter() - t1)
            lat[name] = round(float(np.median(ts[10:])) * 1e6, 2)
        extra["recorded_step"] = {"us_per_step_back_to_back": round(g_s / 200 * 1e6, 2),
                                  "qps_back_to_back": round(200 * B / g_s),
                                  "host_latency_us_median": lat,
                                  "note": "same batch replayed (weights, tables and access pattern as in the timed region)"}
        log(f"recorded step: {extra['recorded_step']}")
        graph.close()

    # ---- k chosen per query inside the pass (ACLO): Confidence LSH tables trained on the build
    #      set with c(k, x) = -cross-entropy(full prediction, prediction at k) (Eq. 3) ----
    if args.aclo and mixed is None and not ell and cfg.hashed_layers[0] == 0:
        grid = sorted(set(float(k) for k in cfg.keeps))
        nb_ = min(xb.shape[0], 8192)
        xb_ = xb[:nb_]
        pf = torch.softmax(net.dense_forward(xb_)["out"].double(), dim=1)
        conf = torch.empty((nb_, len(grid)), dtype=torch.float32, device=dev)
        for gi, k in enumerate(grid):
            yk = net.sparse_forward(xb_, k)["out"].double()
            conf[:, gi] = (pf * torch.log_softmax(yk, dim=1)).sum(dim=1).float()
        codes = net.select(0, xb_, 1.0)["codes"]
        pol = slonn.slonn_policy_create(cfg.K, cfg.L, grid)
        slonn.slonn_policy_train_confidence(pol, codes, conf, nb_)
        # one threshold per query, drawn from the training confidences at the middle k, so that
        # a batch mixes queries that are satisfied early with queries that need more nodes
        pick = torch.from_numpy(np.random.default_rng(8).integers(0, nb_, nq)).to(dev)
        thr_all = conf[:, len(grid) // 2][pick].contiguous()
        keep_out = torch.zeros(B, dtype=torch.float32, device=dev)

        def run_aclo(steps, first=0):
            for i in range(steps):
                b = (first + i) % n_batches
                slonn.slonn_sparse_forward_aclo(net.model, net.tables, pol, batches[b], B,
                                                thr_all[b * B:(b + 1) * B], 1, keep_out, out, None, ws, stream)
        run_aclo(20)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        run_aclo(120, 20)
        e1.record(stream)
        torch.cuda.synchronize()
        a_s = max(e0.elapsed_time(e1) / 1e3, time.perf_counter() - t0)
        chosen = []
        for b in range(min(n_batches, 16)):
            run_aclo(1, b)
            chosen.append(keep_out.cpu().numpy().copy())
        chosen = np.concatenate(chosen)
        extra["aclo"] = {"qps": round(120 * B / a_s), "us_per_step": round(a_s / 120 * 1e6, 2),
                         "k_grid": grid,
                         "share_of_queries_per_k": [round(float((chosen == np.float32(k)).mean()), 4) for k in grid],
                         "mean_keep": round(float(chosen.mean()), 4),
                         "confidence": "-cross-entropy(softmax(full), softmax(at k)) on the first "
                                       f"{nb_} build inputs; per-query thresholds drawn from those at k = {grid[len(grid) // 2]}"}
        log(f"ACLO: {extra['aclo']}")

    # ---- CPU baseline: the oracle as it stands, on the host cores, bounded sample ----
    cpu = None
    blob_bytes = slonn.slonn_tables_export_bytes(net.tables)
    if not args.no_cpu_baseline and blob_bytes > (4 << 30):
        log(f"CPU baseline skipped: the tables are {blob_bytes / 2**30:.1f} GiB; rerun with --build-inputs 4096")
    elif not args.no_cpu_baseline:
        from oracle import slonn_oracle
        onet = slonn_oracle.OracleNet(layers, first_layer_rows_are_inputs=ell,
                                      hash_nodes_always_active=args.hash_nodes_always_active)
        onet.import_tables(net.export_tables())
        n_s = min(nq, 4096)
        Xs = tuple(a[:n_s] for a in X_query) if ell else X_query[:n_s]
        ks = args.keep if mixed is None else mixed[:n_s].cpu().numpy()
        # passes over the sample until about ten seconds of CPU work have been timed
        done, dt = 0, 0.0
        while dt < 10.0 and done < 400 * n_s:
            t0 = time.perf_counter()
            onet.sparse_forward(Xs, ks, taps=False)
            dt += time.perf_counter() - t0
            done += n_s
        # the same oracle on one thread, briefly (about three seconds)
        one = slonn_oracle.OracleNet(layers, threads=1, first_layer_rows_are_inputs=ell,
                                     hash_nodes_always_active=args.hash_nodes_always_active)
        one.tables = onet.tables
        n_1 = min(n_s, 256)
        X1 = tuple(a[:n_1] for a in Xs) if ell else Xs[:n_1]
        k1 = ks if np.ndim(ks) == 0 else ks[:n_1]
        done1, dt1 = 0, 0.0
        while dt1 < 3.0 and done1 < 400 * n_1:
            t0 = time.perf_counter()
            one.sparse_forward(X1, k1, taps=False)
            dt1 += time.perf_counter() - t0
            done1 += n_1
        extra["cpu_baseline_one_thread_qps"] = round(done1 / dt1, 1)
        cpu = {"value": round(done / dt, 1), "unit": "queries/s", "cores": onet.threads, "kind": "oracle",
               "sample": f"first {n_s} queries of the same query set, {done // n_s} passes ({dt:.1f} s of CPU work), "
                         f"keep {args.keep if mixed is None else 'per query'}, all layers, "
                         f"{onet.threads} threads over queries"}

    line = {
        "metric": "queries/sec and effective HBM GB/s (vs peak) for sparse forward at keep-fraction",
        "value": round(qps, 1), "unit": "queries/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(secs / K * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if cfg.w_dtype == wl.W_F32 else "bf16 weights, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{args.config}: MLP {'-'.join(map(str, cfg.dims))}, K={cfg.K} L={cfg.L} on "
                               f"{len(cfg.hashed_layers)} hidden layers, {nq} queries", "batch": B,
                   "keep": args.keep if mixed is None else f"per query U[{cfg.keep_range[0]}, {cfg.keep_range[1]}]",
                   "queries_per_step": B, "path": args.path,
                   "hash_nodes_always_active": bool(args.hash_nodes_always_active)},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    line.update(extra)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
