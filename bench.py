#!/usr/bin/env python3
"""Benchmark of the SLO-NN hot path on one MI355X.

A step is one pass of the whole path (FreeHash projection, key + bucket lookup + merge,
gathered-row forward, for every layer) over the WHOLE synthetic query set of the workload,
processed in batches of B (the last batch is the ragged remainder); inputs, weights and tables
sit in HBM before the timed region starts.  Headline workload: the largest configuration, the
deep 1024-8192x6-1000 MLP with bf16 weights, K=12 L=64 on six hidden layers, 20 000 queries
with one keep fraction per query drawn from U[0.02, 0.3], batch 2048.  Beside it, briefly and
in the same JSON line: the 3072-4096^3-100 fp32 MLP at batch 1024 and the 784-1024^2-10 fp32
MLP at batch 256 over their keep-fraction sweeps, each with the full network (all nodes) as
the baseline every speed-up is quoted against.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
F16_PEAK_TFLOPS = 2500.0        # dense fp16 (and bf16) MFMA
FP32_MFMA_PEAK_TFLOPS = 157.3
KERNEL_OF_KIND = {"fused": "fused_", "tiles": "masked_tiles_kernel", "gather": "gather_blocked_kernel",
                  "select": "select_block_kernel", "hash": "hash projection kernels", "dense": "dense_layer_kernel",
                  "ell": "ell_layer_kernel", "finalize": "finalize_kernel"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# The side streams of the lanes, shared by every workload of the process: a process has four hardware
# queues, and streams beyond that share them (a workload with fresh streams of its own may find two
# of its lanes on one queue).
_LANE_STREAMS = []


def lane_stream(torch, dev, i):
    while len(_LANE_STREAMS) < i:
        _LANE_STREAMS.append(torch.cuda.Stream(device=dev))
    return _LANE_STREAMS[i - 1]


class Workload:
    """One configuration set up on the device: weights, hash nodes, tables, the query set cut
    into batches, output buffers and the workspace."""

    def __init__(self, name, B, args, n_queries=0, n_build=0, top_keep=None):
        import numpy as np
        import torch
        from paper_2204_08400_amd import runtime, slonn, workloads as wl
        self.np, self.torch, self.slonn, self.wl, self.runtime = np, torch, slonn, wl, runtime
        self.name, self.args = name, args
        cfg = self.cfg = wl.CONFIGS[name]
        self.B = B or cfg.batches[-1]
        dev = self.dev = torch.device("cuda:0")
        t0 = time.time()
        layers = self.layers = wl.make_mlp(cfg.dims, seed=0, w_dtype=cfg.w_dtype, last_act=cfg.last_act)
        self.n_build = n_build or cfg.n_inputs
        self.nq = n_queries or cfg.n_inputs
        if args.input_clusters > 0 and cfg.input_kind != "ell":
            # not a benchmark configuration: inputs with class structure, for --cluster-by-key
            X_build = wl.inputs_clustered(self.n_build, cfg.dims[0], 1, args.input_clusters)
            self.X_query = wl.inputs_clustered(self.nq, cfg.dims[0], 2, args.input_clusters)
        else:
            X_build = wl.make_inputs(cfg, self.n_build, seed=1)
            self.X_query = wl.make_inputs(cfg, self.nq, seed=2)
        log(f"{name}: generated weights, {self.n_build} table-training inputs and {self.nq} queries in {time.time() - t0:.1f}s")
        ell = self.ell = cfg.input_kind == "ell"
        if ell:     # wide sparse-input model: first layer stored input-major on the device
            layers[0].W = np.ascontiguousarray(layers[0].W.T)
        # hash nodes: variance of the full network's activations on the build set (device dense pass)
        plain = runtime.Network(layers, first_layer_rows_are_inputs=ell)
        self.xb = self.to_dev(X_build)
        dn = plain.dense_forward(self.xb, layer_outs=True)
        keeps = [k for k in cfg.keeps if k < 1.0] + ([cfg.keep_range[1]] if cfg.keep_range else [])
        top = max(keeps + ([top_keep] if top_keep else []))
        for l in cfg.hashed_layers:
            layers[l].K, layers[l].L = cfg.K, cfg.L
            # lists never need more entries than the largest budget below d_out that will be asked for
            layers[l].list_cap = min(layers[l].d_out, int(np.ceil(top * layers[l].d_out)) + 1)
            layers[l].hash_nodes = runtime.hash_nodes_by_variance(dn["layers"][l], cfg.K, cfg.L,
                                                                  wl.hash_node_draws(cfg.K, cfg.L, seed=3 + l))
        del plain, dn
        self.net = runtime.Network(layers, first_layer_rows_are_inputs=ell)
        t0 = time.time()
        self.net.build_tables(self.xb)
        self.net.set_path(args.path)
        self.net.set_hash_nodes_always_active(args.hash_nodes_always_active)
        torch.cuda.synchronize()
        log(f"{name}: tables built on the device in {time.time() - t0:.2f}s")

        self.xq = self.to_dev(self.X_query)
        self.nq_all = self.nq
        # Lanes: consecutive batches of a step go to HIP streams in turn (default priority), each with
        # its own workspace and output buffers, so that the launch- and latency-bound kernels of one
        # batch (hash, select) run beside the matrix-core kernels of another.  Lane 0 is the current
        # stream.  Two lanes for large batches, four for batches of up to 256 queries, whose kernels are
        # chains of dependent memory round trips; the library is told how many batches are in flight.
        self.stream = torch.cuda.current_stream()
        self.graphs, self.keep_tensors = {}, {}
        self.all_lanes = []
        self.lanes = []
        self.set_batch(self.B, self.nq)
        self.out, self.ws, self.out_arg = self.lanes[0]["out"], self.lanes[0]["ws"], self.lanes[0]["arg"]
        self.mixed = None
        if cfg.keep_range:        # one keep fraction per query (mixed SLOs in one batch)
            self.mixed_host = wl.keep_uniform(self.nq, cfg.keep_range[0], cfg.keep_range[1], seed=6)
            self.mixed = torch.from_numpy(self.mixed_host).to(dev)

    def _lane(self, i):
        torch, slonn, dev, B = self.torch, self.slonn, self.dev, self.B
        n_last = self.cfg.dims[-1]
        lane = {"stream": self.stream if i == 0 else lane_stream(torch, dev, i),
                "ws": torch.empty(slonn.slonn_workspace_bytes(self.net.model, B), dtype=torch.uint8, device=dev),
                "arg": torch.empty(B, dtype=torch.int32, device=dev),
                "yd": torch.empty((B, n_last), dtype=torch.float32, device=dev)}
        if self.layers[-1].K > 0:      # activated output layer: compact (id, value) output, no dense row
            lane["o"] = (torch.empty((B, n_last), dtype=torch.int32, device=dev),
                         torch.empty((B, n_last), dtype=torch.float32, device=dev),
                         torch.empty(B, dtype=torch.int32, device=dev))
            lane["out"] = slonn.make_output(idx=lane["o"][0], val=lane["o"][1], cnt=lane["o"][2], stride=n_last,
                                            argmax=lane["arg"])
        else:
            lane["o"] = torch.empty((B, n_last), dtype=torch.float32, device=dev)
            lane["out"] = slonn.make_output(dense=lane["o"], argmax=lane["arg"])
        return lane

    def set_batch(self, B, nq=0):
        """the query set (its first nq queries) cut into batches of B, ragged tail included; buffers and
        workspace are sized for the batch the workload was created with, so B may only shrink"""
        slonn, xq = self.slonn, self.xq
        assert B <= self.B
        self.batch = B
        # (a model of under a million weights is a 13 us launch: more streams only add host work)
        small_model = sum(l.d_in * l.d_out for l in self.layers) < (1 << 20)
        self.n_streams = self.args.streams if self.args.streams > 0 else (4 if B <= 256 and not small_model else 2)
        while len(self.all_lanes) < self.n_streams:
            self.all_lanes.append(self._lane(len(self.all_lanes)))
        self.lanes = self.all_lanes[:self.n_streams]
        slonn.slonn_model_set_batches_in_flight(self.net.model, self.n_streams)
        self.nq = min(nq or self.nq_all, self.nq_all)
        self.sizes = [min(B, self.nq - s) for s in range(0, self.nq, B)]
        self.batches = []
        for i, nb in enumerate(self.sizes):
            s = i * B
            if self.ell:
                self.batches.append(slonn.make_input(idx=xq[0][s:s + nb], val=xq[1][s:s + nb], nnz=xq[2][s:s + nb]))
            else:
                self.batches.append(slonn.make_input(x=xq[s:s + nb]))

    def to_dev(self, X):
        torch, np = self.torch, self.np
        if self.ell:
            return tuple(torch.from_numpy(np.ascontiguousarray(a)).to(self.dev) for a in X)
        return torch.from_numpy(X).to(self.dev)

    # ---- one step = the whole query set ----
    def _fork(self, lanes):
        for ln in lanes[1:]:
            ln["stream"].wait_stream(self.stream)

    def _join(self, lanes):
        for ln in lanes[1:]:
            self.stream.wait_stream(ln["stream"])

    def step(self, keep_t, one_lane=False, uniform=False):
        s, B = self.slonn, self.batch
        lanes = self.lanes[:1] if one_lane else self.lanes
        self._fork(lanes)
        # (measured: replaying wins where the host's launches bind -- one or two queries a batch with four
        # batches in flight, C3 batch 1: 25.7 -> 37.9 k queries/s -- and loses about 5 % on one stream)
        recorded = not one_lane and ((self.args.graphs and B <= 32) or (B <= 2 and len(lanes) >= 4))
        for i, nb in enumerate(self.sizes):
            ln = lanes[i % len(lanes)]
            if recorded:
                # small batches are bound by the host's launches (11 per query on C3): each batch's pass is
                # recorded once (its input, keep fractions, outputs and workspace are fixed device buffers)
                # and replayed with one call
                mixed = self.mixed is not None and not uniform
                key = (B, i, len(lanes), "mixed" if mixed else keep_t.data_ptr())
                g = self.graphs.get(key)
                if g is None:
                    # (create runs a pass on a stream of its own: nothing else may be using this lane's
                    # workspace and outputs meanwhile)
                    self.torch.cuda.synchronize()
                    kp = self.mixed[i * B:i * B + nb] if mixed else keep_t
                    g = self.graphs[key] = s.slonn_forward_graph_create(
                        self.net.model, self.net.tables, self.batches[i], nb, kp, 1 if mixed else 0, 0, ln["out"], ln["ws"])
                g.launch(ln["stream"])
                continue
            if self.mixed is not None and not uniform:
                s.slonn_sparse_forward(self.net.model, self.net.tables, self.batches[i], nb,
                                       self.mixed[i * B:i * B + nb], 1, 0, ln["out"], None, ln["ws"], ln["stream"])
            else:
                s.slonn_sparse_forward(self.net.model, self.net.tables, self.batches[i], nb, keep_t, 0, 0,
                                       ln["out"], None, ln["ws"], ln["stream"])
        self._join(lanes)

    def dense_step(self):
        self._fork(self.lanes)
        for i, nb in enumerate(self.sizes):
            ln = self.lanes[i % len(self.lanes)]
            self.slonn.slonn_dense_forward(self.net.model, self.batches[i], nb, ln["yd"], ln["arg"], None,
                                           ln["ws"], ln["stream"])
        self._join(self.lanes)

    def marker(self):
        """a kernel nothing else here launches, so that a profiler's dispatch list shows where the
        timed region starts and ends (--markers)"""
        a = self.torch.ones(64, dtype=self.torch.float32, device=self.dev)
        self.torch.nextafter(a, a)

    def timed(self, fn, steps, warm, mark=False):
        """K steps between two synchronisations; returns (seconds, per-step milliseconds).  The
        slower of the device clock (events on the launch stream) and the host clock counts."""
        torch = self.torch
        for _ in range(warm):
            fn()
        if mark:
            self.marker()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        ev[0].record(self.stream)
        for i in range(steps):
            fn()
            ev[i + 1].record(self.stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        if mark:
            self.marker()
        per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
        return max(ev[0].elapsed_time(ev[steps]) / 1e3, wall), per

    def keep_tensor(self, keep):
        k = float(keep if keep is not None else 1.0)
        if k not in self.keep_tensors:       # (one tensor per value: recorded passes bake its address in)
            self.keep_tensors[k] = self.torch.full((1,), k, dtype=self.torch.float32, device=self.dev)
        return self.keep_tensors[k]

    def time_sparse(self, keep, steps, warm, mark=False, uniform=False):
        kt = self.keep_tensor(keep)
        return self.timed(lambda: self.step(kt, uniform=uniform), steps, warm, mark)

    def steps_for(self, fn, steps, warm, min_seconds=0.1):
        """(steps, warm-up steps) for a side measurement: at least the given ones, and enough of both for
        a timed region of about min_seconds behind a warm-up of half that -- a step of a small workload
        is a millisecond, and a GPU coming out of idle runs its first milliseconds at a low clock"""
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        t = max(time.perf_counter() - t0, 1e-5)
        return (min(500, max(steps, int(min_seconds / t) + 1)), min(250, max(warm, int(0.5 * min_seconds / t) + 1)))

    def latency_us(self, keep, uniform=False):
        """Mean time per batch with one batch in flight: the query set pass after pass on one stream
        (eager launches, a batch's kernels start when the batch before has finished), in microseconds."""
        kt = self.keep_tensor(keep)
        self.slonn.slonn_model_set_batches_in_flight(self.net.model, 1)
        fn = lambda: self.step(kt, one_lane=True, uniform=uniform)
        steps, warm = self.steps_for(fn, 3, 1, min_seconds=0.05)
        secs, _ = self.timed(fn, steps, warm)
        self.slonn.slonn_model_set_batches_in_flight(self.net.model, self.n_streams)
        return round(secs / steps / len(self.sizes) * 1e6, 1)

    def profile_sparse(self, keep, steps):
        """Per-kernel-kind durations over `steps` more steps: every launch bracketed by two HIP events
        on the launch stream inside the library."""
        kt = self.keep_tensor(keep)
        per_step = len(self.sizes) * (12 * len(self.layers) + 8)
        self.slonn.slonn_profile_begin(steps * per_step)
        for _ in range(steps):
            self.step(kt, one_lane=True)       # one stream: a kernel's duration without a neighbour on the chip
        return self.slonn.slonn_profile_end()

    # ---- the method's own work ----
    def budgets(self, keep, n):
        """node budgets of the queries in a layer of n nodes (nearest whole node, at least one)"""
        np = self.np
        k = self.mixed_host[:self.nq].astype(np.float64) if keep is None else np.full(self.nq, np.float32(keep), np.float64)
        return np.clip(np.floor(k * n + 0.5), 1, n)

    def gathered_bytes_per_step(self, keep, activated_only=True):
        """weight bytes the method must evaluate for the whole query set: budget x row bytes for every
        activated layer (+ the whole matrix per query for layers computed in full, on request)"""
        tot = 0.0
        for lay in self.layers:
            esz = 4 if lay.w_dtype == self.wl.W_F32 else 2
            if lay.K > 0:
                tot += float(self.budgets(keep, lay.d_out).sum()) * lay.d_in * esz
            elif not activated_only:
                rows = self.cfg.ell_nnz if (self.ell and lay is self.layers[0]) else lay.d_out
                cols = lay.d_out if (self.ell and lay is self.layers[0]) else lay.d_in
                tot += float(self.nq) * rows * cols * esz
        return tot

    def dense_flops_per_query(self):
        return 2.0 * sum(l.d_in * l.d_out for l in self.layers if not (self.ell and l is self.layers[0]))


def load_traffic(key):
    """HBM bytes per launch and per step from the committed rocprofv3 counter summaries
    (profiles/hbm_traffic.json; FETCH_SIZE / WRITE_SIZE scaled by a plain copy of known size)."""
    p = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        return json.load(open(p)).get(key)
    except Exception:
        return None


def roofline_of(w, keep, prof, steps, secs_per_step, traffic_key):
    """The dominant kernel of the step against the resource that bounds it."""
    np = w.np
    per_step_us = {k: v[0] * 1e3 / steps for k, v in prof.items() if v[1]}
    dom = max(per_step_us, key=per_step_us.get)
    ms, n = prof[dom]
    avg_s = ms / 1e3 / n
    launches_per_step = n / steps
    gathered = w.gathered_bytes_per_step(keep)
    tr = load_traffic(traffic_key) or {}
    cand = {k: v for k, v in (tr.get("kernels") or {}).items() if k.startswith(KERNEL_OF_KIND[dom])}
    tk = cand[max(cand, key=lambda k: cand[k]["launches_per_step"])] if cand else None
    traffic = int(tk["fetch_bytes_per_launch"] + tk["write_bytes_per_launch"]) if tk else None
    hbm_step = tr.get("hbm_bytes_per_step")
    nominal = gathered / secs_per_step / 1e9
    common = {"kernel": KERNEL_OF_KIND[dom], "avg_launch_us": round(avg_s * 1e6, 2),
              "launches_per_step": round(launches_per_step, 2), "share_of_step": round(per_step_us[dom] / sum(per_step_us.values()), 3),
              "traffic": traffic,
              "gathered_bytes_per_step": int(gathered),
              "nominal_gathered_GBps": round(nominal, 1),
              "nominal_gathered_over_hbm_peak": round(nominal / HBM_PEAK_GBPS, 4),
              "hbm_bytes_per_step_from_counters": hbm_step,
              "hbm_GBps_from_counters": round(hbm_step / secs_per_step / 1e9, 1) if hbm_step else None,
              "hbm_frac_from_counters": round(hbm_step / secs_per_step / 1e9 / HBM_PEAK_GBPS, 4) if hbm_step else None,
              "traffic_source": (f"profiles/hbm_traffic.json[{traffic_key}] (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE at this "
                                 "workload, scaled by a plain copy; not measured in this run)") if tr else None}
    if dom == "tiles":
        # masked tiles on the fp16 matrix cores: one launch per activated layer and batch.  The method's
        # own flops are 2 d per selected (query, node) pair; the kernel issues every pair of its tiles,
        # and 2 (bf16 weights) or 3 (fp32 weights in two parts) fp16 products per fp32-class product.
        act = [l for l in w.layers if l.K > 0]
        own = sum(2.0 * float(w.budgets(keep, l.d_out).sum()) * l.d_in for l in act)
        issued = sum(2.0 * w.nq * l.d_in * l.d_out * (2 if l.w_dtype == w.wl.W_BF16 else 3) for l in act)
        own_l, issued_l = own / (n / steps), issued / (n / steps)
        r = {"bound": "mfma", "achieved": round(own_l / avg_s / 1e12, 2), "peak": F16_PEAK_TFLOPS, "unit": "TFLOP/s",
             "frac": round(own_l / avg_s / 1e12 / F16_PEAK_TFLOPS, 4),
             "method_flops_per_launch": int(own_l), "issued_flops_per_launch": int(issued_l),
             "issued_TFLOPs": round(issued_l / avg_s / 1e12, 1),
             "issued_frac": round(issued_l / avg_s / 1e12 / F16_PEAK_TFLOPS, 4),
             "mfma_rate_from_registers_TFLOPs": None, "issued_frac_of_mfma_rate_from_registers": None,
             "note": "achieved = the method's own flops (2 d per selected pair) per launch over the mean launch duration; "
                     "issued = what the tile kernel executes for them: every (query, node) pair of a served 128-query tile, "
                     "each fp32-class product as 2 (bf16 weights) or 3 (fp32 weights) fp16 MFMA products.  "
                     "nominal_gathered_GBps is the north-star figure (budget x row bytes over the step time); it exceeds the "
                     "HBM peak because a weight tile is fetched once per 128 queries, so it is not a roofline fraction.  "
                     "mfma_rate_from_registers = a register-only loop of the same MFMAs on this device in this run "
                     "(slonn_probe_mfma_rate): what the matrix cores deliver at the clock they hold under load"}
        try:      # the yardstick beside the published peak, measured now
            scratch = w.torch.empty(1 << 22, dtype=w.torch.uint8, device=w.dev)
            rate = w.slonn.slonn_probe_mfma_rate(scratch, w.stream)
            r["mfma_rate_from_registers_TFLOPs"] = round(rate, 1)
            r["issued_frac_of_mfma_rate_from_registers"] = round(issued_l / avg_s / 1e12 / rate, 4)
        except Exception as e:      # (a library without the probe)
            log(f"no MFMA rate probe: {e}")
    else:
        # gather-type kernels: bytes of the rows this kernel kind evaluates per launch
        per_launch = w.gathered_bytes_per_step(keep, activated_only=(dom != "fused")) / launches_per_step
        if dom in ("select", "hash", "dense", "finalize", "ell"):
            per_launch = None
        ach = per_launch / avg_s / 1e9 if per_launch else None
        r = {"bound": "hbm", "achieved": round(ach, 1) if ach else None, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
             "frac": round(ach / HBM_PEAK_GBPS, 4) if ach else None,
             "algorithmic_bytes_per_launch": int(per_launch) if per_launch else None,
             "note": "achieved = the weight rows the method evaluates per launch (budget x row bytes; whole matrix for layers "
                     "computed in full) over the mean launch duration.  Where the weights fit the 4 MiB L2 slices / 256 MiB "
                     "Infinity Cache the rows are served from cache to many queries and the figure is not bounded by the HBM "
                     "peak: hbm_*_from_counters is what reached HBM"}
    r.update(common)
    return r, per_step_us


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--keep", type=float, default=0.25, help="keep fraction of the headline (configurations with one keep per query ignore it)")
    ap.add_argument("--config", default="C5")
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--queries", type=int, default=0, help="size of the query set (default: the configuration's)")
    ap.add_argument("--build-inputs", type=int, default=0, help="size of the table-training set (default: the configuration's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="headline only: no keep sweep, no dense baseline, no other workloads")
    ap.add_argument("--no-others", action="store_true", help="skip the other workloads reported beside the headline")
    ap.add_argument("--path", default="auto", choices=["auto", "layers", "fused"])
    ap.add_argument("--hash-nodes-always-active", action="store_true",
                    help="Section 3.4 variant: hash nodes always computed, never selected (default off)")
    ap.add_argument("--aclo", action="store_true",
                    help="also time the pass with k chosen per query inside it (ACLO, Confidence LSH tables)")
    ap.add_argument("--cluster-by-key", action="store_true",
                    help="Section 6 (future work): also order each batch by its first-layer LSH keys before the pass; "
                         "reports the union of 16 / 128 queries' active rows over one list, and the rate, both ways")
    ap.add_argument("--input-clusters", type=int, default=0,
                    help="inputs with class structure instead of the configuration's (study of --cluster-by-key only)")
    ap.add_argument("--streams", type=int, default=0,
                    help="HIP streams the batches of a step are dealt to in turn (each with its own workspace); "
                         "0: two for batches above 256 queries and for tiny models, else four")
    ap.add_argument("--graphs", action="store_true",
                    help="batches of up to 32 queries: record each batch's pass once (HIP graph) and replay it "
                         "(always done for batches of one or two queries dealt to four streams)")
    ap.add_argument("--full-network", choices=["fp32", "f16"], default=None,
                    help="time only the full-network pass (the baseline) in the given arithmetic, for profilers")
    ap.add_argument("--markers", action="store_true",
                    help="launch a marker kernel (nextafter) right before and after the timed steps, for profilers")
    ap.add_argument("--no-profile", action="store_true", help="skip the event-instrumented pass (profiler runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy, for scaling rocprofv3 byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the path is data-parallel over queries with nothing "
                 "exchanged between GPUs, and this build has no multi-GPU leg (run with --gpus 1)")

    import numpy as np
    import torch
    from paper_2204_08400_amd import slonn, workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    slonn.load()
    dev = torch.device("cuda:0")
    K, W = args.steps, args.warmup

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
    # ---- what the compute units draw from L2 (the bound of the gathers on cache-resident weights) ----
    l2_all = l2_one = None
    if hasattr(slonn, "slonn_probe_l_two_read_rate"):
        scratch = torch.zeros(4 << 20, dtype=torch.uint8, device=dev)
        l2_all, l2_one = slonn.slonn_probe_l_two_read_rate(scratch, torch.cuda.current_stream())
        del scratch
        log(f"16-byte loads of an L2-resident window: {l2_all:,.0f} GB/s with every compute unit busy, {l2_one:,.0f} GB/s for one unit alone")

    # ---- headline ----
    w = Workload(args.config, args.batch, args, n_queries=args.queries, n_build=args.build_inputs, top_keep=args.keep)
    cfg, B = w.cfg, w.B
    head_keep = None if w.mixed is not None else args.keep
    if args.full_network:
        # profiler runs of the baseline alone: the full-network pass between the markers, nothing else
        slonn.slonn_model_set_dense_arithmetic(w.net.model, 1 if args.full_network == "f16" else 0)
        secs, per = w.timed(w.dense_step, K, W, mark=args.markers)
        print(json.dumps({"metric": "queries/s of the full-network pass (all nodes: the baseline, not the method)",
                          "value": round(K * w.nq / secs, 1), "unit": "queries/s", "n_gpus": 1, "steps": K, "warmup": W,
                          "ms_per_step": round(secs / K * 1e3, 5), "higher_is_better": True,
                          "TFLOPs": round(w.dense_flops_per_query() * K * w.nq / secs / 1e12, 2),
                          "config": {"workload": args.config, "batch": B, "arithmetic": args.full_network,
                                     "queries_per_step": w.nq, "streams": w.n_streams}}), flush=True)
        return
    secs, per = w.time_sparse(head_keep, K, W, mark=args.markers)
    qps = K * w.nq / secs
    gathered = w.gathered_bytes_per_step(head_keep)
    eff_gbps = gathered * K / secs / 1e9
    log(f"{args.config} batch {B}: {qps:,.0f} q/s, {secs / K * 1e3:.3f} ms/step ({len(w.sizes)} batches), "
        f"nominal {eff_gbps:,.0f} GB/s on gathered bytes")
    keep_label = head_keep if head_keep is not None else f"per query U[{cfg.keep_range[0]}, {cfg.keep_range[1]}]"
    head_config = {"workload": f"{args.config}: MLP {'-'.join(map(str, cfg.dims))}, K={cfg.K} L={cfg.L} on "
                               f"{len(cfg.hashed_layers)} layers", "batch": B, "keep": keep_label,
                   "queries_per_step": w.nq, "batches_per_step": len(w.sizes), "table_training_inputs": w.n_build,
                   "streams": w.n_streams,
                   "path": args.path, "hash_nodes_always_active": bool(args.hash_nodes_always_active)}
    traffic_key = f"{args.config}_B{B}_keep{head_keep if head_keep is not None else 'mixed'}"
    extra = {"ms_per_step_median": round(float(np.median(per)), 4),
             "nominal_gathered_GBps": round(eff_gbps, 1),
             "measured_copy_GBps": round(copy_gbps, 1),
             "measured_l2_read_GBps_all_units": round(l2_all, 1) if l2_all else None,
             "measured_l2_read_GBps_one_unit": round(l2_one, 1) if l2_one else None}
    roofline = None
    if not args.no_profile:
        prof = w.profile_sparse(head_keep, K)
        roofline, per_step_us = roofline_of(w, head_keep, prof, K, secs / K, traffic_key)
        if roofline.get("bound") == "hbm" and roofline.get("achieved") and l2_all:
            # every gathered byte passes from L2 (or beyond) into a compute unit: the measured rate of
            # that path bounds the kernel also where HBM does not
            roofline["measured_l2_read_GBps_all_units"] = round(l2_all, 1)
            roofline["frac_of_measured_l2_read_rate"] = round(roofline["achieved"] / l2_all, 4)
            if roofline["frac"] and roofline["frac"] > 1.0 and roofline.get("hbm_GBps_from_counters"):
                # cache-resident weights: the gathered bytes over time exceed the HBM peak, so that ratio is no
                # fraction of a roofline; against HBM only the bytes that reached it count
                roofline["nominal_gathered_over_hbm_peak"] = roofline["frac"]
                roofline["nominal_gathered_GBps_per_launch"] = roofline["achieved"]
                roofline["achieved"] = roofline["hbm_GBps_from_counters"]
                roofline["frac"] = roofline["hbm_frac_from_counters"]
                roofline["note"] += ".  The weights are cache-resident here: achieved / frac are the HBM bytes from the counters " \
                                    "over the step time; the kernel is bound by the compute units' path to L2 " \
                                    "(frac_of_measured_l2_read_rate)"
        extra["per_step_us_by_kernel_kind_with_event_overhead"] = {k: round(v, 1) for k, v in per_step_us.items()}
        extra["avg_launch_us_by_kernel_kind_with_event_overhead"] = \
            {k: round(v[0] * 1e3 / v[1], 2) for k, v in prof.items() if v[1]}

    def sweep_and_dense(wk, steps, warm, keeps):
        """the keep fractions of a workload and the full network, a few steps each"""
        res = {"sweep": {}}
        base_steps, base_warm = steps, warm
        for keep in keeps:
            kt_ = wk.keep_tensor(keep)
            steps, warm = wk.steps_for(lambda: wk.step(kt_), base_steps, base_warm)
            s, _ = wk.time_sparse(keep, steps, warm)
            q = steps * wk.nq / s
            res["sweep"][str(keep)] = {"qps": round(q), "ms_per_step": round(s / steps * 1e3, 4),
                                       "nominal_gathered_GBps": round(wk.gathered_bytes_per_step(keep) * steps / s / 1e9, 1)}
        dflops = wk.dense_flops_per_query()
        res["dense_baseline"] = {}
        for mode, label in ((0, "fp32_mfma"), (1, "f16_parts_mfma")):
            if mode and not hasattr(slonn, "slonn_model_set_dense_arithmetic"):
                continue
            if hasattr(slonn, "slonn_model_set_dense_arithmetic"):
                slonn.slonn_model_set_dense_arithmetic(wk.net.model, mode)
            steps, warm = wk.steps_for(wk.dense_step, base_steps, base_warm)
            s, _ = wk.timed(wk.dense_step, steps, warm)
            res["dense_baseline"][label] = {"qps": round(steps * wk.nq / s), "ms_per_step": round(s / steps * 1e3, 4),
                                            "TFLOPs": round(dflops * steps * wk.nq / s / 1e12, 2)}
        if hasattr(slonn, "slonn_model_set_dense_arithmetic"):
            slonn.slonn_model_set_dense_arithmetic(wk.net.model, 0)
        if wk.batch <= 64 and 1.0 not in keeps:
            # small batches: the full network is also run through the sparse path's own kernels with every
            # node active (keep 1.0: no table access, rows spread over all compute units), the "all nodes
            # computed" case of Section 3.4; a matrix-core GEMM has little to offer a handful of queries
            kt_ = wk.keep_tensor(1.0)
            steps, warm = wk.steps_for(lambda: wk.step(kt_, uniform=True), base_steps, base_warm)
            s, _ = wk.time_sparse(1.0, steps, warm, uniform=True)
            res["dense_baseline"]["all_nodes_through_the_gather_kernels"] = {
                "qps": round(steps * wk.nq / s), "ms_per_step": round(s / steps * 1e3, 4),
                "TFLOPs": round(dflops * steps * wk.nq / s / 1e12, 2)}
        best_dense = max(v["qps"] for v in res["dense_baseline"].values())
        for k, v in res["sweep"].items():
            v["sparse_over_best_dense"] = round(v["qps"] / best_dense, 3)
        return res

    if not args.no_sweep:
        keeps = cfg.keeps if w.mixed is None else ()
        r = sweep_and_dense(w, max(2, min(K, 5)), 1, keeps)
        extra.update(r)
        best_dense = max(v["qps"] for v in r["dense_baseline"].values())
        extra["sparse_over_best_dense"] = round(qps / best_dense, 3)

    # ---- k chosen per query inside the pass (ACLO): Confidence LSH tables trained on the build
    #      set with c(k, x) = -cross-entropy(full prediction, prediction at k) (Section 2.1) ----
    if args.aclo and w.mixed is None and not w.ell and cfg.hashed_layers[0] == 0:
        net, xb = w.net, w.xb
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
        pick = torch.from_numpy(np.random.default_rng(8).integers(0, nb_, w.nq)).to(dev)
        thr_all = conf[:, len(grid) // 2][pick].contiguous()
        keep_out = torch.zeros(B, dtype=torch.float32, device=dev)
        chosen = []

        def aclo_step(collect=False):
            for i, nb in enumerate(w.sizes):
                slonn.slonn_sparse_forward_aclo(net.model, net.tables, pol, w.batches[i], nb,
                                                thr_all[i * B:i * B + nb], 1, keep_out, w.out, None, w.ws, w.stream)
                if collect:
                    chosen.append(keep_out[:nb].cpu().numpy().copy())
        a_s, _ = w.timed(aclo_step, max(2, min(K, 5)), 1)
        a_n = max(2, min(K, 5))
        aclo_step(collect=True)
        chosen = np.concatenate(chosen)
        extra["aclo"] = {"qps": round(a_n * w.nq / a_s), "ms_per_step": round(a_s / a_n * 1e3, 4), "k_grid": grid,
                         "share_of_queries_per_k": [round(float((chosen == np.float32(k)).mean()), 4) for k in grid],
                         "mean_keep": round(float(chosen.mean()), 4),
                         "confidence": "-cross-entropy(softmax(full), softmax(at k)) on the first "
                                       f"{nb_} build inputs; per-query thresholds drawn from those at k = {grid[len(grid) // 2]}"}
        log(f"ACLO: {extra['aclo']}")

    # ---- batches ordered by LSH key (Section 6 names clustering a batch into micro-batches as future
    #      work): queries whose first-layer keys agree share the heads of their ranked lists, so groups
    #      of neighbours in that order select overlapping rows.  The keys come from slonn_select; the
    #      reordering of the query rows is a device gather outside the library. ----
    if args.cluster_by_key and w.mixed is None and not w.ell:
        net = w.net
        l0 = cfg.hashed_layers[0]
        nb0 = w.sizes[0]
        xb0 = w.xq[:nb0]
        if l0 > 0:
            xb0 = net.dense_forward(xb0, layer_outs=True)["layers"][l0 - 1]
        codes = net.select(l0, xb0, head_keep)["codes"].cpu().numpy().view(np.uint32)
        order = np.lexsort(codes.T[::-1])             # by table 0's key, then table 1's, ...
        res = {}
        for label, perm in (("arrival_order", np.arange(nb0)), ("ordered_by_first_layer_keys", order)):
            xq_p = w.xq[:nb0][torch.from_numpy(perm).to(dev)].contiguous()
            r = net.sparse_forward(xq_p, head_keep, taps=True)
            stats = {}
            for l in cfg.hashed_layers:
                act = r["taps"]["active"][l].cpu().numpy()
                cnt = r["taps"]["cnt"][l].cpu().numpy()
                for gsz in (16, 128):
                    ratios = []
                    for g0 in range(0, nb0 - gsz + 1, gsz):
                        u = np.unique(np.concatenate([act[q, :cnt[q]] for q in range(g0, g0 + gsz)])).size
                        ratios.append(u / cnt[g0:g0 + gsz].mean())
                    stats[f"layer{l}_union_of_{gsz}_over_one_list"] = round(float(np.mean(ratios)), 3)
            inp = slonn.make_input(x=xq_p)
            kt = w.keep_tensor(head_keep)

            def one():
                slonn.slonn_sparse_forward(net.model, net.tables, inp, nb0, kt, 0, 0, w.out, None, w.ws, w.stream)
            s_, _ = w.timed(one, 30, 5)
            stats["us_per_batch"] = round(s_ / 30 * 1e6, 1)
            res[label] = stats
        extra["cluster_by_key"] = res
        log(f"cluster by key: {res}")

    # ---- CPU baseline: the oracle as it stands, on the host cores, bounded sample ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import slonn_oracle
        net = w.net
        note = ""
        blob_bytes = slonn.slonn_tables_export_bytes(net.tables)
        if blob_bytes > (5 << 30):
            # the full table set is too large to copy to the host twice: the oracle gets tables trained
            # (on the device, same kernels) on the first inputs of the same training set
            nb_small = 1024
            net_small = w.runtime.Network(w.layers, first_layer_rows_are_inputs=w.ell)
            net_small.build_tables(w.xb[:nb_small] if not w.ell else tuple(a[:nb_small] for a in w.xb))
            blob = net_small.export_tables()
            del net_small
            note = f", tables trained on the first {nb_small} of the {w.n_build} training inputs ({len(blob) / 2**30:.1f} GiB)"
        else:
            blob = net.export_tables()
        onet = slonn_oracle.OracleNet(w.layers, first_layer_rows_are_inputs=w.ell,
                                      hash_nodes_always_active=args.hash_nodes_always_active)
        onet.import_tables(blob)
        del blob
        big = cfg.dims[1] >= 4096 and len(cfg.dims) > 3
        n_s = min(w.nq, 512 if big else 4096)
        Xs = tuple(a[:n_s] for a in w.X_query) if w.ell else w.X_query[:n_s]
        ks = args.keep if w.mixed is None else w.mixed_host[:n_s]
        done, dt = 0, 0.0
        while dt < 10.0 and done < 400 * n_s:      # passes over the sample until about ten seconds are timed
            t0 = time.perf_counter()
            onet.sparse_forward(Xs, ks, taps=False)
            dt += time.perf_counter() - t0
            done += n_s
        cpu = {"value": round(done / dt, 1), "unit": "queries/s", "cores": onet.threads, "kind": "oracle",
               "sample": f"first {n_s} queries of the same query set, {done // n_s} passes ({dt:.1f} s of CPU work), "
                         f"keep {keep_label}, all layers, {onet.threads} threads over queries{note}"}
        # the same oracle on one thread (the paper times one query at a time), on the first queries of the
        # sample: about two seconds
        n_1 = max(1, min(n_s, int(2.0 * done / dt / max(onet.threads, 1)) + 1))
        all_threads, onet.threads = onet.threads, 1
        X1 = tuple(a[:n_1] for a in Xs) if w.ell else Xs[:n_1]
        k1 = ks if w.mixed is None else ks[:n_1]
        t0 = time.perf_counter()
        onet.sparse_forward(X1, k1, taps=False)
        cpu["one_thread"] = {"value": round(n_1 / (time.perf_counter() - t0), 2), "unit": "queries/s",
                             "sample": f"first {n_1} queries, one pass"}
        onet.threads = all_threads
        log(f"CPU oracle: {cpu}")
        del onet

    # ---- the other workloads, briefly (their own query sets, whole-set steps) ----
    if not args.no_sweep and not args.no_others and args.config == "C5":
        others = {}
        # the headline model at small batches (the paper serves one query at a time, Section 4)
        for b_, q_ in ((32, 1024), (8, 256), (1, 64)):
            w.set_batch(b_, q_)
            r = sweep_and_dense(w, 3, 1, ())
            kt_ = w.keep_tensor(None)
            n_, w_ = w.steps_for(lambda: w.step(kt_), 3, 1)
            s_, _ = w.time_sparse(None, n_, w_)
            best = max(v["qps"] for v in r["dense_baseline"].values())
            r["sparse"] = {"qps": round(n_ * w.nq / s_), "ms_per_step": round(s_ / n_ * 1e3, 4),
                           "nominal_gathered_GBps": round(w.gathered_bytes_per_step(None) * n_ / s_ / 1e9, 1),
                           "sparse_over_best_dense": round(n_ * w.nq / s_ / best, 3)}
            if b_ == 1:      # the paper's regime: one query at a time, nothing else in flight
                r["sparse"]["latency_us_one_in_flight"] = w.latency_us(None)
                r["dense_baseline"]["all_nodes_through_the_gather_kernels"]["latency_us_one_in_flight"] = \
                    w.latency_us(1.0, uniform=True)
            r["config"] = {"workload": head_config["workload"], "batch": b_, "keep": keep_label,
                           "queries_per_step": w.nq, "streams": w.n_streams}
            others[f"{args.config}_B{b_}"] = r
            log(f"{args.config} batch {b_}: {r}")
        del w
        torch.cuda.empty_cache()
        # (name, batch sizes with the queries per step at each, query set, table-training inputs)
        for name, shapes, nq_, nb_ in (("C3", ((1024, 8192), (32, 2048), (1, 256)), 8192, 8192),
                                       ("C2", ((256, 0),), 0, 0), ("C4", ((128, 0),), 0, 0), ("C1", ((64, 0), (1, 64)), 0, 0)):
            wk = Workload(name, shapes[0][0], args, n_queries=nq_, n_build=nb_)
            for b_, q_ in shapes:
                wk.set_batch(b_, q_)
                r = sweep_and_dense(wk, 3, 1, wk.cfg.keeps)
                if b_ == 1:
                    for k_, v_ in r["sweep"].items():
                        v_["latency_us_one_in_flight"] = wk.latency_us(float(k_))
                    r["dense_baseline"]["all_nodes_through_the_gather_kernels"]["latency_us_one_in_flight"] = \
                        wk.latency_us(1.0, uniform=True)
                r["config"] = {"workload": f"{name}: MLP {'-'.join(map(str, wk.cfg.dims))}, K={wk.cfg.K} L={wk.cfg.L}",
                               "batch": b_, "queries_per_step": wk.nq, "table_training_inputs": wk.n_build,
                               "streams": wk.n_streams}
                others[f"{name}_B{b_}"] = r
                log(f"{name} batch {b_}: {r}")
            del wk
            torch.cuda.empty_cache()
        extra["other_workloads"] = others

    line = {
        "metric": "queries/sec and effective HBM GB/s (vs peak) for sparse forward at keep-fraction",
        "value": round(qps, 1), "unit": "queries/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(secs / K * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if cfg.w_dtype == wl.W_F32 else "bf16 weights, f32 accumulate",
        "data": "synthetic",
        "config": head_config,
        "roofline": roofline, "cpu_baseline": cpu,
    }
    line.update(extra)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
