#!/usr/bin/env python3
"""Benchmark of the PiKV routed sharded-KV decode path on one MI355X.

A "step" is one pass of the whole hot path over one batch of queries against one layer's
expert-sharded cache:  route -> evict (min-utility entry of every selected full shard) ->
append the new token's K/V -> attention over the selected shards -> utility update.
Every step runs in the HIP kernels of libpikv.so through the C ABI; inputs are seeded,
synthetic, and resident in HBM before the timed region starts.

Default workload: the 128K-context / 16-expert long-context configuration (B=1, 32 query
heads over 8 KV heads, D=128, E=16 shards x 8192 tokens, top-k=4, bf16).  One step reads
128 MiB of K/V, which would fit the 256 MB Infinity Cache, so the steps cycle round-robin
over 32 independent layer instances (16 GiB), as a 32-layer model does for every token.

Prints ONE JSON line: `value` = queries/s over the timed steps (B x steps / elapsed), `roofline` =
the attention pass against the 8 TB/s HBM peak: `frac` uses the kernel's average duration from
the committed rocprofv3 kernel trace of this workload (profiles/, which names its command), the
live HIP-event figures of this run are printed beside it; `cpu_baseline` = the CPU oracle on a bounded sample
of the same workload; `other_workloads` = one short line per remaining workload.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
CPU_BASELINE_SECONDS = 10.0   # how long the oracle leg keeps repeating its sample
MIN_PROBE_STEPS = 256         # eager steps with the event pair around the attention pass

# HBM bytes per launch of the dominant kernel as measured by rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE (two runs, scaled by what a plain 1 GiB device copy reads on the same counters);
# the numbers and the commands are in the named files under profiles/.
TRAFFIC_FILES = {
    "c3_long_context": "profiles/c3_long_context_hbm_traffic_pmc.txt",
    "c2_bf16_decode": "profiles/c2_bf16_decode_hbm_traffic_pmc.txt",
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=256)
    ap.add_argument("--config", default="c3_long_context")
    ap.add_argument("--layers", type=int, default=0, help="layer instances cycled (0: per config)")
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph")
    ap.add_argument("--api", choices=["fused", "separate"], default="fused",
                    help="fused: pikv_decode_step (3 launches); separate: the five calls (7 launches)")
    ap.add_argument("--cpu-steps", type=int, default=-1, help="oracle steps timed (0: skip, -1: auto)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short runs of the other workloads (key other_workloads)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--balance", action="store_true",
                    help="widened row: keep the load-balance router penalty on the device and feed "
                         "it back as the routing bias (inside the fused step's last launch)")
    ap.add_argument("--compress", action="store_true",
                    help="widened row (rank > 0 workloads): compress the new token's full-width K/V "
                         "to codes inside the step (one extra small launch)")
    ap.add_argument("--k", type=int, default=0,
                    help="sanity ratio: override the configuration's k (k = E is dense attention)")
    ap.add_argument("--rank", type=int, default=-1,
                    help="sanity ratio: override the configuration's code rank (0 = full-width K/V)")
    ap.add_argument("--histogram", type=int, default=-1, metavar="N",
                    help="route N random queries through layer 0's router and print the empirical "
                         "expert popularity to stderr (default: 4096 for the workloads with a Zipf "
                         "popularity law, 0 = off)")
    ap.add_argument("--policy", choices=["none", "lru", "lru_plus", "sl"], default="none",
                    help="widened row: evict by a Table 3 bookkeeping policy inside the fused step "
                         "(pikv_decode_step_policy) and keep the access stamps and counts up to date")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device copy 8 times and exit (reference for the "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


# layer instances so that consecutive steps cannot be served from the 256 MB Infinity Cache
DEFAULT_LAYERS = {"c1_tiny_f32": 1, "c2_bf16_decode": 2, "c3_long_context": 32, "c4_streaming": 2,
                  "c5_compressed": 16, "c3_long_context_tq4": 32, "c3_long_context_tq8": 32,
                  "c3_kv4_tq16": 32}
RECIPE = {  # how each configuration's inputs are drawn (workloads.make_device_layers arguments)
    "c1_tiny_f32": dict(w_sigma=1.0),
    "c2_bf16_decode": dict(kv="lognormal_token"),
    "c3_long_context": dict(zipf_s=1.1),
    "c4_streaming": dict(utility0="exp"),
    "c5_compressed": dict(zipf_s=1.1),
    "c3_long_context_tq4": dict(zipf_s=1.1, w_sigma=0.01),
    "c3_long_context_tq8": dict(zipf_s=1.1),     # routed by the tile's first query: the router of c3
    "c3_kv4_tq16": dict(zipf_s=1.1),
}
DECAY = {"c4_streaming": 0.9}
OTHER_WORKLOADS = ("c2_bf16_decode", "c4_streaming", "c5_compressed")


class Layer:
    """One layer instance's device state plus the binding calls of one step."""

    def __init__(self, pk, torch, geo, tensors, shared):
        self.pk, self.geo, self.t, self.sh = pk, geo, tensors, shared
        g = geo
        self.desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, rank=g.rank,
                                 dtype=0 if g.dtype == "f32" else 1,
                                 route_rows_per_seq=g.Hq if g.per_head_routing else 1,
                                 tq=g.tq if g.token_major else 1)
        self.K_tab = pk.shard_table(tensors["K"])
        self.V_tab = pk.shard_table(tensors["V"])
        self.decay = DECAY.get(g.name, 1.0)
        self.fused = shared.get("fused", False) and not g.per_head_routing
        import workloads as wl
        self.route_x = wl.routing_rows(g, tensors["q"])   # what pikv_route sees (the queries are fixed)

    def step(self):
        pk, g, t, s = self.pk, self.geo, self.t, self.sh
        if s.get("compress"):
            pk.pikv_compress(self.desc, s["K_full"], s["Wenc_K"], s["K_new"], s["V_full"], s["Wenc_V"],
                             s["V_new"])
        self._step()
        if s.get("balance") and not self.fused:
            pk.pikv_router_penalty(pk.PENALTY_LOAD_BALANCE, s["topk"], g.route_rows, g.k, g.E,
                                   t["load"], None, 0.01, t["bias"])

    def _step(self):
        pk, g, t, s = self.pk, self.geo, self.t, self.sh
        feedback = None
        if self.fused and s.get("balance"):      # the loop closes inside the step's last launch
            feedback = pk.make_router_feedback(pk.PENALTY_LOAD_BALANCE, 0.01, t["load"], t["bias"])
        if self.fused and (s.get("policy") or feedback is not None):
            # the step counter is baked into the captured launch: replays re-stamp with the same
            # value, which costs the same as a running counter
            args = None
            if s.get("policy"):
                args = pk.make_policy_args(s["policy"], 1000, lam=0.5, window=g.S // 2, threshold=1.0 / g.S,
                                           birth=t["birth"], last_access=t["last_access"], freq=t["freq"])
            pk.pikv_decode_step_policy(self.desc, t["q"], t["W_r"], t["bias"], s["K_new"], s["V_new"],
                                       self.K_tab, self.V_tab, t["U_K"], t["U_V"], t["n_valid"], t["utility"],
                                       g.k, pk.COMBINE_LSE, 0.0, self.decay, s["topk"], s["gates"], s["eidx"],
                                       s["ecnt"], s["y"], s["row_max"], s["row_norm"], s["scores"],
                                       s["slot_coef"], s["workspace"], args, feedback=feedback)
            return
        if self.fused:
            pk.pikv_decode_step(self.desc, t["q"], t["W_r"], t["bias"], s["K_new"], s["V_new"],
                                self.K_tab, self.V_tab, t["U_K"], t["U_V"], t["n_valid"], t["utility"],
                                g.k, pk.COMBINE_LSE, 0.0, self.decay, s["topk"], s["gates"], s["eidx"],
                                s["ecnt"], s["y"], s["row_max"], s["row_norm"], s["scores"],
                                s["slot_coef"], s["workspace"])
            return
        pk.pikv_route(self.route_x, t["W_r"], t["bias"], g.route_rows, g.d_r, g.E, g.k, s["topk"],
                      s["gates"], None)
        if not g.per_head_routing:
            pk.pikv_evict(self.desc, t["utility"], t["n_valid"], g.S - 1, s["topk"], g.k, s["eidx"],
                          s["ecnt"], 1, False, None, None)
            pk.pikv_append(self.desc, s["K_new"], s["V_new"], s["topk"], g.k, s["eidx"], s["ecnt"], 1,
                           self.K_tab, self.V_tab, t["utility"], t["n_valid"])
        pk.pikv_sharded_attn(self.desc, t["q"], self.K_tab, self.V_tab, t["U_K"], t["U_V"],
                             t["n_valid"], s["topk"], s["gates"], g.k, pk.COMBINE_LSE, 0.0, s["y"],
                             s["row_max"], s["row_norm"], s["scores"], s["slot_coef"], s["workspace"])
        pk.pikv_update_utility(self.desc, s["scores"], s["slot_coef"], t["n_valid"], s["topk"], g.k,
                               self.decay, t["utility"])


def make_shared(pk, torch, geo, dev):
    g = geo
    tdt = torch.float32 if g.dtype == "f32" else torch.bfloat16
    R, k = g.route_rows, g.k
    desc = pk.make_desc(g.B, g.Hq, g.Hkv, g.D, g.E, g.S, rank=g.rank, dtype=0 if g.dtype == "f32" else 1,
                        route_rows_per_seq=g.Hq if g.per_head_routing else 1,
                        tq=g.tq if g.token_major else 1)
    gen = torch.Generator(device=dev)
    gen.manual_seed(12345)
    return dict(
        topk=torch.zeros((R, k), device=dev, dtype=torch.int32),
        gates=torch.zeros((R, k), device=dev),
        eidx=torch.zeros((g.B, g.E, 1), device=dev, dtype=torch.int32),
        ecnt=torch.zeros((g.B, g.E), device=dev, dtype=torch.int32),
        K_new=torch.randn((g.B, g.Hkv, g.width), device=dev, generator=gen).to(tdt),
        V_new=torch.randn((g.B, g.Hkv, g.width), device=dev, generator=gen).to(tdt),
        y=torch.zeros((g.B, g.Hq, g.D), device=dev),
        row_max=torch.zeros((g.B, g.Hq), device=dev),
        row_norm=torch.zeros((g.B, g.Hq), device=dev),
        scores=torch.zeros((g.B, g.Hq, k, g.S), device=dev),
        slot_coef=torch.zeros((g.B, g.Hq, k, 2), device=dev),
        workspace=torch.empty(pk.pikv_attn_workspace_bytes(desc, k), device=dev, dtype=torch.uint8),
    )


def attn_kernel_name(geo):
    g = geo.Hq // geo.Hkv
    if geo.dtype == "bf16" and geo.rank == 0 and geo.D == 128 and not geo.per_head_routing and 2 <= g <= 64:
        # (row tiles, form of the score output: the second template argument is the library's choice)
        return "attn_partial_gqa128<%d, *>" % (1 if g <= 16 else 2 if g <= 32 else 4)
    gb = g if (not geo.per_head_routing and g in (2, 4, 8)) else 1
    return "attn_partial<%s, %d, %d>" % ("pikv::bf16" if geo.dtype == "bf16" else "float", geo.width, gb)


def read_ceiling(pk, torch, geo, layers, stream):
    """What a pass that only READS a step's K/V bytes reaches here: the library's measurement
    kernel (pikv_stream_read_probe: the attention pass's load shape, no arithmetic) over k shards'
    K and V buffers of every sequence, one launch per layer instance in the same rotation as the
    steps, replayed as a HIP graph.  Context for the roofline fraction, not part of `value`."""
    g = geo
    dev = layers[0].t["K"].device
    elt = 4 if g.dtype == "f32" else 2
    bytes_each = g.Hkv * g.S * g.width * elt
    n = g.B * g.k * 2
    parts = max(1, min(1024 // max(n, 1), bytes_each // 65536))
    tables, outs = [], []
    for L in layers:
        K, V = L.t["K"], L.t["V"]                      # [B, E, Hkv, S, w]
        bufs = [T[b, e] for T in (K, V) for b in range(g.B) for e in range(g.k)]
        tables.append(pk.shard_table(bufs))
        outs.append(torch.zeros(n * parts, device=dev, dtype=torch.int32))
    def launch(i):
        pk.pikv_stream_read_probe(tables[i], n, bytes_each, parts, outs[i], stream=stream.cuda_stream)
    with torch.cuda.stream(stream):
        for i in range(len(layers)):
            launch(i)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(len(layers)):
                launch(i)
        graph.replay()
    stream.synchronize()
    launches = max(512, len(layers))
    replays = -(-launches // len(layers))
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        for _ in range(replays):
            graph.replay()
    stream.synchronize()
    per_launch = (time.perf_counter() - t0) / (replays * len(layers))
    nbytes = n * bytes_each
    return {"GBps": nbytes / per_launch / 1e9, "frac_of_peak": nbytes / per_launch / 1e9 / HBM_PEAK_GBS,
            "us_per_launch": per_launch * 1e6, "bytes_per_launch": nbytes, "blocks": n * parts,
            "launches_timed": replays * len(layers),
            "what": "pikv_stream_read_probe: K and V buffers of k shards per sequence read once with the "
                    "attention pass's load shape and no arithmetic, one launch per layer instance, graph replay"}


def profile_summary(config, kernel):
    """Average duration (ns) of `kernel` in the committed rocprofv3 kernel-trace summary of this
    workload (profiles/<config>_kernel_stats.txt: a table `name calls avg_ns min_ns max_ns pct`)."""
    path = os.path.join(ROOT, "profiles", "%s_kernel_stats.txt" % config)
    if not os.path.exists(path):
        return None, None
    key = re.sub(r"[^A-Za-z0-9_]", "", kernel)
    for line in open(path):
        m = re.match(r"^(.*\S)\s+(\d+)\s+(\d+)\s+(\d+)\s+(\d+)\s+[\d.]+\s*$", line)
        if m and key in re.sub(r"[^A-Za-z0-9_]", "", m.group(1)):
            return float(m.group(3)), os.path.relpath(path, ROOT)
    return None, os.path.relpath(path, ROOT)


def measured_traffic(config):
    """(bytes per launch, file) from the committed FETCH_SIZE / WRITE_SIZE summary, if any."""
    rel = TRAFFIC_FILES.get(config)
    if not rel or not os.path.exists(os.path.join(ROOT, rel)):
        return None, None
    for line in open(os.path.join(ROOT, rel)):
        m = re.match(r"^\s*traffic_bytes_per_launch\s*[:=]\s*(\d+)", line)
        if m:
            return int(m.group(1)), rel
    return None, rel


def cpu_baseline(torch, wl, layers, n_steps):
    """Time the oracle (as it stands) on the same inputs: route + attend + utility per step."""
    from oracle import pikv_oracle as orc
    import numpy as np
    g = layers[0].geo
    dummy = np.zeros((1,), np.float32 if g.dtype == "f32" else np.uint16)
    prepared = []
    for L in layers[:n_steps]:
        t = L.t
        q = wl.to_host(t["q"], g.dtype)
        W = wl.to_host(t["W_r"], g.dtype)
        bias = None if t["bias"] is None else t["bias"].cpu().numpy()
        x = np.ascontiguousarray(wl.routing_rows(g, q))
        idx, gates, _ = orc.route(x, W, g.k, bias=bias, dtype=g.dtype)
        Ks, Vs = [dummy] * (g.B * g.E), [dummy] * (g.B * g.E)
        for row in range(idx.shape[0]):
            b = row // g.Hq if g.per_head_routing else row
            for e in idx[row]:
                i = b * g.E + int(e)
                if Ks[i] is dummy:
                    Ks[i] = wl.to_host(t["K"][b, e], g.dtype)
                    Vs[i] = wl.to_host(t["V"][b, e], g.dtype)
        prepared.append(dict(
            q=q, W=W, bias=bias, x=x, Ks=Ks, Vs=Vs, n=t["n_valid"].cpu().numpy(),
            u=t["utility"].cpu().numpy(),
            UK=None if t["U_K"] is None else wl.to_host(t["U_K"], g.dtype),
            UV=None if t["U_V"] is None else wl.to_host(t["U_V"], g.dtype)))
    # passes over the prepared steps until about 10 s of CPU work are on the clock
    t0 = time.perf_counter()
    done = 0
    while True:
        for p in prepared:
            idx, gates, _ = orc.route(p["x"], p["W"], g.k, bias=p["bias"], dtype=g.dtype)
            orc.attend(p["q"], p["Ks"], p["Vs"], p["n"], idx, gates, Hkv=g.Hkv, E=g.E, S=g.S,
                       dtype=g.dtype, rank=g.rank, U_K=p["UK"], U_V=p["UV"], utility=p["u"],
                       decay=DECAY.get(g.name, 1.0))
            done += 1
        if not prepared or time.perf_counter() - t0 >= CPU_BASELINE_SECONDS:
            break
    dt = time.perf_counter() - t0
    return dt / max(1, done), done, dt


def expert_histogram(pk, torch, geo, t, n_queries, dev):
    """Empirical expert popularity of the configuration's router over a stream of random queries."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    x = torch.randn((n_queries, geo.d_r), device=dev, generator=gen).to(t["W_r"].dtype)
    idx = torch.zeros((n_queries, geo.k), device=dev, dtype=torch.int32)
    gates = torch.zeros((n_queries, geo.k), device=dev)
    pk.pikv_route(x, t["W_r"], t["bias"], n_queries, geo.d_r, geo.E, geo.k, idx, gates, None)
    torch.cuda.synchronize()
    counts = torch.bincount(idx.flatten().long(), minlength=geo.E).cpu().tolist()
    top1 = torch.bincount(idx[:, 0].long(), minlength=geo.E).cpu().tolist()
    total = float(sum(counts))
    order = sorted(range(geo.E), key=lambda e: -counts[e])
    print("expert popularity over %d random queries (top-%d selections), most popular first:" %
          (n_queries, geo.k), file=sys.stderr)
    for r, e in enumerate(order):
        print("  rank %2d expert %2d: share %.4f (top-1 share %.4f)" %
              (r + 1, e, counts[e] / total, top1[e] / float(n_queries)), file=sys.stderr)


class StepRunner:
    """Enqueues steps round-robin over the layer instances on one stream of default priority;
    the same code runs eagerly and under graph capture."""

    def __init__(self, torch, layers):
        self.torch, self.layers = torch, layers
        self.main = torch.cuda.Stream()

    def run(self, i):
        with self.torch.cuda.stream(self.main):
            self.layers[i % len(self.layers)].step()

    def synchronize(self):
        self.main.synchronize()


def measure(args, config, steps, warmup, with_cpu, probe_steps, quiet=False):
    """Build the workload, time `steps` steps, time the attention pass; returns the result dict."""
    import torch
    import paper_2508_06526_amd as pk
    import workloads as wl

    dev = torch.device("cuda:0")
    geo = wl.CONFIGS[config]
    if args.k > 0 or args.rank >= 0:
        import dataclasses
        geo = dataclasses.replace(geo, k=args.k if args.k > 0 else geo.k,
                                  rank=args.rank if args.rank >= 0 else geo.rank)
    n_layers = args.layers or DEFAULT_LAYERS[config]
    raw = wl.make_device_layers(geo, n_layers, args.seed, dev, **RECIPE[config])
    shared = [make_shared(pk, torch, geo, dev)]
    for s in shared:
        s["fused"] = args.api == "fused"
    if args.balance:
        for s in shared:
            s["balance"] = True
        for t in raw:
            t["load"] = torch.zeros(geo.E, device=dev, dtype=torch.int32)
            t["bias"] = torch.zeros(geo.E, device=dev)
    if args.policy != "none":
        for s in shared:
            s["policy"] = {"lru": pk.POLICY_LRU, "lru_plus": pk.POLICY_LRU_PLUS, "sl": pk.POLICY_SL}[args.policy]
        for t in raw:
            t["birth"] = torch.randint(0, 1000, (geo.B, geo.E, geo.S), device=dev, dtype=torch.int32)
            t["last_access"] = torch.randint(0, 1000, (geo.B, geo.E, geo.S), device=dev, dtype=torch.int32)
            t["freq"] = torch.randint(0, 50, (geo.B, geo.E, geo.S), device=dev, dtype=torch.int32)
    if args.compress and geo.rank:
        tdt = torch.bfloat16 if geo.dtype == "bf16" else torch.float32
        gen = torch.Generator(device=dev)
        gen.manual_seed(777)
        rn = lambda *sh: torch.randn(*sh, device=dev, generator=gen)
        extra = dict(compress=True,
                     K_full=rn(geo.B, geo.Hkv, geo.D).to(tdt), V_full=rn(geo.B, geo.Hkv, geo.D).to(tdt),
                     Wenc_K=(rn(geo.Hkv, geo.rank, geo.D) / geo.D ** 0.5).to(tdt),
                     Wenc_V=(rn(geo.Hkv, geo.rank, geo.D) / geo.D ** 0.5).to(tdt))
        for s in shared:
            s.update(extra)
    layers = [Layer(pk, torch, geo, t, shared[0]) for t in raw]
    torch.cuda.synchronize()
    n_hist = args.histogram if args.histogram >= 0 else (4096 if "zipf_s" in RECIPE[config] else 0)
    if n_hist > 0 and not quiet:
        expert_histogram(pk, torch, geo, raw[0], n_hist, dev)

    run = StepRunner(torch, layers)
    K, W = steps, warmup
    for i in range(W):
        run.run(i)
    run.synchronize()
    # The graph holds one round over the layer instances, or fewer steps if fewer are asked for;
    # steps that do not fill a whole replay are launched one by one (both counts are reported).
    graph, per_replay = None, 0
    if args.mode == "graph":
        per_replay = min(n_layers, K)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=run.main):
            for i in range(per_replay):
                run.run(i)
        graph.replay()                 # one untimed replay
        run.main.synchronize()

    # ---- timed region: exactly K steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    replays = K // per_replay if graph is not None else 0
    with torch.cuda.stream(run.main):
        for _ in range(replays):
            graph.replay()
    for i in range(replays * per_replay, K):
        run.run(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    eager_steps = K - replays * per_replay
    if elapsed < 0.010 and not quiet:
        print("bench.py: the timed region of %d steps lasted %.2f ms; use --steps >= 256 for a stable figure"
              % (K, elapsed * 1e3), file=sys.stderr)

    # ---- dominant kernel (the attention pass that streams the K/V bytes): the library records
    # a HIP event pair on the launch stream right around that kernel's launch
    # (pikv_set_profile_events), inside the same steps as above, launched eagerly; the GPU work
    # per step is longer than the launch work, so the queue stays ahead of the GPU
    n_probe = probe_steps
    ev, ev_empty = [], []
    with torch.cuda.stream(run.main):
        for _ in range(n_probe):
            quad = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            for x in quad:
                x.record(run.main)
            ev.append((quad[0], quad[1]))
            ev_empty.append((quad[2], quad[3]))
    for i in range(64):                      # refill the queue after the event creation
        run.run(i)
    for i in range(n_probe):
        pk.pikv_set_profile_events(ev[i][0], ev[i][1])
        run.run(i)
        # an event pair with nothing in between, in the same stream position: what the two
        # marker packets themselves cost
        ev_empty[i][0].record(run.main)
        ev_empty[i][1].record(run.main)
    pk.pikv_set_profile_events(None, None)
    run.synchronize()
    raw_ms = sorted(a.elapsed_time(b2) for a, b2 in ev)
    empty_ms = sorted(a.elapsed_time(b2) for a, b2 in ev_empty)
    raw_avg_ms = sum(raw_ms) / len(raw_ms)
    empty_avg_ms = sum(empty_ms) / len(empty_ms)
    net_avg_ms = raw_avg_ms - empty_avg_ms

    ms_per_step = elapsed * 1e3 / K
    qps = geo.B * geo.tq * K / elapsed
    n_mean = float(torch.stack([L.t["n_valid"].float().mean() for L in layers]).mean().item())
    kv_bytes = geo.kv_bytes_per_step(n_mean)
    gbps = lambda ms: kv_bytes / (ms * 1e-3) / 1e9
    kernel = attn_kernel_name(geo)
    prof_ns, prof_file = profile_summary(config, kernel) if not (args.k > 0 or args.rank >= 0) else (None, None)
    if prof_ns is not None:
        avg_ms, basis = prof_ns * 1e-6, "committed rocprofv3 kernel trace of this workload in this launch mode, " + prof_file
    else:
        avg_ms, basis = raw_avg_ms, "uncorrected HIP event pair of this run (no kernel-trace summary for this workload)"
    traffic, traffic_file = measured_traffic(config)
    out = {
        "metric": "routed sharded-KV decode queries/sec", "value": qps, "unit": "queries/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if geo.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": config, "B": geo.B, "Hq": geo.Hq, "Hkv": geo.Hkv, "D": geo.D,
                   "E": geo.E, "S": geo.S, "k": geo.k, "rank": geo.rank,
                   "overrides": {"k": args.k or None, "rank": args.rank if args.rank >= 0 else None},
                   "queries_per_sequence": geo.tq, "layers_cycled": n_layers,
                   "launch": {"mode": args.mode, "graph_replays": replays, "steps_per_replay": per_replay,
                              "steps_in_replays": replays * per_replay, "steps_launched_eagerly": eager_steps},
                   "timed_region_s": elapsed,
                   "timed_region_note": None if elapsed >= 0.010 else
                   "the timed region is under 10 ms: --steps %d is too few for a stable figure "
                   "(the default run times 4096 steps)" % K,
                   "api": args.api, "balance": bool(args.balance),
                   "compress_on_insert": bool(args.compress and geo.rank), "policy": args.policy,
                   "step": "route+evict1+append+attend+utility"},
        "step_effective_GBps": gbps(ms_per_step),
        "step_frac_of_hbm_peak": gbps(ms_per_step) / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": kernel,
                     "achieved": gbps(avg_ms), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbps(avg_ms) / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_file,
                     "bytes_per_launch": kv_bytes, "avg_ms": avg_ms, "avg_ms_basis": basis,
                     "profile_avg_ms": None if prof_ns is None else prof_ns * 1e-6,
                     "frac_profile": None if prof_ns is None else gbps(prof_ns * 1e-6) / HBM_PEAK_GBS,
                     "live": {"event_pair_raw_avg_ms": raw_avg_ms,
                              "frac_event_pair_raw": gbps(raw_avg_ms) / HBM_PEAK_GBS,
                              "empty_event_pair_avg_ms": empty_avg_ms,
                              "event_pair_minus_empty_avg_ms": net_avg_ms,
                              "frac_event_pair_minus_empty": gbps(net_avg_ms) / HBM_PEAK_GBS,
                              "median_raw_ms": raw_ms[len(raw_ms) // 2], "probe_steps": n_probe,
                              "timed_with": "HIP event pair recorded by the library on the launch stream "
                                            "around the kernel, in eager steps of this run"}},
    }
    out["roofline"]["read_only_probe"] = read_ceiling(pk, torch, geo, layers, run.main)
    if with_cpu:
        n_cpu = args.cpu_steps if args.cpu_steps > 0 else min(n_layers, 8)
        per_step, n_done, secs = cpu_baseline(torch, wl, layers, n_cpu)
        out["cpu_baseline"] = {"value": geo.B * geo.tq / per_step, "unit": "queries/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "kind": "oracle",
                               "sample": "%d steps of %s (%d layer instances, repeated for %.1f s): "
                                         "route+attend+utility, selected shards copied to host"
                                         % (n_done, config, min(n_cpu, n_layers), secs)}
    del layers, raw, shared, run, graph
    gc.collect()
    torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build holds all expert shards on a single MI355X "
              "and has no multi-GPU path; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2508_06526_amd as pk

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)
    pk.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.empty(n, device=dev, dtype=torch.uint8).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "launches": 8}))
        return
    with_cpu = not args.no_cpu and args.cpu_steps != 0
    out = measure(args, args.config, args.steps, args.warmup, with_cpu,
                  max(MIN_PROBE_STEPS, min(args.steps, 512)))
    plain = not (args.balance or args.compress or args.policy != "none" or args.k > 0 or args.rank >= 0)
    if not args.no_others and plain and args.config == "c3_long_context":
        # the other workloads, briefly, in the same launch structure (their own lines, not `value`)
        others = {}
        for name in OTHER_WORKLOADS:
            r = measure(args, name, 256, 32, False, 64, quiet=True)
            rf = r["roofline"]
            others[name] = {"step_us": r["ms_per_step"] * 1e3, "queries_per_s": r["value"],
                            "step_frac_of_hbm_peak": r["step_frac_of_hbm_peak"],
                            "kernel": rf["kernel"], "kernel_frac": rf["frac"], "kernel_avg_ms": rf["avg_ms"],
                            "kernel_frac_basis": rf["avg_ms_basis"],
                            "kernel_frac_event_pair_raw": rf["live"]["frac_event_pair_raw"], "steps": r["steps"]}
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
