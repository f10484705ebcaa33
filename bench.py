#!/usr/bin/env python3
"""Benchmark of one draft-tree speculative step (dt_build_tree + dt_tree_attention + dt_accept).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--copies 16] [--eager] [--per-config 3,4,5]

Prints ONE JSON line.  The headline is tree-verify steps/s on the Llama-3-8B-shaped configuration
(TT=60, d=6, k=10, batch 1, bf16); beside it go the HBM (or MFMA) roofline of the kernel that takes the most
time, measured with HIP events attached to every dispatch of a profiled pass, the same measurement in short
for the other bf16 configurations (`per_config`), and the CPU oracle timed on the host cores on the same inputs.

Inputs are synthetic and resident in HBM before any timed region.  A timed loop rotates over `copies`
distinct input sets (16 x 34 MB > the 256 MB last-level cache) so that every step streams its logits and KV
from HBM.  The rotation is captured once in a HIP graph and replayed (a step is three library calls = seven
kernels; launch overhead would otherwise be most of a 50 us step); --eager times plain stream launches.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0        # dense bf16, published
STEP_KERNEL_IDS = range(7)            # draft rows, row merge, tree, attention, attention combine, target rows, accept


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def step_bytes(cfg, trees_n):
    """Algorithmic HBM bytes of one step: every logit once, prefix+tree K/V once, Q in, O out."""
    e = cfg.elem_bytes()
    tot = 0
    for b in range(cfg.B):
        N, L = trees_n[b], cfg.prefix_len[b]
        tot += e * cfg.V * (cfg.n_rows(b) + N)
        tot += e * 2 * cfg.Hkv * cfg.D * (L + N)
        tot += e * 2 * N * cfg.Hq * cfg.D
    return tot


def pct(v, q):
    return round(v[min(len(v) - 1, int(q * len(v)))], 3)


class Workload:
    """One configuration on the device: `copies` independent input sets, the tree-dependent target rows built
    from the device's own tree, argument lists marshalled once."""

    def __init__(self, ci, copies, kv_head_major=False):
        import torch

        import dt_synth
        from paper_2601_12212_amd.step import Step
        t0 = time.time()
        self.cfg = cfg = dt_synth.config(ci)
        self.tdtype = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        self.R = max(1, copies)
        self.drafts = [dt_synth.draft_rows(cfg, b) for b in range(cfg.B)]
        self.steps = []
        for _ in range(self.R):
            st = Step(cfg.params, cfg.prefix_len, cfg.Hq, cfg.Hkv, cfg.D, cfg.V, dtype=self.tdtype, mode=cfg.mode,
                      temperature=cfg.temperature, philox_seed=cfg.philox_seed, kv_head_major=kv_head_major)
            dt_synth.fill_draft_and_qkv(st, cfg, self.drafts)
            self.steps.append(st)
        # the target rows follow the tree (row of node i = draft row the node owns + noise): build once
        self.steps[0].build_tree()
        torch.cuda.synchronize()
        self.trees = [self.steps[0].tree(b) for b in range(cfg.B)]
        self.targets = [dt_synth.target_rows(cfg, b, self.trees[b]["src_row"], self.drafts[b]) for b in range(cfg.B)]
        for st in self.steps:
            for b in range(cfg.B):
                st.set_target(b, self.targets[b])
            st.prepare()
        torch.cuda.synchronize()
        self.n_nodes = [t["n_nodes"] for t in self.trees]
        self.bytes_step = step_bytes(cfg, self.n_nodes)
        e = cfg.elem_bytes()
        self.kbytes = {"rows_target_chunk": e * cfg.V * sum(self.n_nodes),
                       "rows_draft_chunk": e * cfg.V * sum(cfg.n_rows(b) for b in range(cfg.B)),
                       "attention": sum(e * 2 * cfg.Hkv * cfg.D * (cfg.prefix_len[b] + self.n_nodes[b]) +
                                        e * 2 * self.n_nodes[b] * cfg.Hq * cfg.D for b in range(cfg.B))}
        self.attn_flops = sum(4.0 * self.n_nodes[b] * cfg.Hq * (cfg.prefix_len[b] + self.n_nodes[b]) * cfg.D
                              for b in range(cfg.B))
        log("setup %.1fs: %s, n_nodes=%s, %.1f MB/step, %d input copies"
            % (time.time() - t0, cfg.name, self.n_nodes if cfg.B <= 4 else "%d..%d" % (min(self.n_nodes), max(self.n_nodes)),
               self.bytes_step / 1e6, self.R))

    def run_range(self, stream, i0, n):
        for i in range(i0, i0 + n):
            self.steps[i % self.R].run_prepared(stream, i)

    def capture(self, only_set=None):
        """The R steps of one rotation (or R times the step of one input set) as a HIP graph."""
        import torch
        self.run_range(torch.cuda.current_stream().cuda_stream, 0, self.R)      # first touches before capture
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            gs = torch.cuda.current_stream().cuda_stream
            for i in range(self.R):
                self.steps[i if only_set is None else only_set].run_prepared(gs, i)
        return g

    def replay_times(self, g, n):
        """Per-step microseconds of n single replays, each bracketed by its own HIP event pair, sorted."""
        import torch
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for a, b in evs:
            a.record()
            g.replay()
            b.record()
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) * 1e3 / self.R for a, b in evs)

    def kernel_times(self, P):
        """Average duration of every kernel of the step over P eager steps, from the event pair on each dispatch."""
        import torch

        import paper_2601_12212_amd as dt
        P = max(self.R, P)
        dt.dt_profile_enable(P * 8)
        self.run_range(torch.cuda.current_stream().cuda_stream, 0, P)
        torch.cuda.synchronize()
        kern = {}
        for kid in STEP_KERNEL_IDS:
            name, ms, n = dt.dt_profile_read(kid)
            if n:
                kern[name] = dict(avg_us=ms * 1e3 / n, launches_per_step=n / P)
        dt.dt_profile_enable(0)
        for name, v in kern.items():
            if name in self.kbytes:
                v["bytes"] = self.kbytes[name]
                v["gbps"] = self.kbytes[name] / (v["avg_us"] * 1e-6) / 1e9
        if "attention" in kern:
            kern["attention"]["flops"] = self.attn_flops
            kern["attention"]["tflops"] = self.attn_flops / (kern["attention"]["avg_us"] * 1e-6) / 1e12
        return kern, P

    def traffic(self):
        """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if there is one."""
        out = {}
        path = os.path.join(ROOT, "profiles", "pmc_%s.json" % self.cfg.name)
        if os.path.exists(path):
            pk = json.load(open(path))["kernels"]
            for ours, prefix in (("rows_target_chunk", "dt::row_argmax_kernel"), ("rows_draft_chunk", "dt::row_stream_kernel"),
                                 ("attention", "dt::attn_")):
                # the merge / combine launches of the attention are timed as a kernel of their own
                hit = [v for k, v in pk.items() if k.startswith(prefix) and "merge" not in k and "combine" not in k]
                if hit:
                    out[ours] = sum(v["hbm_bytes"] for v in hit)
        return out, (os.path.relpath(path, ROOT) if out else None)

    def rooflines(self, kern, P):
        """Roofline object of the kernel that takes the most time, of every data-moving kernel, and of the
        latency-bound kernels (no roofline applies: their time is dependent trips to memory and LDS)."""
        import torch
        traffic, source = self.traffic()
        ridge = MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBPS       # flops per byte above which the MFMA peak binds

        def roof(name):
            v = kern[name]
            if name not in self.kbytes:
                return {"bound": "latency", "kernel": name, "achieved": None, "peak": None, "unit": None, "frac": None,
                        "traffic": None, "avg_us": round(v["avg_us"], 3),
                        "note": "a few KB per launch; time is dependent trips to memory / LDS, not bytes or flops"}
            if name == "attention" and self.tdtype == torch.bfloat16 and self.attn_flops / self.kbytes[name] > ridge:
                return {"bound": "mfma", "kernel": name, "achieved": round(v["tflops"], 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(v["tflops"] / MFMA_BF16_PEAK_TFLOPS, 4),
                        "traffic": traffic.get(name), "flops_per_launch": self.attn_flops,
                        "bytes_per_launch": self.kbytes[name], "gbps": round(v["gbps"], 1), "avg_us": round(v["avg_us"], 3)}
            r = {"bound": "hbm", "kernel": name, "achieved": round(v["gbps"], 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                 "frac": round(v["gbps"] / HBM_PEAK_GBPS, 4), "traffic": traffic.get(name),
                 "bytes_per_launch": self.kbytes[name], "avg_us": round(v["avg_us"], 3)}
            if name == "attention" and self.tdtype == torch.bfloat16:
                r["tflops"] = round(v["tflops"], 1)
                r["frac_of_mfma_peak"] = round(v["tflops"] / MFMA_BF16_PEAK_TFLOPS, 4)
            return r

        cost = lambda n: kern[n]["avg_us"] * kern[n]["launches_per_step"]
        movers = [n for n in kern if n in self.kbytes]
        dominant = roof(max(movers, key=cost))                    # the kernel the `roofline` object is about
        dominant["timing"] = "HIP events attached to each dispatch, %d profiled steps, %d rotating input sets" % (P, self.R)
        dominant["traffic_source"] = source
        longest = max(kern, key=cost)
        return dominant, [roof(n) for n in sorted(movers, key=lambda n: -self.kbytes[n])], roof(longest)


def summary(W, replays, P):
    """Short measurement of a configuration: graph-replay step time, bytes, fractions, per-kernel times."""
    g = W.capture()
    for _ in range(3):
        g.replay()
    v = W.replay_times(g, replays)
    del g
    kern, P = W.kernel_times(P)
    dominant, streams, longest = W.rooflines(kern, P)
    med = pct(v, 0.5)
    gbps = W.bytes_step / (med * 1e-6) / 1e9
    out = {"workload": W.cfg.name, "batch": W.cfg.B, "step_us_median": med, "step_us_p10": pct(v, 0.1),
           "step_us_p90": pct(v, 0.9), "replays": len(v), "steps_per_replay": W.R, "steps_per_s": round(1e6 / med, 1),
           "bytes_per_step": W.bytes_step, "hbm_gbps_step": round(gbps, 1), "frac_hbm_peak_step": round(gbps / HBM_PEAK_GBPS, 4),
           "kernels_us": {k: round(x["avg_us"], 2) for k, x in kern.items()},
           "roofline": dominant, "streams": streams, "longest_kernel": longest}
    if "attention" in kern and "tflops" in kern["attention"]:
        out["attention_frac_mfma_peak"] = round(kern["attention"]["tflops"] / MFMA_BF16_PEAK_TFLOPS, 4)
    log("  %s: step %.1f us median (%d replays of %d), %.0f GB/s = %.1f%% of peak; kernels %s"
        % (W.cfg.name, med, len(v), W.R, gbps, 100 * gbps / HBM_PEAK_GBPS, out["kernels_us"]))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--copies", type=int, default=16)
    ap.add_argument("--eager", action="store_true", help="plain stream launches instead of HIP graph replay")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=400)
    ap.add_argument("--per-config", default="3,4,5",
                    help="configurations measured in short after the headline one ('' or 'none': skip)")
    ap.add_argument("--attention-layers", type=int, default=32,
                    help="layers of the separately timed all-layer attention graph (0: skip it)")
    ap.add_argument("--sampled-verify", type=int, default=1,
                    help="also time dt_accept in its distribution-preserving mode (0: skip)")
    ap.add_argument("--policy-features", type=int, default=3 * 4096,
                    help="state size of the separately timed policy step (0: skip it)")
    ap.add_argument("--streaming-build", type=int, default=1,
                    help="also time the level-at-a-time build of the same tree (0: skip)")
    ap.add_argument("--commit-layers", type=int, default=32,
                    help="layers of the separately timed input update (0: skip it)")
    ap.add_argument("--topk-k32", type=int, default=1,
                    help="also time the row top-k at the widest action (k = 32), outside the step (0: skip)")
    ap.add_argument("--kv-layout", choices=["token", "head"], default="token",
                    help="prefix caches as [token, kv head, D] or [kv head, token, D]")
    ap.add_argument("--launch-floor", type=int, default=1,
                    help="also time a graph of dependent one-element kernels (the cost of the step's seven launches alone)")
    ap.add_argument("--read-ceiling-mb", type=int, default=2048,
                    help="size of the read-only pass that measures what a plain stream reaches here (0: skip)")
    ap.add_argument("--calibration-copy-mb", type=int, default=0,
                    help="also run a plain device copy of this many MB (a kernel of known traffic, for scaling "
                         "rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding "
            "in this path). Re-run with --gpus 1." % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch

    import dt_synth
    import paper_2601_12212_amd as dt

    dt.load_library()                    # no fallback: raises if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dt.dt_init()
    W = Workload(args.config, args.copies, args.kv_layout == "head")
    cfg, R, steps, tdtype = W.cfg, W.R, W.steps, W.tdtype
    n_nodes, bytes_step = W.n_nodes, W.bytes_step
    K = -(-args.steps // R) * R              # whole rotations, never fewer steps than asked for
    Wm = -(-args.warmup // R) * R
    sptr = torch.cuda.current_stream().cuda_stream

    # ---- timed region -----------------------------------------------------------------------------
    mode, graph = "eager", None
    if not args.eager:
        try:
            graph = W.capture()
            mode = "hipgraph"
        except Exception as ex:                  # noqa: BLE001 -- report and fall back to eager launches
            log("HIP graph capture failed (%s); timing eager launches" % ex)
            graph = None
    spread, cache_warm = None, None
    if graph is not None:
        for _ in range(Wm // R):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K // R):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        # the headline: median over single replays (one rotation of R steps each), HIP events on the replay's stream
        v = W.replay_times(graph, max(20, min(200, K // R)))
        spread = {"p10_us": pct(v, 0.10), "median_us": pct(v, 0.50), "p90_us": pct(v, 0.90), "samples": len(v),
                  "what": "HIP events around single graph replays of %d steps (one per input set), per step" % R}
        ms_per_step = spread["median_us"] * 1e-3
        # the Infinity Cache holds a small configuration's whole input set: the same step R times on set 0
        try:
            gw = W.capture(only_set=0)
            for _ in range(3):
                gw.replay()
            torch.cuda.synchronize()
            v = W.replay_times(gw, max(20, min(200, K // R)))
            cache_warm = {"median_us": pct(v, 0.50), "p10_us": pct(v, 0.10), "p90_us": pct(v, 0.90),
                          "steps_per_s": round(1e6 / pct(v, 0.50), 1), "input_bytes": bytes_step,
                          "what": "the same graph on one input set only (re-read from the last-level cache when it "
                                  "fits); not the headline value"}
            del gw
        except Exception as ex:                  # noqa: BLE001
            log("cache-warm graph failed (%s)" % ex)
        log("  step time p10 / median / p90: %.2f / %.2f / %.2f us; one input set: %s us; wall over %d steps: %.2f us/step" %
            (spread["p10_us"], spread["median_us"], spread["p90_us"], cache_warm["median_us"] if cache_warm else "-",
             K, wall * 1e6 / K))
    else:
        W.run_range(sptr, 0, Wm)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        W.run_range(sptr, Wm, K)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms_per_step = wall * 1e3 / K
    steps_per_s = 1e3 / ms_per_step

    # ---- eager reference number (always) and per-kernel durations with HIP events --------------
    n_e = min(K, 500)
    W.run_range(sptr, 0, min(Wm, 50))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    W.run_range(sptr, 0, n_e)
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) * 1e3 / n_e

    kern, P = W.kernel_times(args.profile_steps)
    for name, v in kern.items():
        log("  kernel %-20s avg %8.2f us  x%.0f/step%s" % (name, v["avg_us"], v["launches_per_step"],
                                                            "  %.0f GB/s" % v["gbps"] if "gbps" in v else ""))
    roofline, roofline_all, longest = W.rooflines(kern, P)
    e = cfg.elem_bytes()

    # ---- what a plain read-only pass reaches on this machine (context for the fractions of the 8 TB/s
    #      peak, never a denominator of `frac`): torch's row-wise maximum of a [4096, n] fp32 matrix of 2 GiB ------
    ceiling = None
    if args.read_ceiling_mb > 0:
        probe = torch.ones((4096, args.read_ceiling_mb * (1 << 20) // 4 // 4096), dtype=torch.float32, device="cuda")
        best = None
        for _ in range(6):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            probe.amax(dim=1)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None or ms < best else best
        ceiling = {"gbps": round(probe.numel() * 4 / (best * 1e-3) / 1e9, 1), "bytes": probe.numel() * 4,
                   "how": "torch.amax(dim=1) over a [4096, n] fp32 matrix, best of 6, torch events; context only"}
        del probe
        log("  read-only pass over %d MiB: %.0f GB/s" % (args.read_ceiling_mb, ceiling["gbps"]))

    # ---- what seven dependent launches cost on this machine when the kernels do nothing (context for the batch-1
    #      step, which is seven dependent launches): a HIP graph of 7 x 16 one-element torch kernels ----------------
    launch_floor = None
    if args.launch_floor > 0 and not args.eager:
        one = torch.zeros(1, dtype=torch.float32, device="cuda")
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for _ in range(3):
                one.add_(1.0)
            torch.cuda.synchronize()
            gf = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gf, stream=side):
                for _ in range(7 * 16):
                    one.add_(1.0)
        torch.cuda.synchronize()
        ts = []
        for _ in range(24):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            gf.replay()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3 / (7 * 16))
        ts.sort()
        launch_floor = {"us_per_dependent_launch": round(ts[len(ts) // 2], 3), "us_per_7_launches": round(7 * ts[len(ts) // 2], 2),
                        "how": "graph replay of 112 dependent one-element torch kernels, median of 24; context only"}
        del gf
        log("  seven dependent empty launches in a graph: %.2f us" % launch_floor["us_per_7_launches"])

    # ---- the input update that follows the step (not part of the timed step): all layers' K/V rows of
    #      the accepted paths appended to the caches; timed on its own with dispatch-attached events ----
    commit = None
    if args.commit_layers > 0:
        st0 = steps[0]
        nl, cap_rows, L0 = args.commit_layers, 16, 4     # the kernel's work does not depend on the prefix length
        i64 = dict(dtype=torch.int64, device="cuda")
        tk = [torch.randn((cfg.B, st0.TT_cap, cfg.Hkv, cfg.D), device="cuda").to(tdtype) for _ in range(2 * nl)]
        ck = [[torch.zeros((cap_rows, cfg.Hkv, cfg.D), dtype=tdtype, device="cuda") for _ in range(cfg.B)]
              for _ in range(2 * nl)]
        ptr_rows = lambda rows: torch.tensor([[t.data_ptr() for t in row] for row in rows], **i64)
        ktp = torch.tensor([t.data_ptr() for t in tk[:nl]], **i64)
        vtp = torch.tensor([t.data_ptr() for t in tk[nl:]], **i64)
        kpp, vpp = ptr_rows(ck[:nl]), ptr_rows(ck[nl:])
        plen = torch.full((cfg.B,), L0, dtype=torch.int32, device="cuda")
        pcap = torch.full((cfg.B,), cap_rows, dtype=torch.int32, device="cuda")
        new_len = torch.empty_like(plen)
        nroot = torch.empty_like(plen)
        n_c = 200
        dt.dt_profile_enable(n_c + 8)
        for _ in range(n_c):
            dt.dt_commit(tk[0], cfg.Hkv, cfg.D, ktp, vtp, kpp, vpp, plen, pcap, cfg.Hkv * cfg.D, cfg.D, st0.n_nodes,
                         st0.path_nodes, st0.accept_len, st0.out_tokens, st0.TT_cap, new_len, nroot)
        torch.cuda.synchronize()
        name, ms, n = dt.dt_profile_read(8)
        dt.dt_profile_enable(0)
        rows = int((st0.accept_len.cpu() + 1).sum())
        cbytes = 2 * 2 * nl * rows * cfg.Hkv * cfg.D * e            # read + write, K and V, every layer
        commit = {"avg_us": round(ms * 1e3 / max(n, 1), 3), "layers": nl, "rows": rows, "bytes": cbytes,
                  "gbps": round(cbytes / (ms * 1e-3 / max(n, 1)) / 1e9, 1), "in_timed_step": False}
        log("  kernel %-20s avg %8.2f us  (%d layers, %d accepted-path rows, %.2f MB moved; outside the timed step)"
            % ("commit", commit["avg_us"], nl, rows, cbytes / 1e6))

    # ---- all layers' attention of one verification pass as one HIP graph (outside the timed step; the
    #      layers share this step's Q/K/V buffers, so it measures launch chaining, not cache behaviour
    #      across distinct layer data) ---------------------------------------------------------------------
    layers_graph = None
    if args.attention_layers > 0 and not args.eager:
        try:
            nl_a = args.attention_layers
            side = torch.cuda.Stream()
            with torch.cuda.stream(side):
                steps[0].tree_attention()
                torch.cuda.synchronize()
                lg = torch.cuda.CUDAGraph()
                with torch.cuda.graph(lg, stream=side):
                    for _ in range(nl_a):
                        steps[0].tree_attention()
            for _ in range(3):
                lg.replay()
            torch.cuda.synchronize()
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record()
            for _ in range(20):
                lg.replay()
            a1.record()
            torch.cuda.synchronize()
            per_layer = a0.elapsed_time(a1) * 1e3 / (20 * nl_a)
            layers_graph = {"layers": nl_a, "us_per_layer": round(per_layer, 3), "in_timed_step": False}
            log("  attention of %d layers in one graph: %.2f us per layer; outside the timed step" % (nl_a, per_layer))
        except Exception as ex:                  # noqa: BLE001
            log("attention layer graph failed: %s" % ex)

    # ---- distribution-preserving verification (every node draws the target's own token), outside the
    #      timed step: the same target rows, mode DT_ACCEPT_SAMPLED ---------------------------------------
    sampled = None
    if args.sampled_verify:
        st0 = steps[0]
        n_v = 200
        call = lambda i: dt.dt_accept(dt.DT_ACCEPT_SAMPLED, 1.0, st0.target_logits, st0.n_nodes, st0.tokens,
                                      st0.parents, st0.depth, st0.logp, st0.anc_mask, cfg.philox_seed, i,
                                      st0.accept_len, st0.best_node, st0.path_nodes, st0.out_tokens,
                                      st0.node_argmax, st0.ws)
        for i in range(5):
            call(i)
        dt.dt_profile_enable(3 * n_v + 8)
        for i in range(n_v):
            call(i)
        torch.cuda.synchronize()
        t_rows, t_samp, t_acc = (dt.dt_profile_read(kid) for kid in (5, 11, 6))
        dt.dt_profile_enable(0)
        us = lambda t: round(t[1] * 1e3 / max(t[2], 1), 3)
        sampled = {"rows_target_chunk_us": us(t_rows), "node_sample_us": us(t_samp), "accept_us": us(t_acc),
                   "in_timed_step": False}
        log("  sampled verification: target rows %.2f us, per-node draws %.2f us, accept %.2f us; outside the timed step"
            % (sampled["rows_target_chunk_us"], sampled["node_sample_us"], sampled["accept_us"]))
        steps[0].accept(0)          # leave the greedy result behind for what follows
        torch.cuda.synchronize()

    # ---- action selection (policy MLP + action cache), outside the timed step: evaluated at every call
    #      here (interval 1); with the paper's interval of 30 it runs once per 30 steps -------------------
    policy = None
    if args.policy_features > 0:
        F, H = args.policy_features, 128
        table = torch.tensor(dt.dt_action_table(), dtype=torch.int32, device="cuda")
        A = table.shape[0]
        g = torch.Generator(device="cuda").manual_seed(5)
        rn = lambda *sh: torch.randn(*sh, generator=g, device="cuda")
        Wts = [rn(F, H) / F ** 0.5, rn(H) * 0.1, rn(H, H) / H ** 0.5, rn(H) * 0.1, rn(H, A) / H ** 0.5, rn(A) * 0.1]
        feat = rn(cfg.B, F).to(tdtype)
        i32 = dict(dtype=torch.int32, device="cuda")
        cs, ca = torch.zeros(cfg.B, **i32), torch.full((cfg.B,), -1, **i32)
        pout = torch.zeros((cfg.B, 3), **i32)
        wsp = torch.empty(dt.dt_policy_workspace_bytes(cfg.B, F, H), dtype=torch.uint8, device="cuda")
        n_p = 200
        for _ in range(5):
            dt.dt_policy_step(feat, *Wts, table, 1, 0, 0, 0, cs, ca, pout, None, None, None, wsp)
        dt.dt_profile_enable(2 * n_p + 8)
        for i in range(n_p):
            dt.dt_policy_step(feat, *Wts, table, 1, 0, 0, i, cs, ca, pout, None, None, None, wsp)
        torch.cuda.synchronize()
        _, ms1, n1 = dt.dt_profile_read(9)
        _, ms2, n2 = dt.dt_profile_read(10)
        dt.dt_profile_enable(0)
        pbytes = F * H * 4 + cfg.B * F * e
        policy = {"layer1_us": round(ms1 * 1e3 / max(n1, 1), 3), "head_us": round(ms2 * 1e3 / max(n2, 1), 3),
                  "features": int(F), "hidden": int(H), "actions": int(A), "layer1_bytes": int(pbytes),
                  "layer1_gbps": round(pbytes / (ms1 * 1e-3 / max(n1, 1)) / 1e9, 1), "in_timed_step": False}
        log("  policy: layer 1 %.2f us (%.1f MB, %.0f GB/s), head %.2f us; %d features, %d actions; outside the timed step"
            % (policy["layer1_us"], pbytes / 1e6, policy["layer1_gbps"], policy["head_us"], F, A))

    # ---- the same tree built one level at a time (a draft model would run between the calls); outside
    #      the timed step.  Level l's rows are the draft rows the one-shot build reads for that level. ----
    streaming = None
    if args.streaming_build and len(set(cfg.params)) == 1:
        TT0, d0, k0 = cfg.params[0]
        st0 = steps[0]
        rows_b = [st0.draft_logits[int(st0.host_row_off[b]):int(st0.host_row_off[b + 1])] for b in range(cfg.B)]
        lvl = [torch.stack([r[0] for r in rows_b])]
        for l in range(2, d0 + 1):
            lvl.append(torch.cat([r[1 + (l - 2) * k0:1 + (l - 1) * k0] for r in rows_b]).contiguous())
        state = torch.zeros(dt.dt_level_state_bytes(cfg.B), dtype=torch.uint8, device="cuda")
        ws2 = torch.empty(dt.dt_workspace_bytes(cfg.B, cfg.B * k0, cfg.V, st0.TT_cap, 1, 1), dtype=torch.uint8,
                          device="cuda")
        i32 = dict(dtype=torch.int32, device="cuda")
        nx = torch.zeros(cfg.B, **i32)
        ex = [torch.zeros((cfg.B, 32), **i32) for _ in range(4)]
        em = torch.zeros((cfg.B, 32, 4), dtype=torch.int64, device="cuda")
        outs = [torch.zeros_like(st0.n_nodes), torch.zeros_like(st0.tokens), torch.zeros_like(st0.parents),
                torch.zeros_like(st0.depth), torch.zeros_like(st0.score), torch.zeros_like(st0.logp),
                torch.zeros_like(st0.src_row), torch.zeros_like(st0.anc_mask)]

        def build_by_levels():
            for l in range(1, d0 + 1):
                dt.dt_expand_level(l, st0.params, lvl[l - 1], k0, st0.prefix_len, st0.TT_cap, state, nx, *ex, em, ws2)
            dt.dt_finish_tree(st0.params, cfg.V, st0.root_token, st0.TT_cap, state, *outs)

        for _ in range(5):
            build_by_levels()
        torch.cuda.synchronize()
        same = bool(torch.equal(outs[1], st0.tokens) and torch.equal(outs[2], st0.parents) and
                    torch.equal(outs[0], st0.n_nodes))
        n_s = 100
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record()
        for _ in range(n_s):
            build_by_levels()
        s1.record()
        torch.cuda.synchronize()
        streaming = {"us_per_build": round(s0.elapsed_time(s1) * 1e3 / n_s, 2), "levels": d0, "calls": d0 + 1,
                     "launches": 3 * d0 + 1, "same_tree_as_one_shot": same, "in_timed_step": False}
        log("  level-at-a-time build: %.1f us for %d levels + finish (%d launches, eager); same tree: %s"
            % (streaming["us_per_build"], d0, 3 * d0 + 1, same))

    # ---- the row top-k at the widest action of the paper's action space (k = 32; the step above uses the
    #      configuration's own k), outside the timed step: TT=128, d=8 gives 225 draft rows -------------------
    topk32 = None
    if args.topk_k32 and tdtype == torch.bfloat16:
        rows32, k32 = 225, 32
        g = torch.Generator(device="cuda").manual_seed(9)
        x = (torch.randn((rows32, cfg.V), generator=g, device="cuda") * 3).to(torch.bfloat16)
        lse = torch.empty(rows32, dtype=torch.float32, device="cuda")
        ws3 = torch.empty(dt.dt_workspace_bytes(1, rows32, cfg.V, 8, 1, 64), dtype=torch.uint8, device="cuda")
        res = {}
        for kk in (10, k32):
            v_ = torch.empty((rows32, kk), dtype=torch.float32, device="cuda")
            i_ = torch.empty((rows32, kk), dtype=torch.int32, device="cuda")
            for _ in range(3):
                dt.dt_topk_rows(x, kk, v_, i_, lse, ws3)
            dt.dt_profile_enable(2 * 50 + 8)
            for _ in range(50):
                dt.dt_topk_rows(x, kk, v_, i_, lse, ws3)
            torch.cuda.synchronize()
            _, ms_s, n_s = dt.dt_profile_read(7)
            _, ms_m, n_m = dt.dt_profile_read(1)
            dt.dt_profile_enable(0)
            res["k%d" % kk] = {"stream_us": round(ms_s * 1e3 / max(n_s, 1), 2), "select_us": round(ms_m * 1e3 / max(n_m, 1), 2)}
        topk32 = {"rows": rows32, "V": cfg.V, **res, "in_timed_step": False}
        log("  row top-k of %d rows: k=10 stream %.2f + select %.2f us; k=32 stream %.2f + select %.2f us; outside the timed step"
            % (rows32, res["k10"]["stream_us"], res["k10"]["select_us"], res["k32"]["stream_us"], res["k32"]["select_us"]))

    if args.calibration_copy_mb > 0:
        n = args.calibration_copy_mb * 1000 * 1000 // 4
        src = torch.arange(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(4):
            dst.copy_(src)          # reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        log("calibration copy: 4 launches of %d bytes read + %d bytes written" % (n * 4, n * 4))

    # ---- the other configurations, in short (graph replay, median of >= 20 replays, per-kernel events) -----
    per_config = []
    wanted = [int(x) for x in args.per_config.split(",") if x.strip().isdigit()]
    main_summary = {"workload": cfg.name, "batch": cfg.B, "step_us_median": round(ms_per_step * 1e3, 3),
                    "steps_per_s": round(steps_per_s, 1), "bytes_per_step": bytes_step,
                    "frac_hbm_peak_step": round(bytes_step / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                    "kernels_us": {k: round(x["avg_us"], 2) for k, x in kern.items()}, "roofline": roofline,
                    "longest_kernel": longest}
    if "attention" in kern and "tflops" in kern["attention"]:
        main_summary["attention_frac_mfma_peak"] = round(kern["attention"]["tflops"] / MFMA_BF16_PEAK_TFLOPS, 4)
    per_config.append(main_summary)
    if wanted and not args.eager:
        del graph
        W.steps = steps = None                   # free the headline configuration's buffers
        torch.cuda.empty_cache()
        for ci in wanted:
            if ci == args.config:
                continue
            try:
                Wc = Workload(ci, 16 if ci <= 3 else 2, args.kv_layout == "head")
                per_config.append(summary(Wc, 24, 48))
                Wc.steps = None
                del Wc
                torch.cuda.empty_cache()
            except Exception as ex:              # noqa: BLE001
                log("per-config measurement of configuration %d failed: %s" % (ci, ex))

    # ---- the oracle on the host cores, same inputs (nothing but the oracle inside the timed legs) -------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ref
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        qkv = [dt_synth.qkv(cfg, b) for b in range(cfg.B)]
        legs = {"build_tree": 0.0, "tree_attention": 0.0, "accept": 0.0}
        done, ok = 0, True
        budget_start = time.perf_counter()
        while done < 8 and (time.perf_counter() - budget_start) < 12.0:
            for b in range(cfg.B):
                TT, d, k = cfg.params[b]
                t0 = time.perf_counter()
                t = ref.build_tree(W.drafts[b], TT, d, k, dt_synth.root_token(cfg, b))
                t1 = time.perf_counter()
                q, kt, vt, kp, vp = qkv[b]
                N = t["n_nodes"]
                ref.tree_attention(q[:N], kt[:N], vt[:N], kp, vp, t["anc_mask"], 1.0 / float(np.sqrt(cfg.D)))
                t2 = time.perf_counter()
                ok = ok and np.array_equal(t["src_row"], W.trees[b]["src_row"])   # so the GPU's target rows apply
                ref.accept(cfg.mode, W.targets[b], t["tokens"], t["parents"], t["depth"], logp=t["logp"],
                           temperature=cfg.temperature, seed=cfg.philox_seed, step=done, seq=b)
                t3 = time.perf_counter()
                legs["build_tree"] += t1 - t0
                legs["tree_attention"] += t2 - t1
                legs["accept"] += t3 - t2
            done += 1
        cpu_s = sum(legs.values()) / done
        cpu = {"value": round(1.0 / cpu_s, 4), "unit": "steps/s", "cores": threads, "kind": "oracle",
               "sample": "%d whole steps of the same workload, inputs generated beforehand (tree build single-threaded, "
                         "attention and row scans OpenMP over %d threads)" % (done, threads),
               "seconds_per_step": {k: round(v / done, 4) for k, v in legs.items()},
               "same_tree_as_gpu": bool(ok)}
        log("cpu oracle: %.3f s/step on %d threads %s" % (cpu_s, threads, cpu["seconds_per_step"]))

    out = {
        "metric": "tree_verify_steps_per_sec", "value": round(steps_per_s, 1), "unit": "steps/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": "%s: Hq=%d Hkv=%d D=%d V=%d prefix=%s (TT,d,k)=%s batch=%d, one layer's attention"
                               % (cfg.name, cfg.Hq, cfg.Hkv, cfg.D, cfg.V, cfg.prefix_len[:4], cfg.params[:4], cfg.B),
                   "launch": mode, "input_copies": R, "n_nodes": n_nodes},
        "value_is": ("1 / median step time over single HIP-graph replays (HIP events on the replay's stream)"
                     if mode == "hipgraph" else "steps / wall time of eager launches"),
        "wall_ms_per_step": round(wall * 1e3 / K, 5),
        "eager_ms_per_step": round(eager_ms, 5),
        "bytes_per_step": bytes_step,
        "hbm_gbps_step": round(bytes_step / (ms_per_step * 1e-3) / 1e9, 1),
        "pct_hbm_peak_step": round(100.0 * bytes_step / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
        "step_time_spread": spread,
        "one_input_set": cache_warm,
        "kernels": {k: {kk: (round(vv, 3) if isinstance(vv, float) else vv) for kk, vv in v.items()}
                    for k, v in kern.items()},
        "input_update": commit,
        "streaming_build": streaming,
        "policy": policy,
        "sampled_verification": sampled,
        "attention_layers_graph": layers_graph,
        "topk_k32": topk32,
        "roofline": roofline,
        "roofline_all_streams": roofline_all,
        "longest_kernel": longest,
        "per_config": per_config,
        "hbm_read_ceiling": ceiling,
        "launch_floor": launch_floor,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
