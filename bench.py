#!/usr/bin/env python3
"""Tree-verify step throughput on one MI355X.

One step = one lpp_tree_attention call (one layer) + one lpp_relaxed_verify call
for the whole batch, on synthetic inputs shaped like the LlamaGen-XXL workload
(workload config 3; see workloads/configs.py).  Inputs are resident in HBM before
the timed region; R replicas of the input set are rotated so that consecutive
steps do not find their inputs in the 256 MB last-level cache.

Prints ONE JSON line (rank 0 / the only process).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
# HBM bytes per launch (fetched + written) per workload config from rocprofv3 FETCH_SIZE / WRITE_SIZE
# runs of this script, scaled by the same counters' reading for a copy of known size (the summary and
# the commands: profiles/verify_attention_hbm_bytes_all_configs.txt).  They hold for the plain step
# (one layer, multi-head, no front end, default options); otherwise the bench reports null.
TRAFFIC = {1: {"tree_attention": 4.49e6, "relaxed_verify": 0.35e6},
           2: {"tree_attention": 5.08e6, "relaxed_verify": 3.40e6},
           3: {"tree_attention": 29.14e6, "relaxed_verify": 30.21e6},
           4: {"tree_attention": 50.37e6, "relaxed_verify": 4.19e6},
           5: {"tree_attention": 450.42e6, "relaxed_verify": 256.42e6}}
FP32_MFMA_PEAK_TFLOPS = 157.3


def algorithmic_bytes(cfg, n_parents):
    """Bytes one step has to move (each needed input read once, outputs written once)."""
    e = 2 if cfg.kv_dtype == "bf16" else 4
    B, H, M, S, Dh, V, k, N = cfg.B, cfg.H, cfg.M, cfg.S, cfg.Dh, cfg.V, cfg.k, cfg.N
    attn = 2 * B * H * S * Dh * e + 3 * B * H * M * Dh * e + 4 * B * H * M * Dh
    verify = 4 * B * V * (M + n_parents) + 4 * B * N * k
    return attn, verify


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=3, help="workload config 1..5 (3 = the metric's shape)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-rotate", action="store_true", help="one replica only (cache-resident inputs)")
    ap.add_argument("--replicas", type=int, default=0,
                    help="input replicas to rotate over (default: enough for R x working set >= 512 MB, at most 64)")
    ap.add_argument("--no-cached", action="store_true",
                    help="leave out the cache-resident pass (so that a kernel trace of this run holds HBM-resident "
                         "calls only)")
    ap.add_argument("--no-knn-timing", action="store_true", help="build the neighbour table once, untimed")
    ap.add_argument("--no-two-batches", action="store_true",
                    help="leave out the pass with two batches in flight (so that a kernel trace of this run holds "
                         "kernels that had the device to themselves only)")
    ap.add_argument("--frontend", action="store_true",
                    help="verify through lpp_relaxed_verify_sampled (guidance 3.0 + top-k 2000 fused; reads one more "
                         "target row set); not the headline configuration")
    ap.add_argument("--rule", choices=["prefix", "skip"], default="prefix",
                    help="choice of A inside B_k (lpp_relaxed_verify_opts when not the default)")
    ap.add_argument("--siblings", choices=["iid", "distinct"], default="iid",
                    help="sibling scheme (lpp_relaxed_verify_opts when not the default)")
    ap.add_argument("--layers", type=int, default=1,
                    help="attention layers per step, each on its own K/V cache (a target's layer count), through "
                         "lpp_tree_attention_layers; the headline step has one")
    ap.add_argument("--layer-loop", action="store_true",
                    help="with --layers: one lpp_tree_attention call per layer instead of lpp_tree_attention_layers")
    ap.add_argument("--kv-heads", type=int, default=0,
                    help="key/value heads shared by groups of query heads (lpp_tree_attention_gqa); 0 = multi-head")
    ap.add_argument("--out-bf16", action="store_true", help="bf16 attention output (lpp_tree_attention_gqa)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three device copies of 256 MiB (a known size to scale rocprofv3 byte counters by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 "
              "(the path shards by batch item with no exchange, nothing to measure across GPUs)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2502_06352_amd as lpp
    from workloads import (CONFIGS, static_tree, children_lists, make_codebook,
                           make_attention_inputs, make_verify_inputs)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    lpp.lib()                                     # fails loudly if liblpp.so is not built

    cfg = CONFIGS[args.config]
    parent = static_tree(cfg.branching, cfg.N)
    kids = children_lists(parent)
    n_parents = sum(1 for c in kids if c)
    tree = lpp.Tree(parent)
    B, H, M, S, Dh, V, k = cfg.B, cfg.H, cfg.M, cfg.S, cfg.Dh, cfg.V, cfg.k
    depth = max(tree.depth, 1)

    # ---- inputs (CPU, seeded) -> HBM
    E = make_codebook(cfg)
    att = make_attention_inputs(cfg)
    Hkv = args.kv_heads if args.kv_heads > 0 else H
    L = max(1, args.layers)
    gqa_call = Hkv != H or args.out_bf16
    if H % Hkv != 0:
        print("bench.py: --kv-heads must divide the head count %d" % H, file=sys.stderr)
        sys.exit(2)
    if Hkv != H:
        import dataclasses
        kv = make_attention_inputs(dataclasses.replace(cfg, H=Hkv), salt=1)
        for n in ("kc", "vc", "kt", "vt"):
            att[n] = kv[n]
            if n + "_bits" in kv:
                att[n + "_bits"] = kv[n + "_bits"]
    ver = make_verify_inputs(cfg, parent, rho=0.8)
    ver_uncond = make_verify_inputs(cfg, parent, rho=0.0, salt=100) if args.frontend else None

    def up(x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(dev)

    def up_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    dE = up(E)
    neigh = torch.empty((V, k), dtype=torch.int32, device=dev)
    knn_ws = torch.empty(lpp.lpp_build_neighbours_workspace(V, cfg.D, k), dtype=torch.uint8, device=dev)
    lpp.lpp_build_neighbours(dE, k, neigh, knn_ws)         # warm-up / result used below
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    knn_reps = 0 if args.no_knn_timing else 3
    ev[0].record()
    for _ in range(knn_reps):
        lpp.lpp_build_neighbours(dE, k, neigh, knn_ws)
    ev[1].record()
    torch.cuda.synchronize()
    knn_ms = ev[0].elapsed_time(ev[1]) / knn_reps if knn_reps else None
    del knn_ws

    if args.calibrate_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    attn_bytes, verify_bytes = algorithmic_bytes(cfg, n_parents)
    if gqa_call:
        e = 2 if cfg.kv_dtype == "bf16" else 4
        attn_bytes = (2 * B * Hkv * S * Dh * e + B * (H + 2 * Hkv) * M * Dh * e
                      + (2 if args.out_bf16 else 4) * B * H * M * Dh)
    if args.frontend:
        verify_bytes += 4 * B * V * M            # the null-conditioned target rows
    step_bytes = L * attn_bytes + verify_bytes
    R = 1 if args.no_rotate else max(2, int(np.ceil(512e6 / step_bytes)))
    R = min(R, 64)
    if args.replicas > 0 and not args.no_rotate:
        R = args.replicas
    reps = []
    for r in range(R):
        d = {}
        if cfg.kv_dtype == "bf16":
            for n in ("q", "kc", "vc", "kt", "vt"):
                d[n] = up_bf16(att[n + "_bits"])
        else:
            for n in ("q", "kc", "vc", "kt", "vt"):
                d[n] = up(att[n])
        for n in ("target_logits", "drafter_logits", "tokens", "u_accept", "u_final"):
            d[n] = up(ver[n])
        if args.frontend:
            d["uncond_logits"] = up(ver_uncond["target_logits"])
        # further layers: device copies of the first layer's tensors (distinct addresses, same values)
        d["layers"] = [{n: (d[n] if l == 0 else d[n].clone()) for n in ("q", "kc", "vc", "kt", "vt")} for l in range(L)]
        d["out_attn"] = torch.empty((B, H, M, Dh), dtype=torch.bfloat16 if args.out_bf16 else torch.float32,
                                    device=dev)
        # (several layers: one call, every layer with an output of its own)
        d["layer_table"] = [dict(q=x["q"], k_cache=x["kc"], v_cache=x["vc"], k_tree=x["kt"], v_tree=x["vt"],
                                 out=d["out_attn"] if l == 0 else torch.empty_like(d["out_attn"]))
                            for l, x in enumerate(d["layers"])]
        d["vout"] = {"accept_len": torch.empty((B,), dtype=torch.int32, device=dev),
                     "path": torch.empty((B, depth), dtype=torch.int32, device=dev),
                     "final_token": torch.empty((B,), dtype=torch.int32, device=dev),
                     "decision": torch.empty((B, M), dtype=torch.uint8, device=dev),
                     "ratio": torch.empty((B, M), dtype=torch.float32, device=dev)}
        reps.append(d)
    attn_ws = torch.empty(max(256, lpp.lpp_tree_attention_layers_workspace(tree, L, B, H, S, Dh)), dtype=torch.uint8,
                          device=dev)
    ver_ws = torch.empty(lpp.lpp_relaxed_verify_workspace(tree, B, V, k), dtype=torch.uint8, device=dev)
    dtype = lpp.LPP_BF16 if cfg.kv_dtype == "bf16" else lpp.LPP_F32
    stream = torch.cuda.current_stream()

    ctx0 = {"tree": tree, "attn_ws": attn_ws, "ver_ws": ver_ws}

    def attention(d, st=None, ctx=ctx0):
        st = stream if st is None else st
        tree, attn_ws = ctx["tree"], ctx["attn_ws"]
        if L > 1 and not args.layer_loop:
            lpp.lpp_tree_attention_layers(tree, dtype, lpp.LPP_BF16 if args.out_bf16 else lpp.LPP_F32, d["layer_table"],
                                          None, B, H, Hkv, S, Dh, 0.0, attn_ws, st)
            return
        for x in d["layers"]:
            if gqa_call:
                lpp.lpp_tree_attention_gqa(tree, dtype, lpp.LPP_BF16 if args.out_bf16 else lpp.LPP_F32, x["q"], x["kc"],
                                           x["vc"], x["kt"], x["vt"], None, B, H, Hkv, S, Dh, 0.0, d["out_attn"],
                                           attn_ws, st)
            else:
                lpp.lpp_tree_attention(tree, dtype, x["q"], x["kc"], x["vc"], x["kt"], x["vt"], None,
                                       B, H, S, Dh, 0.0, d["out_attn"], attn_ws, st)

    def verify(d, st=None, ctx=ctx0):
        st = stream if st is None else st
        tree, ver_ws = ctx["tree"], ctx["ver_ws"]
        if args.rule != "prefix" or args.siblings != "iid":
            lpp.lpp_relaxed_verify_opts(tree, d["target_logits"], d["drafter_logits"], cfg.ldv, cfg.vocab_offset, V, B,
                                        d["tokens"], neigh, k, k, d["u_accept"], d["u_final"], d["vout"], ver_ws, st,
                                        bound=lpp.LPP_BOUND_MULTIPLICATIVE, bound_value=cfg.lam,
                                        rule=lpp.LPP_RULE_SKIP if args.rule == "skip" else lpp.LPP_RULE_PREFIX,
                                        siblings=lpp.LPP_SIBLINGS_DISTINCT if args.siblings == "distinct"
                                        else lpp.LPP_SIBLINGS_IID,
                                        uncond_logits=d["uncond_logits"] if args.frontend else None,
                                        cfg_scale=3.0 if args.frontend else 0.0, top_k=2000 if args.frontend else 0)
        elif args.frontend:
            lpp.lpp_relaxed_verify_sampled(tree, d["target_logits"], d["uncond_logits"], 3.0, 2000, d["drafter_logits"],
                                           cfg.ldv, cfg.vocab_offset, V, B, d["tokens"], neigh, k, k, cfg.lam,
                                           d["u_accept"], d["u_final"], d["vout"], ver_ws, st)
        else:
            lpp.lpp_relaxed_verify(tree, d["target_logits"], d["drafter_logits"], cfg.ldv, cfg.vocab_offset, V, B,
                                   d["tokens"], neigh, k, k, cfg.lam, d["u_accept"], d["u_final"], d["vout"],
                                   ver_ws, st)

    def step(i):
        d = reps[i % R]
        attention(d)
        verify(d)

    # ---- launch path: HIP graphs (one with a step on every replica, one per replica for the
    # remainder), captured after an eager warm-up; eager launches if capture is not available
    for i in range(max(R, 3)):
        step(i)
    torch.cuda.synchronize()
    launch = "hipgraph"
    try:
        side = torch.cuda.Stream()
        def capture(fn):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                global_stream[0] = side
                with torch.cuda.graph(g, stream=side):
                    fn()
                global_stream[0] = torch.cuda.current_stream()
            return g
        global_stream = [stream]
        def attention_s(d):
            attention(d, global_stream[0])
        def verify_s(d):
            verify(d, global_stream[0])
        g_all = capture(lambda: [(attention_s(d), verify_s(d)) for d in reps])
        g_one = [capture(lambda d=d: (attention_s(d), verify_s(d))) for d in reps]
        g_same = capture(lambda: [(attention_s(reps[0]), verify_s(reps[0])) for _ in reps])   # R steps on one replica
        g_attn = capture(lambda: [attention_s(d) for d in reps])
        g_ver = capture(lambda: [verify_s(d) for d in reps])
        torch.cuda.synchronize()

        def run_steps(n):
            for _ in range(n // R):
                g_all.replay()
            for i in range(n % R):
                g_one[i].replay()

    except Exception as e:             # pragma: no cover - depends on the runtime
        launch = "eager (graph capture failed: %s)" % type(e).__name__
        g_attn = g_ver = g_same = None

        def run_steps(n):
            for i in range(n):
                step(i)

    # ---- timed region: W warm-up steps, then exactly K steps between synchronisations.  With
    # graphs, a run of up to 512 steps is ONE graph of exactly that many steps (replicas in rotation),
    # so that a short run pays one launch, not one per replica round.
    g_k = None
    if launch == "hipgraph" and args.steps <= 512:
        g_k = capture(lambda: [(attention_s(reps[i % R]), verify_s(reps[i % R])) for i in range(args.steps)])
        g_k.replay()                   # (its first replay uploads the graph: kept out of the timed region)
        torch.cuda.synchronize()
    run_steps(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if g_k is not None:
        g_k.replay()
    else:
        run_steps(args.steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    steps_per_s = 1e3 / ms_per_step
    mean_accept = float(torch.stack([d["vout"]["accept_len"] for d in reps]).float().mean().item())

    # ---- distributions: HIP events on the launch stream between back-to-back graph replays (R
    # launches each), at least 200 of them whatever --steps says; per-launch time = replay time / R
    def replay_samples(g, fallback, n_replays, per):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_replays + 1)]
        for _ in range(3):
            g.replay() if g is not None else fallback()
        evs[0].record()
        for i in range(n_replays):
            g.replay() if g is not None else fallback()
            evs[i + 1].record()
        torch.cuda.synchronize()
        return np.array([evs[i].elapsed_time(evs[i + 1]) / per for i in range(n_replays)])

    def dist(x):
        return {"mean": float(x.mean()), "median": float(np.median(x)), "p10": float(np.percentile(x, 10)),
                "p90": float(np.percentile(x, 90)), "samples": int(x.size)}

    n_rep_d = max(200, args.steps // R)
    step_d = dist(replay_samples(g_all if launch == "hipgraph" else None, lambda: [step(i) for i in range(R)],
                                 n_rep_d, R))

    # ---- the same step when its inputs are still in the 256 MB last-level cache (one replica over and
    # over: what a step sees whose logits and K/V were written just before it); reported beside the
    # HBM-resident figure above, never in place of it
    cached_ms = None
    if R > 1 and not args.no_cached:
        cached_ms = float(np.median(replay_samples(g_same, lambda: [step(0) for _ in range(R)], 60, R)))

    # ---- per-kernel device time: back-to-back launches of one kernel over the rotating replicas
    # (includes the gap between dependent launches)
    attn_d = dist(replay_samples(g_attn, lambda: [attention(d) for d in reps], n_rep_d, R * L))   # per launch (one layer)
    ver_d = dist(replay_samples(g_ver, lambda: [verify(d) for d in reps], n_rep_d, R))
    attn_ms, verify_ms = attn_d["mean"], ver_d["mean"]

    # ---- two batches in flight (a server with two independent sequences' batches): the replicas
    # are dealt to two branches of one graph, each branch a chain of whole steps with a tree handle
    # and workspaces of its own, so the attention of one batch runs beside the verify of the other.
    # Reported beside `value`, never in place of it: `value` is one batch, its steps one after the other.
    two = None
    if launch == "hipgraph" and L == 1 and R >= 2 and not args.no_two_batches:
        try:
            ctx1 = {"tree": lpp.Tree(parent), "attn_ws": torch.empty_like(attn_ws), "ver_ws": torch.empty_like(ver_ws)}
            s2 = torch.cuda.Stream()

            def two_branches():
                s2.wait_stream(side)
                for d in reps[0::2]:
                    attention(d, side, ctx0)
                    verify(d, side, ctx0)
                for d in reps[1::2]:
                    attention(d, s2, ctx1)
                    verify(d, s2, ctx1)
                side.wait_stream(s2)

            for d in reps[1::2]:               # eager warm-up of the second handle
                attention(d, stream, ctx1)
                verify(d, stream, ctx1)
            torch.cuda.synchronize()
            g_two = capture(two_branches)
            torch.cuda.synchronize()
            two_d = dist(replay_samples(g_two, None, n_rep_d, R))
            gave_up = tree.walk_gave_up() + ctx1["tree"].walk_gave_up()
            two = {"value": 1e3 / two_d["mean"], "unit": "steps/s", "ms_per_step": round(two_d["mean"], 5),
                   "ms_per_step_median": round(two_d["median"], 5), "batches_in_flight": 2,
                   "walks_that_gave_up": gave_up,
                   "note": "two independent batches, one graph branch each (own tree handle and workspaces); "
                           "every step still runs attention then verify in order"}
        except Exception as e:         # pragma: no cover - depends on the runtime
            two = {"value": None, "note": "not measured (%s)" % type(e).__name__}

    # ---- streaming-read ceiling of this device: a plain read of 1 GiB (four times the last-level
    # cache) by the library's probe kernel, best of a few grid sizes
    stream_gbs = None
    try:
        big = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        big.zero_()
        best = 0.0
        for blocks in (2048, 4096, 8192, 16384):
            lpp.lpp_probe_stream_read(big, blocks)
            torch.cuda.synchronize()
            ev[0].record()
            for _ in range(5):
                lpp.lpp_probe_stream_read(big, blocks)
            ev[1].record()
            torch.cuda.synchronize()
            best = max(best, 5 * big.numel() / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9)
        stream_gbs = best
        del big
    except Exception:                  # pragma: no cover
        stream_gbs = None

    kern = {"tree_attention": {"d": attn_d, "bytes": attn_bytes, "GBs": attn_bytes / attn_ms / 1e6},
            "relaxed_verify": {"d": ver_d, "bytes": verify_bytes, "GBs": verify_bytes / verify_ms / 1e6}}
    dom = max(kern, key=lambda n: kern[n]["d"]["mean"])
    traffic = TRAFFIC.get(cfg.idx, {}) if (L == 1 and not gqa_call and not args.frontend
                                           and args.rule == "prefix" and args.siblings == "iid") else {}
    roofline = {"bound": "hbm", "kernel": dom, "achieved": kern[dom]["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": kern[dom]["GBs"] / HBM_PEAK_GBS, "traffic": traffic.get(dom),
                "stream_read_ceiling_GBs": stream_gbs,
                "frac_of_stream_read_ceiling": kern[dom]["GBs"] / stream_gbs if stream_gbs else None,
                "per_call": {n: {"ms": round(v["d"]["mean"], 5), "ms_median": round(v["d"]["median"], 5),
                                 "ms_p10": round(v["d"]["p10"], 5), "ms_p90": round(v["d"]["p90"], 5),
                                 "algorithmic_bytes": v["bytes"], "traffic": traffic.get(n),
                                 "GBs": round(v["GBs"], 1), "frac": round(v["GBs"] / HBM_PEAK_GBS, 4),
                                 "frac_of_stream_read_ceiling": round(v["GBs"] / stream_gbs, 4) if stream_gbs else None}
                             for n, v in kern.items()},
                "step_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "ms_per_step_events": {k2: round(v2, 5) if isinstance(v2, float) else v2 for k2, v2 in step_d.items()},
                "cache_resident_ms_per_step": cached_ms}
    knn = None
    if knn_ms:
        knn_flops = 2.0 * V * V * cfg.D             # the method's contraction: every pair of codes once
        knn = {"ms": knn_ms, "mfma_dtype": "f32" if cfg.D <= 16 else "bf16 filter, float64 keys",
               "contraction_TFLOPs": knn_flops / (knn_ms * 1e-3) / 1e12,
               "frac_of_fp32_mfma_peak": knn_flops / (knn_ms * 1e-3) / 1e12 / FP32_MFMA_PEAK_TFLOPS,
               "note": "one-time per codebook; whole build (select, float64 re-rank, ordering) against the 2 V^2 D "
                       "flops of the definition; sweeps beyond the first are not counted as work"}

    # ---- CPU baseline: the float64 numpy oracle, as it stands, on this host: once held to one
    # thread, once with the host's threading
    cpu = None
    if not args.no_cpu_baseline and L == 1:      # (the oracle's step has one attention layer)
        from oracle import relaxed_verify, tree_attention
        neigh_h = neigh.cpu().numpy()           # input table for the oracle's verify step
        nb = min(B, 1 if cfg.idx >= 5 else B)

        def oracle_steps(budget_s):
            n_rep, t_cpu = 0, 0.0
            while t_cpu < budget_s and n_rep < 500:
                t0 = time.perf_counter()
                tree_attention(att["q"][:nb], att["kc"][:nb], att["vc"][:nb], att["kt"][:nb], att["vt"][:nb], parent)
                relaxed_verify(parent, ver["target_logits"][:nb], ver["drafter_logits"][:nb], cfg.vocab_offset, V,
                               ver["tokens"][:nb], neigh_h, k, cfg.lam, ver["u_accept"][:nb], ver["u_final"][:nb])
                t_cpu += time.perf_counter() - t0
                n_rep += 1
            return n_rep * (nb / B) / t_cpu, n_rep, t_cpu

        threads_all = len(os.sched_getaffinity(0))
        one = None
        try:
            from threadpoolctl import threadpool_info, threadpool_limits
            pools = [pi.get("num_threads", 1) for pi in threadpool_info()]
            threads_all = max(pools) if pools else 1
            with threadpool_limits(limits=1):
                one = oracle_steps(8.0)
        except ImportError:            # pragma: no cover
            pass
        v_all, n_rep, t_cpu = oracle_steps(10.0)
        cpu = {"value": v_all, "unit": "steps/s", "cores": threads_all,
               "kind": "oracle", "sample": f"{nb} of {B} batch items of one step, {n_rep} times "
               f"({t_cpu:.1f} s of CPU work; numpy float64, {threads_all} BLAS threads on "
               f"{len(os.sched_getaffinity(0))} host cores)",
               "one_thread": None if one is None else {"value": one[0], "unit": "steps/s", "cores": 1,
                                                       "sample": f"same sample, {one[1]} times ({one[2]:.1f} s)"}}

    out = {"metric": "tree_verify_steps_per_sec", "value": steps_per_s, "unit": "steps/s",
           "verified_nodes_per_sec": steps_per_s * B * cfg.N,
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "ms_per_step_median": step_d["median"], "ms_per_step_p10": step_d["p10"], "ms_per_step_p90": step_d["p90"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "dtype_note": "verify: f32; attention: %s inputs on MFMA, f32 softmax/accumulate" % cfg.kv_dtype,
           "data": "synthetic",
           "config": {"workload": f"config {cfg.idx} ({cfg.name}): B={B} H={H}x{Dh} S={S} M={M} V={V} k={k} "
                                  f"lambda={cfg.lam}", "replicas_rotated": R, "mean_accept_len": mean_accept,
                      "frontend": "cfg 3.0 + top-k 2000 fused" if args.frontend else "none (final logits handed in)",
                      "rule": args.rule, "siblings": args.siblings,
                      "attention_layers_per_step": L, "kv_heads": Hkv,
                      "attention_out": "bf16" if args.out_bf16 else "f32",
                      "launch": launch},
           "roofline": roofline, "cpu_baseline": cpu, "knn_build": knn, "two_batches_in_flight": two}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
