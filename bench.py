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
# HBM bytes per launch at config 3 from rocprofv3 FETCH_SIZE / WRITE_SIZE runs (profiles/), scaled
# by the same counters' reading for a copy of known size; None until measured for a kernel.
TRAFFIC = {"tree_attention": 29.11e6, "relaxed_verify": 30.20e6}   # config 3; profiles/config3_step_hbm_bytes.txt
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
    ap.add_argument("--frontend", action="store_true",
                    help="verify through lpp_relaxed_verify_sampled (guidance 3.0 + top-k 2000 fused; reads one more "
                         "target row set); not the headline configuration")
    ap.add_argument("--rule", choices=["prefix", "skip"], default="prefix",
                    help="choice of A inside B_k (lpp_relaxed_verify_opts when not the default)")
    ap.add_argument("--siblings", choices=["iid", "distinct"], default="iid",
                    help="sibling scheme (lpp_relaxed_verify_opts when not the default)")
    ap.add_argument("--layers", type=int, default=1,
                    help="attention launches per step, each on its own K/V cache (a target's layer count); "
                         "the headline step has one")
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
    knn_reps = 3
    ev[0].record()
    for _ in range(knn_reps):
        lpp.lpp_build_neighbours(dE, k, neigh, knn_ws)
    ev[1].record()
    torch.cuda.synchronize()
    knn_ms = ev[0].elapsed_time(ev[1]) / knn_reps
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
        d["vout"] = {"accept_len": torch.empty((B,), dtype=torch.int32, device=dev),
                     "path": torch.empty((B, depth), dtype=torch.int32, device=dev),
                     "final_token": torch.empty((B,), dtype=torch.int32, device=dev),
                     "decision": torch.empty((B, M), dtype=torch.uint8, device=dev),
                     "ratio": torch.empty((B, M), dtype=torch.float32, device=dev)}
        reps.append(d)
    attn_ws = torch.empty(max(256, lpp.lpp_tree_attention_workspace(tree, B, H, S, Dh)), dtype=torch.uint8, device=dev)
    ver_ws = torch.empty(lpp.lpp_relaxed_verify_workspace(tree, B, V, k), dtype=torch.uint8, device=dev)
    dtype = lpp.LPP_BF16 if cfg.kv_dtype == "bf16" else lpp.LPP_F32
    stream = torch.cuda.current_stream()

    def attention(d, st=None):
        st = stream if st is None else st
        for x in d["layers"]:
            if gqa_call:
                lpp.lpp_tree_attention_gqa(tree, dtype, lpp.LPP_BF16 if args.out_bf16 else lpp.LPP_F32, x["q"], x["kc"],
                                           x["vc"], x["kt"], x["vt"], None, B, H, Hkv, S, Dh, 0.0, d["out_attn"],
                                           attn_ws, st)
            else:
                lpp.lpp_tree_attention(tree, dtype, x["q"], x["kc"], x["vc"], x["kt"], x["vt"], None,
                                       B, H, S, Dh, 0.0, d["out_attn"], attn_ws, st)

    def verify(d, st=None):
        st = stream if st is None else st
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

        def run_kernel(g, n):          # n launches of one kernel, R per replay
            for _ in range(n // R):
                g.replay()
            return (n // R) * R
    except Exception as e:             # pragma: no cover - depends on the runtime
        launch = "eager (graph capture failed: %s)" % type(e).__name__
        g_attn = g_ver = g_same = None

        def run_steps(n):
            for i in range(n):
                step(i)

        def run_kernel(g, n):
            fn = attention if run_kernel.which == "a" else verify
            for i in range(n):
                fn(reps[i % R])
            return n

    # ---- timed region: W warm-up steps, then exactly K steps between synchronisations
    run_steps(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    steps_per_s = 1e3 / ms_per_step
    mean_accept = float(torch.stack([d["vout"]["accept_len"] for d in reps]).float().mean().item())

    # ---- the same step when its inputs are still in the 256 MB last-level cache (one replica over and
    # over: what a step sees whose logits and K/V were written just before it); reported beside the
    # HBM-resident figure above, never in place of it
    cached_ms = None
    if R > 1:
        n_c = max(200, min(args.steps, 2000)) // R * R

        def run_same(n):
            if g_same is not None:
                for _ in range(n // R):
                    g_same.replay()
            else:
                for _ in range(n):
                    step(0)
        run_same(2 * R)
        torch.cuda.synchronize()
        tc0 = time.perf_counter()
        run_same(n_c)
        torch.cuda.synchronize()
        cached_ms = (time.perf_counter() - tc0) * 1e3 / n_c

    # ---- per-kernel device time: HIP events on the launch stream around back-to-back launches of
    # one kernel over the rotating replicas (includes the gap between dependent launches)
    def device_ms(which):
        run_kernel.which = which
        g = g_attn if which == "a" else g_ver
        ev[0].record()
        n = run_kernel(g, max(args.steps, R))
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / n

    attn_ms = device_ms("a") / L             # per launch (one layer)
    verify_ms = device_ms("v")
    kern = {"tree_attention": {"ms": attn_ms, "bytes": attn_bytes, "GBs": attn_bytes / attn_ms / 1e6},
            "relaxed_verify": {"ms": verify_ms, "bytes": verify_bytes, "GBs": verify_bytes / verify_ms / 1e6}}
    dom = max(kern, key=lambda n: kern[n]["ms"])
    roofline = {"bound": "hbm", "kernel": dom, "achieved": kern[dom]["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": kern[dom]["GBs"] / HBM_PEAK_GBS, "traffic": TRAFFIC.get(dom) if cfg.idx == 3 else None,
                "per_call": {n: {"ms": round(v["ms"], 5), "algorithmic_bytes": v["bytes"],
                                 "GBs": round(v["GBs"], 1), "frac": round(v["GBs"] / HBM_PEAK_GBS, 4)}
                             for n, v in kern.items()},
                "step_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "cache_resident_ms_per_step": cached_ms}
    knn_flops = 2.0 * 2.0 * V * V * cfg.D       # the contraction is swept twice
    knn = {"ms": knn_ms, "mfma_dtype": "f32", "contraction_TFLOPs": knn_flops / (knn_ms * 1e-3) / 1e12,
           "frac_of_fp32_mfma_peak": knn_flops / (knn_ms * 1e-3) / 1e12 / FP32_MFMA_PEAK_TFLOPS,
           "note": "one-time per codebook; whole build incl. select, float64 re-rank and sort"}

    # ---- CPU baseline: the float64 numpy oracle, as it stands, on this host
    cpu = None
    if not args.no_cpu_baseline and L == 1:      # (the oracle's step has one attention layer)
        from oracle import relaxed_verify, tree_attention
        neigh_h = neigh.cpu().numpy()           # input table for the oracle's verify step
        nb = min(B, 1 if cfg.idx >= 5 else B)
        n_rep, t_cpu = 0, 0.0
        while t_cpu < 10.0 and n_rep < 500:     # about 10 s of CPU work
            t0 = time.perf_counter()
            tree_attention(att["q"][:nb], att["kc"][:nb], att["vc"][:nb], att["kt"][:nb], att["vt"][:nb], parent)
            relaxed_verify(parent, ver["target_logits"][:nb], ver["drafter_logits"][:nb], cfg.vocab_offset, V,
                           ver["tokens"][:nb], neigh_h, k, cfg.lam, ver["u_accept"][:nb], ver["u_final"][:nb])
            t_cpu += time.perf_counter() - t0
            n_rep += 1
        cpu = {"value": n_rep * (nb / B) / t_cpu, "unit": "steps/s", "cores": len(os.sched_getaffinity(0)),
               "kind": "oracle", "sample": f"{nb} of {B} batch items of one step, {n_rep} times "
               f"({t_cpu:.1f} s of CPU work; numpy float64, BLAS threads as configured by the host)"}

    out = {"metric": "tree_verify_steps_per_sec", "value": steps_per_s, "unit": "steps/s",
           "verified_nodes_per_sec": steps_per_s * B * cfg.N,
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
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
           "roofline": roofline, "cpu_baseline": cpu, "knn_build": knn}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
