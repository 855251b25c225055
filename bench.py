#!/usr/bin/env python3
"""Benchmark of the DES MoE-layer hot path on one MI355X.

A "step" is one pass of the whole path - router, coreset election,
constrained re-routing, permutation, grouped SwiGLU expert FFN, combine - over
one block of synthetic tokens, through the C ABI (des_moe_forward).  The
workload is the 128-expert bf16 layer (D=2048, F=768, K=8, N=32, Zipf-skewed
router bias) under DES-Vote with a coreset of 32; inputs are resident in HBM
before the timed region.  To keep the 256 MB last-level cache from serving the
expert weights, successive steps rotate over several replicas of the layer's
weights at different addresses.

Prints one JSON line: metric = microseconds per block (lower is better), plus
  roofline     - the dominant kernel (gate/up projection) against the 8 TB/s
                 HBM peak, its duration measured with HIP events in this run;
  cpu_baseline - the CPU oracle timed on this host on the same block.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic of the dominant kernel from rocprofv3 counters, in bytes per
# launch (FETCH_SIZE / WRITE_SIZE scaled by a copy kernel of known size).  It
# is NOT measured by the run that prints it (counters need a profiler run of
# their own): each entry names the committed summary it was read from and the
# commit whose kernels that run profiled, and goes stale when the kernel changes.
MEASURED_TRAFFIC = {
    ("m128_zipf", "vote", "packed"): {
        "bytes": 202684211 + 1586483,  # 202,684,211 B read + 1,586,483 B written
        "profile": "profiles/hbm_traffic_m128_zipf_vote_c32_packed.txt",
        "kernel_commit": "c737a12",
    },
}

# HBM floors of the benchmark definition: unique expert bytes / 8 TB/s.
def floor_us(unique_bytes):
    return unique_bytes / (HBM_PEAK_GBS * 1e9) * 1e6


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="m128_zipf",
                    choices=["m128_zipf", "m256_shared", "tiny_f32", "stack48"])
    ap.add_argument("--mode", default="vote", choices=["vanilla", "seq", "vote"])
    ap.add_argument("--coreset", type=int, default=None)
    ap.add_argument("--n-tokens", type=int, default=None)
    ap.add_argument("--layout", default="packed", choices=["packed", "rowmajor"])
    ap.add_argument("--replicas", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of the other benchmark configurations (256-expert layer "
                         "with a shared expert, block-length sweep, 48-layer stack) that the default "
                         "run adds under other_configs")
    ap.add_argument("--graph", action="store_true", help="also time the steps replayed from a HIP graph")
    ap.add_argument("--sweep", action="store_true",
                    help="block-length sweep N = 4..128, vanilla against DES-Vote C=32, and the "
                         "affine latency law of Eq. 2/3 fitted over the coreset size at N=32")
    ap.add_argument("--k-route", type=int, default=0,
                    help="experts per token inside the coreset (0 = K); Sec. 5.3 of the paper")
    ap.add_argument("--skip-beta", type=float, default=0.0,
                    help="cumulative-probability skipping threshold (0 = off); Sec. 5.1, Baselines")
    ap.add_argument("--variants", action="store_true",
                    help="routing variants on the 128-expert layer: top-k baseline, skipping, "
                         "DES-Vote with k = 8 and k = 4 in the same coreset")
    ap.add_argument("--selection-only", action="store_true",
                    help="time coreset selection alone (one fused HIP launch) beside the same "
                         "selection written with torch ops (Sec. 4.3 / Fig. 6 of the paper)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_00879_amd import binding as B
    from paper_2602_00879_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()  # fails loudly if the HIP library has not been built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.selection_only:
        return bench_selection(args, torch, B, W, dev)
    if args.sweep:
        return bench_sweep(args, torch, B, W, dev)
    if args.variants:
        return bench_variants(args, torch, B, W, dev)
    if args.workload == "stack48":
        return bench_stack(args, torch, B, W, dev)
    cfg = W.CONFIGS[args.workload]
    if args.n_tokens:
        cfg = cfg.with_(n_tokens=args.n_tokens)
    C = args.coreset if args.coreset else cfg.coreset
    layer = W.make_layer(cfg)

    def dev_t(a):
        if a is None:
            return None
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    packed = args.layout == "packed" and cfg.dtype == "bf16"
    layout = B.DES_LAYOUT_PACKED if packed else B.DES_LAYOUT_ROWMAJOR
    shape = B.make_shape(cfg.n_seqs, cfg.n_tokens, cfg.hidden, cfg.n_experts, cfg.ffn, cfg.top_k, C,
                         args.mode, cfg.dtype, ffn_shared=cfg.ffn_shared, weight_layout=layout,
                         k_route=args.k_route, skip_beta=args.skip_beta)
    x = dev_t(layer["x"])
    w_router, bias = dev_t(layer["w_router"]), dev_t(layer["bias"])

    def prep(a):
        t = dev_t(a)
        return B.des_pack_expert_weights(t) if packed else t

    base = [prep(layer[k]) for k in ("w_gate", "w_up", "w_down")]
    shared = tuple(prep(m) for m in layer["shared"]) if layer["shared"] else None
    torch.cuda.synchronize()
    # replicas: same values at different addresses, so that a step never finds
    # its expert weights in the last-level cache
    replicas = [base] + [[t.clone() for t in base] for _ in range(max(1, args.replicas) - 1)]
    bufs = B.MoeBuffers(shape, dev, x.dtype)

    def step(i):
        wg, wu, wd = replicas[i % len(replicas)]
        B.des_moe_forward(shape, x, w_router, bias, wg, wu, wd, shared=shared, buffers=bufs)

    # warm-up: at least one full rotation, so that every replica's pages have been
    # touched before the timed region whatever --warmup says
    for i in range(max(args.warmup, len(replicas))):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    n_unique = int(bufs.n_unique.cpu()[0])

    # per-kernel durations: the same steps again with an event pair around
    # every kernel on the launch stream
    B.des_kernel_timing_enable(True)
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    kt = B.des_kernel_timing_read()
    B.des_kernel_timing_enable(False)
    kernels_us = {k: (v[0] * 1e3 / v[1]) for k, v in kt.items() if v[1] > 0}

    # distribution of the step time: one event before every step (the launch
    # queue stays backed up, so consecutive events are one step apart)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    for i in range(args.steps):
        evs[i].record()
        step(i)
    evs[args.steps].record()
    torch.cuda.synchronize()
    per_step = np.sort(np.array([evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(args.steps)]))
    step_us = {"median": float(np.median(per_step)), "p10": float(per_step[int(0.1 * (len(per_step) - 1))]),
               "p90": float(per_step[int(0.9 * (len(per_step) - 1))])}

    # the machine's practical ceiling: a bare streaming read of as many bytes as
    # the gate/up kernel must fetch, rotating over the same replicas
    el = 2 if cfg.dtype == "bf16" else 4
    gateup_bytes = n_unique * 2 * cfg.hidden * cfg.ffn * el + 2 * cfg.hidden * cfg.ffn_shared * el
    probe_bytes = min(gateup_bytes, base[0].numel() * base[0].element_size()) // 65536 * 65536
    ceiling = None
    if probe_bytes > 0:
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        B.des_kernel_timing_enable(True)
        for i in range(60):
            B.des_hbm_read_probe(replicas[i % len(replicas)][0], probe_bytes, sink)
        torch.cuda.synchronize()
        pr = B.des_kernel_timing_read()["read_probe"]
        B.des_kernel_timing_enable(False)
        pus = pr[0] * 1e3 / pr[1]
        ceiling = {"bytes": probe_bytes, "us": pus, "GB/s": probe_bytes / (pus * 1e-6) / 1e9}

    graph_us = None
    if args.graph:
        g = torch.cuda.CUDAGraph()
        n_rep = len(replicas)
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            for i in range(3):
                step(i)
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=s):
                for i in range(n_rep):
                    step(i)
        torch.cuda.synchronize()
        reps = max(1, args.steps // n_rep)
        g.replay()
        torch.cuda.synchronize()
        tg0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - tg0) * 1e6 / (reps * n_rep)

    per_expert = 3 * cfg.hidden * cfg.ffn * el
    unique_bytes = n_unique * per_expert + (3 * cfg.hidden * cfg.ffn_shared * el)
    dom_us = kernels_us.get("gateup")
    achieved = gateup_bytes / (dom_us * 1e-6) / 1e9 if dom_us else None
    roofline = {
        "bound": "hbm", "kernel": "gateup", "achieved": achieved, "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
        "traffic": (MEASURED_TRAFFIC.get((args.workload, args.mode, args.layout)) or {}).get("bytes"),
        "traffic_source": MEASURED_TRAFFIC.get((args.workload, args.mode, args.layout)),
        "algorithmic_bytes_per_launch": gateup_bytes, "avg_launch_us": dom_us,
        "read_ceiling": ceiling,
        "frac_of_read_ceiling": (achieved / ceiling["GB/s"]) if (achieved and ceiling) else None,
    }
    ffn_us = sum(kernels_us.get(k, 0.0) for k in ("gateup", "down"))
    expert_gbs_step = unique_bytes / (ms_per_step * 1e-3) / 1e9
    expert_gbs_ffn = unique_bytes / (ffn_us * 1e-6) / 1e9 if ffn_us else None

    out = {
        "metric": "MoE-layer us per N-token block (DES-Vote, whole hot path)",
        "value": ms_per_step * 1e3, "unit": "us/block", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "warmup_steps_run": max(args.warmup, len(replicas)),
        "ms_per_step": ms_per_step, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: M={cfg.n_experts} D={cfg.hidden} F={cfg.ffn} "
                               f"Fs={cfg.ffn_shared} K={cfg.top_k} N={cfg.n_tokens} B={cfg.n_seqs} "
                               f"mode={args.mode} C={C} zipf_s={cfg.zipf_s}"
                               + (f" k_route={args.k_route}" if args.k_route else "")
                               + (f" skip_beta={args.skip_beta}" if args.skip_beta else ""),
                   "weight_layout": args.layout, "weight_replicas": len(replicas)},
        "n_unique_experts": n_unique,
        "unique_expert_bytes": unique_bytes,
        "expert_weight_GBps_whole_step": expert_gbs_step,
        "expert_weight_GBps_ffn_kernels": expert_gbs_ffn,
        "pct_of_hbm_peak_whole_step": 100.0 * expert_gbs_step / HBM_PEAK_GBS,
        "pct_of_hbm_peak_ffn_kernels": (100.0 * expert_gbs_ffn / HBM_PEAK_GBS) if expert_gbs_ffn else None,
        "step_us": step_us,
        "kernel_us": kernels_us,
        "graph_replay_us_per_block": graph_us,
        "roofline": roofline,
    }

    default_run = (args.workload == "m128_zipf" and args.mode == "vote" and not args.n_tokens
                   and not args.coreset and not args.k_route and not args.skip_beta and packed)
    if default_run and not args.no_other_configs:
        out["other_configs"] = other_configs(args, torch, B, W, dev, cfg, layer, replicas, w_router, bias)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, layer, args.mode, C)
    print(json.dumps(out))


def _timed_layer(torch, B, shape, x, w_router, bias, replicas, shared, steps, warm):
    """us per block of des_moe_forward on `shape`, weights rotated over `replicas`."""
    bufs = B.MoeBuffers(shape, x.device, x.dtype)

    def step(i):
        wg, wu, wd = replicas[i % len(replicas)]
        B.des_moe_forward(shape, x, w_router, bias, wg, wu, wd, shared=shared, buffers=bufs)

    for i in range(max(warm, len(replicas))):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e6 / steps, int(bufs.n_unique.cpu()[0])


def other_configs(args, torch, B, W, dev, cfg2, layer2, replicas2, w_router2, bias2):
    """Short runs of the other benchmark configurations, each with its HBM floor
    (unique expert bytes / 8 TB/s): the 256-expert layer with a shared expert under
    DES-Vote and DES-Seq at C = 16 / 32 / 64; the block-length sweep N = 4..128 on the
    128-expert layer, vanilla against DES-Vote C = 32; the 48-layer stack when enough
    HBM is free.  Context for the headline line above, same build, same run."""
    steps, warm = 100, 10
    res = {}

    def dev_t(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    def row(us, U, per_expert, shared_bytes=0):
        ub = U * per_expert + shared_bytes
        return {"us": round(us, 2), "n_unique": U, "floor_us": round(floor_us(ub), 2),
                "pct_of_hbm_peak_whole_step": round(100.0 * floor_us(ub) / us, 1)}

    # ---- block-length sweep on the 128-expert layer (the benchmark layer's weights)
    per2 = 3 * cfg2.hidden * cfg2.ffn * 2
    sweep = []
    for N in (4, 8, 16, 32, 64, 128):
        rng = np.random.default_rng([cfg2.seed, N])
        x = dev_t(W._normal(rng, (1, N, cfg2.hidden), 1.0, cfg2.dtype))
        for mode in ("vanilla", "vote"):
            shape = B.make_shape(1, N, cfg2.hidden, cfg2.n_experts, cfg2.ffn, cfg2.top_k, cfg2.coreset, mode,
                                 cfg2.dtype, weight_layout=B.DES_LAYOUT_PACKED)
            us, U = _timed_layer(torch, B, shape, x, w_router2, bias2, replicas2, None, steps, warm)
            sweep.append({"N": N, "mode": mode, **row(us, U, per2)})
    res["m128_sweep"] = {"workload": "128-expert layer, N = 4..128, vanilla vs DES-Vote C=32", "rows": sweep}

    # ---- 256 experts + shared expert
    cfg3 = W.CONFIGS["m256_shared"]
    layer3 = W.make_layer(cfg3)
    x3, wr3 = dev_t(layer3["x"]), dev_t(layer3["w_router"])
    base3 = [B.des_pack_expert_weights(dev_t(layer3[k])) for k in ("w_gate", "w_up", "w_down")]
    shared3 = tuple(B.des_pack_expert_weights(dev_t(m)) for m in layer3["shared"])
    torch.cuda.synchronize()
    reps3 = [base3] + [[t.clone() for t in base3] for _ in range(5)]  # 6 x 1.6 GB
    per3 = 3 * cfg3.hidden * cfg3.ffn * 2
    sh3 = 3 * cfg3.hidden * cfg3.ffn_shared * 2
    rows3 = []
    for mode in ("vote", "seq"):
        for C in (16, 32, 64):
            shape = B.make_shape(1, cfg3.n_tokens, cfg3.hidden, cfg3.n_experts, cfg3.ffn, cfg3.top_k, C, mode,
                                 cfg3.dtype, ffn_shared=cfg3.ffn_shared, weight_layout=B.DES_LAYOUT_PACKED)
            us, U = _timed_layer(torch, B, shape, x3, wr3, None, reps3, shared3, steps, warm)
            rows3.append({"mode": mode, "C": C, **row(us, U, per3, sh3)})
    res["m256_shared"] = {"workload": "256-expert layer + shared expert, N=32, C = 16 / 32 / 64", "rows": rows3}
    del reps3, base3, shared3, layer3
    torch.cuda.empty_cache()

    res["decoder_step"] = decoder_breakdown(torch, B, W, dev)
    res["decoder_step_batch8"] = decoder_breakdown(torch, B, W, dev, n_seqs=8, modes=("vote",))

    # ---- 48-layer stack: needs ~60 GB for the weights and a transient for packing
    free, _ = torch.cuda.mem_get_info()
    if free < 75e9:
        res["stack48"] = {"skipped": f"only {free / 1e9:.0f} GB of HBM free"}
        return res
    from paper_2602_00879_amd import device_workloads as DW
    cfg5 = W.CONFIGS["stack48"]
    st = DW.make_stack(cfg5, dev)
    for k in ("w_gate", "w_up", "w_down"):
        for l in range(cfg5.n_layers):
            st[k][l] = B.des_pack_expert_weights(st[k][l])
    torch.cuda.synchronize()
    shape = B.make_shape(cfg5.n_seqs, cfg5.n_tokens, cfg5.hidden, cfg5.n_experts, cfg5.ffn, cfg5.top_k,
                         cfg5.coreset, "vote", cfg5.dtype, weight_layout=B.DES_LAYOUT_PACKED, residual=1)
    bufs = B.StackBuffers(shape, cfg5.n_layers, dev, torch.bfloat16)

    def sstep():
        B.des_moe_stack_forward(shape, cfg5.n_layers, st["x"], st["w_router"], st["bias"], st["w_gate"],
                                st["w_up"], st["w_down"], buffers=bufs)

    for _ in range(2):
        sstep()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(10):
        sstep()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / 10
    uniq = bufs.n_unique.cpu().numpy()
    ub = int(uniq.sum()) * per2
    res["stack48"] = {"workload": "48 layers x 8 sequences x 32 tokens, DES-Vote C=32 per sequence and layer",
                      "ms_per_step": round(ms, 3), "unique_experts_per_layer_mean": round(float(uniq.mean()), 1),
                      "floor_ms": round(floor_us(ub) / 1e3, 3),
                      "pct_of_hbm_peak_whole_step": round(100.0 * floor_us(ub) / (ms * 1e3), 1)}
    return res


def decoder_breakdown(torch, B, W, dev, n_layers=12, steps=20, warm=3, n_seqs=1, modes=("vanilla", "vote")):
    """Where the time of a decoding step goes once attention sits around the MoE layers
    (the paper's Fig. 2 left, re-measured here with synthetic weights): a stack of
    `n_layers` decoder layers (attention with 32 query / 4 key-value heads of width 128
    over 16 + 16 cached positions and the block, then the 128-expert MoE layer), one
    block of 32 tokens, vanilla routing against DES-Vote C = 32.  Every layer has its own
    weights (14.5 GB for 12 layers), so each is read cold once per step."""
    from paper_2602_00879_amd import device_workloads as DW
    cfg = W.CONFIGS["m128_zipf"].with_(n_layers=n_layers, seed=61, n_seqs=n_seqs)
    acfg = W.ATTN_CONFIGS["attn_block32" if n_seqs == 1 else "attn_batch8"]
    assert acfg.n_seqs == n_seqs
    st = DW.make_stack(cfg, dev)
    at = DW.make_decoder_attention(cfg, acfg, dev)
    for k in ("w_gate", "w_up", "w_down"):
        for l in range(n_layers):
            st[k][l] = B.des_pack_expert_weights(st[k][l])
    torch.cuda.synchronize()
    attn = B.make_attn_shape(acfg.n_heads, acfg.n_kv_heads, acfg.head_dim, acfg.n_prefix, acfg.n_suffix)
    attn_bytes = 2 * (2 * cfg.hidden * acfg.n_heads * acfg.head_dim + 2 * cfg.hidden * acfg.n_kv_heads * acfg.head_dim)
    per = 3 * cfg.hidden * cfg.ffn * 2
    rows = []
    for mode in modes:
        shape = B.make_shape(cfg.n_seqs, cfg.n_tokens, cfg.hidden, cfg.n_experts, cfg.ffn, cfg.top_k, cfg.coreset,
                             mode, cfg.dtype, weight_layout=B.DES_LAYOUT_PACKED, residual=1)
        bufs = B.DecoderBuffers(shape, attn, n_layers, dev, torch.bfloat16)

        def step():
            B.des_decoder_stack_forward(shape, attn, n_layers, st["x"], at["wq"], at["wk"], at["wv"], at["wo"],
                                        at["k_cache"], at["v_cache"], st["w_router"], st["bias"], st["w_gate"],
                                        st["w_up"], st["w_down"], buffers=bufs)

        for _ in range(warm):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        us_layer = (time.perf_counter() - t0) * 1e6 / steps / n_layers
        B.des_kernel_timing_enable(True)
        for _ in range(5):
            step()
        torch.cuda.synchronize()
        kt = B.des_kernel_timing_read()
        B.des_kernel_timing_enable(False)
        k_us = {k: v[0] * 1e3 / v[1] for k, v in kt.items() if v[1] > 0}
        a_us = sum(k_us.get(k, 0.0) for k in ("attn_proj", "attn_core", "attn_out"))
        m_us = sum(k_us.get(k, 0.0) for k in ("routing", "gateup", "down", "combine"))
        U = float(bufs.n_unique.float().mean())
        rows.append({"mode": mode, "us_per_layer": round(us_layer, 2), "n_unique_mean": round(U, 1),
                     "kernel_us": {k: round(v, 2) for k, v in k_us.items() if k.startswith("attn") or k in
                                   ("routing", "gateup", "down", "combine")},
                     "attention_us": round(a_us, 2), "moe_us": round(m_us, 2),
                     "moe_share_of_kernel_time": round(m_us / (a_us + m_us), 3),
                     "floor_us": round(floor_us(U * per + attn_bytes), 2),
                     "attention_floor_us": round(floor_us(attn_bytes), 2)})
    del st, at
    torch.cuda.empty_cache()
    return {"workload": f"{n_layers} decoder layers (attention 32/4 heads x 128 over 16+16 cached + block, then "
                        f"128-expert MoE), {n_seqs} block(s) x 32 tokens, per layer", "rows": rows}


def bench_selection(args, torch, B, W, dev):
    """DES-Vote coreset selection alone: des_select_coreset (one launch) against
    the same selection composed from torch ops on the same GPU (softmax, top-k,
    gather, scatter-add, top-k, sort) - the comparison of Sec. 4.3 / Fig. 6."""
    cfg = W.CONFIGS["m128_zipf" if args.workload == "stack48" else args.workload]
    N = args.n_tokens or cfg.n_tokens
    M, K = cfg.n_experts, cfg.top_k
    C = args.coreset or cfg.coreset
    logits = torch.from_numpy(W.make_logits(N, M, cfg.seed, zipf_s=cfg.zipf_s)).to(dev).reshape(1, N, M)
    shape = B.make_shape(1, N, 32, M, 32, K, C, "vote", "f32")

    def torch_select(L):
        P = torch.softmax(L, dim=-1)
        idx = torch.topk(L, K, dim=-1).indices            # ranking on the logits
        w = torch.gather(P, -1, idx)
        V = torch.zeros(M, device=L.device, dtype=L.dtype).scatter_add_(0, idx.reshape(-1), w.reshape(-1))
        nominated = torch.zeros(M, device=L.device, dtype=torch.bool).index_fill_(0, idx.reshape(-1), True)
        score = torch.where(nominated, V, torch.full_like(V, -1.0))
        core = torch.topk(score, min(C, M)).indices
        return torch.sort(core).values

    def timed(fn, iters):
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / iters

    iters = max(args.steps, 200)
    outs = B.des_select_coreset(shape, logits)  # outputs allocated once, as a serving loop would
    hip_us = timed(lambda: B.des_select_coreset(shape, logits, out=outs), iters)
    # the same launch with the votes added by floating-point LDS atomics (arrival order)
    shape_at = B.make_shape(1, N, 32, M, 32, K, C, "vote", "f32", vote_atomic=1)
    atomic_us = timed(lambda: B.des_select_coreset(shape_at, logits, out=outs), iters)
    at = B.des_select_coreset(shape_at, logits)
    torch_us = timed(lambda: torch_select(logits[0]), iters)
    # same coreset (the torch version breaks exact ties arbitrarily; none occur here)
    ours = B.des_select_coreset(shape, logits)
    n = int(ours["coreset_size"][0])
    same = ours["coreset_idx"][0, :n].tolist() == torch_select(logits[0]).tolist()[:n]
    same_atomic = torch.equal(at["coreset_idx"], ours["coreset_idx"])
    kern = {}
    for name, sh in (("fixed_order", shape), ("atomic", shape_at)):
        B.des_kernel_timing_enable(True)
        for _ in range(50):
            B.des_select_coreset(sh, logits)
        torch.cuda.synchronize()
        kt = B.des_kernel_timing_read()
        B.des_kernel_timing_enable(False)
        kern[name] = kt["select"][0] * 1e3 / max(1, kt["select"][1])
    print(json.dumps({
        "metric": "DES-Vote coreset selection us per block (host wall-clock per call)",
        "value": hip_us, "unit": "us/block", "n_gpus": 1, "steps": iters, "higher_is_better": False,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"selection only: N={N} M={M} K={K} C={C} zipf_s={cfg.zipf_s}"},
        "hip_launches": 1, "hip_kernel_us": kern["fixed_order"],
        "torch_ops_us": torch_us, "speedup_vs_torch_ops": torch_us / hip_us,
        "same_coreset": bool(same),
        "vote_reduction": {"fixed_order_us": hip_us, "atomic_us": atomic_us,
                           "fixed_order_kernel_us": kern["fixed_order"], "atomic_kernel_us": kern["atomic"],
                           "same_coreset": bool(same_atomic)},
    }))


def bench_sweep(args, torch, B, W, dev):
    """Block-length sweep on the 128-expert layer: vanilla routing against
    DES-Vote with a coreset of 32 for N = 4..128 (Fig. 1 / Fig. 7 of the paper:
    latency follows the number of unique experts, not N), then the latency law
    of Eq. 2/3 at fixed N*K: us per block against unique experts as the coreset
    size varies, fitted by least squares to t = t0 + b*U."""
    cfg = W.CONFIGS["m128_sweep"]
    layer = W.make_layer(cfg.with_(n_tokens=128))

    def dev_t(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    packed = args.layout == "packed"
    layout = B.DES_LAYOUT_PACKED if packed else B.DES_LAYOUT_ROWMAJOR
    x_all = dev_t(layer["x"])
    w_router, bias = dev_t(layer["w_router"]), dev_t(layer["bias"])
    base = []
    for k in ("w_gate", "w_up", "w_down"):
        t = dev_t(layer[k])
        base.append(B.des_pack_expert_weights(t) if packed else t)
    torch.cuda.synchronize()
    replicas = [base] + [[t.clone() for t in base] for _ in range(max(1, args.replicas) - 1)]
    per_expert = 3 * cfg.hidden * cfg.ffn * 2
    steps, warm = min(args.steps, 100), min(args.warmup, 10)

    def run(mode, N, C):
        shape = B.make_shape(1, N, cfg.hidden, cfg.n_experts, cfg.ffn, cfg.top_k, C, mode, cfg.dtype,
                             weight_layout=layout)
        x = x_all[:, :N].contiguous()
        bufs = B.MoeBuffers(shape, dev, x.dtype)

        def step(i):
            wg, wu, wd = replicas[i % len(replicas)]
            B.des_moe_forward(shape, x, w_router, bias, wg, wu, wd, buffers=bufs)

        for i in range(warm):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / steps
        B.des_kernel_timing_enable(True)
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        kt = B.des_kernel_timing_read()
        B.des_kernel_timing_enable(False)
        ku = {k: round(v[0] * 1e3 / v[1], 2) for k, v in kt.items() if v[1] > 0}
        U = int(bufs.n_unique.cpu()[0])
        return {"mode": mode, "N": N, "C": C, "n_unique": U, "us": round(us, 2),
                "expert_GBps_whole_step": round(U * per_expert / us / 1e3, 1),
                "expert_GBps_ffn_kernels": round(U * per_expert / (ku.get("gateup", 0) + ku.get("down", 0)) / 1e3, 1),
                "kernel_us": ku}

    rows = []
    for N in (4, 8, 16, 32, 64, 128):
        for mode in ("vanilla", "vote"):
            rows.append(run(mode, N, cfg.coreset))
            print("# " + json.dumps(rows[-1]), file=sys.stderr, flush=True)
    law = [run("vote", 32, C) for C in (8, 16, 24, 32, 48, 64, 96, 128)]
    U = np.array([r["n_unique"] for r in law], dtype=np.float64)
    t = np.array([r["us"] for r in law], dtype=np.float64)
    A = np.stack([np.ones_like(U), U], axis=1)
    (t0_fit, b_fit), *_ = np.linalg.lstsq(A, t, rcond=None)
    resid = t - A @ np.array([t0_fit, b_fit])
    r2 = 1.0 - float(resid @ resid) / float(((t - t.mean()) ** 2).sum())
    print(json.dumps({
        "metric": "MoE-layer us per block over block length N, vanilla vs DES-Vote C=32",
        "unit": "us/block", "n_gpus": 1, "steps": steps, "warmup": warm, "higher_is_better": False,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"m128_sweep: M={cfg.n_experts} D={cfg.hidden} F={cfg.ffn} K={cfg.top_k} "
                               f"zipf_s={cfg.zipf_s} N in 4..128", "weight_layout": args.layout,
                   "weight_replicas": len(replicas)},
        "sweep": rows,
        "latency_law": {"fixed": "N=32, K=8 (N*K = 256 routed pairs)", "points": [[r["C"], r["n_unique"], r["us"]] for r in law],
                        "t0_us": float(t0_fit), "b_us_per_expert": float(b_fit), "r2": r2,
                        "implied_GBps_per_expert_slope": per_expert / float(b_fit) / 1e3},
    }))


def bench_variants(args, torch, B, W, dev):
    """Routing variants that reuse the same FFN kernels, on the 128-expert layer
    (N = 32): the top-k baseline (fewer experts per token, Table 1 of the paper),
    cumulative-probability skipping (Sec. 5.1, Baselines), and DES-Vote with
    k = 8 against k = 4 experts per token inside the same coreset (Sec. 5.3),
    and a sigmoid router limited to 4 of 8 expert groups (another routing function
    sigma of Sec. 4.1) under vanilla, DES-Vote and DES-Seq.
    Latency and expert counts only: accuracy needs trained weights."""
    cfg = W.CONFIGS["m128_zipf"]
    layer = W.make_layer(cfg)

    def dev_t(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    x, w_router, bias = dev_t(layer["x"]), dev_t(layer["w_router"]), dev_t(layer["bias"])
    base = [B.des_pack_expert_weights(dev_t(layer[k])) for k in ("w_gate", "w_up", "w_down")]
    torch.cuda.synchronize()
    replicas = [base] + [[t.clone() for t in base] for _ in range(max(1, args.replicas) - 1)]
    steps, warm = min(args.steps, 200), min(args.warmup, 20)
    rows = []
    plain = dict(router_act="softmax", n_group=0, topk_group=0, group_score="max")
    grouped = dict(router_act="sigmoid", n_group=8, topk_group=4, group_score="top2sum")
    for name, mode, k_route, beta, router in (
            ("vanilla K=8", "vanilla", 0, 0.0, plain),
            ("top-k baseline k=4", "vanilla", 4, 0.0, plain),
            ("vanilla + skipping beta=0.1", "vanilla", 0, 0.1, plain),
            ("vanilla + skipping beta=0.2", "vanilla", 0, 0.2, plain),
            ("vanilla + skipping beta=0.3", "vanilla", 0, 0.3, plain),
            ("DES-Vote C=32 k=8", "vote", 0, 0.0, plain),
            ("DES-Vote C=32 k=4 (same coreset)", "vote", 4, 0.0, plain),
            ("DES-Vote C=32 + skipping beta=0.2", "vote", 0, 0.2, plain),
            ("sigmoid router, 8 groups keep 4: vanilla K=8", "vanilla", 0, 0.0, grouped),
            ("sigmoid router, 8 groups keep 4: DES-Vote C=32", "vote", 0, 0.0, grouped),
            ("sigmoid router, 8 groups keep 4: DES-Seq C=32", "seq", 0, 0.0, grouped)):
        shape = B.make_shape(1, cfg.n_tokens, cfg.hidden, cfg.n_experts, cfg.ffn, cfg.top_k, cfg.coreset,
                             mode, cfg.dtype, weight_layout=B.DES_LAYOUT_PACKED, k_route=k_route,
                             skip_beta=beta, **router)
        bufs = B.MoeBuffers(shape, dev, x.dtype)

        def step(i):
            wg, wu, wd = replicas[i % len(replicas)]
            B.des_moe_forward(shape, x, w_router, bias, wg, wu, wd, buffers=bufs)

        for i in range(warm):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / steps
        pairs = int((bufs.topk_idx >= 0).sum().cpu())
        rows.append({"variant": name, "us": round(us, 2), "n_unique": int(bufs.n_unique.cpu()[0]),
                     "routed_pairs": pairs, "experts_per_token": round(pairs / cfg.n_tokens, 2)})
        print("# " + json.dumps(rows[-1]), file=sys.stderr, flush=True)
    print(json.dumps({
        "metric": "MoE-layer us per block under routing variants", "unit": "us/block", "n_gpus": 1,
        "steps": steps, "warmup": warm, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"m128_zipf: M={cfg.n_experts} D={cfg.hidden} F={cfg.ffn} K={cfg.top_k} "
                               f"N={cfg.n_tokens} zipf_s={cfg.zipf_s}", "weight_layout": "packed",
                   "weight_replicas": len(replicas)},
        "variants": rows}))


def bench_stack(args, torch, B, W, dev):
    """The 48-layer residual stack (8 sequences x 32 tokens, DES-Vote C=32 per
    sequence and layer, ~58 GB of expert weights resident): us per decoding step.
    A context figure: the headline metric is the single layer above."""
    from paper_2602_00879_amd import device_workloads as DW
    cfg = W.CONFIGS["stack48"]
    st = DW.make_stack(cfg, dev)
    packed = args.layout == "packed"
    if packed:
        for k in ("w_gate", "w_up", "w_down"):
            for l in range(cfg.n_layers):  # layer by layer: bounds the temporary
                st[k][l] = B.des_pack_expert_weights(st[k][l])
    torch.cuda.synchronize()
    layout = B.DES_LAYOUT_PACKED if packed else B.DES_LAYOUT_ROWMAJOR
    shape = B.make_shape(cfg.n_seqs, cfg.n_tokens, cfg.hidden, cfg.n_experts, cfg.ffn, cfg.top_k,
                         args.coreset or cfg.coreset, args.mode, cfg.dtype, weight_layout=layout,
                         residual=1)
    bufs = B.StackBuffers(shape, cfg.n_layers, dev, torch.bfloat16)

    def step():
        B.des_moe_stack_forward(shape, cfg.n_layers, st["x"], st["w_router"], st["bias"],
                                st["w_gate"], st["w_up"], st["w_down"], buffers=bufs)

    steps = max(1, min(args.steps, 50))
    for _ in range(min(args.warmup, 5)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    uniq = bufs.n_unique.cpu().numpy()
    B.des_kernel_timing_enable(True)
    step()
    torch.cuda.synchronize()
    kt = B.des_kernel_timing_read()
    B.des_kernel_timing_enable(False)
    per_expert = 3 * cfg.hidden * cfg.ffn * 2
    unique_bytes = int(uniq.sum()) * per_expert
    out = {
        "metric": "48-layer MoE stack us per decoding step (DES-Vote per sequence and layer)",
        "value": ms * 1e3, "unit": "us/step", "n_gpus": 1, "steps": steps, "warmup": min(args.warmup, 5),
        "ms_per_step": ms, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"stack48: L={cfg.n_layers} B={cfg.n_seqs} N={cfg.n_tokens} M={cfg.n_experts} "
                               f"D={cfg.hidden} F={cfg.ffn} K={cfg.top_k} mode={args.mode} C={args.coreset or cfg.coreset}",
                   "weight_layout": args.layout},
        "unique_experts_per_layer_mean": float(uniq.mean()),
        "unique_expert_bytes_per_step": unique_bytes,
        "expert_weight_GBps_whole_step": unique_bytes / (ms * 1e-3) / 1e9,
        "pct_of_hbm_peak_whole_step": 100.0 * unique_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kernel_us_per_layer": {k: v[0] * 1e3 / v[1] for k, v in kt.items() if v[1] > 0},
    }
    print(json.dumps(out))


def cpu_baseline(cfg, layer, mode, C):
    """The CPU oracle, as it stands, on the same block: whole blocks (router,
    election, re-routing and every token's expert FFNs) repeated until about
    12 s of CPU work have been timed."""
    from oracle import des_oracle as O
    from paper_2602_00879_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:  # pragma: no cover
        threads = 1
    x = W.to_f64(layer["x"])
    wr = W.to_f64(layer["w_router"])
    bias = None if layer["bias"] is None else layer["bias"].astype(np.float64)

    class Lazy:  # widen one expert at a time (exact), as the oracle's cache asks for it
        def __init__(self, a):
            self.a = a

        def __getitem__(self, e):
            return W.to_f64(self.a[e])

    wg, wu, wd = Lazy(layer["w_gate"]), Lazy(layer["w_up"]), Lazy(layer["w_down"])
    shared = tuple(W.to_f64(m) for m in layer["shared"]) if layer["shared"] else None

    def run(budget_s):
        blocks, t0 = 0, time.perf_counter()
        while True:
            O.moe_forward(x, wr, bias, wg, wu, wd, cfg.top_k, C, mode, shared=shared)
            blocks += 1
            dt = time.perf_counter() - t0
            if dt >= budget_s or blocks >= 200:
                return blocks, dt

    blocks, dt = run(10.0)
    single = None
    try:  # the same oracle held to one thread
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            b1, d1 = run(8.0)
        single = {"value": d1 / b1 * 1e6, "unit": "us/block", "cores": 1,
                  "sample": f"{b1} whole blocks in {d1:.1f} s (float64 numpy, one BLAS thread)"}
    except Exception:  # pragma: no cover
        pass
    return {"value": dt / blocks * 1e6, "unit": "us/block", "cores": threads, "kind": "oracle",
            "sample": f"{blocks} whole blocks of the same workload in {dt:.1f} s "
                      f"(float64 numpy, BLAS threads = cores)",
            "single_thread": single,
            "host_cpus": len(os.sched_getaffinity(0))}


if __name__ == "__main__":
    main()
