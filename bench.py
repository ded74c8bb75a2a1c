#!/usr/bin/env python3
"""Benchmark of the SDVG hot path on one MI355X.

One step = one video block's worth of the hot path at the 14B target shape (40 layers x 40
heads x 128, 4680 tokens per block, 6 cached blocks -> 32760 keys):
    S x L = 4 x 40 block-attention calls (each layer attends over its own slice of a real
    [40][7*4680][40][128] K/V cache), then the worst-frame router on 12 frame scores, the commit
    of the block's K/V into slot 6 of all 40 layers, and the rollback that removes it again.
Inputs are synthetic (seeded torch RNG on the device) and resident in HBM before timing.

Prints ONE JSON line. `value` is whole-step throughput in attention TFLOP/s (algorithmic
FLOPs 4*n_q*n_k*d*H per call over the full step time, router/commit/rollback included).
`roofline` is the attention kernel against the bf16 dense MFMA peak, from HIP-event timing of
the launches inside the timed region; `hbm_kernels` gives commit/rollback GB/s the same way.
`cpu_baseline` times the fp64 oracle on a bounded row sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E peak
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this workload and
# scaled by what the same counters read for the commit kernel, a plain copy of known size
# (FETCH_SIZE reads half the known bytes, WRITE_SIZE all of them). Only valid for the target workload.
TRAFFIC_TARGET = {"block_attn": 0.9875e9 + 0.0479e9, "kv_commit": 2 * 3.834e9, "kv_rollback": 3.835e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="target", choices=["target", "drafter", "tiny"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--denoise-steps", type=int, default=4)
    ap.add_argument("--sweep", action="store_true",
                    help="also time attention at 0..8 cached blocks (adds launches of other shapes)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by heads with no exchange "
              "inside it); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import sdvg_inputs as si
    import paper_2604_17397_amd as P
    from paper_2604_17397_amd import build as sdvg_build

    if not os.path.exists(P.binding.LIB_PATH):
        sdvg_build.build()
    P.lib()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = si.CONFIGS[args.workload]
    H, T, L, D = cfg["n_heads"], cfg["block_tokens"], cfg["n_layers"], cfg["head_dim"]
    nb = cfg["cached_blocks"]
    S = args.denoise_steps
    c_len = nb * T
    n_k = c_len + T
    cap = (nb + 1) * T

    k_all = si.device_normal_bf16((L, cap, H, D), si.SEED, si.TID_K_CACHE, device=dev)
    v_all = si.device_normal_bf16((L, cap, H, D), si.SEED, si.TID_V_CACHE, device=dev)
    cache = P.KVCache(k_all, v_all, T, cache_len=c_len)
    k_blk = si.device_normal_bf16((L, T, H, D), si.SEED, si.TID_K_BLK, device=dev)
    v_blk = si.device_normal_bf16((L, T, H, D), si.SEED, si.TID_V_BLK, device=dev)
    q = si.device_normal_bf16((T, H, D), si.SEED, si.TID_Q, device=dev)
    out = torch.empty_like(q)
    n_rounds = args.steps + args.warmup
    scores = torch.from_numpy(si.frame_scores_correlated(si.SEED, n_rounds)).to(dev)
    tau = -0.7

    flops_call = si.attn_flops(T, n_k, H, D)
    payload = 2.0 * L * T * H * D * 2   # bytes of K+V of one block over all layers

    def step(i, ev=None):
        if ev:
            ev[0].record()
        for _ in range(S):
            for l in range(L):
                kc, vc = cache.layer(l)
                P.block_attn(q, kc, vc, k_blk[l], v_blk[l], c_len, out=out)
        if ev:
            ev[1].record()
        dec, _ = P.worst_frame_route(scores[i], tau, nb)
        if ev:
            ev[2].record()
        P.kv_commit(cache, k_blk, v_blk, nb)
        if ev:
            ev[3].record()
        P.kv_rollback(cache, c_len)
        if ev:
            ev[4].record()
        return dec

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    accepted = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        accepted += step(args.warmup + i, evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_step = (t1 - t0) * 1e3 / args.steps
    per_step_attn = sorted(e[0].elapsed_time(e[1]) / (S * L) for e in evs)
    attn_ms = sum(per_step_attn) / args.steps
    route_us = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps * 1e3
    commit_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
    rollback_ms = sum(e[3].elapsed_time(e[4]) for e in evs) / args.steps

    value = flops_call * S * L / (ms_step * 1e-3) / 1e12
    attn_tflops = flops_call / (attn_ms * 1e-3) / 1e12
    commit_gbps = 2 * payload / (commit_ms * 1e-3) / 1e9
    rollback_gbps = payload / (rollback_ms * 1e-3) / 1e9

    line = {
        "metric": "block-attn TFLOP/s & % bf16 MFMA peak at 14B shape; KV-commit GB/s",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s-shape block: %d layers x %d heads x %d, %d query tokens x %d keys "
                               "(cache %d + block %d), %d denoising steps, then route + commit + rollback"
                               % (args.workload, L, H, D, T, n_k, c_len, T, S),
                   "attn_calls_per_step": S * L, "attn_flops_per_call": flops_call,
                   "commit_payload_bytes": payload, "tau": tau},
        "roofline": {"kernel": "block_attn_bf16_kernel", "bound": "mfma",
                     "achieved": round(attn_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": TRAFFIC_TARGET["block_attn"] if args.workload == "target" else None,
                     "avg_launch_ms": round(attn_ms, 4),
                     "median_launch_ms": round(per_step_attn[len(per_step_attn) // 2], 4),
                     "min_launch_ms": round(per_step_attn[0], 4)},
        "hbm_kernels": {
            "kv_commit": {"bound": "hbm", "achieved": round(commit_gbps, 1), "peak": PEAK_HBM_GBPS,
                          "unit": "GB/s", "frac": round(commit_gbps / PEAK_HBM_GBPS, 4),
                          "bytes": 2 * payload, "ms": round(commit_ms, 4),
                          "traffic": TRAFFIC_TARGET["kv_commit"] if args.workload == "target" else None},
            "kv_rollback": {"bound": "hbm", "achieved": round(rollback_gbps, 1), "peak": PEAK_HBM_GBPS,
                            "unit": "GB/s", "frac": round(rollback_gbps / PEAK_HBM_GBPS, 4),
                            "bytes": payload, "ms": round(rollback_ms, 4),
                            "traffic": TRAFFIC_TARGET["kv_rollback"] if args.workload == "target" else None},
            "route_us": round(route_us, 1)},
        "accepted_blocks": int(accepted),
    }

    # attention rate against the cache length, up to the paper's 9-block protocol (8 cached blocks)
    if args.sweep:
        sw_k = si.device_normal_bf16((8 * T, H, D), si.SEED, si.TID_K_CACHE + 50, device=dev)
        sw_v = si.device_normal_bf16((8 * T, H, D), si.SEED, si.TID_V_CACHE + 50, device=dev)
        sweep = []
        for kb_ in range(9):
            c_ = kb_ * T
            P.block_attn(q, sw_k, sw_v, k_blk[0], v_blk[0], c_, out=out)
            torch.cuda.synchronize()
            we = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            we[0].record()
            for _ in range(10):
                P.block_attn(q, sw_k, sw_v, k_blk[0], v_blk[0], c_, out=out)
            we[1].record()
            torch.cuda.synchronize()
            sweep.append(round(si.attn_flops(T, c_ + T, H, D) / (we[0].elapsed_time(we[1]) / 10 * 1e-3) / 1e12, 1))
        line["roofline"]["tflops_by_cached_blocks_0_to_8"] = sweep
        del sw_k, sw_v

    # snapshot / restore of an opaque buffer (1 GiB), outside the step: a next-row kernel
    snap_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    snap_dst = torch.empty_like(snap_src)
    P.buffer_snapshot(snap_dst, snap_src)
    torch.cuda.synchronize()
    se = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    se[0].record()
    for _ in range(5):
        P.buffer_snapshot(snap_dst, snap_src)
    se[1].record()
    torch.cuda.synchronize()
    snap_ms = se[0].elapsed_time(se[1]) / 5
    snap_gbps = 2.0 * (1 << 30) / (snap_ms * 1e-3) / 1e9
    line["hbm_kernels"]["buffer_snapshot"] = {"bound": "hbm", "achieved": round(snap_gbps, 1), "peak": PEAK_HBM_GBPS,
                                              "unit": "GB/s", "frac": round(snap_gbps / PEAK_HBM_GBPS, 4),
                                              "bytes": 2.0 * (1 << 30), "ms": round(snap_ms, 4)}
    del snap_src, snap_dst

    # what the matrix cores of this chip deliver with nothing else going on, and at what clock
    P.probe_mfma(4000)
    torch.cuda.synchronize()
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    pe[0].record()
    probe_flops, probe_cycles = P.probe_mfma(40000)
    pe[1].record()
    torch.cuda.synchronize()
    probe_ms = pe[0].elapsed_time(pe[1])
    line["roofline"]["mfma_only_probe"] = {
        "tflops": round(probe_flops / (probe_ms * 1e-3) / 1e12, 1),
        "clock_ghz": round(int(probe_cycles.item()) / (probe_ms * 1e-3) / 1e9, 3),
        "note": "register-only bf16 MFMA loop on the same chip; the 2500 peak assumes 2.4 GHz"}

    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(np, torch, si, cache, q, k_blk, v_blk, c_len, out, P)
    print(json.dumps(line))


def cpu_baseline(np, torch, si, cache, q, k_blk, v_blk, c_len, out, P):
    """Time the fp64 oracle on a bounded row sample of layer 0 and check the GPU rows on it."""
    import oracle
    from oracle import build as oracle_build
    oracle_build.build(force=False)

    def bits(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

    kc, vc = cache.layer(0)
    P.block_attn(q, kc, vc, k_blk[0], v_blk[0], c_len, out=out)
    torch.cuda.synchronize()
    hq, hkc, hvc = bits(q), bits(kc[:max(c_len, 1)]), bits(vc[:max(c_len, 1)])
    hkb, hvb, hout = bits(k_blk[0]), bits(v_blk[0]), bits(out)
    n_q, H, D = hq.shape
    n_k = c_len + hkb.shape[0]
    threads = oracle.num_threads()
    # aim at roughly 15 s: calibrate on 2 rows, then size the sample
    rows_all = si.parity_rows(n_q)
    t = time.perf_counter()
    oracle.block_attn(hq, hkc, hvc, hkb, hvb, c_len, rows=rows_all[:2])
    per_row = max((time.perf_counter() - t) / 2, 1e-6)
    n_rows = int(max(2, min(len(rows_all), 15.0 / per_row)))
    rows = rows_all[np.linspace(0, len(rows_all) - 1, n_rows).astype(np.int64)]
    rows = np.unique(rows)
    t = time.perf_counter()
    ref = oracle.block_attn(hq, hkc, hvc, hkb, hvb, c_len, rows=rows)
    dt = time.perf_counter() - t
    flops = 4.0 * len(rows) * n_k * D * H
    g = si.bf16_bits_to_f64(hout[rows])
    err = g - ref
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": threads,
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": "%d of %d query rows x all %d heads of layer 0, all %d keys (fp64, OpenMP)"
                      % (len(rows), n_q, H, n_k),
            "gpu_vs_oracle_on_sample": {"max_abs_err": float(np.max(np.abs(err))),
                                        "rel_rms": float(math.sqrt(np.sum(err * err) / np.sum(ref * ref)))}}


if __name__ == "__main__":
    main()
