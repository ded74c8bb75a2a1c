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
After the timed region (nothing below touches `value` or `roofline.achieved`) the line also
reports, under `other_shapes`: the drafter-shaped layer (plain, key-split, two items per launch),
the target-shaped layer with two items per launch, attention by cache length (0..8 cached
blocks), and the 7-block streaming aggregate at both shapes; and `cpu_baseline`: the fp64 oracle
timed on a bounded row sample of the same workload, with the GPU's rows checked on it, plus the
oracle's nested-loop commit on a slice. The run exits non-zero if the sampled parity breaks the
stated bounds.
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
BF16_MAX_ABS, BF16_REL_RMS = 2e-2, 1e-2   # parity bounds of the bf16 attention path
# HBM bytes per launch of the target workload, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this file; written next to the counter summaries, with the commit and commands that made them.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "bench_target_traffic.json")


def load_traffic():
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f)
    except (OSError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="target", choices=["target", "drafter", "tiny"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-shapes", action="store_true",
                    help="skip the untimed extra measurements (profiling runs)")
    ap.add_argument("--denoise-steps", type=int, default=4)
    ap.add_argument("--input-std", type=float, default=1.0,
                    help="standard deviation of the synthetic q/k/v (1 = the workload's N(0,1)); the "
                         "attention rate depends on the operand values through the chip's power management")
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

    def normal(shape, tid, seed=si.SEED):
        t = si.device_normal_bf16(shape, seed, tid, device=dev)
        if args.input_std != 1.0:
            t.mul_(args.input_std)
        return t

    cfg = si.CONFIGS[args.workload]
    H, T, L, D = cfg["n_heads"], cfg["block_tokens"], cfg["n_layers"], cfg["head_dim"]
    nb = cfg["cached_blocks"]
    S = args.denoise_steps
    c_len = nb * T
    n_k = c_len + T
    cap = (nb + 1) * T

    k_all = normal((L, cap, H, D), si.TID_K_CACHE)
    v_all = normal((L, cap, H, D), si.TID_V_CACHE)
    cache = P.KVCache(k_all, v_all, T, cache_len=c_len)
    k_blk = normal((L, T, H, D), si.TID_K_BLK)
    v_blk = normal((L, T, H, D), si.TID_V_BLK)
    q = normal((T, H, D), si.TID_Q)
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

    traffic = load_traffic() if args.workload == "target" else None

    def traffic_of(kernel):
        if not traffic or kernel not in traffic.get("kernels", {}):
            return None
        k = traffic["kernels"][kernel]
        return k["fetch_bytes"] + k["write_bytes"]

    line = {
        "metric": "block-attn TFLOP/s & % bf16 MFMA peak at 14B shape; KV-commit GB/s",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s-shape block: %d layers x %d heads x %d, %d query tokens x %d keys "
                               "(cache %d + block %d), %d denoising steps, then route + commit + rollback"
                               % (args.workload, L, H, D, T, n_k, c_len, T, S),
                   "attn_calls_per_step": S * L, "attn_flops_per_call": flops_call,
                   "commit_payload_bytes": payload, "tau": tau, "input_std": args.input_std},
        "roofline": {"kernel": "block_attn_bf16_kernel", "bound": "mfma",
                     "achieved": round(attn_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic_of("block_attn"),
                     "traffic_source": (None if not traffic else
                                        "profiles/bench_target_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                        "runs of this file at commit %s, not this run)" % traffic.get("commit")),
                     "avg_launch_ms": round(attn_ms, 4),
                     "median_launch_ms": round(per_step_attn[len(per_step_attn) // 2], 4),
                     "min_launch_ms": round(per_step_attn[0], 4)},
        "hbm_kernels": {
            "kv_commit": {"bound": "hbm", "achieved": round(commit_gbps, 1), "peak": PEAK_HBM_GBPS,
                          "unit": "GB/s", "frac": round(commit_gbps / PEAK_HBM_GBPS, 4),
                          "bytes": 2 * payload, "ms": round(commit_ms, 4), "traffic": traffic_of("kv_commit")},
            "kv_rollback": {"bound": "hbm", "achieved": round(rollback_gbps, 1), "peak": PEAK_HBM_GBPS,
                            "unit": "GB/s", "frac": round(rollback_gbps / PEAK_HBM_GBPS, 4),
                            "bytes": payload, "ms": round(rollback_ms, 4), "traffic": traffic_of("kv_rollback")},
            "route_us": round(route_us, 1)},
        "accepted_blocks": int(accepted),
    }

    def time_calls(fn, n):
        fn()
        torch.cuda.synchronize()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record()
        for _ in range(n):
            fn()
        e[1].record()
        torch.cuda.synchronize()
        return e[0].elapsed_time(e[1]) / n

    def rate(flops, ms):
        t = flops / (ms * 1e-3) / 1e12
        return {"tflops": round(t, 1), "frac": round(t / PEAK_BF16_TFLOPS, 4), "ms": round(ms, 4)}

    if not args.no_other_shapes and args.workload == "target":
        other = {}
        # -- the target layer with two items per launch (conditional + unconditional pass)
        q2, out2 = normal((T, H, D), si.TID_Q, seed=si.SEED + 1), torch.empty_like(q)
        kc0, vc0 = cache.layer(0)
        kc1, vc1 = cache.layer(1)
        ms = time_calls(lambda: P.block_attn_batch([q, q2], [kc0, kc1], [vc0, vc1], [k_blk[0], k_blk[1]],
                                                   [v_blk[0], v_blk[1]], c_len, outs=[out, out2]), 10)
        other["target_two_items_per_launch"] = rate(2 * flops_call, ms)
        # -- attention against the cache length, up to the paper's 9-block protocol (8 cached blocks)
        sw_k = normal((8 * T, H, D), si.TID_K_CACHE + 50)
        sw_v = normal((8 * T, H, D), si.TID_V_CACHE + 50)
        other["target_tflops_by_cached_blocks_0_to_8"] = [
            round(si.attn_flops(T, kb_ * T + T, H, D) /
                  (time_calls(lambda: P.block_attn(q, sw_k, sw_v, k_blk[0], v_blk[0], kb_ * T, out=out), 10) * 1e-3)
                  / 1e12, 1) for kb_ in range(9)]
        del sw_k, sw_v, q2, out2
        # -- the block's last denoising step with its commit: 40 attention launches then the commit
        #    kernel, against 40 launches with the commit fused in (sdvg_block_attn_commit)
        def last_step_separate():
            for l in range(L):
                kc_, vc_ = cache.layer(l)
                P.block_attn(q, kc_, vc_, k_blk[l], v_blk[l], c_len, out=out)
            P.kv_commit(cache, k_blk, v_blk, nb)
            cache.c.cache_len = c_len            # (timing only: the slot is overwritten again next call)

        def last_step_fused():
            for l in range(L):
                kc_, vc_ = cache.layer(l)
                P.block_attn_commit(q, kc_, vc_, k_blk[l], v_blk[l], c_len, out=out)
        ms_sep, ms_fus = time_calls(last_step_separate, 3), time_calls(last_step_fused, 3)
        other["last_step_plus_commit_ms"] = {"separate": round(ms_sep, 3), "fused": round(ms_fus, 3),
                                             "commit_hidden_ms": round(ms_sep - ms_fus, 3)}
        P.kv_rollback(cache, c_len)              # scrub the slot the fused launches filled

        # -- speculative rounds by threshold (optimistic mode: the draft's K/V are staged in the slot, the
        #    router decides, a reject scrubs the slot). 64 seeded rounds per tau, correlated frame scores.
        def rounds(tau_, n=64):
            sc = torch.from_numpy(si.frame_scores_correlated(si.SEED + 7, n)).to(dev)
            ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n)]
            acc = 0
            for i in range(n):
                ev[i][0].record()
                P.kv_commit(cache, k_blk, v_blk, nb)
                ev[i][1].record()
                dec_, _ = P.worst_frame_route(sc[i], tau_, nb)
                ev[i][2].record()
                P.kv_rollback(cache, c_len)      # on accept too: every round starts from the same cache
                ev[i][3].record()
                acc += int(dec_)
            torch.cuda.synchronize()
            c_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / n
            return {"rounds": n, "accepted": acc,
                    "commit_gbps": round(2 * payload / (c_ms * 1e-3) / 1e9, 1),
                    "route_us": round(sum(e[1].elapsed_time(e[2]) for e in ev) / n * 1e3, 1),
                    "rollback_gbps": round(payload / (sum(e[2].elapsed_time(e[3]) for e in ev) / n * 1e-3) / 1e9, 1)}
        other["speculative_rounds_by_tau"] = {str(t_): rounds(t_) for t_ in (-1.0, -0.7, -0.4)}

        # -- 7-block streaming generation, attention only: block k = 0..6 runs S x L calls at cache_len 4680 k
        def streaming(Ls, Hs, kk, vv, kb_, vb_, qq, oo):
            fl, ms_tot = 0.0, 0.0
            for b in range(7):
                def calls():
                    for l in range(Ls):
                        P.block_attn(qq, kk[l], vv[l], kb_[l], vb_[l], b * T, out=oo)
                ms_tot += time_calls(calls, S) * S
                fl += S * Ls * si.attn_flops(T, b * T + T, Hs, D)
            return {"attention_tflop": round(fl / 1e12, 1), "seconds": round(ms_tot * 1e-3, 3),
                    "tflops": round(fl / (ms_tot * 1e-3) / 1e12, 1),
                    "frac": round(fl / (ms_tot * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        other["streaming_7_blocks"] = {"target": streaming(L, H, k_all, v_all, k_blk, v_blk, q, out)}

        # -- the drafter-shaped layer (12 heads, 2 cached blocks) and the drafter's streaming run
        dcfg = si.CONFIGS["drafter"]
        Hd, Ld = dcfg["n_heads"], dcfg["n_layers"]
        dk = normal((Ld, 7 * T, Hd, D), si.TID_K_CACHE + 60)
        dv = normal((Ld, 7 * T, Hd, D), si.TID_V_CACHE + 60)
        dkb = normal((Ld, T, Hd, D), si.TID_K_BLK + 60)
        dvb = normal((Ld, T, Hd, D), si.TID_V_BLK + 60)
        dq = normal((T, Hd, D), si.TID_Q + 60)
        dq2 = normal((T, Hd, D), si.TID_Q + 61)
        do, do2 = torch.empty_like(dq), torch.empty_like(dq)
        dc = dcfg["cached_blocks"] * T
        dflops = si.attn_flops(T, dc + T, Hd, D)
        drafter = rate(dflops, time_calls(lambda: P.block_attn(dq, dk[0], dv[0], dkb[0], dvb[0], dc, out=do), 20))
        need = P.block_attn_workspace_bytes(dq, dk[0], dv[0], dkb[0], dvb[0], dc, split="always")
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
        drafter["key_split_forced"] = rate(dflops, time_calls(
            lambda: P.block_attn_batch([dq], [dk[0]], [dv[0]], [dkb[0]], [dvb[0]], dc, outs=[do], workspace=ws,
                                       split="always"), 20))
        drafter["key_split_forced"]["workspace_bytes"] = need
        drafter["two_items_per_launch"] = rate(2 * dflops, time_calls(
            lambda: P.block_attn_batch([dq, dq2], [dk[0], dk[1]], [dv[0], dv[1]], [dkb[0], dkb[1]], [dvb[0], dvb[1]],
                                       dc, outs=[do, do2]), 20))
        other["drafter_layer_12_heads_4680x14040"] = drafter
        other["streaming_7_blocks"]["drafter"] = streaming(Ld, Hd, dk, dv, dkb, dvb, dq, do)
        del dk, dv, dkb, dvb, dq, dq2, do, do2, ws
        line["other_shapes"] = other

    # snapshot / restore of an opaque buffer (1 GiB), outside the step: a next-row kernel
    snap_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    snap_dst = torch.empty_like(snap_src)
    snap_ms = time_calls(lambda: P.buffer_snapshot(snap_dst, snap_src), 5)
    snap_gbps = 2.0 * (1 << 30) / (snap_ms * 1e-3) / 1e9
    line["hbm_kernels"]["buffer_snapshot"] = {"bound": "hbm", "achieved": round(snap_gbps, 1), "peak": PEAK_HBM_GBPS,
                                              "unit": "GB/s", "frac": round(snap_gbps / PEAK_HBM_GBPS, 4),
                                              "bytes": 2.0 * (1 << 30), "ms": round(snap_ms, 4)}
    del snap_src, snap_dst
    # the commit with the rotary embedding of K fused into the copy (same traffic plus the angle tables)
    ang = torch.rand((T, 64), device=dev) * 6.283
    cos_t, sin_t = torch.cos(ang).contiguous(), torch.sin(ang).contiguous()

    def commit_rope():
        P.kv_commit_rope(cache, k_blk, v_blk, nb, cos_t, sin_t)
        cache.c.cache_len = c_len                # (timing only: the slot is scrubbed below)
    cr_ms = time_calls(commit_rope, 5)
    P.kv_commit_rope(cache, k_blk, v_blk, nb, cos_t, sin_t)
    P.kv_rollback(cache, c_len)
    cr_gbps = 2 * payload / (cr_ms * 1e-3) / 1e9
    line["hbm_kernels"]["kv_commit_rope"] = {"bound": "hbm", "achieved": round(cr_gbps, 1), "peak": PEAK_HBM_GBPS,
                                             "unit": "GB/s", "frac": round(cr_gbps / PEAK_HBM_GBPS, 4),
                                             "bytes": 2 * payload, "ms": round(cr_ms, 4)}

    # the rotary embedding alone, on one layer's q (what a step pays for q and for the block's own K)
    rope_out = torch.empty_like(q)
    rope_ms = time_calls(lambda: P.rope(q, cos_t, sin_t, out=rope_out), 20)
    rope_bytes = 2.0 * q.numel() * 2
    line["hbm_kernels"]["rope_one_layer_q"] = {"bound": "hbm", "achieved": round(rope_bytes / (rope_ms * 1e-3) / 1e9, 1),
                                               "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                               "frac": round(rope_bytes / (rope_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                                               "bytes": rope_bytes, "ms": round(rope_ms, 4)}
    del rope_out

    # what the matrix cores of this chip deliver with nothing else going on, and at what clock:
    # with two operand registers that never change, and with operands that change as a kernel's do
    def probe(changing):
        P.probe_mfma(4000, changing=changing)
        torch.cuda.synchronize()
        pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        pe[0].record()
        probe_flops, probe_cycles = P.probe_mfma(40000, changing=changing)
        pe[1].record()
        torch.cuda.synchronize()
        probe_ms = pe[0].elapsed_time(pe[1])
        return {"tflops": round(probe_flops / (probe_ms * 1e-3) / 1e12, 1),
                "clock_ghz": round(int(probe_cycles.item()) / (probe_ms * 1e-3) / 1e9, 3)}
    line["roofline"]["mfma_only_probe"] = dict(
        probe(False), note="register-only bf16 MFMA loop on the same chip, constant operands; "
                           "the 2500 peak assumes 2.4 GHz")
    line["roofline"]["mfma_only_probe_changing_operands"] = dict(
        probe(True), note="the same loop with a different random A operand for every MFMA and a "
                          "different B operand every second one, as in the attention kernel")

    parity_ok = True
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(np, torch, si, cache, q, k_blk, v_blk, c_len, out, P)
        par = line["cpu_baseline"]["gpu_vs_oracle_on_sample"]
        parity_ok = (par["max_abs_err"] <= BF16_MAX_ABS and par["rel_rms"] <= BF16_REL_RMS and
                     par["worst_head_rel_rms"] <= BF16_REL_RMS)
        par["within_bounds"] = parity_ok
    print(json.dumps(line))
    if not parity_ok:
        print("bench.py: the GPU rows disagree with the oracle beyond max|err| %.0e / rel-RMS %.0e"
              % (BF16_MAX_ABS, BF16_REL_RMS), file=sys.stderr)
        sys.exit(3)


def cpu_baseline(np, torch, si, cache, q, k_blk, v_blk, c_len, out, P):
    """Time the fp64 oracle on a bounded row sample of layer 0 and check the GPU rows on it; time
    the oracle's nested-loop commit on a slice of the layers."""
    from concurrent.futures import ThreadPoolExecutor

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
    num, den = np.sum(err * err, axis=(0, 2)), np.sum(ref * ref, axis=(0, 2))
    per_head = np.sqrt(num / den)

    # the oracle's commit (nested loops over layer, token, head, dim) on a slice of the layers:
    # one thread as it stands, then one such call per host thread on its own layer
    Lc = min(4, k_blk.shape[0])
    T = k_blk.shape[1]
    blk_k, blk_v = bits(k_blk[:Lc]), bits(v_blk[:Lc])
    slice_bytes = 2.0 * blk_k.nbytes                     # K and V of the slice
    mirror = oracle.KVMirror(1, T, H, D, T)
    t = time.perf_counter()
    oracle.kv_commit(mirror, blk_k[:1], blk_v[:1], 0)
    one_layer_s = time.perf_counter() - t
    n_par = max(1, min(threads, os.cpu_count() or 1))
    mirrors = [oracle.KVMirror(1, T, H, D, T) for _ in range(n_par)]
    with ThreadPoolExecutor(n_par) as pool:
        t = time.perf_counter()
        list(pool.map(lambda i: oracle.kv_commit(mirrors[i], blk_k[i % Lc:i % Lc + 1], blk_v[i % Lc:i % Lc + 1], 0),
                      range(n_par)))
        par_s = time.perf_counter() - t
    layer_bytes = slice_bytes / Lc
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": threads,
            "host_logical_cpus": os.cpu_count(), "kind": "oracle", "seconds": round(dt, 2),
            "sample": "%d of %d query rows x all %d heads of layer 0, all %d keys (fp64, OpenMP)"
                      % (len(rows), n_q, H, n_k),
            "extrapolated_seconds_for_one_full_call": round(dt * n_q / len(rows), 1),
            "gpu_vs_oracle_on_sample": {"max_abs_err": float(np.max(np.abs(err))),
                                        "rel_rms": float(math.sqrt(num.sum() / den.sum())),
                                        "worst_head_rel_rms": float(per_head.max()),
                                        "worst_head": int(per_head.argmax())},
            "oracle_commit": {"sample": "K and V of one layer (%d tokens x %d heads x %d, %.1f MB payload) per call"
                                        % (T, H, D, layer_bytes / 1e6),
                              "one_thread_seconds": round(one_layer_s, 4),
                              "one_thread_gbps": round(2 * layer_bytes / one_layer_s / 1e9, 3),
                              "threads": n_par, "all_threads_seconds": round(par_s, 4),
                              "all_threads_gbps": round(2 * layer_bytes * n_par / par_s / 1e9, 3),
                              "note": "read + write bytes; the GPU commit moves 40 such layers per launch"}}


if __name__ == "__main__":
    main()
