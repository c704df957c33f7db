#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A step is one pass of the whole layer over one batch of seeded synthetic tokens that are already
resident in HBM: gate + routing, dispatch, expert FFN, combine, and (for the fwd+bwd workload)
combine backward, expert FFN backward, dispatch backward and gate backward.  The default
workload is the 6.7B-base, 16-expert, tensor-parallel-shard layer forward + backward
(T=16384, h=4096, E=16, f=4096, capacity factor 1.25).

Prints ONE JSON line: tokens/s of the whole step, the roofline figure of the dominant kernel (the
grouped bf16 MFMA GEMM, timed live with events on the launch stream) and the CPU oracle timed on
a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0

RIDGE_ROWS = 300     # kept rows per expert below which an expert GEMM is bound by streaming its weights (peak flops / peak bytes)


def measured_gemm_traffic(workload: str):
    """HBM bytes per GEMM launch (average over the launches of a step) as measured with rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE, scaled by what the same counters read for a plain copy of known size.  Read
    from the committed summary profiles/gemm_traffic.txt (written by paper_2303_06318_amd/profile_summary.py
    from the raw counter CSVs of one run; it names the commit it was measured at).  None if the workload
    has no entry."""
    path = os.path.join(ROOT, "profiles", "gemm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        kv = dict(item.split("=", 1) for item in line.split())
        if kv.get("workload") == workload:
            return float(kv["bytes_per_launch"]), kv.get("commit")
    return None, None


def bench_optimizer(args, wl, layer, w1, w2):
    """Tiled mixed-precision AdamW step over the layer's expert parameters (two flat groups, W1 and W2, of
    E*h*f parameters each), with the gradients the last backward left in HBM.  Three variants of the same
    step: the paper's tiling with its fp32 staging tile (ts parameters), the same with a 16x larger tile,
    and the up-cast done in registers (no temporary).  Algorithmic bytes per parameter: 14 read + 14
    written (bf16 gradient and parameter copy, fp32 master weight and two moments)."""
    import torch
    from paper_2303_06318_amd import moe
    groups = []
    for w, g in ((w1, layer.d_w1), (w2, layer.d_w2)):
        gf = g.reshape(-1).float()
        groups.append(dict(n=w.numel(), grad=g.reshape(-1), master=w.reshape(-1).float(), m=0.3 * gf, v=gf * gf,
                           param=torch.empty_like(w.reshape(-1))))
        del gf
    n_total = sum(gr["n"] for gr in groups)
    cpu = None
    if not args.no_cpu_baseline:
        # the oracle's step on the first 16 M parameters of the first group, from the same state
        from oracle import moe_oracle as orc
        S = min(16 << 20, groups[0]["n"])
        h_ = {k: groups[0][k][:S].float().cpu().numpy() for k in ("grad", "master", "m", "v")}
        tc0 = time.perf_counter()
        orc.adamw_tiled(h_["grad"], h_["master"], h_["m"], h_["v"], ts=args.tile_size, lr=3e-4, beta1=0.9, beta2=0.95,
                        eps=1e-8, weight_decay=0.1, step=1)
        tc1 = time.perf_counter()
        cpu = {"value": round(S / (tc1 - tc0), 1), "unit": "params/s", "cores": 1, "kind": "oracle",
               "sample": f"first {S} parameters of W1's group, one step, ts = {args.tile_size}, {tc1 - tc0:.2f} s"}
        del h_
    big_ts = 16 * args.tile_size
    staging = torch.empty(big_ts, dtype=torch.float32, device="cuda")
    res = {"params": n_total, "groups": len(groups), "dtype": "f32 update, bf16 gradients and parameter copy",
           "bytes_per_param": 28, "peak_GBs": PEAK_HBM_GBS, "cpu_baseline": cpu}
    step_no = 0
    for name, ts, stg in (("tiled", args.tile_size, staging), ("tiled_16x", big_ts, staging), ("register_upcast", 1, None)):
        ms = []
        for it in range(2 + 5):
            step_no += 1
            hp = moe.make_adamw(3e-4, 0.9, 0.95, 1e-8, 0.1, step_no)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for gr in groups:
                moe.moe_adamw_tiled(gr["n"], ts, hp, gr["grad"], gr["master"], gr["m"], gr["v"], gr["param"], stg,
                                    moe.MOE_BF16)
            e1.record()
            torch.cuda.synchronize()
            if it >= 2:
                ms.append(e0.elapsed_time(e1))
        t = sum(ms) / len(ms)
        gbs = 28.0 * n_total / (t * 1e-3) / 1e9
        res[name] = {"params_per_s": round(n_total / (t * 1e-3), 1), "ts": None if stg is None else ts, "temporary_bytes": 0 if stg is None else 4 * min(ts, groups[0]["n"]),
                     "launches": len(groups) * (1 if stg is None else 2 * -(-groups[0]["n"] // ts)),
                     "ms": round(t, 4), "GBs": round(gbs, 1), "frac": round(gbs / PEAK_HBM_GBS, 4)}
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5_6p7b_tp4_fwdbwd")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=4096)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (known size) so that HBM counters can be scaled")
    ap.add_argument("--optimizer", action="store_true",
                    help="also time the tiled AdamW step over this layer's expert parameters (reported in an extra "
                         "\"optimizer\" object; never part of ms_per_step)")
    ap.add_argument("--recompute", action="store_true",
                    help="activation recomputation: hact and z_save are not kept, the backward runs GEMM1 again")
    ap.add_argument("--fused", action="store_true",
                    help="dispatch folded into GEMM1's operand load (forward-only workloads) and combine into GEMM2's "
                         "epilogue (moe_expert_ffn_fwd_fused)")
    ap.add_argument("--tile-size", type=int, default=1_800_000, help="ts of the tiled optimizer step")
    ap.add_argument("--no-isolated", action="store_true",
                    help="skip the isolated timings of the HBM-bound phases (clean and dirty caches)")
    ap.add_argument("--dtd", type=int, default=0, metavar="G",
                    help="also time the local halves of duplicate token dropping for a tensor-parallel group of G "
                         "(reported in an extra \"dtd\" object; never part of ms_per_step)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the layer on ONE GPU; --gpus must be 1 "
              "(nothing in this build crosses GPUs)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2303_06318_amd import moe, synth
    from paper_2303_06318_amd.layer import MoeLayer

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 3
    moe.lib()     # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    assert wl.dtype == "bf16", "the benchmark workloads are the bf16 ones"
    inp = synth.make_inputs(wl)

    def up(name):
        a = inp.bits.get(name)
        return None if a is None else torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)

    x, w1, w2, d_out = up("x"), up("w1"), up("w2"), up("d_out")
    wg = torch.from_numpy(inp.wg).cuda()
    bias = None if inp.logit_bias is None else torch.from_numpy(inp.logit_bias).cuda()
    layer = MoeLayer(wl.T, wl.h, wl.E, wl.f, wl.C, moe.MOE_BF16, moe.MOE_GELU_ERF, backward=wl.backward,
                     recompute=args.recompute)
    sh = layer.shape

    if args.fused:
        phases = ["gate"] + (["dispatch"] if wl.backward else []) + ["ffn_fwd"]
    else:
        phases = ["gate", "dispatch", "ffn_fwd", "combine"]
    phases += ["combine_bwd", "gate_bwd", "ffn_bwd", "dispatch_bwd"] if wl.backward else []

    def step(ev=None):
        n_mark = [0]

        def mark():
            if ev is not None:
                ev[n_mark[0]].record()
            n_mark[0] += 1
        mark()
        moe.moe_gate(sh, x, wg, bias, layer.logits, layer.probs, layer.expert, layer.gate_p, layer.slot, layer.counts,
                     layer.kept, layer.token_of_slot, layer.ws)
        mark()
        if args.fused:
            if wl.backward:      # the weight gradient reads the dispatched rows
                moe.moe_dispatch(sh, x, layer.token_of_slot, layer.buf)
                mark()
            moe.moe_expert_ffn_fwd_fused(sh, None if wl.backward else x, layer.buf if wl.backward else None,
                                         layer.token_of_slot, layer.slot, layer.gate_p, w1, w2, layer.kept,
                                         layer.z_save, layer.hact, layer.y if wl.backward else None, layer.out,
                                         layer.ws)
            mark()
        else:
            moe.moe_dispatch(sh, x, layer.token_of_slot, layer.buf)
            mark()
            moe.moe_expert_ffn_fwd(sh, layer.buf, w1, w2, layer.kept, layer.z_save, layer.hact, layer.y, layer.ws)
            mark()
            moe.moe_combine(sh, layer.y, layer.expert, layer.slot, layer.gate_p, layer.out)
            mark()
        if wl.backward:
            moe.moe_combine_bwd(sh, d_out, layer.y, layer.token_of_slot, layer.slot, layer.gate_p, layer.d_y,
                                layer.d_gate_p)
            mark()
            moe.moe_gate_bwd(sh, layer.d_gate_p, layer.probs, layer.expert, x, wg, layer.d_logits, layer.d_w_gate,
                             None, layer.ws)
            mark()
            moe.moe_expert_ffn_bwd(sh, layer.d_y, layer.buf, layer.z_save, layer.hact, w1, w2, layer.kept,
                                   layer.d_buf, layer.d_w1, layer.d_w2, layer.ws)
            mark()
            moe.moe_dispatch_bwd(sh, layer.d_buf, layer.expert, layer.slot, layer.d_x, layer.d_logits, wg)
            mark()

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    nev = len(phases) + 1
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(nev)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    phase_ms = {p: 0.0 for p in phases}
    for k in range(args.steps):
        for i, p in enumerate(phases):
            phase_ms[p] += events[k][i].elapsed_time(events[k][i + 1])
    phase_ms = {p: v / args.steps for p, v in phase_ms.items()}

    step_ms = sorted(events[k][0].elapsed_time(events[k][nev - 1]) for k in range(args.steps))
    median_ms = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])
    phase_med = {}
    for i, p in enumerate(phases):
        v = sorted(events[k][i].elapsed_time(events[k][i + 1]) for k in range(args.steps))
        phase_med[p] = v[len(v) // 2]

    # routing alone (softmax + top-1 from stored logits, histogram, slot assignment: three dependent small
    # launches) against the same number of empty launches: both are latency, not bandwidth
    def timed_us(fn, reps=50):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps
    route_launches = 3
    route_us = timed_us(lambda: moe.moe_gate(sh, None, None, None, layer.logits, layer.probs, layer.expert, layer.gate_p,
                                             layer.slot, layer.counts, layer.kept, layer.token_of_slot, layer.ws))
    floor_us = timed_us(lambda: moe.moe_launch_floor(route_launches))

    kept = layer.kept.cpu().numpy().astype(np.int64)
    counts = layer.counts.cpu().numpy().astype(np.int64)
    n_kept = int(kept.sum())
    # dominant kernel: the grouped bf16 MFMA GEMM.  Algorithmic flops per launch = 2*h*f*N_kept
    # (kept rows only); 2 launches in ffn_fwd, 4 in ffn_bwd.
    n_launch = 2 + ((5 if args.recompute else 4) if wl.backward else 0)
    gemm_ms = phase_ms["ffn_fwd"] + (phase_ms["ffn_bwd"] if wl.backward else 0.0)
    flops_per_launch = 2.0 * wl.hm * wl.fm * n_kept      # model sizes: zero padding to a multiple of 8 is not work
    avg_launch_ms = gemm_ms / n_launch
    achieved = flops_per_launch / (avg_launch_ms * 1e-3) / 1e12
    traffic, traffic_commit = measured_gemm_traffic(wl.name)
    # Which roofline bounds the expert GEMMs: with fewer kept rows per expert than the ridge (peak flops /
    # peak bytes, about 300 rows) a launch is bound by streaming the weights of the experts that hold rows.
    n_active = int((kept > 0).sum())
    rows_per_active = n_kept / max(n_active, 1)
    esz = 2
    bytes_per_launch = n_active * wl.hm * wl.fm * esz + n_kept * (wl.hm + wl.fm) * esz
    if rows_per_active < RIDGE_ROWS:
        gbs = bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": traffic, "traffic_measured_at_commit": traffic_commit,
                    "kernel": "gemm_bf16_kernel", "launches_per_step": n_launch,
                    "avg_launch_ms": round(avg_launch_ms, 4), "bytes_per_launch": bytes_per_launch,
                    "rows_per_active_expert": round(rows_per_active, 1), "active_experts": n_active,
                    "mfma_TFLOPs_for_information": round(achieved, 1),
                    "mfma_frac_for_information": round(achieved / PEAK_BF16_TFLOPS, 4)}
    else:
        roofline = {"bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                    "traffic_measured_at_commit": traffic_commit,
                    "kernel": "gemm_bf16_kernel", "launches_per_step": n_launch,
                    "avg_launch_ms": round(avg_launch_ms, 4), "flops_per_launch": flops_per_launch,
                    "bytes_per_launch": bytes_per_launch}

    hbm = {
        "gate": (wl.T * wl.hm * esz + wl.hm * wl.E * 4 + wl.T * wl.E * 4 * (2 if wl.backward else 1) + wl.T * 8),
        "dispatch": 2 * n_kept * wl.hm * esz + wl.T * 8,
        "combine": n_kept * wl.hm * esz + wl.T * wl.hm * esz + wl.T * 12,
    }
    if wl.backward:
        hbm["combine_bwd"] = 3 * n_kept * wl.hm * esz
        hbm["dispatch_bwd"] = n_kept * wl.hm * esz + wl.T * wl.hm * esz      # gate's d_x term fused in
        hbm["gate_bwd"] = wl.T * wl.hm * esz + wl.T * wl.E * 4 * 2           # d_logits, d_w_gate (reads x once)
    hbm_frac = {p: round(b / (phase_ms[p] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4) for p, b in hbm.items() if p in phase_ms}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import moe_oracle as orc
        S = min(args.cpu_sample_tokens, wl.T)
        Cs = orc.capacity(S, wl.E, wl.capacity_factor)
        tc0 = time.perf_counter()
        fw = orc.layer_forward(inp.x[:S], inp.wg, inp.w1, inp.w2, Cs, logit_bias=inp.logit_bias)
        if wl.backward:
            orc.layer_backward(fw, inp.d_out[:S], inp.x[:S], inp.wg, inp.w1, inp.w2)
        tc1 = time.perf_counter()
        cpu_baseline = {"value": round(S / (tc1 - tc0), 2), "unit": "tokens/s", "cores": orc.max_threads(),
                        "kind": "oracle",
                        "sample": f"first {S} tokens of the same workload through the whole layer "
                                  f"({'fwd+bwd' if wl.backward else 'fwd'}, all {wl.E} experts, capacity {Cs}), "
                                  f"{tc1 - tc0:.1f} s"}

    # The HBM-bound phases once more, each alone: after 1 GiB has been READ (the caches hold clean lines) and after
    # 1 GiB has been WRITTEN (they hold dirty lines, as they do inside a training step, where every phase follows
    # kernels that have just written hundreds of MB: each line a phase brings in then pushes a dirty line out, and
    # that write-back shares the HBM with the phase's own traffic).  Medians, one event pair per call (includes
    # about 6 us of launch and event overhead).
    isolated = None
    if not args.no_isolated:
        big = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        big.zero_()

        def alone_us(fn, flush, n=7):
            ts = []
            for _ in range(n):
                big.sum() if flush == "read" else big.fill_(1.0)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e3)
            return sorted(ts)[n // 2]
        calls = {
            "gate": lambda: moe.moe_gate(sh, x, wg, bias, layer.logits, layer.probs, layer.expert, layer.gate_p, layer.slot,
                                         layer.counts, layer.kept, layer.token_of_slot, layer.ws),
            "dispatch": lambda: moe.moe_dispatch(sh, x, layer.token_of_slot, layer.buf),
            "combine": lambda: moe.moe_combine(sh, layer.y, layer.expert, layer.slot, layer.gate_p, layer.out),
        }
        if wl.backward:
            calls["combine_bwd"] = lambda: moe.moe_combine_bwd(sh, d_out, layer.y, layer.token_of_slot, layer.slot,
                                                               layer.gate_p, layer.d_y, layer.d_gate_p)
            calls["gate_bwd"] = lambda: moe.moe_gate_bwd(sh, layer.d_gate_p, layer.probs, layer.expert, x, wg,
                                                         layer.d_logits, layer.d_w_gate, None, layer.ws)
            calls["dispatch_bwd"] = lambda: moe.moe_dispatch_bwd(sh, layer.d_buf, layer.expert, layer.slot, layer.d_x,
                                                                 layer.d_logits, wg)
        isolated = {"unit": "us", "launch_and_event_overhead": round(alone_us(lambda: moe.moe_launch_floor(1), "read"), 1),
                    "after_1GiB_read": {p: round(alone_us(f, "read"), 1) for p, f in calls.items()},
                    "after_1GiB_write": {p: round(alone_us(f, "write"), 1) for p, f in calls.items()}}
        del big

    dtd = None
    if args.dtd > 1:
        # One rank's drop fused with dispatch (1/G of the rows), the expert FFN reading all G shares in place, the
        # reassembling copy, and for a training step the backward's drop and the dispatch backward from shares.
        G = args.dtd
        Cg = -(-wl.C // G)
        shares = torch.empty((G, wl.E, Cg, wl.h), dtype=torch.bfloat16, device="cuda")
        for r in range(G):
            moe.moe_dispatch_dtd(sh, x, layer.token_of_slot, r, G, shares[r])
        dtd = {"tp_size": G, "share_rows_per_expert": Cg,
               "dispatch_dtd_one_rank_us": round(timed_us(lambda: moe.moe_dispatch_dtd(sh, x, layer.token_of_slot, 0, G, shares[0])), 2),
               "dispatch_whole_chunks_us": round(timed_us(lambda: moe.moe_dispatch(sh, x, layer.token_of_slot, layer.buf)), 2),
               "ffn_fwd_from_shares_us": round(timed_us(lambda: moe.moe_expert_ffn_fwd_dtd(
                   sh, shares, G, w1, w2, layer.kept, layer.z_save, layer.hact, layer.y, layer.ws), 10), 2),
               "ffn_fwd_from_chunks_us": round(timed_us(lambda: moe.moe_expert_ffn_fwd(
                   sh, layer.buf, w1, w2, layer.kept, layer.z_save, layer.hact, layer.y, layer.ws), 10), 2),
               "gather_copy_us": round(timed_us(lambda: moe.moe_dtd_gather(sh, shares, layer.kept, G, layer.buf)), 2)}
        if wl.backward:
            d_shares = torch.empty_like(shares)
            for r in range(G):
                moe.moe_dtd_drop(sh, layer.d_buf, layer.kept, r, G, d_shares[r])
            dtd["drop_d_buf_one_rank_us"] = round(timed_us(lambda: moe.moe_dtd_drop(sh, layer.d_buf, layer.kept, 0, G, d_shares[0])), 2)
            dtd["dispatch_bwd_from_shares_us"] = round(timed_us(lambda: moe.moe_dispatch_bwd_dtd(
                sh, d_shares, G, layer.expert, layer.slot, layer.d_x, layer.d_logits, wg)), 2)
            dtd["dispatch_bwd_from_chunks_us"] = round(timed_us(lambda: moe.moe_dispatch_bwd(
                sh, layer.d_buf, layer.expert, layer.slot, layer.d_x, layer.d_logits, wg)), 2)
        del shares

    optimizer = None
    if args.optimizer:
        optimizer = bench_optimizer(args, wl, layer, w1, w2)

    out = {
        "metric": "MoE-layer tokens/sec " + ("fwd+bwd" if wl.backward else "fwd") + f" at h={wl.hm},E={wl.E} (1 GPU)",
        "value": round(wl.T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(median_ms, 4),
        "kept_tokens_per_s": round(n_kept / (ms_per_step * 1e-3), 1),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name, "T": wl.T, "h": wl.hm, "E": wl.E, "f": wl.fm, "h_stored": wl.h, "f_stored": wl.f,
                   "C": wl.C,
                   "capacity_factor": wl.capacity_factor, "n_kept": n_kept,
                   "count_min": int(counts.min()), "count_max": int(counts.max()), "seed": wl.seed,
                   "pass": "fwd+bwd" if wl.backward else "fwd", "activation_recomputation": bool(args.recompute),
                   "fused_permutations": bool(args.fused)},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "phase_ms": {p: round(v, 4) for p, v in phase_ms.items()},
        "phase_ms_median": {p: round(v, 4) for p, v in phase_med.items()},
        "route": {"us": round(route_us, 2), "launches": route_launches, "empty_launch_floor_us": round(floor_us, 2),
                  "what": "softmax + top-1 from stored logits, histogram, slot assignment (moe_gate with x = NULL) "
                          "against the same number of empty kernels, back to back on one stream"},
        "hbm_frac_of_8TBs": hbm_frac,
    }
    if isolated is not None:
        out["hbm_phases_alone"] = isolated
    if optimizer is not None:
        out["optimizer"] = optimizer
    if dtd is not None:
        out["dtd"] = dtd
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
