#!/usr/bin/env python3
"""Benchmark of the spa2 hot path on one MI355X.

A step is one pass of the whole path over one batch of seeded synthetic input that is
already resident in HBM: block masker (pool, select, column lists), block-sparse
attention forward, backward (D, dK/dV, dQ).  The stage entry points of the C ABI are
called one after the other — exactly the sequence spa2_mask / spa2_fwd / spa2_bwd make —
with a HIP event between them, so every kernel's duration comes out of the timed region.

Prints ONE JSON line.  `value` is the effective throughput of the step: FLOPs of the
executed tiles (4*rows*cols*d forward + 10*rows*cols*d backward, valid rows and columns
only) divided by the step time, masker included.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="wan14b-720p-95")
    ap.add_argument("--dense-steps", type=int, default=1, help="timed dense fwd+bwd passes (0 = skip)")
    ap.add_argument("--overlap-steps", type=int, default=5,
                    help="extra steps with dQ and dK/dV on two streams, reported as two_stream_backward (0 = skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the warm-up, run one plain device-to-device copy of this many MiB (a kernel of "
                         "known HBM traffic against which rocprofv3's FETCH_SIZE / WRITE_SIZE are scaled)")
    return ap.parse_args()


def tile_flops_per_d(mask, N):
    """sum over selected tiles of valid_rows * valid_cols (a torch reduction on the device: bookkeeping
    for the metric, not part of the path)."""
    import torch
    Tm, Tn = mask.shape[-2:]
    rv = torch.full((Tm,), 128.0, device=mask.device, dtype=torch.float64)
    cv = torch.full((Tn,), 64.0, device=mask.device, dtype=torch.float64)
    rv[-1] = N - 128 * (Tm - 1)
    cv[-1] = N - 64 * (Tn - 1)
    per_row = (mask.to(torch.float32) @ cv.to(torch.float32)).to(torch.float64)     # [B,H,Tm]
    return float((per_row * rv).sum().item())


def cpu_baseline(w, q, k, v, do, heads=((0, 0), (0, -1))):
    """The fp64 oracle, as it stands, on two heads of the same workload (the first and the last): pooling,
    pooled map, selection, gather-form attention forward and gradients."""
    import numpy as np
    from oracle import spa2_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    heads = sorted({(b % w.B, h % w.H) for b, h in heads})
    flops, tiles, dt = 0.0, 0, 0.0
    for b, h in heads:
        qd, kd, vd, dod = (t[b, h].to("cpu").double().numpy() for t in (q, k, v, do))
        t0 = time.perf_counter()
        k_cnt = orc.topk_blocks(w.k_frac, w.Tn)
        m, _ = orc.block_mask(qd, kd, k_cnt, float(np.float32(w.top_p)))
        if w.backward:
            orc.attention_bwd_gather(qd, kd, vd, m, dod)
        else:
            orc.attention_gather(qd, kd, vd, m)
        dt += time.perf_counter() - t0
        Tm, Tn = m.shape
        rv = np.full(Tm, 128.0); rv[-1] = w.N - 128 * (Tm - 1)
        cv = np.full(Tn, 64.0); cv[-1] = w.N - 64 * (Tn - 1)
        flops += float((m * rv[:, None] * cv[None, :]).sum()) * (14.0 if w.backward else 4.0) * w.d
        tiles += int(m.sum())
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{len(heads)} of {w.B * w.H} heads {heads} of {w.name}: mask + fwd{' + bwd' if w.backward else ''} in fp64 numpy, "
                      f"{dt:.1f} s, {tiles} tiles"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (the path would shard by head, with no "
              "communication between the shards)", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2602_13515_amd as spa2
    from paper_2602_13515_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    w = wl.CONFIGS[args.workload]
    scale = 1.0 / math.sqrt(w.d)
    q, k, v, do = wl.make_inputs(w, seed=args.seed, device=dev, need_do=True)
    o = torch.empty_like(q); o_res = torch.empty_like(q); dq = torch.empty_like(q); dk = torch.empty_like(q); dv = torch.empty_like(q)
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=dev)
    pat = spa2.alloc_pattern(w.B, w.H, w.N, dev)
    ws_m = torch.empty(spa2.spa2_mask_workspace_bytes(q), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(spa2.spa2_bwd_workspace_bytes(q), dtype=torch.uint8, device=dev)
    ws_f = torch.empty(spa2.spa2_fwd_workspace_bytes(q), dtype=torch.uint8, device=dev)
    k_cnt = spa2.spa2_topk_blocks(w.k_frac, w.Tn)

    stages = ["pool", "select", "columns", "fwd", "delta", "dkdv", "dq"]

    def step(p, events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        spa2.spa2_mask_pool(q, k, ws_m); mark(1)
        spa2.spa2_mask_select(q, k_cnt, w.top_p, scale, p, None, ws_m); mark(2)
        spa2.spa2_mask_columns(q, p); mark(3)
        spa2.spa2_fwd(q, k, v, p, scale, o, lse, o_res, ws_f); mark(4)
        if w.backward:        # a forward-only configuration stops here (its stage times below read 0)
            spa2.spa2_bwd_delta(o, do, ws_b, o_res); mark(5)
            spa2.spa2_bwd_dkdv(q, k, v, do, lse, p, scale, dk, dv, ws_b); mark(6)
            spa2.spa2_bwd_dq(q, k, v, do, lse, p, scale, dq, ws_b); mark(7)
        else:
            mark(5); mark(6); mark(7)

    if args.calibration_copy_mib > 0:
        src = torch.empty(args.calibration_copy_mib << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step(pat)
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(pat, evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    stage_ms = {n: sum(e[i].elapsed_time(e[i + 1]) for e in evs) / args.steps for i, n in enumerate(stages)}

    units = tile_flops_per_d(pat.mask, w.N)            # sum of rows*cols over executed tiles
    n_tiles = int(pat.mask.sum().item())
    density = n_tiles / pat.mask.numel()
    fwd_flops = 4.0 * units * w.d
    bwd_flops = 10.0 * units * w.d if w.backward else 0.0
    value = (fwd_flops + bwd_flops) / (ms_per_step * 1e-3) / 1e12

    # per-kernel rates.  Algorithmic FLOPs: fwd 4*r*c*d; backward 10*r*c*d of which the dK/dV kernel
    # carries S, dP, dV, dK (8) and the dQ kernel carries dQ (2) -- its S and dP are re-computation.
    kern = {
        "spa2_fwd": {"ms": stage_ms["fwd"], "alg_tflops": fwd_flops / stage_ms["fwd"] / 1e9,
                     "executed_tflops": fwd_flops / stage_ms["fwd"] / 1e9},
    }
    if w.backward:
        kern["spa2_bwd_dkdv"] = {"ms": stage_ms["dkdv"], "alg_tflops": 8.0 * units * w.d / stage_ms["dkdv"] / 1e9,
                                 "executed_tflops": 8.0 * units * w.d / stage_ms["dkdv"] / 1e9}
        kern["spa2_bwd_dq"] = {"ms": stage_ms["dq"], "alg_tflops": 2.0 * units * w.d / stage_ms["dq"] / 1e9,
                               "executed_tflops": 6.0 * units * w.d / stage_ms["dq"] / 1e9}
    pool_bytes = 2.0 * w.B * w.H * w.N * w.d * 2
    delta_bytes = 3.0 * w.B * w.H * w.N * w.d * 2 + 4.0 * w.B * w.H * w.N      # O, O residual, dO; D
    hbm = {
        "spa2_mask_pool": {"ms": stage_ms["pool"], "alg_gbs": pool_bytes / stage_ms["pool"] / 1e6},
    }
    if w.backward:
        hbm["spa2_bwd_delta"] = {"ms": stage_ms["delta"], "alg_gbs": delta_bytes / stage_ms["delta"] / 1e6}
    dom = max(kern, key=lambda n: kern[n]["ms"])
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(w.name, {}).get(dom)
        except Exception:
            traffic = None
    roofline = {"kernel": dom, "bound": "mfma", "achieved": kern[dom]["alg_tflops"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": kern[dom]["alg_tflops"] / PEAK_BF16_TFLOPS, "traffic": traffic,
                "ms_per_launch": kern[dom]["ms"],
                # not measured in this run: counters need rocprofv3 around the process
                "traffic_source": "profiles/traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE runs of this command, see profiles/)"
                                  if traffic is not None else None}

    # the same step with the two backward kernels launched at the same time on two streams (the operator's
    # overlap_backward option).  Reported beside the headline, never as it: per-kernel durations, and with them
    # the roofline above, only mean something when the kernels run one after the other.
    two_stream = None
    if w.backward and args.overlap_steps > 0:
        from paper_2602_13515_amd.autograd import backward_two_streams

        def overlapped_step():
            spa2.spa2_mask_pool(q, k, ws_m)
            spa2.spa2_mask_select(q, k_cnt, w.top_p, scale, pat, None, ws_m)
            spa2.spa2_mask_columns(q, pat)
            spa2.spa2_fwd(q, k, v, pat, scale, o, lse, o_res, ws_f)
            backward_two_streams(q, k, v, o, do, lse, pat, scale, dq, dk, dv, ws_b, o_res)
        overlapped_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.overlap_steps):
            overlapped_step()
        torch.cuda.synchronize()
        ov_ms = (time.perf_counter() - t1) * 1e3 / args.overlap_steps
        two_stream = {"ms_per_step": ov_ms, "tflops": (fwd_flops + bwd_flops) / ov_ms / 1e9, "steps": args.overlap_steps}

    # dense attention through the same kernels (all-ones pattern), same tensors
    dense = None
    if args.dense_steps > 0:
        full = spa2.alloc_pattern(w.B, w.H, w.N, dev)
        spa2.spa2_pattern_full(q, full)

        def dense_step():
            spa2.spa2_fwd(q, k, v, full, scale, o, lse, o_res, ws_f)
            if w.backward:
                spa2.spa2_bwd(q, k, v, o, do, lse, full, scale, dq, dk, dv, ws_b, o_res)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.dense_steps):
            dense_step()
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1) / args.dense_steps
        dense_flops = (14.0 if w.backward else 4.0) * float(w.B * w.H) * float(w.N) * float(w.N) * w.d
        dense = {"ms": dense_ms, "tflops": dense_flops / dense_ms / 1e9,
                 "speedup_attention_only": dense_ms / (stage_ms["fwd"] + stage_ms["delta"] + stage_ms["dkdv"] + stage_ms["dq"]),
                 "speedup_with_masker": dense_ms / ms_per_step}
        del full

    out = {
        "metric": "sparse_attn_fwd_bwd_effective_tflops_at_95pct_block_sparsity",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d": w.d, "k_frac": w.k_frac,
                   "top_p": w.top_p, "topk_blocks": k_cnt, "block_q": 128, "block_kv": 64,
                   "executed_tiles": n_tiles, "block_sparsity": 1.0 - density},
        "stage_ms": stage_ms,
        "mask_ms": stage_ms["pool"] + stage_ms["select"] + stage_ms["columns"],
        "fwd_ms": stage_ms["fwd"], "bwd_ms": stage_ms["delta"] + stage_ms["dkdv"] + stage_ms["dq"],
        "fwd_tflops": kern["spa2_fwd"]["alg_tflops"],
        "bwd_tflops": (bwd_flops / (stage_ms["delta"] + stage_ms["dkdv"] + stage_ms["dq"]) / 1e9) if w.backward else None,
        "dense": dense,
        "two_stream_backward": two_stream,
        "roofline": roofline, "kernels": kern, "hbm_kernels": hbm,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, q, k, v, do)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
