#!/usr/bin/env python3
"""Serves a synthetic API-augmented trace on one MI355X for real: the LAMPS scheduler
(lamps_sched.h) picks the batch every iteration and the library's GPU calls execute it
(append + decode attention, swap out / in, discard + recompute through prefill attention).

    python -m paper_2410_18248_amd.serve_live [--policy lamps|fcfs|sjf] [--requests 32] [--layers 4]

There is no model (no GEMMs): per-layer q / k / v come from a seeded random source, so
the numbers are those of the cache-management and attention path alone.  API durations are
the paper's API-table classes scaled by --time-scale so that a run takes seconds.
Prints one JSON object.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2410_18248_amd as P  # noqa: E402
from paper_2410_18248_amd.engine import DeviceSource, LiveEngine, RandomSource  # noqa: E402
from paper_2410_18248_amd.serve_sim import synthetic_trace  # noqa: E402


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--policy", default="lamps", choices=["fcfs", "sjf", "sjf_total", "lamps"])
    ap.add_argument("--requests", type=int, default=32)
    ap.add_argument("--rate", type=float, default=200.0, help="arrivals per second (of scaled time)")
    ap.add_argument("--time-scale", type=float, default=1e-3, help="API durations are multiplied by this")
    ap.add_argument("--layers", type=int, default=4)
    ap.add_argument("--heads", type=int, default=40)
    ap.add_argument("--kv-heads", type=int, default=40)
    ap.add_argument("--memory-tokens", type=int, default=6000)
    ap.add_argument("--max-batch", type=int, default=16)
    ap.add_argument("--seed", type=int, default=2410)
    ap.add_argument("--source", default="device", choices=["device", "host"],
                    help="where the random q / k / v rows are made (host: slow, the tests' source)")
    ap.add_argument("--layered-swap", action="store_true", help="swap layer-major (a returning request runs layer by layer)")
    a = ap.parse_args()
    import torch
    pol = {"fcfs": P.LAMPS_POLICY_FCFS, "sjf": P.LAMPS_POLICY_SJF, "sjf_total": P.LAMPS_POLICY_SJF_TOTAL,
           "lamps": P.LAMPS_POLICY_LAMPS}[a.policy]
    bs, D = 16, 128
    nb = a.memory_tokens // bs + a.requests + 8
    cfg = P.LampsConfig(a.layers, a.heads, a.kv_heads, D, bs, nb, 256, a.max_batch, P.LAMPS_BF16, 0.0, 0, 0)
    M = float(P.lamps_kv_bytes_per_token(cfg))
    # cost model used for the handling decision and the rank only (time itself is measured)
    cost = P.LampsCostModel(2e-3, 2e-8 * a.layers, 1e-3, 3e-6 * a.layers, 3e-4, 3.7e-7 * a.layers, 0, 0)
    scfg = P.LampsSchedConfig(pol, a.max_batch, a.memory_tokens, 100, 1, 2048, 0.5 * a.memory_tokens, M, cost)
    make = DeviceSource if a.source == "device" else RandomSource
    eng = LiveEngine(cfg, scfg, make(a.seed, a.heads, a.kv_heads, D, torch.bfloat16), layered_swap=a.layered_swap)
    trace = synthetic_trace(a.seed, a.requests, a.rate)
    for rid, arr, prompt, segs, _ in trace:
        eng.add(rid, arr, prompt, [(n, None if d is None else d * a.time_scale, rho, None) for n, d, rho in segs])
    t0 = time.perf_counter()
    stats = eng.run(progress=100)
    wall = time.perf_counter() - t0
    lat, ttft, mix = [], [], [0, 0, 0]
    for rid, arr, prompt, segs, _ in trace:
        c, f, h = eng.sched.result(rid, len(segs))
        lat.append(c - arr)
        ttft.append(f - arr)
        for x in h[:-1]:
            mix[x] += 1
    free_ok = eng.lam.num_free() == nb
    out = {"policy": a.policy, "requests": a.requests, "layers": a.layers, "heads": a.heads, "kv_heads": a.kv_heads,
           "memory_tokens": a.memory_tokens, "wall_s": wall, "scheduler_time_s": eng.sched.now(), **stats,
           "generated_tokens_per_s": stats["decode_tokens"] / wall,
           "mean_latency_s": float(np.mean(lat)), "p99_latency_s": float(np.percentile(lat, 99)),
           "mean_ttft_s": float(np.mean(ttft)), "handling_preserve_discard_swap": mix,
           "all_blocks_free_at_end": bool(free_ok),
           "note": "no model: q/k/v are seeded random tensors (made on the %s); gpu_s is the time from the first "
                   "enqueue of an iteration to the compute stream running dry, the iteration time the scheduler "
                   "is given" % a.source}
    eng.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
