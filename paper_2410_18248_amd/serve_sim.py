#!/usr/bin/env python3
"""LAMPS against FCFS on one MI355X: the library's scheduler (lamps_sched.h) run
over a synthetic API-augmented request trace, with the engine's times measured
on the GPU through the library's own decode and swap calls.

    python -m paper_2410_18248_amd.serve_sim [--requests 600] [--rates 2,4,6,8] [--memory-gb 40]

What is measured and what is assumed
  * iteration time = weights + attention.  Attention per context token (it_b)
    is MEASURED: lamps_decode_attn over all layers of a Vicuna-13B-shaped cache
    (40 layers, 40 heads of 128, bf16; Section 6 names the model) at several
    batch compositions, least-squares line through the points.  The weight pass
    (it_a) is not part of this library: it is taken as parameter bytes over the
    read bandwidth the decode kernel itself achieves, and said so in the output.
  * T_swap(C) is MEASURED: lamps_swap_out + lamps_swap_in of C tokens' blocks.
    The library overlaps swaps with decode (swap_stalls = 0); the paper's
    substrate stalls the batch (equation (3)), which --paper-substrate models.
  * T_fwd(C) (recompute after Discard) needs a prefill pass, which this library
    does not have: fwd_b is 2 * parameters flop per token over an assumed
    fraction of the dense bf16 matrix peak.
  * The trace stands in for the paper's INFERCEPT mix (not available): six API
    classes with the (mean, std) durations and call counts of the paper's API
    table, prompts and segment lengths drawn uniformly; Poisson arrivals.
    Predictions are perfect (the paper's predictor needs its training data).

Prints one JSON object: per policy the paper's metrics (mean / P99 end-to-end
latency and time to first token, throughput) and the handling mix chosen by
equations (1)-(3).
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

# (duration mean, std) seconds and (calls mean, std) per request: the paper's API table
API_CLASSES = {
    "math": ((9e-5, 6e-5), (3.75, 1.3)),
    "qa": ((0.69, 0.17), (2.52, 1.73)),
    "ve": ((0.09, 0.014), (28.18, 15.2)),
    "chatbot": ((28.6, 15.6), (4.45, 1.96)),
    "image": ((20.03, 7.8), (6.91, 3.93)),
    "tts": ((17.24, 7.6), (6.91, 3.93)),
}
PARAM_BYTES = 13.0e9 * 2          # Vicuna 13B in bf16
FLOP_PER_TOKEN = 2 * 13.0e9
MFMA_PEAK = 2.5e15
PREFILL_EFFICIENCY = 0.4          # assumed share of the dense bf16 peak a prefill pass reaches


def synthetic_trace(seed, n, rate):
    """n requests: (id, arrival, prompt, [(n_out, api_duration|None, response), ...], class)."""
    rng = np.random.default_rng(seed)
    names = list(API_CLASSES)
    t = 0.0
    out = []
    for i in range(n):
        t += rng.exponential(1.0 / rate)
        cls = names[int(rng.integers(len(names)))]
        (dm, ds), (nm, ns) = API_CLASSES[cls]
        calls = int(min(32, max(1, round(rng.normal(nm, ns)))))
        segs = []
        for _ in range(calls):
            segs.append((int(rng.integers(8, 129)), float(max(1e-5, rng.normal(dm, ds))),
                         int(rng.integers(4, 65))))
        segs.append((int(rng.integers(8, 129)), None, 0))
        out.append((i, t, int(rng.integers(32, 513)), segs, cls))
    return out


def calibrate(verbose=False):
    """Measures attention time per context token and swap time per token on cuda:0."""
    import torch
    L, H, D, bs = 40, 40, 128, 16
    dev = torch.device("cuda:0")
    points = [(64, 256), (128, 256), (256, 256), (256, 512)]      # (batch, context each)
    max_b = max(b for b, _ in points)
    nb = max(b * ((c + bs - 1) // bs) for b, c in points) + 300
    cfg = P.LampsConfig(L, H, H, D, bs, nb, 64, max_b, P.LAMPS_BF16, 0.0, 0, 0)
    shape = (nb, L, H, bs * D)
    k_pool = torch.empty(shape, dtype=torch.bfloat16, device=dev).normal_()
    v_pool = torch.empty(shape, dtype=torch.bfloat16, device=dev).normal_()
    ws = torch.empty(P.lamps_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
    cs, so, si = (torch.cuda.Stream(dev) for _ in range(3))
    torch.cuda.synchronize()
    lam = P.Lamps(cfg, k_pool, v_pool, ws, cs.cuda_stream, so.cuda_stream, si.cuda_stream)
    ids = lam.alloc_blocks(nb)
    perm = torch.randperm(nb - 300, device="cpu").to(torch.int32)
    xs, ys = [], []
    for B, C in points:
        per = (C + bs - 1) // bs
        table = torch.full((B, 64), -1, dtype=torch.int32)
        table[:, :per] = perm[:B * per].reshape(B, per)
        td = table.to(dev)
        cd = torch.full((B,), C, dtype=torch.int32, device=dev)
        md = torch.ones(B, dtype=torch.uint8, device=dev)
        q = torch.empty((B, H, D), dtype=torch.bfloat16, device=dev).normal_()
        out = torch.empty_like(q)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for rep in range(3):
            e0.record(cs)
            for layer in range(L):
                lam.decode_attn(layer, B, q, td, cd, md, out)
            e1.record(cs)
            cs.synchronize()
        xs.append(B * C)
        ys.append(e0.elapsed_time(e1) * 1e-3)
        if verbose:
            print("decode B=%d C=%d: %.3f ms" % (B, C, ys[-1] * 1e3), file=sys.stderr)
    A = np.vstack([np.ones(len(xs)), np.array(xs, dtype=np.float64)]).T
    (att_a, att_b), *_ = np.linalg.lstsq(A, np.array(ys), rcond=None)
    read_bw = (P.lamps_kv_bytes_per_token(cfg) * xs[-1]) / ys[-1]
    # swap: out then in, n blocks (16 tokens each)
    sx, sy = [], []
    block_bytes = P.lamps_block_bytes(cfg)
    host = torch.empty(256 * block_bytes, dtype=torch.uint8).pin_memory()
    for nblk in (4, 16, 64, 256):
        sel = [int(x) for x in ids[nb - 300:nb - 300 + nblk]]
        for rep in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            lam.ticket_wait(lam.swap_out(sel, host))
            lam.ticket_wait(lam.swap_in(host, sel))
            dt = time.perf_counter() - t0
        sx.append(nblk * bs)
        sy.append(dt / 2)                            # one direction
        if verbose:
            print("swap %d blocks: %.3f ms each way" % (nblk, sy[-1] * 1e3), file=sys.stderr)
    A = np.vstack([np.ones(len(sx)), np.array(sx, dtype=np.float64)]).T
    (sw_a, sw_b), *_ = np.linalg.lstsq(A, np.array(sy), rcond=None)
    lam.destroy()
    return {"attention_per_iteration_s": float(max(att_a, 0.0)), "attention_per_token_s": float(att_b),
            "decode_read_GBs": float(read_bw / 1e9), "swap_fixed_s": float(max(sw_a, 0.0)),
            "swap_per_token_s": float(sw_b), "kv_bytes_per_token": int(P.lamps_kv_bytes_per_token(cfg)),
            "points_decode": list(zip(xs, ys)), "points_swap": list(zip(sx, sy))}


def run_policy(policy, trace, cost, memory_tokens, max_batch, c_other, M, starvation, refresh):
    cfg = P.LampsSchedConfig(policy, max_batch, memory_tokens, starvation, refresh, 2048, c_other, M, cost)
    s = P.LampsSched(cfg)
    for rid, arr, prompt, segs, _ in trace:
        s.add(rid, arr, prompt, [(a, b, c, None) for a, b, c in segs])
    t0 = time.perf_counter()
    s.run()
    wall = time.perf_counter() - t0
    lat, ttft, mix = [], [], [0, 0, 0]
    tokens = 0
    for rid, arr, prompt, segs, _ in trace:
        c, f, h = s.result(rid, len(segs))
        lat.append(c - arr)
        ttft.append(f - arr)
        tokens += sum(x[0] for x in segs)
        for x in h[:-1]:
            mix[x] += 1
    iters, peak, pre = s.stats()
    end = s.now()
    s.destroy()
    lat, ttft = np.array(lat), np.array(ttft)
    return {"mean_latency_s": float(lat.mean()), "p99_latency_s": float(np.percentile(lat, 99)),
            "mean_ttft_s": float(ttft.mean()), "p99_ttft_s": float(np.percentile(ttft, 99)),
            "throughput_req_s": len(trace) / end, "throughput_tok_s": tokens / end,
            "handling_preserve_discard_swap": mix, "iterations": iters, "peak_memory_tokens": peak,
            "out_of_memory_discards": pre, "scheduler_us_per_iteration": wall / max(iters, 1) * 1e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--requests", type=int, default=600)
    ap.add_argument("--rates", default="2,4,6,8", help="arrival rates to run, requests per second")
    ap.add_argument("--memory-gb", type=float, default=40.0,
                    help="GPU memory for weights + KV cache (the paper limits its GPUs to 40 GB)")
    ap.add_argument("--max-batch", type=int, default=256)
    ap.add_argument("--seed", type=int, default=2410)
    ap.add_argument("--paper-substrate", action="store_true",
                    help="swaps stall the running batch, as in the paper's equation (3)")
    ap.add_argument("--no-gpu", action="store_true", help="use stored stand-in times (no calibration)")
    a = ap.parse_args()
    if a.no_gpu:
        cal = {"attention_per_iteration_s": 6e-4, "attention_per_token_s": 1.45e-7, "decode_read_GBs": 5700.0,
               "swap_fixed_s": 2e-4, "swap_per_token_s": 1.5e-5, "kv_bytes_per_token": 819200,
               "note": "stand-in values, not measured in this run"}
    else:
        cal = calibrate(verbose=True)
    M = cal["kv_bytes_per_token"]
    weights_s = PARAM_BYTES / (cal["decode_read_GBs"] * 1e9)
    fwd_b = FLOP_PER_TOKEN / (MFMA_PEAK * PREFILL_EFFICIENCY)
    cost = P.LampsCostModel(weights_s + cal["attention_per_iteration_s"], cal["attention_per_token_s"],
                            weights_s, fwd_b, cal["swap_fixed_s"], cal["swap_per_token_s"],
                            1 if a.paper_substrate else 0, 0)
    memory_tokens = int((a.memory_gb * 1e9 - PARAM_BYTES) / M)
    c_other = 0.5 * memory_tokens                    # half the cache in use by others, as an estimate
    runs = []
    for rate in [float(x) for x in a.rates.split(",")]:
        trace = synthetic_trace(a.seed, a.requests, rate)
        res = {}
        for name, pol in (("fcfs", P.LAMPS_POLICY_FCFS), ("sjf", P.LAMPS_POLICY_SJF),
                          ("sjf_total", P.LAMPS_POLICY_SJF_TOTAL), ("lamps", P.LAMPS_POLICY_LAMPS)):
            res[name] = run_policy(pol, trace, cost, memory_tokens, a.max_batch, c_other, float(M), 100, 1)
        runs.append({"rate_per_s": rate, "policies": res,
                     "lamps_vs_fcfs": {k: res["lamps"][k] / res["fcfs"][k] for k in
                                       ("mean_latency_s", "p99_latency_s", "mean_ttft_s", "p99_ttft_s",
                                        "throughput_req_s")}})
    out = {"trace": {"requests": a.requests, "seed": a.seed,
                     "classes": "paper's API table (mean, std) durations and call counts; synthetic lengths"},
           "engine": {"model": "Vicuna-13B-shaped (40 layers, 40 heads x 128, bf16)",
                      "memory_tokens": memory_tokens, "max_batch": a.max_batch,
                      "iteration_fixed_s": cost.it_a, "iteration_per_context_token_s": cost.it_b,
                      "weights_pass_s (assumed: parameter bytes / measured read bandwidth)": weights_s,
                      "t_fwd_per_token_s (assumed: 2*params flop at %.0f%% of 2.5 PFLOP/s)"
                      % (100 * PREFILL_EFFICIENCY): fwd_b,
                      "t_swap_fixed_s": cost.sw_a, "t_swap_per_token_s": cost.sw_b,
                      "swaps_stall_batch": bool(a.paper_substrate), "calibration": cal},
           "runs": runs}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
