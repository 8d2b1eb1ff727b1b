#!/usr/bin/env python3
"""Benchmark of the LAMPS decode hot path on one MI355X.

A "step" is one pass of the hot path over one synthetic batch: paged decode
attention for the running requests of the batch (one call per layer through
the C ABI), while the batch's Swap-state requests have their blocks swapped
out to pinned host memory, freed, re-allocated and swapped back in on side
streams, Preserve-state requests stay masked, and Discard-state requests'
blocks are freed.  Inputs are resident in HBM before the timed region.

Timing rule.  A second host thread keeps the Swap-state requests' blocks moving
the way the configuration states it -- configuration 1: out to pinned host
memory; 2: back in from it, into freshly allocated blocks; 3 and 4: out, freed,
re-allocated and back in -- round after round (at most two groups of 128 MiB to
1 GiB in flight at a time), from before the warm-up steps until after the timed
steps, so the host link is busy in those directions throughout.  The warm-up
steps run, the compute stream is synchronised, exactly K steps are timed (host
clock from before the first call until the compute stream has drained; HIP
events on the compute stream for the kernel time), then the swap thread is told
to stop and what it started is drained outside the timed region.  `value` =
running requests x K / that time: tokens/s of one full decode-attention step
with swaps in flight, whatever K is; the swap GB/s achieved during the timed
steps is reported next to it.

With no --config the line's headline is configuration 4 (the largest: 40
layers, 113 GB of pools) and configurations 1-3 are measured the same way and
reported under "per_config".  Prints ONE JSON line with the HBM roofline of the
decode kernel and the CPU oracle timed on the host cores as a reported baseline.
"""
import argparse
import collections
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E bandwidth

# HBM bytes per decode launch measured with rocprofv3 --pmc (FETCH_SIZE run + WRITE_SIZE run,
# each scaled by the same counter's reading for a plain 1 GiB copy: x2.0 and x1.0), keyed by
# workload name; summaries in profiles/.  None where not measured.
MEASURED_TRAFFIC_BYTES = {
    "cfg1-7b-mha-bf16": 889187000,     # decode_balanced + decode_merge_balanced
    "cfg2-8b-gqa-bf16": 1713836000,
    "cfg3-long-gqa-bf16": 1546508000,
    "cfg4-13b-40layer-bf16": 2177279000,   # per layer
    # prefill_mfma, fetched + written (same counters, same scale factors)
    "prefill-4x4096-new-on-0-cached-H32-Hkv8-D128": 359935000,
    "prefill-4x4096-new-on-0-cached-H40-Hkv40-D128": 693023000,
    "prefill-64x8-new-on-2048-cached-H32-Hkv8-D128": 550227000,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="0 = enough steps for ~50 ms of decode")
    ap.add_argument("--warmup", type=int, default=-1)
    ap.add_argument("--config", type=int, default=0,
                    help="workload 1..4 alone; 0 (default) = 4 as the headline and 1-3 under per_config")
    ap.add_argument("--graph", type=int, default=-1,
                    help="1: replay each step (all layers) from a HIP graph captured once per rotation; "
                         "0: eager calls; -1 (default): graph for workloads of more than one layer")
    ap.add_argument("--clock-warmup-ms", type=float, default=30.0,
                    help="untimed decode steps run before the warm-up steps for about this long, so "
                         "that the timed region does not start on clocks that are still ramping up")
    ap.add_argument("--rotations", type=int, default=0, help="disjoint KV regions cycled over")
    ap.add_argument("--part-tokens", type=int, default=-1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-swap", action="store_true", help="decode only (for profiling)")
    ap.add_argument("--swap-layered", default="", metavar="L,Hkv,D,blocks",
                    help="measure the layer-major swap-in of one request instead of the decode step")
    ap.add_argument("--staging-mib", type=int, default=0, help="lamps_config.staging_bytes in MiB (0 = default)")
    ap.add_argument("--direct-copy-bytes", type=int, default=0,
                    help="lamps_config.direct_copy_bytes (0 = the library default: blocks of 4 MiB and more per pool; -1 = never)")
    ap.add_argument("--zero-copy", type=int, default=0, metavar="WORKGROUPS",
                    help="lamps_config.zero_copy_workgroups (0 = off, the default)")
    ap.add_argument("--ctx-override", type=int, default=0,
                    help="diagnostic: give every request this context length")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device-to-device copies (a kernel of known "
                         "traffic, for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--geom", default="",
                    help="diagnostic: override geometry, e.g. H=8,Hkv=8,bs=32,B=64,MB=128,NB=50000")
    ap.add_argument("--ctx-long", type=int, default=0,
                    help="diagnostic: after the overrides, request 0 runs with this many tokens "
                         "(a skewed batch: one long context among the others)")
    ap.add_argument("--prefill", default="",
                    help="measure lamps_prefill_attn instead (Discard's recompute): "
                         "'H,Hkv,D,requests,tokens[,cached]', e.g. 40,40,128,4,4096")
    ap.add_argument("--swap-directions", choices=["", "out", "in", "both"], default="",
                    help="which way the Swap-state blocks move during the timed steps (default: as the "
                         "configuration states it: 1 out, 2 in, 3 and 4 both)")
    ap.add_argument("--table", choices=["random", "sequential"], default="random",
                    help="physical placement of the blocks (sequential is a diagnostic)")
    return ap.parse_args()


class Job:
    """Device-resident state of one benchmark workload."""

    def __init__(self, cfg_id, rotations, part_tokens, table_kind="random", ctx_override=0,
                 geom_override="", direct_copy_bytes=0, staging_mib=0, zero_copy=0, ctx_long=0, swap_mode=""):
        import torch

        import lamps_workloads as W
        import paper_2410_18248_amd as P
        self.torch, self.W, self.P = torch, W, P
        wl = W.workload(cfg_id)
        if geom_override:
            import dataclasses
            kv = dict(x.split("=") for x in geom_override.split(","))
            names = {"H": "num_q_heads", "Hkv": "num_kv_heads", "bs": "block_size",
                     "MB": "max_blocks_per_req", "NB": "num_blocks", "D": "head_dim",
                     "L": "num_layers"}
            wl.geom = dataclasses.replace(wl.geom, **{names[k]: int(v) for k, v in kv.items()
                                                      if k in names})
            if "B" in kv:
                wl.batch = int(kv["B"])
                wl.ctx_lens = np.resize(wl.ctx_lens, wl.batch)
                wl.state = np.resize(wl.state, wl.batch)
            wl.name += "-" + geom_override
        if ctx_override:
            wl.ctx_lens[:] = ctx_override
            wl.name += "-ctx%d" % ctx_override
        if ctx_long:
            wl.ctx_lens[0] = ctx_long
            wl.state[0] = W.RUNNING
            wl.name += "-long%d" % ctx_long
        g = wl.geom
        self.wl, self.g = wl, g
        dev = torch.device("cuda:0")
        self.dev = dev
        need = sum(g.blocks_for(c) for c in wl.ctx_lens)
        if rotations <= 0:
            rotations = 8
        rotations = max(1, min(rotations, (g.num_blocks - need // 4) // need))
        self.R = rotations
        if part_tokens < 0:
            part_tokens = wl.part_tokens
        self.cfg = P.LampsConfig(g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim,
                                 g.block_size, g.num_blocks, g.max_blocks_per_req, wl.batch,
                                 P.LAMPS_BF16 if g.dtype == "bf16" else P.LAMPS_F32, 0.0,
                                 part_tokens, staging_mib << 20, direct_copy_bytes, zero_copy)
        tdt = torch.bfloat16 if g.dtype == "bf16" else torch.float32
        seed = W.config_seed(cfg_id)
        gen = torch.Generator(device=dev).manual_seed(seed)
        self.k_pool = torch.empty(g.pool_shape, dtype=tdt, device=dev).normal_(generator=gen)
        self.v_pool = torch.empty(g.pool_shape, dtype=tdt, device=dev).normal_(generator=gen)
        self.ws = torch.empty(P.lamps_workspace_bytes(self.cfg), dtype=torch.uint8, device=dev)
        self.compute = torch.cuda.Stream(dev)
        self.s_out = torch.cuda.Stream(dev)
        self.s_in = torch.cuda.Stream(dev)
        torch.cuda.synchronize()
        self.lam = P.Lamps(self.cfg, self.k_pool, self.v_pool, self.ws, self.compute.cuda_stream,
                           self.s_out.cuda_stream, self.s_in.cuda_stream)
        # decode steps are enqueued far ahead here and the swapped requests are paused (none of
        # that work touches their blocks): the swap calls need not wait for the compute stream
        self.lam.set_swap_fence(False)
        # every block starts allocated to the harness; what no batch uses goes back
        self.lam.alloc_blocks(g.num_blocks)
        perm = W.permutation(seed + 3, g.num_blocks)
        if table_kind == "sequential":
            perm = np.arange(g.num_blocks, dtype=np.int64)
        self.running = (wl.state == W.RUNNING).astype(np.uint8)
        self.n_running = int(self.running.sum())
        self.tables, self.q, self.out, self.tab_d = [], [], [], []
        pos = 0
        for b in range(self.R):
            table, used = W.deal_block_table(perm, wl.ctx_lens, g, start=pos)
            pos += used
            self.tables.append(table)
            self.tab_d.append(torch.as_tensor(table, device=dev))
            self.q.append(torch.empty((wl.batch, g.num_q_heads, g.head_dim), dtype=tdt,
                                      device=dev).normal_(generator=gen))
            self.out.append(torch.zeros((wl.batch, g.num_q_heads, g.head_dim), dtype=tdt,
                                        device=dev))
        self.lam.free_blocks([int(x) for x in perm[pos:]])
        self.ctx_d = torch.as_tensor(wl.ctx_lens.astype(np.int32), device=dev)
        self.mask_d = torch.as_tensor(self.running, device=dev)
        # Swap-state requests of all rotation batches: their block ids in groups of 128 MiB to
        # 1 GiB (a quarter of everything in between), each with a pinned buffer of its own, so
        # that the swap-in of one group runs while the next group is still on its way out
        self.block_bytes = P.lamps_block_bytes(self.cfg)
        ids = []
        for b in range(self.R):
            for r in np.flatnonzero(wl.state == W.SWAP):
                ids += [int(x) for x in self.tables[b][r, :g.blocks_for(wl.ctx_lens[r])]]
        want = min(1 << 30, max(128 << 20, len(ids) * self.block_bytes // 4))
        per_group = max(1, want // self.block_bytes)
        self.swap_groups = []                           # [ids, pinned buffer] pairs
        for i in range(0, len(ids), per_group):
            part = ids[i:i + per_group]
            self.swap_groups.append([part, torch.empty(len(part) * self.block_bytes,
                                                       dtype=torch.uint8).pin_memory()])
        # Discard-state requests: their blocks are simply freed (and re-allocated next train)
        self.discard_ids = []
        for b in range(self.R):
            ids = []
            for r in np.flatnonzero(wl.state == W.DISCARD):
                ids += [int(x) for x in self.tables[b][r, :g.blocks_for(wl.ctx_lens[r])]]
            self.discard_ids.append(ids)
        self.swap_bytes = sum(len(i) for i, _ in self.swap_groups) * self.block_bytes   # one round, each way
        # which way the Swap-state blocks move while the steps are timed, as the configurations
        # state it: 1 swaps out, 2 swaps in, 3 and 4 do both (anything else: both)
        self.swap_mode = swap_mode or {1: "out", 2: "in"}.get(cfg_id, "both")
        for ids, host in self.swap_groups:                  # the host images exist before anything comes back in
            self.lam.ticket_wait(self.lam.swap_out(ids, host))
        self.graphs = None
        torch.cuda.synchronize()
        # algorithmic bytes of one decode launch: K and V of the running requests' tokens,
        # q in, out, and the block-table entries walked
        tok = int(wl.ctx_lens[self.running == 1].sum())
        self.run_tokens = tok
        self.algo_bytes = (tok * g.token_bytes_per_layer
                           + 2 * self.n_running * g.num_q_heads * g.head_dim * g.elem_bytes
                           + 4 * sum(g.blocks_for(c) for c in wl.ctx_lens[self.running == 1]))

    def swap_group(self, grp):
        """One turn of one Swap-state group, by the workload's swap directions:
        "both": out, freed, allocated again (other blocks) and back in;
        "out":  out (the requests entered their API call; the blocks stay listed for the next turn);
        "in":   back in from the host image into freshly allocated blocks, the old ones freed
                (the requests return from their API call).
        Returns (swap-out ticket or None, swap-in ticket or None)."""
        lam = self.lam
        old, host = grp
        if self.swap_mode == "out":
            return lam.swap_out(old, host), None
        new = lam.alloc_blocks(len(old))                    # different physical blocks
        t_out = lam.swap_out(old, host) if self.swap_mode == "both" else None
        lam.free_blocks(old)
        t_in = lam.swap_in(host, new)
        grp[0] = new
        return t_out, t_in

    def recycle_discards(self):
        """Discard-state requests: their blocks are freed and allocated again."""
        lam = self.lam
        for b in range(self.R):
            if self.discard_ids[b]:
                lam.free_blocks(self.discard_ids[b])
                self.discard_ids[b] = lam.alloc_blocks(len(self.discard_ids[b]))

    def enqueue_swaps(self):
        """One swap round, every group once, enqueued at once; returns the last ticket."""
        last = None
        for grp in self.swap_groups:
            t_out, t_in = self.swap_group(grp)
            last = t_in if t_in is not None else t_out
        self.recycle_discards()
        return last

    def use_graphs(self):
        """Captures one step (all layers) per rotation batch in a HIP graph; decode_steps replays
        them from then on.  The calls have run eagerly before (the calibration trains)."""
        torch = self.torch
        lam, L, B = self.lam, self.g.num_layers, self.wl.batch
        self.graphs = []
        for b in range(self.R):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=self.compute):
                for layer in range(L):
                    lam.decode_attn(layer, B, self.q[b], self.tab_d[b], self.ctx_d, self.mask_d, self.out[b])
            self.graphs.append(gr)

    def decode_steps(self, k, first=0):
        lam, L, B = self.lam, self.g.num_layers, self.wl.batch
        if self.graphs is not None:
            with self.torch.cuda.stream(self.compute):
                for i in range(first, first + k):
                    self.graphs[i % self.R].replay()
            return
        for i in range(first, first + k):
            b = i % self.R
            for layer in range(L):
                lam.decode_attn(layer, B, self.q[b], self.tab_d[b], self.ctx_d, self.mask_d,
                                self.out[b])

    def train(self, k, with_swap, warmup=0, clock_warmup_s=0.0, per_step_s=0.0):
        """`warmup` untimed steps, then k timed ones.  Returns a dict: wall seconds of the k
        steps (host clock, compute stream drained at both ends), their HIP-event seconds on the
        compute stream, and what the swaps moved meanwhile.

        With swaps: a second host thread keeps swap rounds going from before the warm-up until
        after the timed steps (SwapFeeder); the decode steps never wait for them (the swapped
        requests are masked)."""
        torch = self.torch
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        n_clock = int(clock_warmup_s / per_step_s) + 1 if clock_warmup_s > 0 and per_step_s > 0 else 0
        torch.cuda.synchronize()
        feeder = None
        if with_swap and self.swap_bytes:
            feeder = SwapFeeder(self)
            feeder.start()
            feeder.first_done.wait()                     # the link is busy in both directions from here on
        self.decode_steps(n_clock + warmup, first=0)
        self.compute.synchronize()
        t0 = time.perf_counter()
        e0.record(self.compute)
        self.decode_steps(k, first=n_clock + warmup)
        e1.record(self.compute)
        self.compute.synchronize()
        t1 = time.perf_counter()
        res = {"wall_s": t1 - t0, "event_s": e0.elapsed_time(e1) * 1e-3, "swaps_in_flight_at_end": False,
               "swap_out_GBs_meanwhile": 0.0, "swap_in_GBs_meanwhile": 0.0}
        if feeder:
            res["swaps_in_flight_at_end"] = feeder.is_alive() and not feeder.failed
            feeder.stop = True
            feeder.join()
            if feeder.failed:
                raise feeder.failed
            res["swap_out_GBs_meanwhile"], res["swap_in_GBs_meanwhile"] = feeder.rates(t0, t1)
        torch.cuda.synchronize()
        if os.environ.get("LAMPS_BENCH_DEBUG"):
            print("train k=%d swap=%s: warm-up %d+%d steps, timed %.3f ms, swaps meanwhile %.1f out / %.1f in GB/s" %
                  (k, with_swap, n_clock, warmup, (t1 - t0) * 1e3, res["swap_out_GBs_meanwhile"],
                   res["swap_in_GBs_meanwhile"]), file=sys.stderr)
        return res

    def swap_alone(self):
        """GB/s of one batch's swap-out and swap-in with nothing else running, and of
        a plain pinned copy of the same size (the host link as this machine delivers it)."""
        torch, lam = self.torch, self.lam
        if not self.swap_groups:
            return None
        ids, host = self.swap_groups[0]
        nbytes = len(ids) * self.block_bytes
        res = {}
        for _ in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            lam.ticket_wait(lam.swap_out(ids, host))
            t1 = time.perf_counter()
            lam.ticket_wait(lam.swap_in(host, ids))
            t2 = time.perf_counter()
            res["swap_out_GBs"] = nbytes / (t1 - t0) / 1e9
            res["swap_in_GBs"] = nbytes / (t2 - t1) / 1e9
        dbuf = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
        for _ in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            host[:nbytes].copy_(dbuf, non_blocking=True)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            dbuf.copy_(host[:nbytes], non_blocking=True)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            res["memcpy_d2h_GBs"] = nbytes / (t1 - t0) / 1e9
            res["memcpy_h2d_GBs"] = nbytes / (t2 - t1) / 1e9
        res["bytes_each_way"] = nbytes
        return res

    def unpage(self, b, r, layer):
        """Logical K, V of request r of rotation batch b in one layer, as numpy (oracle input)."""
        torch, g = self.torch, self.g
        C = int(self.wl.ctx_lens[r])
        ids = torch.as_tensor(self.tables[b][r, :g.blocks_for(C)].astype(np.int64), device=self.dev)

        def logical(pool, index_map):
            x = pool[ids, layer].cpu()                          # [nb][Hkv][tile]
            x = x.view(torch.int16).numpy().view(np.uint16) if x.dtype == torch.bfloat16 else x.numpy()
            return self.W.tiles_to_logical(x, index_map, C)
        k_index, v_index = g.tile_index_maps()
        return logical(self.k_pool, k_index), logical(self.v_pool, v_index)


class SwapFeeder(threading.Thread):
    """Keeps the Swap-state groups of a Job going out and coming back, round after round, from a
    host thread of its own, until told to stop; then waits for what it started.  At most DEPTH
    groups are in flight: with more copies queued than that, the runtime's copy path drops into
    a mode four times slower (measured; the queue depth, not the decode kernels, sets it off),
    so a caller that wants the link's rate feeds it like this.  The thread makes block-management
    calls only (alloc, free, swap, ticket wait); the main thread makes decode calls only."""
    DEPTH = 2

    def __init__(self, job):
        super().__init__(daemon=True)
        self.job, self.stop, self.failed = job, False, None
        self.first_done = threading.Event()
        self.done = []                                   # (host time, is_out, bytes) per finished copy

    def run(self):
        job, lam = self.job, self.job.lam
        pend = collections.deque()

        def wait(ticket):                                # polled: a blocking host wait on an event of a
            while not lam.ticket_query(ticket):          # busy device has been seen to return late
                time.sleep(0.0001)

        def retire():
            t_out, t_in, n = pend.popleft()
            if t_out is not None:
                wait(t_out)
                self.done.append((time.perf_counter(), True, n))
            if t_in is not None:
                wait(t_in)
                self.done.append((time.perf_counter(), False, n))
            self.first_done.set()
        try:
            while not self.stop:
                for grp in job.swap_groups:
                    if self.stop:
                        break
                    while len(pend) >= self.DEPTH:
                        retire()
                    t_out, t_in = job.swap_group(grp)
                    pend.append((t_out, t_in, len(grp[0]) * job.block_bytes))
                job.recycle_discards()
            while pend:
                retire()
        except Exception as e:                           # reported by the main thread
            self.failed = e
        self.first_done.set()

    def rates(self, t0, t1):
        """GB/s out and in over [t0, t1], from the copies that finished inside it (whole copies)."""
        out = sum(n for t, is_out, n in self.done if is_out and t0 <= t <= t1)
        inn = sum(n for t, is_out, n in self.done if not is_out and t0 <= t <= t1)
        return out / (t1 - t0) / 1e9, inn / (t1 - t0) / 1e9


def _host_bits(t, torch):
    t = t.cpu()
    return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()


def oracle_check(job, layers, requests):
    """max |GPU - oracle| over the listed requests (all their query heads) in the listed layers
    of rotation batch 0, each layer run once more into a buffer of its own."""
    import oracle
    torch, g, B = job.torch, job.g, job.wl.batch
    q = _host_bits(job.q[0], torch)
    pick = np.zeros(B, dtype=np.uint8)
    pick[list(requests)] = 1
    worst = 0.0
    for layer in layers:
        out = torch.zeros_like(job.out[0])
        job.lam.decode_attn(layer, B, job.q[0], job.tab_d[0], job.ctx_d, job.mask_d, out)
        job.compute.synchronize()
        K, V = [None] * B, [None] * B
        for r in requests:
            K[r], V[r] = job.unpage(0, r, layer)
        ref = oracle.decode_attn(q, K, V, job.wl.ctx_lens, pick, threads=len(os.sched_getaffinity(0)))
        got = out.cpu().to(torch.float64).numpy()
        sel = pick == 1
        worst = max(worst, float(np.abs(got[sel] - ref[sel]).max()))
    return worst


def cpu_baseline(job):
    """The oracle, as it stands, on the host cores: all running requests of one
    batch, one layer.  Un-paging is done before the clock starts."""
    import oracle
    torch = job.torch
    cores = len(os.sched_getaffinity(0))
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = min(cores, int(env))
    q = _host_bits(job.q[0], torch)
    B = job.wl.batch
    K, V = [None] * B, [None] * B
    last = job.g.num_layers - 1                     # job.out holds the last layer's result
    for r in np.flatnonzero(job.running):
        K[r], V[r] = job.unpage(0, r, last)
    reps, t0 = 0, time.perf_counter()
    while True:                                     # the same pass again until about a second of wall
        ref = oracle.decode_attn(q, K, V, job.wl.ctx_lens, job.running, threads=cores)   # time (cores x that of CPU work)
        reps += 1
        dt = (time.perf_counter() - t0) / reps
        if dt * reps >= 1.0 and reps >= 3:
            break
    got = job.out[0].cpu().to(torch.float64).numpy()
    run = job.running == 1
    err = float(np.abs(got[run] - ref[run]).max())
    t1 = time.perf_counter()                        # and once on a single thread
    oracle.decode_attn(q, K, V, job.wl.ctx_lens, job.running, threads=1)
    dt1 = time.perf_counter() - t1
    return {"value": job.n_running / (dt * job.g.num_layers), "unit": "tokens/s", "cores": cores,
            "kind": "oracle", "value_one_thread": job.n_running / (dt1 * job.g.num_layers),
            "sample": "all %d running requests of one batch, 1 of %d layer(s), %d passes of %.3f s; "
                      "scaled by the layer count" % (job.n_running, job.g.num_layers, reps, dt),
            "max_abs_err_gpu_vs_oracle": err}


MFMA_BF16_PEAK_TFLOPS = 2500.0    # MI355X published dense bf16 matrix peak


def swap_layered_bench(a):
    """Layer-major swap against the block-major one for one returning request: `blocks` blocks of a
    cache with L layers of Hkv kv heads of D (bf16, 16-token blocks).  Reports the rates of both and
    how long the compute stream waits before the attention of layer 0, of the middle layer and of
    the last layer may start (lamps_compute_wait_layer against lamps_compute_wait)."""
    import torch

    import paper_2410_18248_amd as P
    L, Hkv, D, blocks = [int(x) for x in a.swap_layered.split(",")]
    nb = blocks + 8
    dev = torch.device("cuda:0")
    cfg = P.LampsConfig(L, Hkv, Hkv, D, 16, nb, blocks, 1, P.LAMPS_BF16, 0.0, 0, a.staging_mib << 20,
                        a.direct_copy_bytes or -1)      # the block-major side of the comparison is the staged path
    elems = P.lamps_pool_bytes(cfg) // 2
    k_pool = torch.empty(elems, dtype=torch.bfloat16, device=dev).normal_()
    v_pool = torch.empty(elems, dtype=torch.bfloat16, device=dev).normal_()
    ws = torch.empty(P.lamps_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
    cs, so, si = (torch.cuda.Stream(dev) for _ in range(3))
    torch.cuda.synchronize()
    lam = P.Lamps(cfg, k_pool, v_pool, ws, cs.cuda_stream, so.cuda_stream, si.cuda_stream)
    ids = lam.alloc_blocks(nb)[:blocks]
    nbytes = blocks * P.lamps_block_bytes(cfg)
    host = torch.empty(nbytes, dtype=torch.uint8).pin_memory()

    def ready_times(layered, layers):
        """ms from the swap-in call until the compute stream is released for each listed layer."""
        ticket = None
        lam.ticket_wait(lam.swap_out(ids, host, layered=layered))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ticket = lam.swap_in(host, ids, layered=layered)
        evs = []
        for layer in layers:
            if layered:
                lam.compute_wait_layer(ticket, layer)
            else:
                lam.compute_wait(ticket)
            e = torch.cuda.Event()
            e.record(cs)
            evs.append(e)
        done = [None] * len(evs)
        while any(d is None for d in done):         # polled: a host wait on such an event returns only
            for i, e in enumerate(evs):             # when the whole copy stream has drained
                if done[i] is None and e.query():
                    done[i] = (time.perf_counter() - t0) * 1e3
        lam.ticket_wait(ticket)
        return done, (time.perf_counter() - t0) * 1e3

    layers = sorted(set([0, L // 2, L - 1]))
    best = {}
    for layered in (False, True):
        runs = [ready_times(layered, layers) for _ in range(6)]
        runs.sort(key=lambda r: r[1])               # the runtime now and then blocks a copy call for ms: take the median
        done, total = runs[len(runs) // 2]
        best[layered] = {"ready_ms": dict(zip(["layer_%d" % x for x in layers], done)), "all_ms": total,
                         "GBs": nbytes / total / 1e6}
    line = {"metric": "swap-in of one request: ms until a layer's attention may start", "unit": "ms",
            "value": best[True]["ready_ms"]["layer_0"], "higher_is_better": False, "n_gpus": 1, "data": "synthetic",
            "config": {"workload": "swap-in-%d-blocks-L%d-Hkv%d-D%d" % (blocks, L, Hkv, D), "bytes": nbytes},
            "block_major": best[False], "layer_major": best[True]}
    print(json.dumps(line))
    lam.destroy()


def prefill_bench(a):
    """lamps_kv_append_tokens + lamps_prefill_attn for `requests` requests of `tokens` new tokens
    each on top of `cached` old ones (0 = a discarded context recomputed from scratch), one layer,
    bf16.  Bound by the matrix cores: flops = 4 * D * H * (query, key) pairs."""
    import torch

    import lamps_workloads as W
    import oracle
    import paper_2410_18248_amd as P
    f = [int(x) for x in a.prefill.split(",")]
    H, Hkv, D, n_req, n_new = f[:5]
    cached = f[5] if len(f) > 5 else 0
    bs = 16
    C = cached + n_new
    per = (C + bs - 1) // bs
    nb = n_req * per + 8
    dev = torch.device("cuda:0")
    cfg = P.LampsConfig(1, H, Hkv, D, bs, nb, per, n_req, P.LAMPS_BF16, 0.0, 0, 0)
    g = W.Geometry(1, H, Hkv, D, bs, nb, per, "bf16")
    gen = torch.Generator(device=dev).manual_seed(W.config_seed(5))
    k_pool = torch.empty(g.pool_shape, dtype=torch.bfloat16, device=dev).normal_(generator=gen)
    v_pool = torch.empty(g.pool_shape, dtype=torch.bfloat16, device=dev).normal_(generator=gen)
    ws = torch.empty(P.lamps_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
    cs = torch.cuda.Stream(dev)
    torch.cuda.synchronize()
    lam = P.Lamps(cfg, k_pool, v_pool, ws, cs.cuda_stream, cs.cuda_stream, cs.cuda_stream)
    lam.alloc_blocks(nb)
    perm = W.permutation(W.config_seed(5) + 1, nb)
    table, _ = W.deal_block_table(perm, [C] * n_req, g)
    td = torch.as_tensor(table, device=dev)
    cd = torch.full((n_req,), C, dtype=torch.int32, device=dev)
    sd = torch.arange(0, (n_req + 1) * n_new, n_new, dtype=torch.int32, device=dev)
    total = n_req * n_new
    q = torch.empty((total, H, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
    kn = torch.empty((total, Hkv, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
    vn = torch.empty((total, Hkv, D), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
    out = torch.empty_like(q)
    steps = a.steps if a.steps > 0 else 20

    def run(k, append):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(cs)
        for _ in range(k):
            if append:
                lam.kv_append_tokens(0, n_req, total, kn, vn, sd, td, cd)
            lam.prefill_attn(0, n_req, total, q, sd, td, cd, out, max_new_tokens=n_new)
        e1.record(cs)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, e0.elapsed_time(e1) * 1e-3
    # the kernel gets faster over its first 20-30 ms after an idle period (clocks ramp up):
    # warm up for about 40 ms unless told otherwise
    _, probe = run(3, True)
    warmup = a.warmup if a.warmup >= 0 else max(3, int(0.04 / (probe / 3)))
    if a.copy_calibration:                             # a kernel of known traffic, for scaling counter readings
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    run(warmup, True)
    wall, dev_s = run(steps, True)
    _, attn_s = run(steps, False)
    pairs = n_req * sum(cached + i + 1 for i in range(n_new))
    flops = 4.0 * D * H * pairs
    achieved = flops / (attn_s / steps) / 1e12
    hbm_bytes = n_req * C * 2 * Hkv * D * 2 + 2 * total * H * D * 2
    # parity on sampled rows against the oracle (un-paged by the harness)
    k_index, v_index = g.tile_index_maps()

    def logical(pool, index_map, r):
        ids = torch.as_tensor(table[r, :per].astype(np.int64), device=dev)
        x = pool[ids, 0].cpu().view(torch.int16).numpy().view(np.uint16)
        return W.tiles_to_logical(x, index_map, C)
    rows = sorted(set([0, 1, n_new // 2, n_new - 1]))
    K, V = logical(k_pool, k_index, 0), logical(v_pool, v_index, 0)
    qh = q[:n_new].cpu().view(torch.int16).numpy().view(np.uint16)
    got = out[:n_new].cpu().to(torch.float64).numpy()
    t0 = time.perf_counter()
    ref = oracle.decode_attn(qh[rows], [K] * len(rows), [V] * len(rows), [cached + i + 1 for i in rows],
                             [1] * len(rows), threads=len(os.sched_getaffinity(0)))
    cpu_s = time.perf_counter() - t0
    err = float(np.abs(got[rows] - ref).max())
    cpu_pairs = sum(cached + i + 1 for i in rows)
    workload = "prefill-%dx%d-new-on-%d-cached-H%d-Hkv%d-D%d" % (n_req, n_new, cached, H, Hkv, D)
    line = {"metric": "prefill-attention tokens/s (Discard's recompute, one layer)",
            "value": total * steps / wall, "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": wall / steps * 1e3, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": workload},
            "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": MEASURED_TRAFFIC_BYTES.get(workload),
                         "kernel": "prefill_mfma",
                         "algorithmic_flops_per_launch": flops, "kernel_us": attn_s / steps * 1e6,
                         "append_plus_attention_us": dev_s / steps * 1e6},
            # with few new tokens per request the same kernel is a stream over the cache instead:
            # K and V once per (request, kv head), q in, out
            "hbm": {"achieved": hbm_bytes / (attn_s / steps) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": hbm_bytes / (attn_s / steps) / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": hbm_bytes},
            "cpu_baseline": {"value": cpu_pairs / cpu_s * (total / pairs), "unit": "tokens/s",
                             "cores": len(os.sched_getaffinity(0)), "kind": "oracle",
                             "sample": "%d rows of request 0 (%d query-key pairs, %.2f s), scaled by pairs per token"
                                       % (len(rows), cpu_pairs, cpu_s),
                             "max_abs_err_gpu_vs_oracle": err}}
    if line["hbm"]["frac"] > line["roofline"]["frac"]:     # the stream over the cache is what binds
        mf = line["roofline"]
        line["roofline"] = dict(line["hbm"], bound="hbm", traffic=mf["traffic"], kernel="prefill_mfma", kernel_us=mf["kernel_us"],
                                append_plus_attention_us=mf["append_plus_attention_us"])
        line["mfma"] = {k: mf[k] for k in ("achieved", "peak", "unit", "frac", "algorithmic_flops_per_launch")}
        del line["hbm"]
    lam.destroy()
    print(json.dumps(line))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build measures one MI355X; --gpus %d is not supported "
              "(no collectives or sharding are part of it)" % a.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if a.swap_layered:
        swap_layered_bench(a)
        return
    if a.prefill:
        prefill_bench(a)
        return
    if a.config:
        line = measure_config(a, a.config, True)
    else:
        line = measure_config(a, 4, True)
        line["per_config"] = [measure_config(a, c, False) for c in (1, 2, 3)]
    print(json.dumps(line))


def measure_config(a, cfg_id, headline):
    """One workload measured by the timing rule of the module docstring.  headline: the whole
    bench line (exactly --steps timed steps, oracle timed as cpu_baseline); otherwise a compact
    record for "per_config" (at least --steps steps and at least about 60 ms of them)."""
    import torch
    job = Job(cfg_id, a.rotations, a.part_tokens, a.table, a.ctx_override, a.geom, a.direct_copy_bytes, a.staging_mib,
              a.zero_copy, a.ctx_long, a.swap_directions)
    with_swap = not a.no_swap
    L = job.g.num_layers

    # calibrate: short trains to size the run (and the eager calls every capture needs first)
    job.train(2 * job.R, False)
    per_step = job.train(2 * job.R, False)["event_s"] / (2 * job.R)
    graph = a.graph == 1 or (a.graph < 0 and L > 1)
    if graph:
        job.use_graphs()
        per_step = job.train(2 * job.R, False)["event_s"] / (2 * job.R)
    steps = a.steps if a.steps > 0 else int(min(4000, max(job.R, 0.05 / per_step)))
    if not headline:                                    # long enough for a dozen swap copies to finish inside
        steps = max(steps, int(np.ceil(0.06 / per_step)))
    warmup = a.warmup if a.warmup >= 0 else max(job.R, steps // 4)
    clock_s = a.clock_warmup_ms * 1e-3

    if a.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=job.dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    swap = None
    if with_swap:
        # the runtime sets up its copy path lazily (first large copies block the host for
        # milliseconds each); get that out of the way before anything is timed
        for _ in range(2):
            job.enqueue_swaps()
            torch.cuda.synchronize()
        swap = job.swap_alone()
    under = job.train(steps, with_swap, warmup, clock_s, per_step)
    alone = job.train(steps, False, warmup, clock_s, per_step) if with_swap else under
    if swap:
        swap["swap_out_GBs_during_timed_steps"] = under["swap_out_GBs_meanwhile"]
        swap["swap_in_GBs_during_timed_steps"] = under["swap_in_GBs_meanwhile"]

    # spread over repeated trains (decode alone, each at least about 20 ms on the compute stream)
    n_each = max(job.R, int(0.02 / per_step))
    per = sorted(job.train(n_each, False)["event_s"] / n_each * 1e3 for _ in range(20))
    spread = {"trains": len(per), "steps_each": n_each, "ms_per_step_min": per[0],
              "ms_per_step_median": 0.5 * (per[9] + per[10]), "ms_per_step_p95": per[18]}

    launches = steps * L
    kernel_s = under["event_s"] / launches
    achieved = job.algo_bytes / kernel_s / 1e9
    alone_GBs = job.algo_bytes / (alone["event_s"] / launches) / 1e9
    rule = ("a second host thread keeps the Swap-state groups going out and coming back (at most %d groups "
            "in flight) from before the warm-up until after the timed steps; the decode steps are timed "
            "on the compute stream meanwhile; swaps drained afterwards" % SwapFeeder.DEPTH
            if with_swap else "decode alone")
    cfgd = {"workload": job.wl.name, "batch": job.wl.batch, "running": job.n_running,
            "running_tokens": job.run_tokens, "layers": L,
            "q_heads": job.g.num_q_heads, "kv_heads": job.g.num_kv_heads,
            "head_dim": job.g.head_dim, "block_size": job.g.block_size,
            "num_blocks": job.g.num_blocks, "rotations": job.R,
            "part_tokens": int(job.cfg.part_tokens),
            "timing_rule": rule, "hip_graph": bool(graph), "clock_warmup_ms": a.clock_warmup_ms,
            "swap_directions": job.swap_mode if with_swap else "none",
            "swap_bytes_each_way_per_round": 0 if not with_swap else job.swap_bytes,
            "swaps_in_flight_when_timed_steps_ended": under["swaps_in_flight_at_end"]}
    roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(job.wl.name),
            "kernel": "decode_balanced" if int(job.cfg.part_tokens) == 0 else "decode_partial",
            "algorithmic_bytes_per_launch": job.algo_bytes,
            "kernel_us": kernel_s * 1e6,
            "timing": "HIP events on the compute stream around the timed steps / launches "
                      "(includes the small merge kernel that follows each launch)"}
    if headline:
        line = {
            "metric": "decode-attention tokens/s (achieved HBM GB/s in roofline; swap GB/s in swap)",
            "value": job.n_running * steps / under["wall_s"],
            "unit": "tokens/s",
            "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": under["wall_s"] / steps * 1e3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": job.g.dtype, "data": "synthetic",
            "config": cfgd,
            "roofline": roof,
            "decode_alone": {"ms_per_step": alone["event_s"] / steps * 1e3,
                             "tokens_per_s": job.n_running * steps / alone["wall_s"],
                             "GBs": alone_GBs, "frac": alone_GBs / HBM_PEAK_GBS},
            "decode_alone_trains": spread,
            "decode_slowdown_under_swap": under["event_s"] / alone["event_s"],
        }
        if swap:
            line["swap"] = swap
        if not a.no_cpu_baseline:
            line["cpu_baseline"] = cpu_baseline(job)
            if L > 1:                                   # the other layers, on a seeded sample of requests
                run = np.flatnonzero(job.running)
                sample = sorted(int(x) for x in run[job.W.permutation(job.W.config_seed(cfg_id) + 77, len(run))[:64]])
                line["cpu_baseline"]["max_abs_err_sampled_layers"] = {
                    "layers": [0, L // 2 - 1, L - 1], "requests": len(sample),
                    "max_abs_err_gpu_vs_oracle": oracle_check(job, [0, L // 2 - 1, L - 1], sample)}
    else:
        line = {"workload": job.wl.name, "steps": steps, "warmup": warmup,
                "tokens_per_s": job.n_running * steps / under["wall_s"],
                "ms_per_step": under["wall_s"] / steps * 1e3,
                "frac_under_swap": achieved / HBM_PEAK_GBS, "frac_alone": alone_GBs / HBM_PEAK_GBS,
                "decode_slowdown_under_swap": under["event_s"] / alone["event_s"],
                "kernel_us_under_swap": kernel_s * 1e6, "kernel_us_alone": alone["event_s"] / launches * 1e6,
                "algorithmic_bytes_per_launch": job.algo_bytes,
                "traffic": MEASURED_TRAFFIC_BYTES.get(job.wl.name),
                "decode_alone_trains": spread, "swap": swap, "config": cfgd}
        if not a.no_cpu_baseline:
            line["max_abs_err_gpu_vs_oracle"] = oracle_check(job, [L - 1], [int(r) for r in np.flatnonzero(job.running)])
            line["oracle_checked"] = "all %d running requests, every query head" % job.n_running
    job.lam.destroy()
    del job
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    return line


if __name__ == "__main__":
    main()
