"""A live serving loop over liblamps: the scheduler (lamps_sched.h) decides, the
GPU calls of lamps.h execute.

Every iteration of Algorithm 1 (arXiv 2410.18248) becomes:
  lamps_sched_next_batch  -> which requests run, and what each brings back first
      swap_in   > 0 : lamps_alloc_blocks + lamps_swap_in + lamps_compute_wait   (Swap; or the
                      layer-major calls, each layer's work behind lamps_compute_wait_layer)
      recompute > 0 : lamps_alloc_blocks + lamps_kv_append_tokens + lamps_prefill_attn
                      per layer (Discard's recompute, a prompt, an API response)
      otherwise     : lamps_kv_append + lamps_decode_attn per layer (one new token)
  lamps_sched_commit(measured iteration time) -> who reached an API call and how it leaves
      Preserve: nothing;  Discard: lamps_free_blocks;
      Swap: lamps_swap_out to a pinned buffer, then lamps_free_blocks
      finished: lamps_free_blocks

There is no model here: the per-layer query / key / value vectors that a
transformer would produce are drawn by a caller-supplied ``source`` (seeded
random tensors by default), so that everything the library is responsible for
-- block management, append, swap, recompute, attention -- runs for real while
the GEMMs are absent.  torch is plumbing: device memory, streams, the clock.
"""
import time

import numpy as np
import torch

from . import binding as P


class RandomSource:
    """q / k / v of request `rid` at position `pos` in `layer`: N(0,1) bf16 or fp32,
    a pure function of (seed, rid, pos, layer) so that a recompute reproduces them."""

    def __init__(self, seed, num_q_heads, num_kv_heads, head_dim, dtype):
        self.seed, self.H, self.Hkv, self.D, self.dtype = seed, num_q_heads, num_kv_heads, head_dim, dtype

    def rows(self, rid, first_pos, count, layer):
        g = torch.Generator()
        out = torch.empty((count, self.H + 2 * self.Hkv, self.D))
        for i in range(count):                      # one seed per position: any range costs its own length
            g.manual_seed((((self.seed * 1000003 + rid) * 8191 + layer) * 1048573 + first_pos + i) & 0x7FFFFFFFFFFFFFFF)
            torch.randn(out.shape[1:], generator=g, out=out[i])
        x = out.to(self.dtype)
        return x[:, :self.H], x[:, self.H:self.H + self.Hkv], x[:, self.H + self.Hkv:]


class DeviceSource:
    """The same contract as RandomSource -- a pure function of (seed, rid, pos, layer) -- but made
    on the device by integer hashing (uniform, zero mean, unit variance), so that a serving run is
    not dominated by the host making its inputs."""

    def __init__(self, seed, num_q_heads, num_kv_heads, head_dim, dtype, device="cuda:0"):
        self.seed, self.H, self.Hkv, self.D, self.dtype = seed, num_q_heads, num_kv_heads, head_dim, dtype
        self.dev = torch.device(device)
        self.idx = torch.arange((num_q_heads + 2 * num_kv_heads) * head_dim, dtype=torch.int64, device=self.dev)

    def rows(self, rid, first_pos, count, layer):
        key = ((((self.seed * 1000003 + rid) * 8191 + layer) * 1048573) & 0x3FFFFFFFFFFF)
        pos = torch.arange(first_pos, first_pos + count, dtype=torch.int64, device=self.dev)[:, None]
        z = self.idx[None, :] * 0x9E3779B1 + pos * 0x85EBCA77 + key      # int64 arithmetic wraps
        z = (z ^ ((z >> 29) & 0x7FFFFFFFF)) * 0xBF58476D
        z = (z ^ ((z >> 32) & 0xFFFFFFFF)) * 0x94D049BB
        z = z ^ ((z >> 31) & 0x1FFFFFFFF)
        u = (z & 0xFFFFFF).to(torch.float32) * (1.0 / (1 << 24)) - 0.5
        x = (u * 12.0 ** 0.5).view(count, self.H + 2 * self.Hkv, self.D).to(self.dtype)
        return x[:, :self.H], x[:, self.H:self.H + self.Hkv], x[:, self.H + self.Hkv:]


class LiveEngine:
    def __init__(self, cfg, sched_cfg, source, device="cuda:0", observer=None, layered_swap=False):
        """cfg: LampsConfig (pools are allocated here); sched_cfg: LampsSchedConfig whose
        memory_tokens must not exceed num_blocks * block_size; observer(kind, rid, layer, first_pos,
        out_rows): called with the attention output of every processed token (tests);
        layered_swap: swap layer-major, so that a returning request's first layers run while the
        later ones are still on their way."""
        self.cfg, self.dev, self.source, self.observer = cfg, torch.device(device), source, observer
        self.layered = layered_swap
        self.tdtype = torch.bfloat16 if cfg.dtype == P.LAMPS_BF16 else torch.float32
        elems = P.lamps_pool_bytes(cfg) // (2 if cfg.dtype == P.LAMPS_BF16 else 4)
        self.k_pool = torch.zeros(elems, dtype=self.tdtype, device=self.dev)
        self.v_pool = torch.zeros(elems, dtype=self.tdtype, device=self.dev)
        self.ws = torch.empty(P.lamps_workspace_bytes(cfg), dtype=torch.uint8, device=self.dev)
        self.cs, self.so, self.si = (torch.cuda.Stream(self.dev) for _ in range(3))
        torch.cuda.synchronize()
        self.lam = P.Lamps(cfg, self.k_pool, self.v_pool, self.ws, self.cs.cuda_stream,
                           self.so.cuda_stream, self.si.cuda_stream)
        assert sched_cfg.memory_tokens <= cfg.num_blocks * cfg.block_size
        assert sched_cfg.max_batch <= cfg.max_batch
        self.sched = P.LampsSched(sched_cfg)
        self.block_bytes = P.lamps_block_bytes(cfg)
        self.blocks = {}        # rid -> physical block ids of its context, in order
        self.ctx = {}           # rid -> tokens of context that are in the cache
        self.host = {}          # rid -> (pinned buffer, n blocks, tokens) while swapped out
        self._inflight = []     # (ticket, pinned buffer) of copies that may still be running
        self.stats = {"iterations": 0, "decode_tokens": 0, "prefill_tokens": 0, "swapped_out_blocks": 0,
                      "swapped_in_blocks": 0, "discarded_blocks": 0, "gpu_s": 0.0}

    def close(self):
        torch.cuda.synchronize()
        self.sched.destroy()
        self.lam.destroy()

    def add(self, rid, arrival, prompt_tokens, segments, priority=0.0):
        self.sched.add(rid, arrival, prompt_tokens, segments, priority)
        self.blocks[rid], self.ctx[rid] = [], 0

    # ---- helpers
    def _grow(self, rid, tokens):
        """Blocks for `tokens` more positions of request rid."""
        bs = self.cfg.block_size
        need = (self.ctx[rid] + tokens + bs - 1) // bs - len(self.blocks[rid])
        if need > 0:
            new = self.lam.alloc_blocks(need)
            self.lam.compute_wait_blocks(new)       # they may still be the source of a swap-out
            self.blocks[rid] += new

    def _tables(self, rids):
        t = np.full((len(rids), self.cfg.max_blocks_per_req), -1, dtype=np.int32)
        for i, r in enumerate(rids):
            t[i, :len(self.blocks[r])] = self.blocks[r]
        return torch.from_numpy(t).to(self.dev, non_blocking=True)

    def _release(self, rid):
        if self.blocks[rid]:
            self.lam.free_blocks(self.blocks[rid])
        self.blocks[rid] = []

    # ---- one iteration of Algorithm 1; returns False when every request has finished
    def step(self):
        cfg, lam = self.cfg, self.lam
        batch = self.sched.next_batch()
        for rid in self.sched.take_discards():      # dropped by the scheduler for lack of memory
            self.stats["discarded_blocks"] += len(self.blocks[rid])
            self._release(rid)
            self.ctx[rid] = 0
            self.host.pop(rid, None)
        if not batch:
            return False
        self._inflight = [(t, b) for t, b in self._inflight if not lam.ticket_query(t)]
        t0 = time.perf_counter()
        dec, pre = [], []                           # (rid,) / (rid, count)
        landing = []                                # layer-major swap-ins of this iteration
        with torch.cuda.stream(self.cs):
            for rid, swap_in, recompute, _ in batch:
                if swap_in:                         # Swap: back from pinned host memory into fresh blocks
                    buf, nblk, tokens = self.host.pop(rid)
                    assert tokens == swap_in
                    ids = lam.alloc_blocks(nblk)
                    ticket = lam.swap_in(buf, ids, layered=self.layered)
                    if self.layered:
                        landing.append(ticket)      # each layer's work waits for its own slice only
                    else:
                        lam.compute_wait(ticket)
                    self._inflight.append((ticket, buf))    # the buffer lives until the copy is done
                    self.blocks[rid], self.ctx[rid] = ids, tokens
                    self.stats["swapped_in_blocks"] += nblk
                if recompute:
                    pre.append((rid, recompute))
                else:
                    dec.append(rid)
            L = cfg.num_layers
            if pre:                                 # several new tokens per request
                rids = [r for r, _ in pre]
                first = [self.ctx[r] for r in rids]
                for r, n in pre:
                    self._grow(r, n)
                    self.ctx[r] += n
                counts = [n for _, n in pre]
                qs = torch.tensor(np.concatenate([[0], np.cumsum(counts)]), dtype=torch.int32, device=self.dev)
                td = self._tables(rids)
                cd = torch.tensor([self.ctx[r] for r in rids], dtype=torch.int32, device=self.dev)
                total = int(sum(counts))
                for layer in range(L):
                    for ticket in landing:
                        lam.compute_wait_layer(ticket, layer)
                    parts = [self.source.rows(r, f, n, layer) for r, f, n in zip(rids, first, counts)]
                    q = torch.cat([p[0] for p in parts]).contiguous().to(self.dev)
                    k = torch.cat([p[1] for p in parts]).contiguous().to(self.dev)
                    v = torch.cat([p[2] for p in parts]).contiguous().to(self.dev)
                    out = torch.empty_like(q)
                    lam.kv_append_tokens(layer, len(rids), total, k, v, qs, td, cd)
                    lam.prefill_attn(layer, len(rids), total, q, qs, td, cd, out, max_new_tokens=max(counts))
                    if self.observer:
                        o = out.float().cpu()
                        at = 0
                        for r, f, n in zip(rids, first, counts):
                            self.observer("prefill", r, layer, f, o[at:at + n])
                            at += n
                self.stats["prefill_tokens"] += total
            if dec:                                 # one new token per request
                for r in dec:
                    self._grow(r, 1)
                td = self._tables(dec)
                cd = torch.tensor([self.ctx[r] for r in dec], dtype=torch.int32, device=self.dev)
                md = torch.ones(len(dec), dtype=torch.uint8, device=self.dev)
                for layer in range(L):
                    for ticket in landing:
                        lam.compute_wait_layer(ticket, layer)
                    parts = [self.source.rows(r, self.ctx[r], 1, layer) for r in dec]
                    q = torch.cat([p[0] for p in parts]).contiguous().to(self.dev)
                    k = torch.cat([p[1] for p in parts]).contiguous().to(self.dev)
                    v = torch.cat([p[2] for p in parts]).contiguous().to(self.dev)
                    out = torch.empty_like(q)
                    # the new token's key and value go in first and attention sees them: lengths + 1
                    # (on the last layer the append has already advanced the device lengths)
                    lam.kv_append(layer, len(dec), k, v, td, cd, md, layer == L - 1)
                    lam.decode_attn(layer, len(dec), q, td, cd if layer == L - 1 else cd + 1, md, out)
                    if self.observer:
                        o = out.float().cpu()
                        for i, r in enumerate(dec):
                            self.observer("decode", r, layer, self.ctx[r], o[i:i + 1])
                for r in dec:
                    self.ctx[r] += 1
                self.stats["decode_tokens"] += len(dec)
        self.cs.synchronize()
        dt = time.perf_counter() - t0
        self.stats["gpu_s"] += dt
        self.stats["iterations"] += 1
        for rid, what, handling, context in self.sched.commit(dt):
            assert context == self.ctx[rid], (rid, context, self.ctx[rid])
            if what == 1 or handling == P.LAMPS_DISCARD:
                self.stats["discarded_blocks"] += len(self.blocks[rid]) if what == 0 else 0
                self._release(rid)
                if what == 0:
                    self.ctx[rid] = 0               # everything is recomputed on return
            elif handling == P.LAMPS_SWAP:
                ids = self.blocks[rid]
                buf = torch.empty(max(1, len(ids) * self.block_bytes), dtype=torch.uint8).pin_memory()
                ticket = lam.swap_out(ids, buf, layered=self.layered)   # the library orders the blocks' reuse behind the copy
                self._inflight.append((ticket, buf))
                self.host[rid] = (buf, len(ids), self.ctx[rid])
                self.stats["swapped_out_blocks"] += len(ids)
                self._release(rid)
                self.ctx[rid] = 0
        return True

    def run(self, max_iterations=10 ** 9, progress=None):
        n = 0
        while n < max_iterations and self.step():
            n += 1
            if progress and n % progress == 0:
                import sys
                print("iteration %d, scheduler time %.3f s, %d tokens generated"
                      % (n, self.sched.now(), self.stats["decode_tokens"]), file=sys.stderr, flush=True)
        torch.cuda.synchronize()
        return self.stats
