"""Logical (un-paged) model of the growing KV cache (test infrastructure, see
package doc).

Section 2.2 / 2.2.1: every decode iteration produces, in every layer, one key
and one value vector per kv head for the token being generated; they are
appended to the request's cache, whose size therefore grows by one position
per iteration.  A request that is not in the running batch (Algorithm 1)
appends nothing.

The model keeps, per layer and request, the sequences K[C][H_kv][D] and
V[C][H_kv][D] in the storage type (float32, or uint16 bf16 bit patterns) and
knows nothing of blocks or layouts: the GPU's paged result is compared with it
through the harness' un-pager.
"""
import numpy as np


class LogicalCache:
    def __init__(self, num_layers, ctx_lens, K, V):
        """K[layer][r], V[layer][r]: arrays [ctx_lens[r]][H_kv][D] (copied)."""
        self.ctx = [int(c) for c in ctx_lens]
        self.K = [[np.array(K[l][r], copy=True) for r in range(len(self.ctx))]
                  for l in range(num_layers)]
        self.V = [[np.array(V[l][r], copy=True) for r in range(len(self.ctx))]
                  for l in range(num_layers)]
        for l in range(num_layers):
            for r, c in enumerate(self.ctx):
                assert self.K[l][r].shape[0] == c and self.V[l][r].shape[0] == c

    def append(self, layer, k_new, v_new, running, advance):
        """Position ctx[r] of every running request r gets k_new[r], v_new[r]
        ([B][H_kv][D]) in `layer`.  With `advance` the context length of the
        running requests then grows by one (the caller passes it on the last
        layer of an iteration); without it a later call for the same layer
        overwrites the same position."""
        for r, on in enumerate(running):
            if not on:
                continue
            t = self.ctx[r]
            for seq, new in ((self.K, k_new), (self.V, v_new)):
                s = seq[layer][r]
                row = np.asarray(new[r], dtype=s.dtype)[None]
                if s.shape[0] == t:
                    seq[layer][r] = np.concatenate([s, row], axis=0)
                else:                                 # position t was written before (no advance since)
                    assert s.shape[0] == t + 1
                    s[t] = row[0]
        if advance:
            for r, on in enumerate(running):
                if on:
                    self.ctx[r] += 1
