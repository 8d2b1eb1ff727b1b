"""Byte- and integer-exact model of the KV block pool under the three handling
strategies of Section 1 / Section 4.2 (test infrastructure, see package doc).

Preserve: nothing moves, blocks stay allocated.
Discard : blocks go back to the free list; contents become undefined.
Swap    : the request's KV cache is offloaded to CPU memory and reloaded when
          the API returns; a block id denotes the block in all layers, keys
          and values.  Host image of block i = key-pool bytes of that block
          followed by value-pool bytes of that block.  A second, layer-major
          image holds the same bytes layer by layer (a reload in that order
          lets the first layers run while the rest is on its way).

The pools are opaque byte rows here: the model knows nothing of the layout
inside a block.
"""
import numpy as np


def kv_bytes_per_token(num_layers, num_kv_heads, head_dim, elem_bytes):
    """M of equations (1)-(3): one key and one value vector per layer per head
    (Section 2.2.1: memory grows with sequence length, layers, hidden size)."""
    return 2 * num_layers * num_kv_heads * head_dim * elem_bytes


class PoolModel:
    """Key pool and value pool as uint8[num_blocks][half_bytes]."""

    def __init__(self, k_bytes, v_bytes):
        self.k = np.array(k_bytes, dtype=np.uint8, copy=True)
        self.v = np.array(v_bytes, dtype=np.uint8, copy=True)
        assert self.k.ndim == 2 and self.k.shape == self.v.shape

    @property
    def half_bytes(self):
        return self.k.shape[1]

    def swap_out(self, block_ids):
        """Returns the host image uint8[n][2*half]; the pool is unchanged."""
        ids = list(block_ids)
        host = np.empty((len(ids), 2 * self.half_bytes), dtype=np.uint8)
        for i, b in enumerate(ids):
            host[i, :self.half_bytes] = self.k[b]
            host[i, self.half_bytes:] = self.v[b]
        return host

    def swap_in(self, host, block_ids):
        """Writes image i into block block_ids[i]; every other block is untouched."""
        ids = list(block_ids)
        host = np.asarray(host, dtype=np.uint8).reshape(len(ids), 2 * self.half_bytes)
        assert len(set(ids)) == len(ids), "duplicate destination block"
        for i, b in enumerate(ids):
            self.k[b] = host[i, :self.half_bytes]
            self.v[b] = host[i, self.half_bytes:]


    def swap_out_layered(self, block_ids, num_layers):
        """The layer-major host image uint8[layers][n][2][half / layers]: the request's cache
        layer by layer (a block's half is its layers one after the other), so that a reload
        can hand over layer 0 first.  The pool is unchanged."""
        ids = list(block_ids)
        lb = self.half_bytes // num_layers
        assert lb * num_layers == self.half_bytes
        host = np.empty((num_layers, len(ids), 2, lb), dtype=np.uint8)
        for layer in range(num_layers):
            for i, b in enumerate(ids):
                host[layer, i, 0] = self.k[b, layer * lb:(layer + 1) * lb]
                host[layer, i, 1] = self.v[b, layer * lb:(layer + 1) * lb]
        return host

    def swap_in_layered(self, host, block_ids, num_layers, layers=None):
        """Writes a layer-major image back (only the listed layers, if given: what has landed
        when the reload is `layers` layers in); every other byte is untouched."""
        ids = list(block_ids)
        lb = self.half_bytes // num_layers
        host = np.asarray(host, dtype=np.uint8).reshape(num_layers, len(ids), 2, lb)
        assert len(set(ids)) == len(ids), "duplicate destination block"
        for layer in (range(num_layers) if layers is None else layers):
            for i, b in enumerate(ids):
                self.k[b, layer * lb:(layer + 1) * lb] = host[layer, i, 0]
                self.v[b, layer * lb:(layer + 1) * lb] = host[layer, i, 1]


class AllocatorModel:
    """LIFO free list: a fresh pool hands out 0, 1, 2, ...; ``free`` pushes ids
    in the order given, so the last id freed is the next one allocated."""

    def __init__(self, num_blocks):
        self.num_blocks = num_blocks
        self.stack = list(range(num_blocks - 1, -1, -1))
        self.live = set()

    @property
    def num_free(self):
        return len(self.stack)

    def alloc(self, n):
        if n < 0 or n > len(self.stack):
            raise MemoryError("pool exhausted")
        ids = [self.stack.pop() for _ in range(n)]
        self.live.update(ids)
        return ids

    def free(self, ids):
        ids = list(ids)
        if len(set(ids)) != len(ids):
            raise ValueError("duplicate id")
        for b in ids:
            if not 0 <= b < self.num_blocks:
                raise IndexError("id out of range")
            if b not in self.live:
                raise ValueError("double free")
        for b in ids:
            self.live.remove(b)
            self.stack.append(b)
