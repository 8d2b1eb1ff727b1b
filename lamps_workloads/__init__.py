"""Seeded synthetic inputs for the paged decode + KV swap path.

This module serves both the GPU tests / benchmark and the CPU oracle's tests.
It draws numbers, deals block tables and moves bytes between a request's
logical key/value sequence and the block pool; it contains none of the
method's arithmetic (no scores, no softmax, no merging) and imports neither
the oracle nor the GPU package.

The paper's workloads (the INFERCEPT request mix and ToolBench, Section 6) are
not reproduced: the five configurations below stand in for them, keeping the
batch sizes, the head geometry of the served models (Section 6: GPT-J 6B,
Vicuna 13B), the spread of context lengths and the share of requests that sit
in an API call under each handling strategy (Section 1).
"""
from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 241018248
_MASK = (1 << 64) - 1


def config_seed(cfg, rep=0):
    return SEED_BASE + 1000 * cfg + rep


# ---------------------------------------------------------------- generators
def splitmix64(seed, n):
    """n outputs of the splitmix64 sequence started at `seed` (uint64 array).

    Counter form: output i mixes seed + (i+1)*golden-gamma, so any slice can be
    produced without the ones before it."""
    with np.errstate(over="ignore"):
        z = (np.uint64(seed & _MASK)
             + (np.arange(1, n + 1, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed, n):
    """n doubles in (0, 1): top 53 bits of splitmix64, offset by half a step."""
    return ((splitmix64(seed, n) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / (1 << 53))


def normal_f32(seed, n):
    """n standard normal float32 draws (Box-Muller on uniform01 pairs)."""
    m = (n + 1) // 2
    u = uniform01(seed, 2 * m)
    rad = np.sqrt(-2.0 * np.log(u[0::2]))
    ang = 2.0 * np.pi * u[1::2]
    z = np.empty(2 * m, dtype=np.float64)
    z[0::2] = rad * np.cos(ang)
    z[1::2] = rad * np.sin(ang)
    return z[:n].astype(np.float32)


def permutation(seed, n):
    """Fisher-Yates shuffle of 0..n-1 driven by splitmix64(seed)."""
    p = np.arange(n, dtype=np.int64)
    rnd = splitmix64(seed, max(n - 1, 0))
    for i in range(n - 1, 0, -1):
        j = int(rnd[n - 1 - i] % np.uint64(i + 1))
        p[i], p[j] = p[j], p[i]
    return p


# ---------------------------------------------------------------- bf16 bits
def f32_to_bf16_bits(x):
    """float32 -> bf16 bit patterns (uint16), round to nearest even; NaN kept quiet."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = ((b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


BF16_NAN = np.uint16(0x7FC0)


# ---------------------------------------------------------------- geometry
@dataclass(frozen=True)
class Geometry:
    """Shape of the KV pool.  Keys and values live in separate pools of the same
    shape, pool[block][layer][kv_head][tile]; a tile holds the block_size x
    head_dim elements of one (block, layer, kv head) in the order given by
    `tile_index_maps` (the library's documented layout)."""
    num_layers: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    num_blocks: int
    max_blocks_per_req: int
    dtype: str  # "f32" | "bf16"

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.uint16

    @property
    def tile_elems(self):
        return self.block_size * self.head_dim

    @property
    def pool_shape(self):
        return (self.num_blocks, self.num_layers, self.num_kv_heads, self.tile_elems)

    @property
    def kv_layout(self):
        """"tiled" for bf16 with grouped query heads, else "plain"."""
        grouped = self.num_q_heads // self.num_kv_heads >= 2
        return "tiled" if self.dtype == "bf16" and grouped else "plain"

    @property
    def block_half_bytes(self):
        """Bytes of one block in ONE pool (all layers)."""
        return self.num_layers * self.num_kv_heads * self.tile_elems * self.elem_bytes

    @property
    def token_bytes_per_layer(self):
        """Key + value bytes of one token in one layer."""
        return 2 * self.num_kv_heads * self.head_dim * self.elem_bytes

    def blocks_for(self, ctx_len):
        return (int(ctx_len) + self.block_size - 1) // self.block_size

    def tile_index_maps(self):
        """(k_index, v_index): int arrays [block_size][head_dim] giving the element
        offset of (slot, dim) inside a tile of the key pool / the value pool."""
        s = np.arange(self.block_size)[:, None]
        d = np.arange(self.head_dim)[None, :]
        if self.kv_layout == "plain":
            idx = s * self.head_dim + d
            return idx, idx
        base = (s // 16) * 16 * self.head_dim
        t = s % 16
        k = base + ((d // 8) * 16 + t) * 8 + d % 8
        v = base + ((((d // 32) * 4 + t // 4) * 16 + d % 16) * 2 + (d % 32) // 16) * 4 + t % 4
        return k, v


def deal_block_table(perm, ctx_lens, geom, start=0):
    """Deal physical ids from `perm` (starting at `start`) to requests in order.

    Returns (table int32[B][max_blocks_per_req] with -1 in unused entries,
    number of ids consumed)."""
    B = len(ctx_lens)
    table = np.full((B, geom.max_blocks_per_req), -1, dtype=np.int32)
    pos = start
    for r, c in enumerate(ctx_lens):
        nb = geom.blocks_for(c)
        assert nb <= geom.max_blocks_per_req, "context longer than the table row"
        assert pos + nb <= len(perm), "pool too small for this batch"
        table[r, :nb] = perm[pos:pos + nb]
        pos += nb
    return table, pos - start


def page(pool, layer, table_row, seq, index_map):
    """Scatter a logical sequence seq[C][H_kv][D] into pool (numpy array of shape
    Geometry.pool_shape) through one block-table row; index_map is the pool's
    entry of Geometry.tile_index_maps().  Slots past C are left as they are."""
    C = seq.shape[0]
    bs = index_map.shape[0]
    for j in range((C + bs - 1) // bs):
        n = min(bs, C - j * bs)
        # pool[block, layer] is [H_kv][tile]; seq chunk is [slot][H_kv][D]
        pool[table_row[j], layer][:, index_map[:n].ravel()] = \
            np.swapaxes(seq[j * bs:j * bs + n], 0, 1).reshape(seq.shape[1], -1)


def tiles_to_logical(tiles, index_map, C):
    """tiles[nb][H_kv][tile] (the blocks of one request, in logical order) ->
    the first C cached positions as [C][H_kv][D]."""
    bs, D = index_map.shape
    x = tiles[..., index_map.ravel()]                       # [nb][H_kv][bs * D] in (slot, dim) order
    x = x.reshape(tiles.shape[0], tiles.shape[1], bs, D)
    return np.ascontiguousarray(np.swapaxes(x, 1, 2).reshape(-1, tiles.shape[1], D)[:C])


def unpage(pool, layer, table_row, C, index_map):
    """Gather the first C cached positions of one request back into [C][H_kv][D]."""
    nb = (C + index_map.shape[0] - 1) // index_map.shape[0]
    ids = np.asarray(table_row[:nb], dtype=np.int64)
    return tiles_to_logical(pool[ids, layer], index_map, C)


# ---------------------------------------------------------------- context lengths
def ctx_uniform(seed, B, lo, hi):
    """Integers uniform on [lo, hi]."""
    u = uniform01(seed, B)
    return (lo + np.floor(u * (hi - lo + 1))).astype(np.int64).clip(lo, hi)


def ctx_lognormal(seed, B, median, sigma, lo, hi):
    """round(exp(ln median + sigma z)), clipped to [lo, hi]."""
    z = normal_f32(seed, B).astype(np.float64)
    return np.clip(np.rint(np.exp(np.log(median) + sigma * z)), lo, hi).astype(np.int64)


def ctx_zipf_rank(seed, B, s, lo, hi):
    """C = lo - 1 + k with P(k) proportional to k^-s on k = 1 .. hi-lo+1
    (rank 1 is the shortest context)."""
    k = np.arange(1, hi - lo + 2, dtype=np.float64)
    cdf = np.cumsum(k ** (-s))
    cdf /= cdf[-1]
    u = uniform01(seed, B)
    return (lo + np.searchsorted(cdf, u, side="left")).astype(np.int64).clip(lo, hi)


# ---------------------------------------------------------------- configurations
@dataclass
class Workload:
    """One synthetic batch description (no tensors)."""
    name: str
    geom: Geometry
    batch: int
    ctx_lens: np.ndarray            # int64[B]
    state: np.ndarray               # uint8[B]: RUNNING / PRESERVE / SWAP / DISCARD
    part_tokens: int = 0            # 0 = library default
    notes: dict = field(default_factory=dict)


RUNNING, PRESERVE, SWAP, DISCARD = 0, 1, 2, 3


def _pick(seed, B, n):
    """n distinct request indices chosen by seed, in draw order."""
    return permutation(seed, B)[:n]


def workload(cfg, rep=0, num_blocks=None):
    """The five configurations.  cfg 0 is the tiny fp32 parity case; 1..4 are
    the serving-shaped ones.  `rep` changes the draw, not the shape."""
    seed = config_seed(cfg, rep)
    if cfg == 0:
        g = Geometry(1, 8, 8, 64, 16, 64, 13, "f32")
        ctx = np.array([17, 64, 130, 200], dtype=np.int64)
        st = np.zeros(4, dtype=np.uint8)
        st[2] = SWAP
        return Workload("cfg0-tiny-fp32", g, 4, ctx, st)
    if cfg == 1:
        g = Geometry(1, 32, 32, 128, 16, num_blocks or 40000, 128, "bf16")
        B = 64
        ctx = ctx_uniform(seed + 1, B, 128, 2048)
        st = np.zeros(B, dtype=np.uint8)
        paused = _pick(seed + 2, B, int(round(0.2 * B)))
        st[paused[:len(paused) // 2]] = PRESERVE
        st[paused[len(paused) // 2:]] = SWAP
        return Workload("cfg1-7b-mha-bf16", g, B, ctx, st)
    if cfg == 2:
        B = 256
        ctx = ctx_lognormal(seed + 1, B, 1024.0, 1.0, 32, 8192)
        need = int(sum((int(c) + 15) // 16 for c in ctx))
        g = Geometry(1, 32, 8, 128, 16, num_blocks or int(need * 1.5) + 1, 512, "bf16")
        st = np.zeros(B, dtype=np.uint8)
        st[_pick(seed + 2, B, int(round(0.1 * B)))] = SWAP
        return Workload("cfg2-8b-gqa-bf16", g, B, ctx, st)
    if cfg == 3:
        B = 32
        ctx = ctx_uniform(seed + 1, B, 4096, 32768)
        nb = [(int(c) + 31) // 32 for c in ctx]
        g = Geometry(1, 32, 8, 128, 32, num_blocks or int(sum(nb) * 1.5) + 1, 1024, "bf16")
        st = np.zeros(B, dtype=np.uint8)
        order = permutation(seed + 2, B)
        covered = 0
        for r in order:  # requests in seed order until 40 % of allocated blocks are covered
            if covered >= 0.4 * sum(nb):
                break
            st[r] = SWAP
            covered += nb[r]
        return Workload("cfg3-long-gqa-bf16", g, B, ctx, st)
    if cfg == 4:
        B = 512
        ctx = ctx_zipf_rank(seed + 1, B, 1.2, 64, 4096)
        need = int(sum((int(c) + 15) // 16 for c in ctx))
        g = Geometry(40, 40, 40, 128, 16, num_blocks or int(need * 1.1) + 1, 256, "bf16")
        st = np.zeros(B, dtype=np.uint8)
        out = _pick(seed + 2, B, int(round(0.15 * B)))
        q = len(out) // 4  # Preserve : Discard : Swap = 1 : 1 : 2
        st[out[:q]] = PRESERVE
        st[out[q:2 * q]] = DISCARD
        st[out[2 * q:]] = SWAP
        return Workload("cfg4-13b-40layer-bf16", g, B, ctx, st)
    raise ValueError("cfg must be 0..4")


def logical_kv(seed, geom, ctx_len):
    """Logical key and value sequences [C][H_kv][D] ~ N(0,1) in the geometry's
    storage type (float32, or bf16 bit patterns rounded once here)."""
    n = int(ctx_len) * geom.num_kv_heads * geom.head_dim
    shape = (int(ctx_len), geom.num_kv_heads, geom.head_dim)
    k = normal_f32(seed, n).reshape(shape)
    v = normal_f32(seed ^ 0x5DEECE66D, n).reshape(shape)
    if geom.dtype == "bf16":
        return f32_to_bf16_bits(k), f32_to_bf16_bits(v)
    return k, v


def queries(seed, geom, batch):
    q = normal_f32(seed ^ 0xA5A5A5A5, batch * geom.num_q_heads * geom.head_dim)
    q = q.reshape(batch, geom.num_q_heads, geom.head_dim)
    return f32_to_bf16_bits(q) if geom.dtype == "bf16" else q


def poison(geom):
    """Value that must never influence a result: NaN in the storage type."""
    return np.float32(np.nan) if geom.dtype == "f32" else BF16_NAN
