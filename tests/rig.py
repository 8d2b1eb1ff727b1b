"""Test-side plumbing for the GPU tests: torch owns the device memory and the
streams, the library does the work.  Nothing here computes attention."""
import numpy as np
import torch

import lamps_workloads as W
import paper_2410_18248_amd as P


def make_config(geom, max_batch, part_tokens=0, staging_bytes=0, scale=0.0, direct_copy_bytes=0,
                zero_copy_workgroups=0, max_swaps_in_flight=0):
    return P.LampsConfig(geom.num_layers, geom.num_q_heads, geom.num_kv_heads, geom.head_dim,
                         geom.block_size, geom.num_blocks, geom.max_blocks_per_req, max_batch,
                         P.LAMPS_BF16 if geom.dtype == "bf16" else P.LAMPS_F32, scale,
                         part_tokens, staging_bytes, direct_copy_bytes, zero_copy_workgroups, max_swaps_in_flight)


def t2n(t):
    """torch tensor (cpu) -> numpy in the oracle's convention (bf16 as uint16 bits)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def n2t(a, device):
    """numpy (float32, or uint16 bf16 bits) -> torch tensor on device."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


class Rig:
    """Pools, workspace, streams and a Lamps context for one geometry."""

    def __init__(self, geom, max_batch, part_tokens=0, staging_bytes=0, poison=True,
                 side_streams=True, scale=0.0, direct_copy_bytes=0, zero_copy_workgroups=0,
                 max_swaps_in_flight=0):
        self.geom = geom
        self.dev = torch.device("cuda:0")
        self.tdtype = torch.bfloat16 if geom.dtype == "bf16" else torch.float32
        self.cfg = make_config(geom, max_batch, part_tokens, staging_bytes, scale, direct_copy_bytes,
                               zero_copy_workgroups, max_swaps_in_flight)
        assert P.lamps_pool_bytes(self.cfg) == int(np.prod(geom.pool_shape)) * geom.elem_bytes
        assert P.lamps_kv_layout(self.cfg) == (P.LAMPS_LAYOUT_TILED if geom.kv_layout == "tiled"
                                               else P.LAMPS_LAYOUT_PLAIN)
        self.k_index, self.v_index = geom.tile_index_maps()
        self.k_pool = torch.empty(geom.pool_shape, dtype=self.tdtype, device=self.dev)
        self.v_pool = torch.empty(geom.pool_shape, dtype=self.tdtype, device=self.dev)
        if poison:
            self.k_pool.fill_(float("nan"))
            self.v_pool.fill_(float("nan"))
        self.workspace = torch.empty(P.lamps_workspace_bytes(self.cfg), dtype=torch.uint8,
                                     device=self.dev)
        self.compute = torch.cuda.Stream(self.dev)
        self.s_out = torch.cuda.Stream(self.dev) if side_streams else self.compute
        self.s_in = torch.cuda.Stream(self.dev) if side_streams else self.compute
        torch.cuda.synchronize()
        self.lamps = P.Lamps(self.cfg, self.k_pool, self.v_pool, self.workspace,
                             self.compute.cuda_stream, self.s_out.cuda_stream,
                             self.s_in.cuda_stream)

    def close(self):
        torch.cuda.synchronize()
        self.lamps.destroy()

    # ---- paging (host mirror -> device) for logical-first inputs
    def host_pools(self):
        return t2n(self.k_pool), t2n(self.v_pool)

    def upload_pools(self, kp, vp):
        self.k_pool.copy_(n2t(kp, self.dev))
        self.v_pool.copy_(n2t(vp, self.dev))
        torch.cuda.synchronize()

    def page_requests(self, layer, table, K, V):
        kp, vp = self.host_pools()
        kp, vp = kp.copy(), vp.copy()
        for r in range(len(K)):
            if K[r] is not None:
                W.page(kp, layer, table[r], K[r], self.k_index)
                W.page(vp, layer, table[r], V[r], self.v_index)
        self.upload_pools(kp, vp)

    # ---- un-paging (device -> logical) for physical-first inputs
    def unpage_request(self, layer, table_row, C):
        nb = self.geom.blocks_for(C)
        ids = torch.as_tensor(np.asarray(table_row[:nb], dtype=np.int64), device=self.dev)
        kb = t2n(self.k_pool[ids, layer])            # [nb][Hkv][tile]
        vb = t2n(self.v_pool[ids, layer])
        return W.tiles_to_logical(kb, self.k_index, C), W.tiles_to_logical(vb, self.v_index, C)

    # ---- one decode call through the C ABI
    def decode(self, layer, q, table, ctx, running, out=None, sentinel=None):
        B = len(ctx)
        g = self.geom
        with torch.cuda.stream(self.compute):
            qd = q if torch.is_tensor(q) else n2t(q, self.dev)
            td = torch.as_tensor(np.ascontiguousarray(table, dtype=np.int32), device=self.dev)
            cd = torch.as_tensor(np.asarray(ctx, dtype=np.int32), device=self.dev)
            md = torch.as_tensor(np.asarray(running, dtype=np.uint8), device=self.dev)
            if out is None:
                out = torch.empty((B, g.num_q_heads, g.head_dim), dtype=self.tdtype, device=self.dev)
                out.fill_(float("nan") if sentinel is None else sentinel)
            self.lamps.decode_attn(layer, B, qd, td, cd, md, out)
        self.compute.synchronize()
        self._keep = (qd, td, cd, md)
        return out


def to_f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def tol(geom):
    """Max-abs error allowed against the fp64 oracle: fp32 path 1e-5, bf16 path 2e-2."""
    return 1e-5 if geom.dtype == "f32" else 2e-2
