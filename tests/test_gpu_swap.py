"""Swap / free-list behaviour of liblamps on the GPU against the oracle's
byte-exact block model (handling strategies of Section 1 / Section 4.2)."""
import numpy as np
import pytest
import torch

import lamps_workloads as W
import oracle
import paper_2410_18248_amd as P
from rig import Rig, t2n, to_f64

pytestmark = pytest.mark.gpu


def _bytes(t):
    return t.detach().cpu().contiguous().view(torch.uint8).numpy()


def _fill_random(rig, seed):
    gen = torch.Generator(device=rig.dev).manual_seed(seed)
    # random BYTES (every bit pattern, NaNs included): the copy must not interpret them
    for pool in (rig.k_pool, rig.v_pool):
        raw = pool.view(torch.uint8)
        raw.copy_(torch.randint(0, 256, raw.shape, dtype=torch.uint8, device=rig.dev, generator=gen))
    torch.cuda.synchronize()


def _model(rig):
    nb = rig.geom.num_blocks
    return oracle.PoolModel(_bytes(rig.k_pool).reshape(nb, -1), _bytes(rig.v_pool).reshape(nb, -1))


def _pinned(n):
    return torch.empty(max(n, 1), dtype=torch.uint8).pin_memory()


# the three ways a block-major image moves: staged through the gather kernels, plain copies
# per block, one kernel that reaches the pinned buffer itself
PATHS = {"staged": {}, "direct": {"direct_copy_bytes": 1}, "zero-copy": {"zero_copy_workgroups": 3}}


@pytest.mark.parametrize("path", list(PATHS))
@pytest.mark.parametrize("dtype,L,Hkv,D,bs,staging_blocks", [
    ("f32", 1, 8, 64, 16, 0), ("bf16", 3, 2, 128, 16, 4), ("bf16", 2, 4, 128, 32, 1)])
def test_swap_out_image_and_round_trip(dtype, L, Hkv, D, bs, staging_blocks, path):
    geom = W.Geometry(L, Hkv, Hkv, D, bs, 48, 8, dtype)
    bb = 2 * geom.block_half_bytes
    rig = Rig(geom, max_batch=2, staging_bytes=staging_blocks * bb,     # small staging: several chunks
              **PATHS[path])
    lam = rig.lamps
    assert P.lamps_block_bytes(rig.cfg) == bb
    _fill_random(rig, 11)
    model = _model(rig)
    ids_all = lam.alloc_blocks(geom.num_blocks)
    assert ids_all == oracle.AllocatorModel(geom.num_blocks).alloc(geom.num_blocks)
    src = [int(x) for x in W.permutation(5, geom.num_blocks)[:11]]
    host = _pinned(len(src) * bb)
    t = lam.swap_out(src, host)
    lam.ticket_wait(t)
    assert lam.ticket_query(t)
    want = model.swap_out(src)
    np.testing.assert_array_equal(host.numpy().reshape(len(src), bb), want)     # image layout, bit-exact
    np.testing.assert_array_equal(_bytes(rig.k_pool).reshape(geom.num_blocks, -1), model.k)  # pool untouched
    np.testing.assert_array_equal(_bytes(rig.v_pool).reshape(geom.num_blocks, -1), model.v)

    # back into different blocks; every other block byte-identical
    dst = [int(x) for x in W.permutation(5, geom.num_blocks)[20:31]]
    t2 = lam.swap_in(host, dst)
    lam.ticket_wait(t2)
    model.swap_in(want, dst)
    np.testing.assert_array_equal(_bytes(rig.k_pool).reshape(geom.num_blocks, -1), model.k)
    np.testing.assert_array_equal(_bytes(rig.v_pool).reshape(geom.num_blocks, -1), model.v)
    rig.close()


@pytest.mark.parametrize("dtype,L,Hkv,D,bs,staging_blocks", [
    ("f32", 1, 8, 64, 16, 0), ("bf16", 3, 2, 128, 16, 4), ("bf16", 5, 4, 128, 32, 1), ("bf16", 40, 2, 64, 16, 0)])
def test_layer_major_swap_image_and_round_trip(dtype, L, Hkv, D, bs, staging_blocks):
    """The layer-major variant: image layout against the oracle's, round trip into other
    blocks, every other block untouched; small staging areas force steps of one layer in
    chunks of blocks, large ones several layers per step."""
    geom = W.Geometry(L, Hkv, Hkv, D, bs, 48, 8, dtype)
    bb = 2 * geom.block_half_bytes
    rig = Rig(geom, max_batch=2, staging_bytes=staging_blocks * bb)
    lam = rig.lamps
    _fill_random(rig, 12)
    model = _model(rig)
    lam.alloc_blocks(geom.num_blocks)
    src = [int(x) for x in W.permutation(6, geom.num_blocks)[:11]]
    host = _pinned(len(src) * bb)
    t = lam.swap_out(src, host, layered=True)
    lam.ticket_wait(t)
    want = model.swap_out_layered(src, L)
    np.testing.assert_array_equal(host.numpy().reshape(want.shape), want)
    np.testing.assert_array_equal(_bytes(rig.k_pool).reshape(geom.num_blocks, -1), model.k)
    dst = [int(x) for x in W.permutation(6, geom.num_blocks)[20:31]]
    t2 = lam.swap_in(host, dst, layered=True)
    for layer in range(L):
        lam.compute_wait_layer(t2, layer)           # enqueues waits on the compute stream; any order is legal
    with pytest.raises(P.LampsError) as e:
        lam.compute_wait_layer(t2, L)
    assert e.value.status == -2
    lam.ticket_wait(t2)
    lam.compute_wait_layer(t2, 0)                   # a finished ticket: nothing to wait for
    model.swap_in_layered(want, dst, L)
    np.testing.assert_array_equal(_bytes(rig.k_pool).reshape(geom.num_blocks, -1), model.k)
    np.testing.assert_array_equal(_bytes(rig.v_pool).reshape(geom.num_blocks, -1), model.v)
    rig.close()


def test_layer_major_swap_in_feeds_decode_layer_by_layer():
    """A swapped-out request comes back layer-major into new blocks; each layer is decoded
    behind lamps_compute_wait_layer only, and matches the oracle."""
    geom = W.Geometry(6, 8, 2, 128, 16, 300, 40, "bf16")
    ctx = [600, 200]
    B = len(ctx)
    rig = Rig(geom, max_batch=B)
    lam = rig.lamps
    lam.alloc_blocks(geom.num_blocks)
    perm = W.permutation(9, geom.num_blocks)
    table, used = W.deal_block_table(perm, ctx, geom)
    lam.free_blocks([int(x) for x in perm[used:]])
    K, V, q = [], [], W.queries(9, geom, B)
    for r, c in enumerate(ctx):
        k, v = W.logical_kv(200 + r, geom, c)
        K.append(k)
        V.append(v)
    for layer in range(geom.num_layers):
        rig.page_requests(layer, table, K, V)       # the same K, V in every layer
    ref = oracle.decode_attn(q, K, V, ctx, [1] * B)
    bb = 2 * geom.block_half_bytes
    old = [int(x) for x in table[0, :geom.blocks_for(ctx[0])]]
    host = _pinned(len(old) * bb)
    lam.swap_out(old, host, layered=True)
    lam.free_blocks(old)
    new = lam.alloc_blocks(len(old))[::-1]          # the same physical blocks in another order
    tab = table.copy()
    tab[0, :len(new)] = new
    with torch.cuda.stream(rig.compute):
        idx = torch.as_tensor(old, device=rig.dev)
        lam.compute_wait_blocks(old)
        rig.k_pool[idx] = 0.0                       # whatever the swap-in has not brought back is wrong
        rig.v_pool[idx] = 0.0
    ticket = lam.swap_in(host, new, layered=True)
    outs = []
    for layer in range(geom.num_layers):
        lam.compute_wait_layer(ticket, layer)
        outs.append(rig.decode(layer, q, tab, ctx, [1] * B))
    for layer, got in enumerate(outs):
        np.testing.assert_allclose(to_f64(got), ref, rtol=0, atol=2e-2, err_msg="layer %d" % layer)
    lam.ticket_wait(ticket)
    rig.close()


def test_empty_list_and_ticket_errors():
    geom = W.Geometry(1, 2, 2, 64, 16, 8, 2, "bf16")
    rig = Rig(geom, max_batch=1)
    lam = rig.lamps
    host = _pinned(16)
    t = lam.swap_out([], host)
    lam.ticket_wait(t)
    assert lam.ticket_query(t)
    t = lam.swap_in(host, [], layered=True)         # an empty layer-major copy is a ticket like any other
    lam.compute_wait_layer(t, 0)
    lam.ticket_wait(t)
    assert lam.ticket_query(t)
    with pytest.raises(P.LampsError) as e:
        lam.ticket_wait(t + 5)
    assert e.value.status == -2
    with pytest.raises(P.LampsError) as e:
        lam.swap_out([3], host)                     # block 3 is not allocated
    assert e.value.status == -4
    rig.close()


def test_freed_block_reuse_waits_for_its_swap_out():
    """swap-out, free, allocate again (LIFO gives the same ids back) and overwrite
    at once: the host image must still hold the old bytes."""
    geom = W.Geometry(8, 8, 8, 128, 16, 160, 8, "bf16")     # 512 KiB images, ~70 MB per swap
    bb = 2 * geom.block_half_bytes
    rig = Rig(geom, max_batch=1)
    lam = rig.lamps
    _fill_random(rig, 21)
    model = _model(rig)
    lam.alloc_blocks(geom.num_blocks)
    ids = list(range(10, 150))
    other = _pinned(len(ids) * bb)
    other.numpy()[:] = 0x5A
    host = _pinned(len(ids) * bb)
    want = model.swap_out(ids)
    t_out = lam.swap_out(ids, host)
    lam.free_blocks(ids)
    again = lam.alloc_blocks(len(ids))
    assert again == ids[::-1]                       # LIFO, as in the oracle's allocator model
    t_in = lam.swap_in(other, again)                # overwrites the same physical blocks
    lam.ticket_wait(t_in)
    lam.ticket_wait(t_out)
    np.testing.assert_array_equal(host.numpy().reshape(len(ids), bb), want)
    assert (_bytes(rig.k_pool[again[0]]) == 0x5A).all()
    rig.close()


def test_compute_stream_writer_is_ordered_by_compute_wait_blocks():
    """A compute-stream writer of a re-allocated block (recompute after Discard,
    KV append) goes behind the block's unfinished swap-out."""
    geom = W.Geometry(8, 8, 8, 128, 16, 160, 8, "bf16")
    bb = 2 * geom.block_half_bytes
    rig = Rig(geom, max_batch=1)
    lam = rig.lamps
    _fill_random(rig, 22)
    model = _model(rig)
    lam.alloc_blocks(geom.num_blocks)
    ids = list(range(5, 145))
    host = _pinned(len(ids) * bb)
    want = model.swap_out(ids)
    t_out = lam.swap_out(ids, host)
    lam.free_blocks(ids)
    again = lam.alloc_blocks(len(ids))
    lam.compute_wait_blocks(again)
    with torch.cuda.stream(rig.compute):
        idx = torch.as_tensor(again, device=rig.dev)
        rig.k_pool[idx] = 0.0
        rig.v_pool[idx] = 0.0
    lam.ticket_wait(t_out)
    rig.compute.synchronize()
    np.testing.assert_array_equal(host.numpy().reshape(len(ids), bb), want)
    assert (_bytes(rig.k_pool[again[0]]) == 0).all()
    rig.close()


def test_backpressure_keeps_the_swap_queue_shallow():
    """max_swaps_in_flight = 2: a swap call returns only when fewer than two copies of its
    direction are unfinished, so right after call k the copies before k - 1 are done; the
    images are what they are without the limit."""
    geom = W.Geometry(8, 8, 8, 128, 16, 400, 8, "bf16")
    bb = 2 * geom.block_half_bytes
    rig = Rig(geom, max_batch=1, max_swaps_in_flight=2)
    lam = rig.lamps
    _fill_random(rig, 29)
    model = _model(rig)
    lam.alloc_blocks(geom.num_blocks)
    groups = [list(range(40 * g, 40 * g + 40)) for g in range(10)]      # 20 MiB each
    hosts = [_pinned(40 * bb) for _ in groups]
    tickets = []
    for ids, host in zip(groups, hosts):
        tickets.append(lam.swap_out(ids, host))
        assert all(lam.ticket_query(t) for t in tickets[:-2])           # at most two still on their way
    for g, (ids, host) in enumerate(zip(groups, hosts)):                # and back in, into the next group's blocks
        t = lam.swap_in(host, groups[(g + 1) % len(groups)])
        tickets.append(t)
        assert all(lam.ticket_query(x) for x in tickets[len(groups):-2])
    lam.ticket_wait(tickets[-1])
    for ids, host in zip(groups, hosts):                                # every swap-out read the blocks before any swap-in wrote them
        np.testing.assert_array_equal(host.numpy().reshape(len(ids), bb), model.swap_out(ids))
    for g, ids in enumerate(groups):                                    # group g + 1 now holds what group g held
        model_after = model.swap_out(ids)
        got = _model(rig).swap_out(groups[(g + 1) % len(groups)])
        np.testing.assert_array_equal(got, model_after)
    rig.close()


@pytest.mark.parametrize("fence", [True, False])
def test_swap_out_behind_a_compute_stream_writer(fence):
    """The swap-out of blocks that compute-stream work still writes comes after that work: by
    itself (the default), or, with the automatic ordering switched off, because the caller
    said so with lamps_swap_wait_compute."""
    geom = W.Geometry(8, 8, 8, 128, 16, 160, 8, "bf16")
    bb = 2 * geom.block_half_bytes
    rig = Rig(geom, max_batch=1)
    lam = rig.lamps
    _fill_random(rig, 23)
    lam.alloc_blocks(geom.num_blocks)
    lam.set_swap_fence(fence)
    ids = list(range(3, 150))
    host = _pinned(len(ids) * bb)
    host.numpy()[:] = 0
    big = torch.empty(1 << 28, dtype=torch.float32, device=rig.dev)
    with torch.cuda.stream(rig.compute):
        for _ in range(8):                              # a few milliseconds of work ahead of the writer
            big.fill_(1.0)
        idx = torch.as_tensor(ids, device=rig.dev)
        rig.k_pool[idx] = 1.5
        rig.v_pool[idx] = -2.0
    if not fence:
        lam.swap_wait_compute()
    t = lam.swap_out(ids, host)
    lam.ticket_wait(t)
    got = host.view(torch.bfloat16).reshape(len(ids), 2, -1)
    assert (got[:, 0] == 1.5).all() and (got[:, 1] == -2.0).all()
    rig.close()


@pytest.mark.parametrize("path", list(PATHS))
def test_swap_in_right_behind_swap_out_through_one_buffer(path):
    geom = W.Geometry(4, 8, 8, 128, 16, 128, 8, "bf16")
    bb = 2 * geom.block_half_bytes
    rig = Rig(geom, max_batch=1, **PATHS[path])
    lam = rig.lamps
    _fill_random(rig, 31)
    model = _model(rig)
    lam.alloc_blocks(geom.num_blocks)
    src, dst = list(range(0, 50)), list(range(60, 110))
    host = _pinned(len(src) * bb)
    host.numpy()[:] = 0
    lam.swap_out(src, host)
    t = lam.swap_in(host, dst)                      # no host wait in between
    lam.ticket_wait(t)
    model.swap_in(model.swap_out(src), dst)
    np.testing.assert_array_equal(_bytes(rig.k_pool).reshape(geom.num_blocks, -1), model.k)
    np.testing.assert_array_equal(_bytes(rig.v_pool).reshape(geom.num_blocks, -1), model.v)
    rig.close()


def test_zero_copy_refuses_memory_the_device_cannot_reach():
    """The copy kernel of the zero-copy path dereferences the host buffer: pageable or
    misaligned memory is turned down on the host, before anything is enqueued."""
    geom = W.Geometry(1, 2, 2, 64, 16, 8, 4, "bf16")
    bb = 2 * geom.block_half_bytes
    rig = Rig(geom, max_batch=1, zero_copy_workgroups=2)
    lam = rig.lamps
    ids = lam.alloc_blocks(2)
    pageable = np.zeros(2 * bb + 64, dtype=np.uint8)
    for call in (lambda: lam.swap_out(ids, pageable), lambda: lam.swap_in(pageable, ids)):
        with pytest.raises(P.LampsError) as e:
            call()
        assert e.value.status == -1
    pinned = _pinned(2 * bb + 16)
    with pytest.raises(P.LampsError) as e:
        lam.swap_out(ids, pinned.data_ptr() + 4)
    assert e.value.status == -1
    t = lam.swap_out(ids, pinned)                   # and the context still works
    lam.ticket_wait(t)
    rig.close()


def test_decode_while_others_swap():
    """Requests in Swap state move out and back on the side streams while the
    others are decoded; outputs match the oracle and paused rows stay untouched;
    after lamps_compute_wait the returned requests decode correctly from their
    new blocks."""
    geom = W.Geometry(2, 8, 2, 128, 16, 400, 40, "bf16")
    ctx = [600, 37, 512, 300, 129, 640]
    B = len(ctx)
    rig = Rig(geom, max_batch=B, part_tokens=128)
    lam = rig.lamps
    lam.alloc_blocks(geom.num_blocks)
    perm = W.permutation(8, geom.num_blocks)
    table, used = W.deal_block_table(perm, ctx, geom)
    lam.free_blocks([int(x) for x in perm[used:]])
    K, V, q = [], [], W.queries(8, geom, B)
    for r, c in enumerate(ctx):
        k, v = W.logical_kv(100 + r, geom, c)
        K.append(k)
        V.append(v)
    for layer in range(geom.num_layers):
        rig.page_requests(layer, table, K, V)
    ref = oracle.decode_attn(q, K, V, ctx, [1] * B)
    swapped = [0, 3]
    running = np.ones(B, dtype=np.uint8)
    running[swapped] = 0
    bb = 2 * geom.block_half_bytes
    tickets, new_tab = [], table.copy()
    bufs = []
    for r in swapped:
        old = [int(x) for x in table[r, :geom.blocks_for(ctx[r])]]
        new = lam.alloc_blocks(len(old))
        host = _pinned(len(old) * bb)
        bufs.append(host)
        lam.swap_out(old, host)
        lam.free_blocks(old)
        tickets.append(lam.swap_in(host, new))
        new_tab[r, :len(new)] = new
    for layer in range(geom.num_layers):            # decode of the others, swaps in flight
        out = rig.decode(layer, q, table, ctx, running, sentinel=9.0)
        got = to_f64(out)
        for r in range(B):
            if running[r]:
                assert np.abs(got[r] - ref[r]).max() <= 2e-2
            else:
                assert (got[r] == 9.0).all()
    for t in tickets:
        lam.compute_wait(t)
    out = rig.decode(1, q, new_tab, ctx, [1] * B)
    assert np.abs(to_f64(out) - ref).max() <= 2e-2
    rig.close()
