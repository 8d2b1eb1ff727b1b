"""The C-ABI library without a GPU: it loads, exports every declared symbol,
and its host logic (sizes, validation, free list) behaves as documented.  No
compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

import lamps_workloads as W
import paper_2410_18248_amd as P
from oracle import AllocatorModel, kv_bytes_per_token

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = os.path.join(ROOT, "tests", "golden")


def _cfg(**kw):
    base = dict(num_layers=2, num_q_heads=8, num_kv_heads=2, head_dim=128, block_size=16,
                num_blocks=32, max_blocks_per_req=8, max_batch=4, dtype=P.LAMPS_BF16,
                softmax_scale=0.0, part_tokens=0, staging_bytes=0)
    base.update(kw)
    return P.LampsConfig(**base)


@pytest.fixture
def ctx():
    buf = ctypes.create_string_buffer(4096)
    a = (ctypes.addressof(buf) + 255) & ~255
    lam = P.Lamps(_cfg(), a, a, a)                 # fake "device" memory: never dereferenced here
    lam._buf = buf
    yield lam
    lam.destroy()


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lamps.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(lamps_[a-z_]+)\s*\(", header)))
    assert len(names) >= 22 and "lamps_kv_append" in names and "lamps_swap_in_layered" in names
    lib = P.load_library()
    for n in names:
        assert hasattr(lib, n), n


def test_sizes():
    c = _cfg()
    half = 2 * 2 * 16 * 128 * 2
    assert P.lamps_block_bytes(c) == 2 * half
    assert P.lamps_pool_bytes(c) == 32 * half
    assert P.lamps_kv_bytes_per_token(c) == kv_bytes_per_token(2, 2, 128, 2)
    assert P.lamps_workspace_bytes(c) >= 4 * 8 * 1 * 130 * 4 + 2 * 2 * half
    g = W.workload(1).geom
    c1 = _cfg(num_layers=1, num_q_heads=32, num_kv_heads=32, num_blocks=40000, max_blocks_per_req=128,
              max_batch=64)
    assert P.lamps_pool_bytes(c1) == g.num_blocks * g.block_half_bytes


def test_layout_query():
    assert P.lamps_kv_layout(_cfg()) == P.LAMPS_LAYOUT_TILED                       # bf16, 8 / 2 heads
    assert P.lamps_kv_layout(_cfg(num_kv_heads=8)) == P.LAMPS_LAYOUT_PLAIN        # bf16 MHA
    assert P.lamps_kv_layout(_cfg(dtype=P.LAMPS_F32)) == P.LAMPS_LAYOUT_PLAIN     # fp32
    assert P.lamps_kv_layout(_cfg(head_dim=96)) == -1


def test_kv_bytes_matches_paper_example():
    L, Hkv, D, s, tokens, quoted = np.loadtxt(os.path.join(GOLD, "kv_cache_size.txt"))
    c = _cfg(num_layers=int(L), num_q_heads=int(Hkv), num_kv_heads=int(Hkv), head_dim=int(D))
    total = P.lamps_kv_bytes_per_token(c) * int(tokens)
    assert abs(total / 2 ** 30 - quoted) / quoted < 0.05


@pytest.mark.parametrize("bad", [
    dict(num_q_heads=7), dict(head_dim=96), dict(block_size=8), dict(block_size=24),
    dict(dtype=5), dict(num_blocks=0), dict(part_tokens=24), dict(staging_bytes=100),
    dict(dtype=P.LAMPS_F32, head_dim=256), dict(zero_copy_workgroups=-1), dict(zero_copy_workgroups=2000),
    dict(zero_copy_workgroups=4, direct_copy_bytes=1)])
def test_invalid_configs_are_rejected(bad):
    c = _cfg(**bad)
    assert P.lamps_block_bytes(c) == 0 and P.lamps_workspace_bytes(c) == 0
    with pytest.raises(P.LampsError) as e:
        P.Lamps(c, 256, 256, 256)
    assert e.value.status == -1


def test_create_rejects_null_and_misaligned():
    for args in [(0, 256, 256), (256, 0, 256), (256, 256, 0), (257, 256, 256)]:
        with pytest.raises(P.LampsError):
            P.Lamps(_cfg(), *args)


def test_allocator_follows_the_lifo_model(ctx):
    model = AllocatorModel(32)
    rnd = W.splitmix64(77, 400)
    held = []
    for i in range(200):
        if rnd[2 * i] % 3 != 0 and model.num_free:
            n = int(rnd[2 * i + 1] % min(5, model.num_free)) + 1
            got = ctx.alloc_blocks(n)
            assert got == model.alloc(n)
            held += got
        elif held:
            n = int(rnd[2 * i + 1] % len(held)) + 1
            p = W.permutation(int(rnd[2 * i + 1] % 1000), len(held))[:n]
            ids = [held[j] for j in p]
            ctx.free_blocks(ids)
            model.free(ids)
            held = [b for b in held if b not in ids]
        assert ctx.num_free() == model.num_free
        assert ctx.num_free() + len(held) == 32                    # conservation


def test_errors_leave_state_unchanged(ctx):
    ids = ctx.alloc_blocks(5)
    assert ids == [0, 1, 2, 3, 4]
    before = ctx.num_free()
    for bad, status in [([1, 1], -3), ([0, 40], -2), ([-1], -2), ([7], -4), ([0, 7], -4)]:
        with pytest.raises(P.LampsError) as e:
            ctx.free_blocks(bad)
        assert e.value.status == status
        assert ctx.num_free() == before
    with pytest.raises(P.LampsError) as e:
        ctx.alloc_blocks(before + 1)
    assert e.value.status == -6 and ctx.num_free() == before
    assert ctx.alloc_blocks(2) == [5, 6]                             # order undisturbed
    assert "not enough free blocks" in ctx.last_error() or ctx.last_error() != ""


def test_free_count_per_handling_strategy(ctx):
    """Preserve keeps the blocks; Discard and (after its copy) Swap release them;
    the API's return takes them back (Section 4.2)."""
    req = ctx.alloc_blocks(9)
    base = ctx.num_free()
    assert ctx.num_free() == base                    # Preserve
    ctx.free_blocks(req)                             # Discard / Swap
    assert ctx.num_free() == base + 9
    assert len(ctx.alloc_blocks(9)) == 9 and ctx.num_free() == base


def test_argument_validation_makes_no_gpu_call(ctx):
    with pytest.raises(P.LampsError) as e:
        ctx.decode_attn(0, 4, 0, 256, 256, 256, 256)                 # null q
    assert e.value.status == -1
    with pytest.raises(P.LampsError) as e:
        ctx.decode_attn(2, 4, 256, 256, 256, 256, 256)               # layer out of range
    assert e.value.status == -2
    with pytest.raises(P.LampsError) as e:
        ctx.decode_attn(0, 5, 256, 256, 256, 256, 256)               # batch > max_batch
    assert e.value.status == -2
    ctx.decode_attn(0, 0, 256, 256, 256, 256, 256)                   # empty batch: nothing to do
    ids = ctx.alloc_blocks(2)
    for bad, status in [([0, 0], -3), ([99], -2), ([5], -4)]:
        with pytest.raises(P.LampsError) as e:
            ctx.swap_out(bad, 256)
        assert e.value.status == status
        with pytest.raises(P.LampsError) as e:
            ctx.swap_in(256, bad)
        assert e.value.status == status
    with pytest.raises(P.LampsError) as e:
        ctx.swap_out(ids, 0)                                         # null host buffer
    assert e.value.status == -1
    with pytest.raises(P.LampsError) as e:
        ctx.ticket_query(1)                                          # no ticket issued yet
    assert e.value.status == -2


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits (before touching a device)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one MI355X" in r.stderr and r.stdout.strip() == ""


def test_static_scratch_decode_checks_its_arguments_before_any_gpu_call():
    """lamps_decode_attn_static: everything the host can see is refused before the device is
    touched (this runs without a GPU), and the text comes back through lamps_last_error(NULL)."""
    buf = ctypes.create_string_buffer(4096)
    a = (ctypes.addressof(buf) + 255) & ~255                      # never dereferenced
    ok = _cfg()

    def call(cfg=ok, layer=0, batch=2, q=a, kp=a, vp=a, table=a, lens=a, mask=a, out=a):
        P.lamps_decode_attn_static(cfg, 0, layer, batch, q, kp, vp, table, lens, mask, out)
    for bad, status, word in ((dict(cfg=_cfg(head_dim=48)), -1, "head_dim"),
                              (dict(cfg=_cfg(part_tokens=64)), -1, "part_tokens"),
                              (dict(q=None), -1, "null"), (dict(vp=None), -1, "null"),
                              (dict(kp=a + 8), -1, "aligned"),
                              (dict(layer=2), -2, "layer"), (dict(layer=-1), -2, "layer"),
                              (dict(batch=5), -2, "batch"), (dict(batch=-1), -2, "batch")):
        with pytest.raises(P.LampsError) as e:
            call(**bad)
        assert e.value.status == status and word in str(e.value), (bad, str(e.value))
    call(batch=0)                                                 # an empty batch is no work and no error
    header = open(os.path.join(ROOT, "include", "lamps.h")).read()
    m = re.search(r"#define\s+LAMPS_STATIC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", header)
    assert m and (int(m.group(1)) << int(m.group(2))) == 33 << 20   # the stated, modest size
