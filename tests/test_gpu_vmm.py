"""GPU tests of independently allocated KV blocks with layer stacking (paper
Sec. 5.1 and 5.2): a pool of 2 MiB physical blocks shared by k = 4 layers of
128 tokens each, decode and prefill over it, a shrink that only permutes the
block list and then really returns memory to the device, and a grow."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import (MAX_ABS, REL_L2, assert_pools_equal, attn_errors, bitmap_ids, fill_pair,
                        make_pair)

pytestmark = pytest.mark.gpu
SEED = 4242
MiB = 1 << 20


_warm = False


def _free_bytes() -> int:
    global _warm
    if not _warm:  # one-time costs of the runtime (first mapping, first kernels) must not count
        w = P.VmmPool(2 * MiB, 4)
        t = torch.as_tensor(P.binding._DeviceSpan(w.alloc(2)[0], 2 * MiB), device="cuda")
        t.fill_(1)
        int(t.sum(dtype=torch.int64))
        del t
        torch.cuda.synchronize()
        w.close()
        _warm = True
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return torch.cuda.mem_get_info()[0]


def _close(delta: int, expected: int) -> bool:
    """device memory accounting is exact to a few MiB (page tables, the runtime's own rounding)"""
    return abs(delta - expected) <= max(8 * MiB, expected // 50)


def test_pool_alloc_free_accounting_and_errors():
    pool = P.VmmPool(2 * MiB, 64)
    free0 = _free_bytes()
    a = pool.alloc(40)
    assert len(set(a)) == 40 and pool.allocated == 40
    assert sorted(a) == a and a[1] - a[0] == 2 * MiB          # lowest positions first
    free1 = _free_bytes()
    assert _close(free0 - free1, 40 * 2 * MiB)                 # physical memory really taken ...
    t = torch.as_tensor(P.binding._DeviceSpan(a[7], 2 * MiB), device="cuda")
    t.fill_(1234)
    assert int(t.sum(dtype=torch.int64)) == 1234 * MiB
    del t
    with pytest.raises(P.PipeliveError) as e:
        pool.alloc(25)                                         # only 24 positions left
    assert e.value.rc == P.E_NOSPACE and pool.allocated == 40
    for bad in ([a[0] + 256], [a[0], a[0]], [a[-1] + 2 * MiB], [1 << 20]):
        with pytest.raises(P.PipeliveError) as e:
            pool.free(bad)
        assert e.value.rc == P.E_INVAL and pool.allocated == 40   # checked before anything is released
    pool.free(a[10:30])
    assert pool.allocated == 20
    assert _close(_free_bytes() - free1, 20 * 2 * MiB)         # ... and really returned
    with pytest.raises(P.PipeliveError):
        pool.free([a[10]])                                     # already released
    b = pool.alloc(20)
    assert sorted(b) == sorted(a[10:30])                       # freed positions are reused, lowest first
    pool.close()
    assert _close(_free_bytes() - free0, 0)


def test_quarter_filled_unit_is_what_stacking_avoids():
    """A 512 KiB block (one layer of 128 tokens) still costs a whole 2 MiB unit; four layers stacked
    into one 2 MiB block cost the same memory for four times the KV."""
    free0 = _free_bytes()
    small = P.VmmPool(512 << 10, 64)
    small.alloc(64)
    used_small = free0 - _free_bytes()
    small.close()
    assert P.pipelive_vmm_backing_bytes(512 << 10) == 2 * MiB
    assert _close(used_small, 64 * 2 * MiB)                    # four times the 32 MiB asked for
    assert _close(_free_bytes() - free0, 0)


def _decode(cfg, dev, layer, table_d, ctx_d):
    q = torch.from_numpy(pin.q_bits(cfg, SEED, layer).view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.full((cfg.num_seqs, cfg.num_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32,
                     device="cuda")
    P.pipelive_paged_attn_decode(dev, layer, q, out, table_d, ctx_d)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_stacked_vmm_region_decode_shrink_release_grow():
    # 8 layers, k = 4 -> 2 groups; 8 KV heads of 128, 128-token blocks: 512 KiB per layer, 2 MiB physical
    cfg = pin.StageConfig("vmm", 8, 32, 8, 128, 128, 12, 100, 1500)
    Bn = 160
    batch = pin.draw_batch(cfg, SEED, num_blocks=Bn)
    n_live = len(batch.live_ids)
    assert n_live < 120
    free0 = _free_bytes()
    host, dev = make_pair(cfg, batch, SEED, capacity=200, stack_k=4, backing="vmm")
    assert dev.phys_bytes == 2 * MiB and dev.groups == 2
    assert dev.pool.allocated == 2 * Bn
    assert _close(free0 - _free_bytes(), 2 * Bn * 2 * MiB)
    fill_pair(cfg, batch, SEED, host, dev)
    table_h = batch.table.copy()
    table_d = torch.from_numpy(batch.table).cuda()
    ctx_d = torch.from_numpy(batch.ctx_lens).cuda()
    used_d = torch.from_numpy(batch.used).cuda()

    # decode over the stacked, individually allocated blocks
    before = {}
    for layer in (0, 3, 5, 7):
        got = _decode(cfg, dev, layer, table_d, ctx_d)
        ref = host.attn_decode(layer, pin.q_bits(cfg, SEED, layer), table_h, batch.ctx_lens, nthreads=8)
        ma, rl = attn_errors(got, ref)
        assert ma <= MAX_ABS and rl <= REL_L2, (layer, ma, rl)
        before[layer] = got

    # shrink 160 -> 120: pointer updates only
    bl0_d = dev.block_list.cpu().numpy().copy()
    bl0_h = host.block_list.copy()
    B_new = 120
    rc_h, remap_h, res_h = host.resize(B_new, [table_h], [batch.used])
    remap_d = torch.full((Bn,), -7, dtype=torch.int32, device="cuda")
    rc_d, res_d = P.pipelive_kv_resize(dev, B_new, [table_d], [used_d], remap_out=remap_d)
    assert rc_h == oracle.OK and rc_d == P.OK
    assert (res_d.n_live, res_d.n_moved, res_d.old_num_blocks, res_d.new_num_blocks) == tuple(int(x) for x in res_h)
    assert res_d.n_moved > 0
    assert np.array_equal(remap_d.cpu().numpy(), remap_h)
    assert np.array_equal(table_d.cpu().numpy(), table_h)
    assert np.array_equal(bitmap_ids(dev.live, 200), host.live_ids())
    # the block list went through the same permutation as the oracle's (compare positions, the
    # addresses themselves are device vs host)
    bl1_d = dev.block_list.cpu().numpy()
    for g in range(dev.groups):
        pos_d = {int(a): i for i, a in enumerate(bl0_d[g, :Bn])}
        pos_h = {int(a): i for i, a in enumerate(bl0_h[g, :Bn])}
        assert [pos_d[int(a)] for a in bl1_d[g, :Bn]] == [pos_h[int(a)] for a in host.block_list[g, :Bn]]
    dev.sync_block_list()
    assert_pools_equal(host, dev, range(cfg.num_layers), host.live_ids())
    for layer in (0, 3, 5, 7):   # same physical blocks under new ids: bit-identical output
        assert np.array_equal(_decode(cfg, dev, layer, table_d, ctx_d).view(np.uint32), before[layer].view(np.uint32))

    # release the 40 blocks per group that no id names any more
    free1 = _free_bytes()
    assert dev.release_tail(Bn) == 2 * (Bn - B_new)
    assert dev.pool.allocated == 2 * B_new
    assert _close(_free_bytes() - free1, 2 * (Bn - B_new) * 2 * MiB)
    for layer in (0, 7):
        assert np.array_equal(_decode(cfg, dev, layer, table_d, ctx_d).view(np.uint32), before[layer].view(np.uint32))

    # grow to 180: new physical blocks appended to the list, new ids not live, usable
    dev.grow_backing(180)
    rc_h, _, _ = host.resize(180, [table_h], [batch.used])
    rc_d, res_d = P.pipelive_kv_resize(dev, 180, [table_d], [used_d])
    assert rc_h == oracle.OK and rc_d == P.OK and dev.num_blocks == 180
    assert np.array_equal(bitmap_ids(dev.live, 200), host.live_ids())
    probe = torch.arange(dev.blk_elems, dtype=torch.int16, device="cuda")[None]
    dev.write_blocks(6, [179], probe)
    assert torch.equal(dev.read_blocks(6, [179]), probe)
    assert np.array_equal(_decode(cfg, dev, 5, table_d, ctx_d).view(np.uint32), before[5].view(np.uint32))
    assert P.pipelive_kv_read_state(dev).status == 0
    del dev, table_d, ctx_d, used_d, remap_d, probe
    # all 640 MiB of the pool returned (the slack covers code objects and workspaces loaded meanwhile)
    assert abs(_free_bytes() - free0) <= 64 * MiB


def test_patch_between_stacked_vmm_regions():
    """Dirty blocks travel between two per-block regions with k = 4 (migration granularity of a group)."""
    cfg = pin.StageConfig("vmm2", 4, 16, 8, 128, 128, 6, 50, 600)
    batch = pin.draw_batch(cfg, SEED, num_blocks=48)
    host, dev = make_pair(cfg, batch, SEED, stack_k=4, backing="vmm")
    fill_pair(cfg, batch, SEED, host, dev)
    tgt_h = oracle.HostKV(4, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, 48,
                          stack_k=4, fill_bits=pin.BF16_NAN)
    tgt_d = P.KVRegion(4, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, 48,
                       stack_k=4, fill_bits=pin.BF16_NAN, backing="vmm")
    live = batch.live_ids
    layers = [0, 1, 2, 3]
    cap = 64 + 256 + len(live) * (4 + 4 * host.blk_bytes)
    patch_h = np.zeros(cap, dtype=np.uint8)
    patch_d = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    assert host.mark_dirty(live, 0) == oracle.OK
    P.pipelive_kv_mark_dirty(dev, torch.from_numpy(np.asarray(live, dtype=np.int32)).cuda(), 0)
    assert host.patch_collect(layers, patch_h) == oracle.OK
    P.pipelive_kv_patch_collect(dev, layers, patch_d)
    torch.cuda.synchronize()
    h = oracle.parse_patch_header(patch_h)
    end = h["payload_offset"] + h["n_blocks"] * 4 * host.blk_bytes
    assert np.array_equal(patch_d.cpu().numpy()[:end], patch_h[:end])
    assert tgt_h.patch_apply(layers, patch_h) == oracle.OK
    P.pipelive_kv_patch_apply(tgt_d, layers, patch_d)
    torch.cuda.synchronize()
    assert_pools_equal(tgt_h, tgt_d, range(4), live)
    assert P.pipelive_kv_read_state(tgt_d).status == 0
