"""GPU parity, Tiny configuration: one decode step over all layers, resize
128 -> 96 with compaction, decode again, round 0 + 3 patch rounds with 10 %
of the live blocks dirty.  Every byte of state is compared with the oracle."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import (MAX_ABS, REL_L2, assert_pools_equal, attn_errors, bitmap_ids, fill_pair,
                        make_pair)

pytestmark = pytest.mark.gpu
SEED = pin.MASTER_SEED


def _decode_all(cfg, dev, table_d, ctx_d, split=0):
    outs = []
    for layer in range(cfg.num_layers):
        q = torch.from_numpy(pin.q_bits(cfg, SEED, layer).view(np.int16)).cuda().view(torch.bfloat16)
        out = torch.full((cfg.num_seqs, cfg.num_q_heads, cfg.head_dim), float("nan"),
                         dtype=torch.float32, device="cuda")
        P.pipelive_paged_attn_decode(dev, layer, q, out, table_d, ctx_d, split_tokens=split)
        outs.append(out.cpu().numpy())
    return outs


def _oracle_all(cfg, host, table, ctx):
    return [host.attn_decode(layer, pin.q_bits(cfg, SEED, layer), table, ctx) for layer in range(cfg.num_layers)]


def test_tiny_end_to_end():
    cfg = pin.CONFIGS["tiny"]
    B = 128
    batch = pin.draw_batch(cfg, SEED, num_blocks=B)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    table_h = batch.table.copy()
    table_d = torch.from_numpy(batch.table).cuda()
    ctx_d = torch.from_numpy(batch.ctx_lens).cuda()
    used_d = torch.from_numpy(batch.used).cuda()

    # 1. decode
    ref = _oracle_all(cfg, host, table_h, batch.ctx_lens)
    got = _decode_all(cfg, dev, table_d, ctx_d, split=64)
    for layer in range(cfg.num_layers):
        ma, rl = attn_errors(got[layer], ref[layer])
        assert ma <= MAX_ABS and rl <= REL_L2, (layer, ma, rl)
        assert ma < 1e-4, "fp32 accumulation should be far inside the tolerance"

    # 2. resize 128 -> 96
    rc_h, remap_h, res_h = host.resize(96, [table_h], [batch.used])
    remap_d = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    rc_d, res_d = P.pipelive_kv_resize(dev, 96, [table_d], [used_d], remap_out=remap_d)
    assert rc_h == oracle.OK and rc_d == P.OK
    assert (res_d.n_live, res_d.n_moved, res_d.old_num_blocks, res_d.new_num_blocks) == tuple(int(x) for x in res_h)
    assert res_d.n_moved > 0
    assert np.array_equal(remap_d.cpu().numpy(), remap_h)
    assert np.array_equal(table_d.cpu().numpy(), table_h)
    assert dev.num_blocks == 96 == host.num_blocks
    assert np.array_equal(bitmap_ids(dev.live, 128), host.live_ids())
    assert_pools_equal(host, dev, range(cfg.num_layers), range(96))

    # 3. decode again: unchanged bit for bit on the GPU, still equal to the oracle
    got2 = _decode_all(cfg, dev, table_d, ctx_d, split=64)
    ref2 = _oracle_all(cfg, host, table_h, batch.ctx_lens)
    for layer in range(cfg.num_layers):
        assert np.array_equal(got2[layer].view(np.uint32), got[layer].view(np.uint32))
        assert np.array_equal(ref2[layer].view(np.uint32), ref[layer].view(np.uint32))

    # 4. patch session into a second region (3 layers; source layers 0,1 -> target layers 2,0)
    live = host.live_ids()
    bt2 = pin.Batch(cfg, SEED, 96, batch.ctx_lens, table_h, batch.used, live)
    tgt_h = oracle.HostKV(3, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, 96,
                          fill_bits=pin.BF16_NAN)
    tgt_d = P.KVRegion(3, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, 96,
                       arenas=2, fill_bits=pin.BF16_NAN)
    layers, dst_layers = [0, 1], [2, 0]
    cap = 64 + 256 + len(live) * (4 + 2 * host.blk_bytes)
    patch_h = np.zeros(cap, dtype=np.uint8)
    patch_d = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    hdr_pin = torch.zeros(64, dtype=torch.uint8).pin_memory()
    sched = 0
    for rnd in range(4):
        if rnd == 0:
            ids, ntok = live, 0
        else:
            ids = pin.draw_dirty_ids(bt2, SEED, rnd, 0.10)
            ntok = cfg.num_seqs
            for layer in range(cfg.num_layers):
                rows = np.stack([pin.kv_block_bits(cfg, SEED, 128, rnd, layer, int(b)) for b in ids])
                for b, row in zip(ids, rows):
                    host.block(layer, int(b))[:] = row
                dev.write_blocks(layer, ids, torch.from_numpy(rows.view(np.int16)).cuda())
        sched += ntok
        assert host.mark_dirty(ids, ntok) == oracle.OK
        P.pipelive_kv_mark_dirty(dev, torch.from_numpy(np.asarray(ids, dtype=np.int32)).cuda(), ntok)
        assert np.array_equal(bitmap_ids(dev.dirty, 96), host.dirty_ids())
        assert host.patch_collect(layers, patch_h) == oracle.OK
        P.pipelive_kv_patch_collect(dev, layers, patch_d, hdr_host=hdr_pin)
        torch.cuda.synchronize()
        h = oracle.parse_patch_header(patch_h)
        assert h["n_blocks"] == len(ids)
        got_p = patch_d.cpu().numpy()
        assert np.array_equal(got_p[:64], patch_h[:64])
        assert np.array_equal(hdr_pin.numpy(), patch_h[:64])
        assert np.array_equal(got_p[64:64 + 4 * h["n_blocks"]], patch_h[64:64 + 4 * h["n_blocks"]])
        end = h["payload_offset"] + h["n_blocks"] * 2 * host.blk_bytes
        assert np.array_equal(got_p[h["payload_offset"]:end], patch_h[h["payload_offset"]:end])
        assert len(bitmap_ids(dev.dirty, 96)) == 0
        assert tgt_h.patch_apply(dst_layers, patch_h) == oracle.OK
        P.pipelive_kv_patch_apply(tgt_d, dst_layers, patch_d)
    st = P.pipelive_kv_read_state(tgt_d)
    assert st.t_applied == sched == tgt_h.t_applied and st.status == 0
    assert P.pipelive_kv_read_state(dev).n_acc == 0 == host.n_acc
    assert_pools_equal(tgt_h, tgt_d, range(3), range(96))          # every byte of the target
    for b in live:                                                  # target == source
        for sl, dl in zip(layers, dst_layers):
            assert np.array_equal(tgt_d.block(dl, int(b)).cpu().numpy(), dev.block(sl, int(b)).cpu().numpy())


def test_tiny_infeasible_busy_and_range_leave_state_untouched():
    cfg = pin.CONFIGS["tiny"]
    batch = pin.draw_batch(cfg, SEED, num_blocks=128)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    table_d = torch.from_numpy(batch.table).cuda()
    used_d = torch.from_numpy(batch.used).cuda()
    n_live = len(batch.live_ids)
    rc, res = P.pipelive_kv_resize(dev, n_live - 1, [table_d], [used_d])
    assert rc == P.E_INFEASIBLE and res.n_live == n_live and res.new_num_blocks == 128
    ids = torch.tensor([int(batch.live_ids[0])], dtype=torch.int32, device="cuda")
    P.pipelive_kv_mark_dirty(dev, ids, 1)
    rc, res = P.pipelive_kv_resize(dev, 100, [table_d], [used_d])
    assert rc == P.E_BUSY
    patch = torch.zeros(64 + 256 + 4 * (4 + 2 * dev.blk_bytes), dtype=torch.uint8, device="cuda")
    P.pipelive_kv_patch_collect(dev, [0, 1], patch)
    bad = table_d.clone()
    free = sorted(set(range(128)) - set(batch.live_ids.tolist()))[0]
    bad[0, 0] = free
    rc, res = P.pipelive_kv_resize(dev, 100, [bad], [used_d])
    assert rc == P.E_RANGE
    rc, res = P.pipelive_kv_resize(dev, 129, [table_d], [used_d])
    assert rc == P.E_NOSPACE
    assert dev.num_blocks == 128
    assert np.array_equal(table_d.cpu().numpy(), batch.table)
    assert np.array_equal(bitmap_ids(dev.live, 128), batch.live_ids)
    assert_pools_equal(host, dev, range(cfg.num_layers), range(128))
    # exactly full is feasible; grow back moves nothing
    table_h = batch.table.copy()
    rc_h, remap_h, res_h = host.resize(n_live, [table_h], [batch.used])
    remap_d = torch.zeros(128, dtype=torch.int32, device="cuda")
    rc, res = P.pipelive_kv_resize(dev, n_live, [table_d], [used_d], remap_out=remap_d)
    assert rc == P.OK == rc_h and res.n_moved == res_h[1]
    assert np.array_equal(remap_d.cpu().numpy(), remap_h) and np.array_equal(table_d.cpu().numpy(), table_h)
    assert_pools_equal(host, dev, range(cfg.num_layers), range(n_live))
    rc_h, remap_h, res_h = host.resize(128, [table_h], [batch.used])
    rc, res = P.pipelive_kv_resize(dev, 128, [table_d], [used_d], remap_out=remap_d)
    assert rc == P.OK and res.n_moved == 0 and dev.num_blocks == 128
    assert np.array_equal(remap_d.cpu().numpy()[:n_live], remap_h[:n_live])
    assert np.array_equal(bitmap_ids(dev.live, 128), host.live_ids())


def test_clipped_drain_matches_oracle():
    cfg = pin.CONFIGS["tiny"]
    batch = pin.draw_batch(cfg, SEED, num_blocks=128)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    ids = batch.live_ids[::3]
    host.mark_dirty(ids, 17)
    P.pipelive_kv_mark_dirty(dev, torch.from_numpy(ids.astype(np.int32)).cuda(), 17)
    cap = 64 + 256 + 5 * (4 + 1 * host.blk_bytes) + 100       # room for 5 blocks
    assert P.pipelive_patch_max_blocks(dev, 1, cap) == 5 == host.patch_max_blocks(1, cap)
    patch_h = np.zeros(cap, dtype=np.uint8)
    patch_d = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    rounds = 0
    while True:
        assert host.patch_collect([1], patch_h) == oracle.OK
        P.pipelive_kv_patch_collect(dev, [1], patch_d)
        h = oracle.parse_patch_header(patch_h)
        g = patch_d.cpu().numpy()
        end = h["payload_offset"] + h["n_blocks"] * host.blk_bytes
        assert np.array_equal(g[:64 + 4 * h["n_blocks"]], patch_h[:64 + 4 * h["n_blocks"]])
        assert np.array_equal(g[h["payload_offset"]:end], patch_h[h["payload_offset"]:end])
        assert np.array_equal(bitmap_ids(dev.dirty, 128), host.dirty_ids())
        assert P.pipelive_kv_read_state(dev).n_acc == host.n_acc
        rounds += 1
        if not h["more_pending"]:
            break
    assert rounds == (len(ids) + 4) // 5
    assert P.pipelive_kv_patch_collect(dev, [1], patch_d[:300], check=False) == P.E_NOSPACE
    assert P.pipelive_kv_patch_collect(dev, [2], patch_d, check=False) == P.E_RANGE


def test_device_status_word_on_bad_ids():
    cfg = pin.CONFIGS["tiny"]
    batch = pin.draw_batch(cfg, SEED, num_blocks=128)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    P.pipelive_kv_mark_dirty(dev, torch.tensor([5, 128, -1], dtype=torch.int32, device="cuda"), 0)
    assert P.pipelive_kv_read_state(dev).status == P.E_RANGE
    assert bitmap_ids(dev.dirty, 128).tolist() == [5]
    P.pipelive_kv_clear_status(dev)
    assert P.pipelive_kv_read_state(dev).status == 0
    # a patch whose ids do not exist in a smaller target: skipped, flagged, nothing written
    small = P.KVRegion(cfg.num_layers, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, 4,
                       fill_bits=pin.BF16_NAN)
    patch = torch.zeros(64 + 256 + 2 * (4 + dev.blk_bytes), dtype=torch.uint8, device="cuda")
    P.pipelive_kv_patch_collect(dev, [0], patch)
    P.pipelive_kv_patch_apply(small, [1], patch)
    assert P.pipelive_kv_read_state(small).status == P.E_RANGE
    for b in range(4):
        assert (small.block(1, b).cpu().numpy().view(np.uint16) == pin.BF16_NAN).all()
    # header mismatch (other number of layers)
    P.pipelive_kv_clear_status(small)
    P.pipelive_kv_patch_apply(small, [0, 1], patch)
    assert P.pipelive_kv_read_state(small).status == P.E_INVAL


@pytest.mark.parametrize("backing", ["arena", "vmm"])
def test_resize_with_no_table_and_with_several_tables(backing):
    """The last kernel of a shrink rewrites every table in one launch and moves the live bits: none, and
    three tables of different shapes (the batch's rows split in two, plus a table that shares blocks with
    them and holds rows without entries)."""
    cfg = pin.CONFIGS["tiny"]
    B = 128
    batch = pin.draw_batch(cfg, SEED, num_blocks=B)
    for n_tables in (0, 3):
        host, dev = make_pair(cfg, batch, SEED, backing=backing)
        fill_pair(cfg, batch, SEED, host, dev)
        half = cfg.num_seqs // 2
        t0, u0 = batch.table[:half].copy(), batch.used[:half].copy()
        t1 = np.ascontiguousarray(np.pad(batch.table[half:], ((0, 0), (0, 5)), constant_values=pin.TABLE_FILL))
        u1 = batch.used[half:].copy()
        t2 = np.full((4, 3), pin.TABLE_FILL, dtype=np.int32)      # prefix sharing: first blocks of four sequences
        u2 = np.zeros(4, dtype=np.int32)
        for k, srow in enumerate((0, half, 1)):
            n = min(3, int(batch.used[srow]))
            t2[k, :n] = batch.table[srow, :n]
            u2[k] = n                                           # row 3 stays empty
        tabs_h = [t0, t1, t2][:n_tables]
        used_h = [u0, u1, u2][:n_tables]
        tabs_d = [torch.from_numpy(t.copy()).cuda() for t in tabs_h]
        used_d = [torch.from_numpy(u.copy()).cuda() for u in used_h]
        rc_h, remap_h, res_h = host.resize(96, tabs_h, used_h)
        remap_d = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        rc_d, res_d = P.pipelive_kv_resize(dev, 96, tabs_d, used_d, remap_out=remap_d)
        assert rc_h == oracle.OK and rc_d == P.OK
        assert (res_d.n_live, res_d.n_moved, res_d.old_num_blocks, res_d.new_num_blocks) == tuple(int(x) for x in res_h)
        assert res_d.n_moved > 0
        assert np.array_equal(remap_d.cpu().numpy(), remap_h)
        for td, th in zip(tabs_d, tabs_h):
            assert np.array_equal(td.cpu().numpy(), th)          # the oracle remapped its tables in place
        assert np.array_equal(bitmap_ids(dev.live, 128), host.live_ids())
        dev.sync_block_list()
        assert_pools_equal(host, dev, range(cfg.num_layers), host.live_ids())
