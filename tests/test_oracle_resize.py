"""Pins for the oracle's ResizeKV / compaction (CPU only).

Paper: Sec. 4.2 primitive ResizeKV(B); Alg. 1 phase 1 (abort when the blocks
in use exceed the shrunken budget); Sec. 5.1 (compaction frees the tail of
the block list, expansion appends)."""
import itertools

import numpy as np
import pytest

import oracle
import pipelive_inputs as pin
from helpers import dense_attention, gather_logical, scatter_dense


def _definition(live, B, B_new):
    """The pairing rule written as sorted lists (independent of the oracle's
    scan): T = live ids in the tail, F = free ids in the head, T[k] -> F[k]."""
    T = sorted(b for b in live if b >= B_new)
    F = sorted(b for b in range(B_new) if b not in live)
    remap = {b: (b if b in live else -1) for b in range(B)}
    for t, f in zip(T, F):
        remap[t] = f
    return remap, len(T)


def _fill_blocks(kv, seed=0):
    rng = np.random.default_rng(seed)
    for layer in range(kv.L):
        for b in range(kv.capacity):
            kv.block(layer, b)[:] = rng.integers(0, 65536, kv.blk_elems, dtype=np.uint16)


def _snapshot(kv):
    return [[kv.block(l, b).copy() for b in range(kv.capacity)] for l in range(kv.L)]


def test_brute_force_all_subsets_of_8_blocks():
    B = 8
    for mask in range(1 << B):
        live = {b for b in range(B) if mask >> b & 1}
        for B_new in range(0, B + 1):
            kv = oracle.HostKV(2, 2, 1, 8, 2, B, arenas=3)
            _fill_blocks(kv, seed=mask)
            before = _snapshot(kv)
            kv.set_live(sorted(live))
            table = np.array([sorted(live) + [pin.TABLE_FILL]], dtype=np.int32) if live else np.full((1, 1), pin.TABLE_FILL, np.int32)
            used = np.array([len(live)], dtype=np.int32)
            t0 = table.copy()
            rc, remap, res = kv.resize(B_new, [table], [used])
            if len(live) > B_new:
                assert rc == oracle.E_INFEASIBLE
                assert kv.num_blocks == B and np.array_equal(table, t0)
                assert set(kv.live_ids()) == live
                for l in range(2):
                    for b in range(B):
                        assert np.array_equal(kv.block(l, b), before[l][b])
                continue
            assert rc == oracle.OK
            exp, n_moved = _definition(live, B, B_new)
            assert [int(x) for x in remap[:B]] == [exp[b] for b in range(B)]
            assert res[0] == len(live) and res[1] == n_moved and res[2] == B and res[3] == B_new
            assert kv.num_blocks == B_new
            assert set(kv.live_ids()) == {exp[b] for b in live}
            assert list(table[0, :len(live)]) == [exp[b] for b in sorted(live)]
            assert table[0, -1] == pin.TABLE_FILL or len(live) == table.shape[1]
            for l in range(2):
                for b in live:  # content followed the block
                    assert np.array_equal(kv.block(l, exp[b]), before[l][b])
                moved_dst = {exp[b] for b in live if exp[b] != b}
                for b in range(B_new):  # nothing else in the kept range was written
                    if b not in moved_dst:
                        assert np.array_equal(kv.block(l, b), before[l][b])


def test_per_block_mode_permutes_the_block_list_and_copies_nothing():
    """Sec. 5.1: with independently allocated blocks compaction is pointer updates only.  On every
    subset of an 8-block pool the logical outcome (remap, table, live set, content by id) equals the
    copying mode's, the block list is a permutation of itself, unmoved ids keep their address, the
    addresses left at ids >= B_new belong to blocks nobody uses, and no arena byte changes."""
    B = 8
    for mask in range(1 << B):
        live = {b for b in range(B) if mask >> b & 1}
        for B_new in range(len(live), B + 1):
            kv = oracle.HostKV(4, 2, 1, 8, 2, B, arenas=3, stack_k=2, per_block=True)
            ref = oracle.HostKV(4, 2, 1, 8, 2, B, arenas=3, stack_k=2)
            _fill_blocks(kv, seed=mask)
            _fill_blocks(ref, seed=mask)
            before = _snapshot(kv)
            arenas0 = [a.copy() for a in kv.arenas]
            bl0 = kv.block_list.copy()
            for r in (kv, ref):
                r.set_live(sorted(live))
            tabs = [np.array([sorted(live) + [pin.TABLE_FILL]], dtype=np.int32) for _ in range(2)]
            used = np.array([len(live)], dtype=np.int32)
            rc, remap, res = kv.resize(B_new, [tabs[0]], [used])
            rc2, remap2, res2 = ref.resize(B_new, [tabs[1]], [used])
            assert rc == rc2 == oracle.OK
            assert np.array_equal(remap, remap2) and list(res) == list(res2)
            assert np.array_equal(tabs[0], tabs[1]) and np.array_equal(kv.live, ref.live)
            for a0, a1 in zip(arenas0, kv.arenas):
                assert np.array_equal(a0, a1)                      # nothing was copied
            exp, _ = _definition(live, B, B_new)
            for g in range(kv.groups):
                assert sorted(kv.block_list[g]) == sorted(bl0[g])  # a permutation
                for b in live:
                    assert kv.block_list[g, exp[b]] == bl0[g, b]   # the id took its physical block along
                used_addrs = {int(bl0[g, b]) for b in live}
                for b in range(B_new, B):
                    assert int(kv.block_list[g, b]) not in used_addrs
                for b in range(B_new):
                    if b not in {exp[x] for x in live if exp[x] != x}:
                        assert kv.block_list[g, b] == bl0[g, b]
            for l in range(kv.L):
                for b in live:
                    assert np.array_equal(kv.block(l, exp[b]), before[l][b])
                    assert np.array_equal(kv.block(l, exp[b]), ref.block(l, exp[b]))


def _tiny_region(seed=pin.MASTER_SEED, B=128, stack_k=1):
    cfg = pin.CONFIGS["tiny"]
    bt = pin.draw_batch(cfg, seed, num_blocks=B)
    kv = oracle.HostKV(cfg.num_layers, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                       cfg.block_tokens, B, layout=cfg.layout, stack_k=stack_k)
    rng = np.random.default_rng(1)
    dense = {}
    for layer in range(cfg.num_layers):
        for s in range(cfg.num_seqs):
            n = int(bt.ctx_lens[s])
            k = pin.f32_to_bf16_bits(rng.standard_normal((n, cfg.num_kv_heads, cfg.head_dim)).astype(np.float32))
            v = pin.f32_to_bf16_bits(rng.standard_normal((n, cfg.num_kv_heads, cfg.head_dim)).astype(np.float32))
            dense[(layer, s)] = (k, v)
            scatter_dense(kv, layer, bt.table[s], k, v)
    kv.set_live(bt.live_ids)
    return cfg, bt, kv, dense


@pytest.mark.parametrize("stack_k", [1, 2])
def test_tiny_shrink_keeps_logical_kv_and_attention(stack_k):
    cfg, bt, kv, dense = _tiny_region(stack_k=stack_k)
    assert len(bt.live_ids) <= 96, "seed must give a feasible draw"
    q = pin.q_bits(cfg, 1, 0)
    before = kv.attn_decode(0, q, bt.table, bt.ctx_lens)
    table = bt.table.copy()
    rc, remap, res = kv.resize(96, [table], [bt.used])
    assert rc == oracle.OK
    n_tail = int((bt.live_ids >= 96).sum())
    assert res[1] == n_tail and n_tail > 0
    live_remap = remap[bt.live_ids]
    assert len(np.unique(live_remap)) == len(live_remap) and live_remap.max() < 96
    keep = bt.live_ids[bt.live_ids < 96]
    assert np.array_equal(remap[keep], keep)
    for s in range(cfg.num_seqs):
        assert (table[s, :bt.used[s]] < 96).all()
        assert (table[s, bt.used[s]:] == pin.TABLE_FILL).all()
        for layer in range(cfg.num_layers):
            k, v = gather_logical(kv, layer, table[s], int(bt.ctx_lens[s]))
            assert np.array_equal(k, dense[(layer, s)][0]) and np.array_equal(v, dense[(layer, s)][1])
    after = kv.attn_decode(0, q, table, bt.ctx_lens)
    assert np.array_equal(before.view(np.uint32), after.view(np.uint32))
    ref = dense_attention(q[3], *dense[(0, 3)], cfg.group)
    assert np.abs(after[3] - ref).max() < 2e-6


def test_infeasible_and_busy_have_no_side_effects():
    cfg, bt, kv, dense = _tiny_region()
    snap = _snapshot(kv)
    table = bt.table.copy()
    n_live = len(bt.live_ids)
    rc, remap, res = kv.resize(n_live - 1, [table], [bt.used])
    assert rc == oracle.E_INFEASIBLE and res[0] == n_live
    assert kv.num_blocks == 128 and np.array_equal(table, bt.table)
    kv.mark_dirty([int(bt.live_ids[0])], 1)
    rc, _, _ = kv.resize(100, [table], [bt.used])
    assert rc == oracle.E_BUSY
    assert kv.num_blocks == 128 and np.array_equal(table, bt.table)
    assert np.array_equal(kv.live_ids(), bt.live_ids)
    for l in range(cfg.num_layers):
        for b in range(128):
            assert np.array_equal(kv.block(l, b), snap[l][b])


def test_exactly_full_is_feasible_and_grow_shrink_is_identity():
    cfg, bt, kv, dense = _tiny_region()
    n_live = len(bt.live_ids)
    table = bt.table.copy()
    rc, remap, res = kv.resize(n_live, [table], [bt.used])
    assert rc == oracle.OK and set(kv.live_ids()) == set(range(n_live))
    t1 = table.copy()
    rc, remap, res = kv.resize(128, [table], [bt.used])       # grow: nothing moves
    assert rc == oracle.OK and res[1] == 0 and kv.num_blocks == 128
    assert np.array_equal(table, t1)
    assert np.array_equal(remap[:n_live], np.arange(n_live))
    rc, remap, res = kv.resize(n_live, [table], [bt.used])    # shrink back: identity
    assert rc == oracle.OK and res[1] == 0 and np.array_equal(table, t1)
    rc, _, _ = kv.resize(129, [table], [bt.used])
    assert rc == oracle.E_NOSPACE


def test_table_entry_must_be_live():
    cfg, bt, kv, dense = _tiny_region()
    table = bt.table.copy()
    free = sorted(set(range(128)) - set(bt.live_ids.tolist()))[0]
    table[0, 0] = free
    rc, _, _ = kv.resize(120, [table], [bt.used])
    assert rc == oracle.E_RANGE and kv.num_blocks == 128


def test_shared_blocks_and_two_tables():
    """Two tables (e.g. running and waiting queues) sharing a prefix block."""
    kv = oracle.HostKV(1, 2, 1, 8, 2, 10)
    _fill_blocks(kv)
    kv.set_live([1, 8, 9])
    ta = np.array([[9, 1]], dtype=np.int32)
    tb = np.array([[9, 8, pin.TABLE_FILL]], dtype=np.int32)
    rc, remap, res = kv.resize(4, [ta, tb], [np.array([2]), np.array([2])])
    assert rc == oracle.OK and res[1] == 2
    assert list(remap) == [-1, 1, -1, -1, -1, -1, -1, -1, 0, 2]
    assert ta.tolist() == [[2, 1]] and tb.tolist() == [[2, 0, pin.TABLE_FILL]]


def test_max_blocks_closed_form():
    # floor((M*u - L*W) / (L*P)) (Alg. 1, MaxBlocks)
    assert oracle.max_blocks(80e9, 0.9, 16, 0.4e9, 65536) == int((80e9 * 0.9 - 16 * 0.4e9) // (16 * 65536))
    assert oracle.max_blocks(100.0, 1.0, 2, 10.0, 4.0) == 10
    assert oracle.max_blocks(100.0, 1.0, 2, 10.0, 4.1) == 9
    assert oracle.max_blocks(10.0, 1.0, 2, 10.0, 4.0) == 0


@pytest.mark.parametrize("gran", [0, 1])
def test_grow_clears_stale_bits_of_the_new_ids_and_moves_nothing(gran):
    """Sec. 5.1: expansion appends newly allocated blocks to the block list.  The ids in [B, B_new) start
    out neither live nor dirty whatever their bits held before (an earlier shrink leaves them behind);
    ids below B, tables and every byte of the pool stay as they are; remap is the identity on live ids."""
    bs, B, cap, B_new = 4, 10, 24, 19
    kv = oracle.HostKV(2, 2, 1, 8, bs, B, capacity_blocks=cap, arenas=3, dirty_gran=gran)
    _fill_blocks(kv, seed=3)
    before = _snapshot(kv)
    live = [0, 3, 4, 9]
    kv.set_live(live)
    upb = bs if gran else 1
    # stale bits: live bits at ids 10, 13, 18 (to be cleared), 19 and 23 (beyond B_new: not the call's business)
    for b in (10, 13, 18, 19, 23):
        kv.live[b >> 3] |= 1 << (b & 7)
    stale_dirty = [10 * upb, 13 * upb + upb - 1, 18 * upb + upb - 1, 19 * upb, 23 * upb + upb - 1]
    for u in stale_dirty:
        kv.dirty[u >> 3] |= 1 << (u & 7)
    table = np.array([[0, 3, 9], [4, pin.TABLE_FILL, pin.TABLE_FILL]], dtype=np.int32)
    used = np.array([3, 1], dtype=np.int32)
    t0 = table.copy()
    rc, remap, res = kv.resize(B_new, [table], [used])
    assert rc == oracle.OK and kv.num_blocks == B_new
    assert res.tolist() == [4, 0, B, B_new]
    assert kv.live_ids().tolist() == live                      # ids [B, B_new) are not live
    all_live = np.nonzero(np.unpackbits(kv.live, bitorder="little")[:cap])[0].tolist()
    assert all_live == live + [19, 23]                         # bits at ids >= B_new were not touched
    all_dirty = np.nonzero(np.unpackbits(kv.dirty, bitorder="little")[:cap * upb])[0].tolist()
    assert all_dirty == [19 * upb, 23 * upb + upb - 1]         # dirty bits of the new ids are gone, too
    assert np.array_equal(table, t0)
    assert remap[:B].tolist() == [b if b in live else -1 for b in range(B)]
    for l in range(2):
        for b in range(cap):
            assert np.array_equal(kv.block(l, b), before[l][b])
    # a grow is refused while a dirty bit below B is pending, and then changes nothing
    kv2 = oracle.HostKV(1, 2, 1, 8, bs, B, capacity_blocks=cap, dirty_gran=gran)
    kv2.set_live(live)
    kv2.live[13 >> 3] |= 1 << (13 & 7)
    assert kv2.mark_dirty([3 * upb], 1) == oracle.OK
    rc, _, _ = kv2.resize(B_new, [], [])
    assert rc == oracle.E_BUSY and kv2.num_blocks == B
    assert (kv2.live[13 >> 3] >> (13 & 7)) & 1
