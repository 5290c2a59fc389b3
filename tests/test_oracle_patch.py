"""Pins for the oracle's dirty bitmap / KV patch cycle (CPU only).

Paper Sec. 6.1 "KV Migration with KV Patch": bitmap starts at zero, written
slots are marked, the sender atomically drains the dirty set, gathers the KV
there into a patch, the receiver writes it; counters T_sched / T_applied with
the n_acc correction."""
import numpy as np

import oracle
import pipelive_inputs as pin


def _region(B=40, L=3, seed=0, layout=0, stack_k=1):
    kv = oracle.HostKV(L, 4, 2, 64, 16, B, layout=layout, stack_k=stack_k)
    rng = np.random.default_rng(seed)
    for l in range(L):
        for b in range(B):
            kv.block(l, b)[:] = rng.integers(0, 65536, kv.blk_elems, dtype=np.uint16)
    return kv


def _patch_buf(kv, n_layers, n_blocks):
    cap = 64 + 256 + n_blocks * (4 + n_layers * kv.blk_bytes)
    return np.full(cap, 0xEE, dtype=np.uint8)


def test_collect_header_ids_payload():
    kv = _region()
    ids = [17, 3, 3, 39, 0]
    assert kv.mark_dirty(ids, 5) == oracle.OK
    layers = [2, 0]
    patch = _patch_buf(kv, 2, 40)
    assert kv.patch_collect(layers, patch) == oracle.OK
    h = oracle.parse_patch_header(patch)
    assert h["magic"] == oracle.PATCH_MAGIC and patch[:4].tobytes() == b"PLKV"
    assert h["n_blocks"] == 4 == len(set(ids))          # popcount, de-duplicated
    assert h["n_layers"] == 2 and h["block_bytes"] == kv.blk_bytes
    assert h["n_acc_tokens"] == 5 and h["more_pending"] == 0
    assert h["max_blocks"] == 40 and h["payload_offset"] == 256
    got = np.frombuffer(patch[64:64 + 16].tobytes(), dtype=np.int32)
    assert got.tolist() == [0, 3, 17, 39]               # strictly ascending
    assert len(kv.dirty_ids()) == 0 and kv.n_acc == 0   # bitmap empty after an unclipped drain
    pay = patch[h["payload_offset"]:].view(np.uint16)
    for r, b in enumerate(got):
        for i, l in enumerate(layers):
            o = (r * 2 + i) * kv.blk_elems
            assert np.array_equal(pay[o:o + kv.blk_elems], kv.block(l, int(b)))


def test_apply_is_idempotent_and_targets_mapped_blocks():
    src = _region(seed=1)
    dst = _region(seed=2, L=4)
    before = [[dst.block(l, b).copy() for b in range(40)] for l in range(4)]
    src.mark_dirty([5, 6, 30], 3)
    patch = _patch_buf(src, 2, 8)
    assert src.patch_collect([0, 2], patch) == oracle.OK
    dmap = np.arange(40, dtype=np.int32)[::-1].copy()    # id b -> 39 - b
    assert dst.patch_apply([3, 1], patch, dmap) == oracle.OK
    snap = [[dst.block(l, b).copy() for b in range(40)] for l in range(4)]
    assert dst.patch_apply([3, 1], patch, dmap) == oracle.OK
    for l in range(4):
        for b in range(40):
            assert np.array_equal(dst.block(l, b), snap[l][b])
            src_b = 39 - b
            if src_b in (5, 6, 30) and l in (3, 1):
                assert np.array_equal(dst.block(l, b), src.block({3: 0, 1: 2}[l], src_b))
            else:
                assert np.array_equal(dst.block(l, b), before[l][b])
    assert dst.t_applied == 6                            # n_acc counted per applied patch


def test_clipped_drain_takes_lowest_ids_and_keeps_n_acc():
    kv = _region()
    marks = [31, 2, 9, 25, 14]
    kv.mark_dirty(marks, 11)
    patch = _patch_buf(kv, 3, 2)                          # room for 2 blocks only
    assert kv.patch_max_blocks(3, patch.nbytes) == 2
    seen = []
    total_acc = 0
    rounds = 0
    while True:
        assert kv.patch_collect([0, 1, 2], patch) == oracle.OK
        h = oracle.parse_patch_header(patch)
        ids = np.frombuffer(patch[64:64 + 4 * h["n_blocks"]].tobytes(), dtype=np.int32).tolist()
        seen += ids
        total_acc += h["n_acc_tokens"]
        rounds += 1
        if rounds == 1:
            assert ids == [2, 9] and h["more_pending"] == 1 and h["n_acc_tokens"] == 0
            assert kv.dirty_ids().tolist() == [14, 25, 31] and kv.n_acc == 11
        if not h["more_pending"]:
            break
    assert seen == sorted(marks) and total_acc == 11 and rounds == 3
    assert kv.patch_collect([0, 1, 2], patch) == oracle.OK   # empty drain is a valid patch
    h = oracle.parse_patch_header(patch)
    assert h["n_blocks"] == 0 and h["n_acc_tokens"] == 0


def test_errors():
    kv = _region()
    assert kv.mark_dirty([40], 1) == oracle.E_RANGE
    assert len(kv.dirty_ids()) == 0 and kv.n_acc == 0
    assert kv.patch_collect([3], _patch_buf(kv, 1, 4)) == oracle.E_RANGE
    small = np.zeros(64 + 256 + 3, dtype=np.uint8)
    assert kv.patch_collect([0], small) == oracle.E_NOSPACE
    kv.mark_dirty([1], 1)
    patch = _patch_buf(kv, 1, 4)
    kv.patch_collect([0], patch)
    other = oracle.HostKV(3, 4, 2, 64, 32, 40)             # other block size
    assert other.patch_apply([0], patch) == oracle.E_INVAL
    dst = _region(B=1)
    kv.mark_dirty([7], 1)
    kv.patch_collect([0], patch)
    assert dst.patch_apply([0], patch) == oracle.E_RANGE    # id 7 outside a 1-block target
    bad = patch.copy(); bad[0] ^= 1
    assert dst.patch_apply([0], bad) == oracle.E_INVAL


def test_session_converges_to_bit_identical_target():
    """Round 0 marks every live block (pre-copy), later rounds rewrite a
    sample of blocks; after the last drain the target equals the source on
    every live block of the migrated layers, and marks / tokens are conserved."""
    cfg = pin.CONFIGS["tiny"]
    B = 128
    bt = pin.draw_batch(cfg, pin.MASTER_SEED, num_blocks=B)
    src = oracle.HostKV(cfg.num_layers, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B)
    dst = oracle.HostKV(cfg.num_layers + 1, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B)
    for l in range(cfg.num_layers):
        for b in bt.live_ids:
            src.block(l, b)[:] = pin.kv_block_bits(cfg, 1, B, 0, l, int(b))
    layers, dst_layers = [0, 1], [2, 0]
    patch = _patch_buf(src, 2, len(bt.live_ids))
    all_marks, all_ids, sched, = set(), [], 0
    for rnd in range(4):
        if rnd == 0:
            ids, ntok = bt.live_ids, 0
        else:
            ids = pin.draw_dirty_ids(bt, 1, rnd, 0.10)
            ntok = cfg.num_seqs
            for l in range(cfg.num_layers):
                for b in ids:
                    src.block(l, b)[:] = pin.kv_block_bits(cfg, 1, B, rnd, l, int(b))
        assert src.mark_dirty(ids, ntok) == oracle.OK
        sched += ntok
        all_marks |= set(int(i) for i in ids)
        assert src.patch_collect(layers, patch) == oracle.OK
        h = oracle.parse_patch_header(patch)
        assert h["n_blocks"] == len(ids)
        all_ids += np.frombuffer(patch[64:64 + 4 * h["n_blocks"]].tobytes(), dtype=np.int32).tolist()
        assert dst.patch_apply(dst_layers, patch) == oracle.OK
    assert set(all_ids) | set(src.dirty_ids().tolist()) == all_marks
    assert dst.t_applied == sched and len(src.dirty_ids()) == 0
    for b in bt.live_ids:
        assert np.array_equal(dst.block(2, b), src.block(0, b))
        assert np.array_equal(dst.block(0, b), src.block(1, b))
    free = sorted(set(range(B)) - set(bt.live_ids.tolist()))
    assert (dst.block(2, free[0]) == 0xFFFF).all() and (dst.block(1, int(bt.live_ids[0])) == 0xFFFF).all()


def test_stacked_layers_patch():
    src = _region(L=4, stack_k=2, seed=4)
    dst = _region(L=4, stack_k=2, seed=5)
    keep = dst.block(2, 9).copy()
    src.mark_dirty([9], 1)
    patch = _patch_buf(src, 1, 2)
    assert src.patch_collect([3], patch) == oracle.OK
    assert dst.patch_apply([3], patch) == oracle.OK
    assert np.array_equal(dst.block(3, 9), src.block(3, 9))
    assert np.array_equal(dst.block(2, 9), keep)          # the sibling layer in the same physical block is untouched
