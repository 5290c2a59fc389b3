"""Pins for the oracle's write side (KV append + dirty marking) and for
slot-granular patches (paper Sec. 6.1: one dirty bit per token slot; the
patch carries the KV of the dirty slots)."""
import numpy as np
import pytest

import oracle
import pipelive_inputs as pin
from helpers import dense_attention, gather_logical, unpack_block


def _bits(rng, shape):
    return pin.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def _region(gran, layout=0, L=2, B=24, bs=16, Hq=4, Hkv=2, D=64):
    return oracle.HostKV(L, Hq, Hkv, D, bs, B, layout=layout, dirty_gran=gran, fill_bits=pin.BF16_NAN)


@pytest.mark.parametrize("bs", [16, 64])
@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("gran", [0, 1])
def test_append_builds_the_same_cache_as_dense_placement(layout, gran, bs):
    rng = np.random.default_rng(3)
    kv = _region(gran, layout, bs=bs)
    S, steps = 3, 37
    table = np.array([[5, 9, 2, 14], [7, 0, 11, 15], [3, 4, 8, 16]], dtype=np.int32)
    start = np.array([0, 10, 16], dtype=np.int32)        # sequences 1, 2 already hold tokens (NaN here)
    dense_k = [[] for _ in range(S)]
    dense_v = [[] for _ in range(S)]
    expect_dirty = set()
    for t in range(steps):
        pos = start + t
        pos[1] = pos[1] if t < 20 else -1                 # sequence 1 stops after 20 tokens
        for layer in range(2):
            k, v = _bits(rng, (S, kv.Hkv, kv.D)), _bits(rng, (S, kv.Hkv, kv.D))
            assert kv.append(layer, k, v, table, pos, mark=True, count_tokens=(layer == 0)) == oracle.OK
            if layer == 1:
                for s in range(S):
                    if pos[s] >= 0:
                        dense_k[s].append(k[s]); dense_v[s].append(v[s])
        for s in range(S):
            if pos[s] >= 0:
                b = int(table[s, pos[s] // kv.bs])
                expect_dirty.add(b * kv.bs + pos[s] % kv.bs if gran else b)
    assert kv.n_acc == steps * 2 + 20                     # counted once per step, not per layer
    assert set(kv.dirty_ids().tolist()) == expect_dirty
    for s in range(S):
        n_total = int(start[s]) + len(dense_k[s])
        k_all, v_all = gather_logical(kv, 1, table[s], n_total)
        assert np.array_equal(k_all[start[s]:], np.stack(dense_k[s]))
        assert np.array_equal(v_all[start[s]:], np.stack(dense_v[s]))
        assert (k_all[:start[s]] == pin.BF16_NAN).all()    # earlier slots untouched
    # attention over the appended tokens of sequence 0 equals dense attention
    q = _bits(rng, (S, kv.Hq, kv.D))
    out = kv.attn_decode(1, q, table, np.array([steps, 0, 0], dtype=np.int32))
    ref = dense_attention(q[0], np.stack(dense_k[0]), np.stack(dense_v[0]), kv.Hq // kv.Hkv)
    assert np.abs(out[0] - ref).max() < 2e-6


def test_append_errors_leave_state_untouched():
    kv = _region(1)
    k = np.zeros((1, kv.Hkv, kv.D), dtype=np.uint16)
    table = np.array([[24]], dtype=np.int32)
    assert kv.append(0, k, k, table, [3]) == oracle.E_RANGE
    assert kv.append(0, k, k, np.array([[1]], dtype=np.int32), [16]) == oracle.E_INVAL   # beyond the table row
    assert len(kv.dirty_ids()) == 0 and kv.n_acc == 0


@pytest.mark.parametrize("layout", [0, 1])
def test_slot_patch_payload_and_apply(layout):
    rng = np.random.default_rng(9)
    src = _region(1, layout, L=3)
    dst = _region(1, layout, L=2, B=30)
    for l in range(3):
        for b in range(24):
            src.block(l, b)[:] = rng.integers(0, 30000, src.blk_elems, dtype=np.uint16)
    before = [[dst.block(l, b).copy() for b in range(30)] for l in range(2)]
    slots = [5 * 16 + 3, 5 * 16 + 4, 0, 23 * 16 + 15, 7 * 16 + 9]
    assert src.mark_dirty(slots + [5 * 16 + 3], 6) == oracle.OK
    cap = 64 + 256 + 8 * (4 + 2 * src.unit_bytes)
    patch = np.zeros(cap, dtype=np.uint8)
    assert src.patch_max_blocks(2, cap) == 8
    assert src.patch_collect([2, 0], patch) == oracle.OK
    h = oracle.parse_patch_header(patch)
    tok_bytes = 2 * src.Hkv * src.D * 2
    assert h["unit_tokens"] == 1 and h["block_bytes"] == tok_bytes and h["n_blocks"] == 5 and h["n_acc_tokens"] == 6
    ids = np.frombuffer(patch[64:64 + 20].tobytes(), dtype=np.int32)
    assert ids.tolist() == sorted(set(slots))
    pay = patch[h["payload_offset"]:].view(np.uint16)
    for r, u in enumerate(ids):
        for i, l in enumerate([2, 0]):
            k_tok, v_tok = unpack_block(layout, src.block(l, u // 16), 16, src.Hkv, src.D)
            o = (r * 2 + i) * (tok_bytes // 2)
            assert np.array_equal(pay[o:o + src.Hkv * src.D], k_tok[u % 16].reshape(-1))
            assert np.array_equal(pay[o + src.Hkv * src.D:o + 2 * src.Hkv * src.D], v_tok[u % 16].reshape(-1))
    dmap = (np.arange(24, dtype=np.int32) + 6)           # block b -> b + 6 in the target
    assert dst.patch_apply([1, 0], patch, dmap) == oracle.OK
    assert dst.patch_apply([1, 0], patch, dmap) == oracle.OK          # idempotent
    assert dst.t_applied == 12
    touched = {}
    for u in ids:
        touched.setdefault(int(u) // 16 + 6, []).append(int(u) % 16)
    for l, sl in [(1, 2), (0, 0)]:
        for b in range(30):
            kd, vd = unpack_block(layout, dst.block(l, b), 16, dst.Hkv, dst.D)
            kb, vb = unpack_block(layout, before[l][b], 16, dst.Hkv, dst.D)
            for t in range(16):
                if b in touched and t in touched[b]:
                    ks, vs = unpack_block(layout, src.block(sl, b - 6), 16, src.Hkv, src.D)
                    assert np.array_equal(kd[t], ks[t]) and np.array_equal(vd[t], vs[t])
                else:
                    assert np.array_equal(kd[t], kb[t]) and np.array_equal(vd[t], vb[t])
    # granularity mismatch between patch and target is refused
    blockwise = _region(0, layout, L=2, B=30)
    assert blockwise.patch_apply([1, 0], patch, dmap) == oracle.E_INVAL


def test_slot_session_converges_and_resize_sees_pending_slots():
    """Decode appends under slot-granular tracking: after the final drain the
    target holds every token of the source, and a pending slot blocks resize."""
    rng = np.random.default_rng(21)
    L, S, bs = 2, 4, 16
    src = _region(1, L=L, B=32)
    dst = _region(1, L=L, B=32)
    table = np.arange(32, dtype=np.int32).reshape(S, 8)
    lens = np.array([30, 5, 64, 17], dtype=np.int32)
    # prefill content + round 0: every slot that holds a token is marked
    for l in range(L):
        for s in range(S):
            for j in range(lens[s]):
                pos = np.full(S, -1, dtype=np.int32); pos[s] = j
                k, v = _bits(rng, (S, src.Hkv, src.D)), _bits(rng, (S, src.Hkv, src.D))
                src.append(l, k, v, table, pos, mark=(l == 0), count_tokens=False)
    assert len(src.dirty_ids()) == int(lens.sum())
    cap = 64 + 256 + 40 * (4 + L * src.unit_bytes)          # 40 slots per patch: round 0 needs several drains
    patch = np.zeros(cap, dtype=np.uint8)
    sched = 0
    for rnd in range(6):
        if rnd:
            for l in range(L):
                k, v = _bits(rng, (S, src.Hkv, src.D)), _bits(rng, (S, src.Hkv, src.D))
                src.append(l, k, v, table, lens, mark=True, count_tokens=(l == 0))
            lens = lens + 1
            sched += S
            rc, _, _ = src.resize(32, [], [])
            assert rc == oracle.E_BUSY                        # pending slots block a resize
        while True:
            assert src.patch_collect([0, 1], patch) == oracle.OK
            assert dst.patch_apply([0, 1], patch) == oracle.OK
            if not oracle.parse_patch_header(patch)["more_pending"]:
                break
    assert dst.t_applied == sched == S * 5 and len(src.dirty_ids()) == 0
    for l in range(L):
        for s in range(S):
            ks, vs = gather_logical(src, l, table[s], int(lens[s]))
            kd, vd = gather_logical(dst, l, table[s], int(lens[s]))
            assert np.array_equal(ks, kd) and np.array_equal(vs, vd)
    assert (dst.block(0, 31) == pin.BF16_NAN).any()          # slots never written stay untouched


@pytest.mark.parametrize("bs", [16, 32, 64])
@pytest.mark.parametrize("gran", [0, 1])
def test_chunk_append_equals_token_by_token_append(gran, bs):
    """A prefill chunk lands exactly where the same tokens appended one at a time would (the single-token
    append is pinned against dense placement above); the dirty set and n_acc agree as well."""
    rng = np.random.default_rng(9)
    a, b = _region(gran, 0, B=40, bs=bs), _region(gran, 0, B=40, bs=bs)
    S = 4
    table = rng.permutation(40)[: S * 8].reshape(S, 8).astype(np.int32)
    ctx = np.array([37, 5, 0, 3 * bs], dtype=np.int32)        # context lengths including the chunk
    qlen = np.array([20, 5, 0, bs + 1], dtype=np.int32)       # unaligned start, whole context, nothing, block + 1
    qo = np.concatenate([[0], np.cumsum(qlen)]).astype(np.int32)
    for layer in range(2):
        k, v = _bits(rng, (int(qo[-1]), a.Hkv, a.D)), _bits(rng, (int(qo[-1]), a.Hkv, a.D))
        assert a.append_chunk(layer, k, v, table, ctx, qo, mark=True, count_tokens=(layer == 0)) == oracle.OK
        for i in range(int(qlen.max())):
            pos = np.where(i < qlen, ctx - qlen + i, -1).astype(np.int32)
            rows = np.minimum(qo[:-1] + i, int(qo[-1]) - 1)
            assert b.append(layer, k[rows], v[rows], table, pos, mark=True, count_tokens=(layer == 0)) == oracle.OK
    assert a.n_acc == b.n_acc == int(qlen.sum())
    assert np.array_equal(a.dirty, b.dirty) and len(a.dirty_ids()) > 0
    for layer in range(2):
        for blk in range(40):
            assert np.array_equal(a.block(layer, blk), b.block(layer, blk)), (layer, blk)


def test_chunk_append_errors_leave_state_untouched():
    kv = _region(1, 0, B=8)
    rng = np.random.default_rng(1)
    before = [kv.block(0, b).copy() for b in range(8)]
    k, v = _bits(rng, (6, kv.Hkv, kv.D)), _bits(rng, (6, kv.Hkv, kv.D))
    table = np.array([[1, 2, 3]], dtype=np.int32)
    qo = np.array([0, 6], dtype=np.int32)
    assert kv.append_chunk(0, k, v, table, np.array([5], np.int32), qo) == oracle.E_INVAL       # chunk longer than context
    assert kv.append_chunk(0, k, v, table, np.array([50], np.int32), qo) == oracle.E_INVAL      # beyond the table row
    assert kv.append_chunk(0, k, v, np.array([[1, 9, 3]], np.int32), np.array([20], np.int32), qo) == oracle.E_RANGE
    assert kv.n_acc == 0 and len(kv.dirty_ids()) == 0
    for b in range(8):
        assert np.array_equal(kv.block(0, b), before[b])
