"""GPU parity of the write side (KV append + dirty marking) and of
slot-granular patches against the oracle: every byte of pool, bitmap, patch."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import MAX_ABS, REL_L2, assert_pools_equal, attn_errors, bitmap_ids

pytestmark = pytest.mark.gpu


def _bits(rng, shape):
    return pin.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def _pair(gran, L, Hq, Hkv, D, bs, B, arenas=3):
    host = oracle.HostKV(L, Hq, Hkv, D, bs, B, dirty_gran=gran, fill_bits=pin.BF16_NAN, arenas=arenas)
    dev = P.KVRegion(L, Hq, Hkv, D, bs, B, dirty_granularity=gran, fill_bits=pin.BF16_NAN, arenas=arenas + 1)
    return host, dev


def _dev16(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)


def _cmp_patch(host, patch_h, patch_d, n_layers):
    h = oracle.parse_patch_header(patch_h)
    g = patch_d.cpu().numpy()
    assert np.array_equal(g[:64], patch_h[:64])
    n = h["n_blocks"]
    assert np.array_equal(g[64:64 + 4 * n], patch_h[64:64 + 4 * n])
    end = h["payload_offset"] + n * n_layers * host.unit_bytes
    assert np.array_equal(g[h["payload_offset"]:end], patch_h[h["payload_offset"]:end])
    return h


@pytest.mark.parametrize("gran", [0, 1])
@pytest.mark.parametrize("shape", [(4, 2, 64, 16), (32, 8, 128, 16), (16, 8, 128, 32), (16, 8, 128, 128),
                                   (4, 2, 64, 64)])
def test_append_then_decode_and_patch(gran, shape):
    Hq, Hkv, D, bs = shape
    rng = np.random.default_rng(17)
    L, S, B = 3, 5, 40
    host, dev = _pair(gran, L, Hq, Hkv, D, bs, B)
    perm = rng.permutation(B)[: S * 6].reshape(S, 6).astype(np.int32)
    table_d = torch.from_numpy(perm).cuda()
    lens0 = np.array([0, 3, bs - 1, bs, 2 * bs + 5], dtype=np.int32)
    lens = np.zeros(S, dtype=np.int32)
    host.set_live(np.sort(perm.reshape(-1)))
    dev.set_live(np.sort(perm.reshape(-1)))
    steps = int(lens0.max()) + 2 * bs + 3
    for t in range(steps):
        pos = lens.copy()
        pos[lens0 > t] = lens[lens0 > t]                       # the first steps fill the ragged starts
        pos[(lens0 <= t) & (t < int(lens0.max()))] = -1        # ... while the other sequences wait
        if t % 5 == 4:
            pos[1] = -1                                        # a sequence that skips this step
        for layer in range(L):
            k, v = _bits(rng, (S, Hkv, D)), _bits(rng, (S, Hkv, D))
            assert host.append(layer, k, v, perm, pos, mark=True, count_tokens=(layer == 0)) == oracle.OK
            P.pipelive_kv_append(dev, layer, _dev16(k), _dev16(v), table_d, torch.from_numpy(pos).cuda(),
                                 mark=True, count_tokens=(layer == 0))
        lens = lens + (pos >= 0)
    units = B * (bs if gran else 1)
    assert np.array_equal(bitmap_ids(dev.dirty, units), host.dirty_ids())
    assert P.pipelive_kv_read_state(dev).n_acc == host.n_acc > 0
    assert P.pipelive_kv_read_state(dev).status == 0
    assert_pools_equal(host, dev, range(L), range(B))
    # decode over what was appended
    for layer in (0, L - 1):
        q = _bits(rng, (S, Hq, D))
        out = torch.full((S, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
        P.pipelive_paged_attn_decode(dev, layer, _dev16(q), out, table_d, torch.from_numpy(lens).cuda())
        ref = host.attn_decode(layer, q, perm, lens)
        ma, rl = attn_errors(out.cpu().numpy(), ref)
        assert ma <= MAX_ABS and rl <= REL_L2, (ma, rl)
    # drain in clipped patches into a second region through a block map
    tgt_h, tgt_d = _pair(gran, 2, Hq, Hkv, D, bs, B + 7, arenas=2)
    dmap = (np.arange(B, dtype=np.int32)[::-1] + 7).copy()
    dmap_d = torch.from_numpy(dmap).cuda()
    n_dirty = len(host.dirty_ids())
    per_patch = max(3, n_dirty // 3)
    cap = 64 + 256 + per_patch * (4 + 2 * host.unit_bytes) + 50
    patch_h = np.zeros(cap, dtype=np.uint8)
    patch_d = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    assert P.pipelive_patch_max_blocks(dev, 2, cap) == per_patch == host.patch_max_blocks(2, cap)
    drains = 0
    while True:
        assert host.patch_collect([2, 0], patch_h) == oracle.OK
        P.pipelive_kv_patch_collect(dev, [2, 0], patch_d)
        h = _cmp_patch(host, patch_h, patch_d, 2)
        assert h["unit_tokens"] == (1 if gran else bs)
        assert np.array_equal(bitmap_ids(dev.dirty, units), host.dirty_ids())
        assert tgt_h.patch_apply([0, 1], patch_h, dmap) == oracle.OK
        P.pipelive_kv_patch_apply(tgt_d, [0, 1], patch_d, dst_block_map=dmap_d)
        drains += 1
        if not h["more_pending"]:
            break
    assert drains >= 3
    assert_pools_equal(tgt_h, tgt_d, range(2), range(B + 7))
    st = P.pipelive_kv_read_state(tgt_d)
    assert st.t_applied == tgt_h.t_applied > 0 and st.status == 0


def test_slot_mode_resize_busy_grow_and_errors():
    host, dev = _pair(1, 2, 4, 2, 64, 16, 20)
    host.c.num_blocks = 20
    k = _bits(np.random.default_rng(1), (1, 2, 64))
    table = np.array([[3, 19]], dtype=np.int32)
    table_d = torch.from_numpy(table).cuda()
    host.set_live([3, 19]); dev.set_live([3, 19])
    used = torch.tensor([2], dtype=torch.int32, device="cuda")
    pos = np.array([17], dtype=np.int32)
    assert host.append(0, k, k, table, pos) == oracle.OK
    P.pipelive_kv_append(dev, 0, _dev16(k), _dev16(k), table_d, torch.from_numpy(pos).cuda())
    assert bitmap_ids(dev.dirty, 320).tolist() == [19 * 16 + 1] == host.dirty_ids().tolist()
    rc, res = P.pipelive_kv_resize(dev, 10, [table_d], [used])
    assert rc == P.E_BUSY                                       # a pending slot blocks the shrink
    patch = torch.zeros(64 + 256 + 4 * (4 + dev.unit_bytes), dtype=torch.uint8, device="cuda")
    P.pipelive_kv_patch_collect(dev, [0], patch)
    rc, res = P.pipelive_kv_resize(dev, 10, [table_d], [used])
    assert rc == P.OK and res.n_moved == 1 and table_d.cpu().numpy().tolist() == [[3, 0]]
    # marks at slot ids of the shrunken pool; ids beyond it are flagged, not written
    P.pipelive_kv_mark_dirty(dev, torch.tensor([159, 160], dtype=torch.int32, device="cuda"), 0)
    assert bitmap_ids(dev.dirty, 320).tolist() == [159]
    assert P.pipelive_kv_read_state(dev).status == P.E_RANGE
    P.pipelive_kv_clear_status(dev)
    P.pipelive_kv_patch_collect(dev, [0], patch)
    # grow: the new ids' slots are not dirty even if stale bits were there
    dev.dirty[20:40] = 0xFF                                     # slots of blocks 10..19 (stale garbage)
    rc, res = P.pipelive_kv_resize(dev, 20, [table_d], [used])
    assert rc == P.OK and len(bitmap_ids(dev.dirty, 320)) == 0
    # append error paths: bad block id, position beyond the table row
    bad = torch.tensor([[25, 1]], dtype=torch.int32, device="cuda")
    P.pipelive_kv_append(dev, 0, _dev16(k), _dev16(k), bad, torch.tensor([0], dtype=torch.int32, device="cuda"))
    assert P.pipelive_kv_read_state(dev).status == P.E_RANGE
    P.pipelive_kv_clear_status(dev)
    P.pipelive_kv_append(dev, 0, _dev16(k), _dev16(k), table_d, torch.tensor([32], dtype=torch.int32, device="cuda"))
    assert P.pipelive_kv_read_state(dev).status == P.E_INVAL
    assert len(bitmap_ids(dev.dirty, 320)) == 0
    # a slot patch is refused by a block-granular target
    blk_tgt = P.KVRegion(2, 4, 2, 64, 16, 20, fill_bits=pin.BF16_NAN)
    P.pipelive_kv_mark_dirty(dev, torch.tensor([5], dtype=torch.int32, device="cuda"), 0)
    P.pipelive_kv_patch_collect(dev, [0], patch)
    P.pipelive_kv_patch_apply(blk_tgt, [0], patch)
    assert P.pipelive_kv_read_state(blk_tgt).status == P.E_INVAL


def test_large_slot_bitmap_uses_the_multi_kernel_drain():
    """320 000 slot bits (5 000 words): ids, clipping, put-back and counters must
    equal the oracle's single sweep."""
    rng = np.random.default_rng(77)
    B, bs = 20000, 16
    host, dev = _pair(1, 1, 1, 1, 64, bs, B, arenas=2)
    units = B * bs
    marks = np.unique(rng.integers(0, units, 6000)).astype(np.int32)
    marks = np.concatenate([marks, [0, 63, 64, units - 1]]).astype(np.int32)
    # give the marked slots' blocks recognisable content on both sides
    blocks = np.unique(marks // bs)
    data = rng.integers(0, 30000, (len(blocks), host.blk_elems), dtype=np.uint16)
    for b, row in zip(blocks, data):
        host.block(0, int(b))[:] = row
    dev.write_blocks(0, blocks, torch.from_numpy(data.view(np.int16)).cuda())
    assert host.mark_dirty(marks, 123) == oracle.OK
    P.pipelive_kv_mark_dirty(dev, torch.from_numpy(marks).cuda(), 123)
    cap = 64 + 256 + 2500 * (4 + host.unit_bytes)
    patch_h = np.zeros(cap, dtype=np.uint8)
    patch_d = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    drains, seen = 0, []
    while True:
        assert host.patch_collect([0], patch_h) == oracle.OK
        P.pipelive_kv_patch_collect(dev, [0], patch_d)
        h = _cmp_patch(host, patch_h, patch_d, 1)
        assert np.array_equal(bitmap_ids(dev.dirty, units), host.dirty_ids())
        assert P.pipelive_kv_read_state(dev).n_acc == host.n_acc
        seen += np.frombuffer(patch_h[64:64 + 4 * h["n_blocks"]].tobytes(), dtype=np.int32).tolist()
        drains += 1
        if not h["more_pending"]:
            break
    assert drains == 3 and seen == sorted(set(marks.tolist()))
