"""GPU tests of the boundary's promises about foreign patches, counters and
writers that race a drain (Sec. 6.1: the patch comes from another sender; the
sender drains while inference keeps writing)."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import assert_pools_equal, bitmap_ids

pytestmark = pytest.mark.gpu


def _pair(gran, L, Hq, Hkv, D, bs, B, fill=0x3C00, arenas=3):
    host = oracle.HostKV(L, Hq, Hkv, D, bs, B, dirty_gran=gran, fill_bits=fill, arenas=arenas)
    dev = P.KVRegion(L, Hq, Hkv, D, bs, B, dirty_granularity=gran, fill_bits=fill, arenas=arenas + 1)
    return host, dev


def _fill_random(host, dev, L, ids, seed):
    rng = np.random.default_rng(seed)
    for l in range(L):
        data = rng.integers(0, 30000, (len(ids), host.blk_elems), dtype=np.uint16)
        for b, row in zip(ids, data):
            host.block(l, int(b))[:] = row
        dev.write_blocks(l, ids, torch.from_numpy(data.view(np.int16)).cuda())


@pytest.mark.parametrize("gran", [0, 1])
def test_apply_checks_a_foreign_patch_and_refuses_it_as_a_whole(gran):
    """Every refusal leaves the target's bytes and T_applied untouched and agrees with the oracle's verdict;
    the same patch, intact and with a map that covers it, is applied like the oracle applies it."""
    L, Hq, Hkv, D, bs, B = 2, 4, 2, 64, 16, 16
    src_h, src_d = _pair(gran, L, Hq, Hkv, D, bs, B)
    ids = np.array([1, 4, 9, 15], dtype=np.int64)
    _fill_random(src_h, src_d, L, ids, 5)
    units = ids if not gran else np.array([1 * bs + 3, 4 * bs, 9 * bs + 15, 15 * bs + 7], dtype=np.int64)
    layers = [0, 1]
    cap = 64 + 256 + 8 * (4 + L * src_h.unit_bytes)
    patch_h = np.zeros(cap, dtype=np.uint8)
    patch_d = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    assert src_h.mark_dirty(units, 11) == oracle.OK
    P.pipelive_kv_mark_dirty(src_d, torch.from_numpy(units.astype(np.int32)).cuda(), 11)
    assert src_h.patch_collect(layers, patch_h) == oracle.OK
    P.pipelive_kv_patch_collect(src_d, layers, patch_d)
    torch.cuda.synchronize()
    assert np.array_equal(patch_d.cpu().numpy()[:64], patch_h[:64])

    def targets():
        th, td = _pair(gran, L, Hq, Hkv, D, bs, 8, fill=0x1234, arenas=2)
        return th, td

    def untouched(td):
        for l in range(L):
            assert (td.read_blocks(l, range(8)).cpu().numpy().view(np.uint16) == 0x1234).all()
        assert P.pipelive_kv_tokens_applied(td) == 0

    full_map = np.full(B, -1, dtype=np.int32)
    full_map[ids] = [0, 3, 5, 7]
    # (1) the map is shorter than the ids the patch names: id 9 and 15 lie beyond it
    th, td = targets()
    short = torch.from_numpy(full_map[:8].copy()).cuda()
    P.pipelive_kv_patch_apply(td, layers, patch_d, dst_block_map=short)
    assert P.pipelive_kv_read_state(td).status == P.E_RANGE
    untouched(td)
    assert th.patch_apply(layers, patch_h, dst_map=np.where(np.arange(B) < 8, full_map, -1)) == oracle.E_RANGE
    # (2) one id that the map sends nowhere among three good ones: nothing at all is written
    th, td = targets()
    holed = full_map.copy()
    holed[9] = -1
    P.pipelive_kv_patch_apply(td, layers, patch_d, dst_block_map=torch.from_numpy(holed).cuda())
    assert P.pipelive_kv_read_state(td).status == P.E_RANGE
    untouched(td)
    assert th.patch_apply(layers, patch_h, dst_map=holed) == oracle.E_RANGE and th.t_applied == 0
    # (3) without a map the ids must exist in the target (8 blocks)
    th, td = targets()
    P.pipelive_kv_patch_apply(td, layers, patch_d)
    assert P.pipelive_kv_read_state(td).status == P.E_RANGE
    untouched(td)
    # (4) a truncated buffer: the payload would end beyond what the caller says may be read
    th, td = targets()
    h = oracle.parse_patch_header(patch_h)
    end = h["payload_offset"] + h["n_blocks"] * L * src_h.unit_bytes
    cut = (end - 256) // 256 * 256
    P.pipelive_kv_patch_apply(td, layers, patch_d[:cut], dst_block_map=torch.from_numpy(full_map).cuda())
    assert P.pipelive_kv_read_state(td).status == P.E_INVAL
    untouched(td)
    # (5) corrupt headers: more ids than the list holds; a payload offset that does not follow the list
    for field, value in (("n_blocks", 9), ("payload_offset", h["payload_offset"] + 256), ("max_blocks", 2 ** 31)):
        th, td = targets()
        bad = patch_d.clone()
        hb = bytearray(patch_h[:64].tobytes())
        off, size = {"n_blocks": (8, 4), "payload_offset": (32, 8), "max_blocks": (40, 4)}[field]
        hb[off:off + size] = int(value).to_bytes(size, "little")
        bad[:64] = torch.frombuffer(hb, dtype=torch.uint8).cuda()
        P.pipelive_kv_patch_apply(td, layers, bad, dst_block_map=torch.from_numpy(full_map).cuda())
        assert P.pipelive_kv_read_state(td).status == P.E_INVAL, field
        untouched(td)
    # (6) intact patch, full map: every byte of the target and the counter as the oracle's
    th, td = targets()
    assert th.patch_apply(layers, patch_h, dst_map=full_map) == oracle.OK
    P.pipelive_kv_patch_apply(td, layers, patch_d, dst_block_map=torch.from_numpy(full_map).cuda())
    st = P.pipelive_kv_read_state(td)
    assert st.status == 0 and st.t_applied == 11 == th.t_applied
    assert P.pipelive_kv_tokens_applied(td) == 11
    assert_pools_equal(th, td, range(L), range(8))


@pytest.mark.parametrize("big", [False, True])
def test_marks_on_a_second_stream_racing_the_drain(big):
    """Marks (each call: a run of fresh unit ids and as many tokens) are issued on one stream while another
    stream drains again and again.  Whatever the interleaving: every mark ends up in exactly one patch or in
    the residual bitmap, the acknowledged tokens add up, and no patch acknowledges tokens of a mark whose
    units neither it nor an earlier patch carries (writers: bit, then count; drain: count, then bits)."""
    gran = 1 if big else 0
    bs = 16
    B = 20000 if big else 4096           # 320 000 slot bits: the three-kernel drain; 4096 bits: one workgroup
    dev = P.KVRegion(1, 1, 1, 64, bs, B, dirty_granularity=gran, fill_bits=0, arenas=2)
    units = B * (bs if gran else 1)
    calls, width = (120, 512) if big else (150, 16)
    assert calls * width <= units
    perm = np.random.default_rng(3).permutation(units)[: calls * width].astype(np.int32)
    marks = [torch.from_numpy(np.ascontiguousarray(perm[m * width:(m + 1) * width])).cuda() for m in range(calls)]
    max_units = calls * width
    cap = 64 + 256 + max_units * (4 + dev.unit_bytes)
    n_drains = 60
    patch = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    log = torch.zeros((n_drains + 1, 64 + 4 * max_units), dtype=torch.uint8, device="cuda")
    s_mark, s_drain = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    d = 0
    for m in range(calls):
        with torch.cuda.stream(s_mark):
            P.pipelive_kv_mark_dirty(dev, marks[m], width)
        if d < n_drains and m % 2 == 1:
            with torch.cuda.stream(s_drain):
                P.pipelive_kv_patch_collect(dev, [0], patch)
                log[d].copy_(patch[: log.shape[1]])
            d += 1
    torch.cuda.synchronize()
    P.pipelive_kv_patch_collect(dev, [0], patch)      # the flush, alone on the default stream
    log[d].copy_(patch[: log.shape[1]])
    d += 1
    torch.cuda.synchronize()
    assert len(bitmap_ids(dev.dirty, units)) == 0
    st = P.pipelive_kv_read_state(dev)
    assert st.n_acc == 0 and st.status == 0
    owner = {int(u): m for m in range(calls) for u in perm[m * width:(m + 1) * width]}
    carried = np.zeros(calls, dtype=np.int64)         # units of each mark call carried so far
    acked, seen = 0, set()
    logs = log[:d].cpu().numpy()
    for k in range(d):
        h = oracle.parse_patch_header(logs[k])
        assert h["more_pending"] == 0 and h["max_blocks"] == max_units
        ids = np.frombuffer(logs[k, 64:64 + 4 * h["n_blocks"]].tobytes(), dtype=np.int32)
        assert (np.diff(ids) > 0).all()
        for u in ids.tolist():
            assert u in owner and u not in seen       # marked once, collected once
            seen.add(u)
            carried[owner[u]] += 1
        acked += h["n_acc_tokens"]
        assert acked <= width * int((carried == width).sum()), k
    assert seen == set(owner) and acked == calls * width


def test_prefill_flags_a_context_beyond_max_ctx_and_skips_it():
    from test_gpu_prefill import _batch
    cfg = pin.StageConfig("pf", 1, 4, 2, 64, 16, 2, 0, 0)
    batch = _batch(cfg, [40, 24], seed=7)
    dev = P.KVRegion(1, 4, 2, 64, 16, batch.num_blocks, fill_bits=0x3F80)     # every K and V element is 1.0
    dev.set_live(batch.live_ids)
    q = torch.zeros((12, 4, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.full((12, 4, 64), 7.0, dtype=torch.float32, device="cuda")
    t, c = torch.from_numpy(batch.table).cuda(), torch.from_numpy(batch.ctx_lens).cuda()
    qo = torch.tensor([0, 8, 12], dtype=torch.int32, device="cuda")
    P.pipelive_paged_attn_prefill(dev, 0, q, out, t, c, qo, 12, max_ctx=32)     # sequence 0 holds 40 tokens
    torch.cuda.synchronize()
    assert P.pipelive_kv_read_state(dev).status == P.E_RANGE
    got = out.cpu().numpy()
    assert (got[:8] == 7.0).all()                      # its rows are left alone
    assert np.allclose(got[8:], 1.0)                   # the other sequence: every V is 1.0


def test_chunk_append_flags_an_overlong_chunk_of_a_late_sequence():
    S = 70
    dev = P.KVRegion(1, 4, 2, 64, 16, 80, fill_bits=pin.BF16_NAN)
    table = torch.arange(S, dtype=torch.int32, device="cuda").view(S, 1).contiguous()
    qlen = np.ones(S, dtype=np.int32)
    ctx = np.full(S, 3, dtype=np.int32)
    qlen[66] = 5                                       # five new tokens in a context of three
    qo = np.concatenate([[0], np.cumsum(qlen)]).astype(np.int32)
    tq = int(qo[-1])
    k = torch.zeros((tq, 2, 64), dtype=torch.bfloat16, device="cuda")
    P.pipelive_kv_append_chunk(dev, 0, k, k, table, torch.from_numpy(ctx).cuda(), torch.from_numpy(qo).cuda(), tq)
    torch.cuda.synchronize()
    assert P.pipelive_kv_read_state(dev).status == P.E_INVAL
    assert (dev.block(0, 66).cpu().numpy().view(np.uint16) == pin.BF16_NAN).all()     # skipped
    assert (dev.block(0, 65).cpu().numpy().view(np.uint16) == 0).any()                # its neighbours were written
    assert (dev.block(0, 67).cpu().numpy().view(np.uint16) == 0).any()
