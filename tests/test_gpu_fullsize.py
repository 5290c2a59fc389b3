"""GPU parity at the full sizes of the four large workloads, in the launch
configuration bench.py times (balanced shares, split_tokens = 0).

Pools of tens of GB cannot be mirrored on the host, so:
  * attention is checked on a seeded sample of (layer, sequence) pairs whose KV
    the oracle side regenerates with numpy from the counter-based generator
    (never copied from the device);
  * tables, remaps, bitmaps, id lists, counters are compared in full against
    the oracle run on a region of the same B with a tiny block geometry (that
    state does not depend on the block size);
  * pool and patch bytes are compared in full on the device against the
    *input* blocks (payload == source blocks, target == source, content
    follows moved blocks), plus sampled blocks against numpy regeneration.
"""
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
from pipelive_inputs.device_fill import fill_live_blocks
import paper_2604_12171_amd as P
from gpu_common import BF16_MAX_ABS, BF16_REL_L2, MAX_ABS, REL_L2, attn_errors, bitmap_ids

pytestmark = pytest.mark.gpu
SEED = pin.MASTER_SEED


def log(*a):
    print(*a, flush=True)


def _state_oracle(B, capacity=None):
    """Oracle region with the same id space and a tiny block: state only."""
    return oracle.HostKV(1, 1, 1, 8, 16, B, capacity_blocks=capacity or B, arenas=1, fill_bits=0)


def _oracle_pair(cfg, batch, capacity, layer, s, epoch=0):
    """Oracle attention of one (layer, sequence) on numpy-regenerated KV."""
    n, u = int(batch.ctx_lens[s]), int(batch.used[s])
    host = oracle.HostKV(1, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, max(u, 1),
                         layout=cfg.layout, arenas=2, fill_bits=pin.BF16_NAN)
    for j in range(u):
        bits = pin.kv_block_bits(cfg, SEED, capacity, epoch, layer, int(batch.table[s, j]))
        valid = min(cfg.block_tokens, n - j * cfg.block_tokens)
        if valid < cfg.block_tokens:
            bits = bits.copy()
            bits[pin.token_slot_mask(cfg.layout, cfg.num_kv_heads, cfg.block_tokens, cfg.head_dim, valid)] = pin.BF16_NAN
        host.block(0, j)[:] = bits
    tab = np.arange(max(u, 1), dtype=np.int32)[None, :]
    q = pin.q_bits(cfg, SEED, layer)[s:s + 1]
    return host.attn_decode(0, q, tab, np.array([n], dtype=np.int32))[0]


def _oracle_pair_after_appends(cfg, batch0, capacity, layer, s, steps):
    """Oracle attention of one (layer, sequence) after `steps` decode steps: the original tokens are
    regenerated from the ids they were written at (content follows a block through every resize), the
    appended ones come from the new-token generator and are placed by the oracle's own append."""
    n0, u0 = int(batch0.ctx_lens[s]), int(batch0.used[s])
    n = n0 + steps
    u = (n + cfg.block_tokens - 1) // cfg.block_tokens
    host = oracle.HostKV(1, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, u,
                         layout=cfg.layout, arenas=2, fill_bits=pin.BF16_NAN)
    for j in range(u0):
        bits = pin.kv_block_bits(cfg, SEED, capacity, 0, layer, int(batch0.table[s, j]))
        valid = min(cfg.block_tokens, n0 - j * cfg.block_tokens)
        if valid < cfg.block_tokens:
            bits = bits.copy()
            bits[pin.token_slot_mask(cfg.layout, cfg.num_kv_heads, cfg.block_tokens, cfg.head_dim, valid)] = pin.BF16_NAN
        host.block(0, j)[:] = bits
    tab = np.arange(u, dtype=np.int32)[None, :]
    for k in range(steps):
        kk, vv = pin.new_token_bits(cfg, SEED, k, layer)
        assert host.append(0, kk[s:s + 1], vv[s:s + 1], tab, np.array([n0 + k], dtype=np.int32), mark=False) == oracle.OK
    q = pin.q_bits(cfg, SEED, layer)[s:s + 1]
    return host.attn_decode(0, q, tab, np.array([n], dtype=np.int32))[0]


def _sample_pairs(cfg, n_pairs, salt):
    h = pin.hash_u64(pin.stream_key(SEED, pin.STREAM_MISC) ^ salt, np.arange(2 * n_pairs, dtype=np.uint64))
    layers = (h[:n_pairs] % np.uint64(cfg.num_layers)).astype(int)
    seqs = (h[n_pairs:] % np.uint64(cfg.num_seqs)).astype(int)
    return sorted(set(zip(layers.tolist(), seqs.tolist())))


class Stage:
    """Device region + tensors of one workload."""

    def __init__(self, cfg, B, capacity=None, arenas=4, stack_k=1, backing="arena", stride_pad=0, allocator=None):
        self.cfg, self.B = cfg, B
        self.cap = capacity or B
        self.batch = pin.draw_batch(cfg, SEED, num_blocks=B, stride_pad=stride_pad)
        self.region = P.KVRegion(cfg.num_layers, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                                 cfg.block_tokens, B, capacity_blocks=self.cap, arenas=arenas, stack_k=stack_k,
                                 backing=backing, allocator=allocator)
        fill_live_blocks(self.region, cfg, self.batch, SEED, self.cap, poison_tail=True)
        self.table = torch.from_numpy(self.batch.table).cuda()
        self.ctx = torch.from_numpy(self.batch.ctx_lens).cuda()
        self.used = torch.from_numpy(self.batch.used).cuda()
        self.max_ctx = int(self.batch.ctx_lens.max())
        self.ws = self.region.attn_workspace(cfg.num_seqs, self.max_ctx + 64 * stride_pad, 0)

    def decode(self, layer):
        cfg = self.cfg
        q = torch.from_numpy(pin.q_bits(cfg, SEED, layer).view(np.int16)).cuda().view(torch.bfloat16)
        out = torch.full((cfg.num_seqs, cfg.num_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        P.pipelive_paged_attn_decode(self.region, layer, q, out, self.table, self.ctx, max_ctx=self.max_ctx,
                                     workspace=self.ws)
        return out

    def append_step(self, bm, step, count_layer=0, mark=True):
        """One decode step's writes: the block manager hands out the slots (new blocks = lowest free id),
        every layer appends its token.  Returns the positions written."""
        cfg = self.cfg
        pos, new_entries = bm.step()
        for s, col, b in new_entries:
            self.table[s, col] = b
        if new_entries:
            self.region.set_live(bm.live_ids())
            self.used.copy_(torch.from_numpy(bm.used))
        pos_d = torch.from_numpy(pos).cuda()
        for l in range(cfg.num_layers):
            kk, vv = pin.new_token_bits(cfg, SEED, step, l)
            P.pipelive_kv_append(self.region, l, torch.from_numpy(kk.view(np.int16)).cuda().view(torch.bfloat16),
                                 torch.from_numpy(vv.view(np.int16)).cuda().view(torch.bfloat16), self.table, pos_d,
                                 mark=mark, count_tokens=(l == count_layer))
        self.ctx.copy_(torch.from_numpy(bm.ctx))
        self.max_ctx = int(bm.ctx.max())
        return pos, new_entries

    def check_attention(self, n_pairs, salt):
        """GPU vs oracle on sampled (layer, sequence) pairs; returns the GPU outputs per layer.
        Call before any resize: block content is a function of the id it was written at."""
        cfg = self.cfg
        pairs = _sample_pairs(cfg, n_pairs, salt)
        outs = {l: self.decode(l).cpu().numpy() for l in sorted({l for l, _ in pairs})}
        bt = self.batch
        oracle.lib()
        with ThreadPoolExecutor(max_workers=12) as ex:
            refs = list(ex.map(lambda ls: _oracle_pair(cfg, bt, self.cap, ls[0], ls[1]), pairs))
        worst = (0.0, 0.0)
        for (l, s), ref in zip(pairs, refs):
            assert np.isfinite(outs[l][s]).all(), (l, s)
            ma, rl = attn_errors(outs[l][s], ref)
            assert ma <= MAX_ABS and rl <= REL_L2, (l, s, ma, rl)
            worst = (max(worst[0], ma), max(worst[1], rl))
        log(f"  attention: {len(pairs)} sampled (layer, seq) pairs, worst max_abs {worst[0]:.2e} rel_l2 {worst[1]:.2e}")
        assert P.pipelive_kv_read_state(self.region).status == 0
        return outs

    def block_sums(self, layer, ids):
        """64-bit wrap-around checksum of every listed block (device side)."""
        return self.region.read_blocks(layer, ids).view(torch.int64).sum(dim=1)


def _resize_and_check(st, B_new, tag, check_content=True):
    """Shrink on both sides, compare all state, check that content followed the blocks."""
    cfg, batch = st.cfg, st.batch
    so = _state_oracle(st.B, st.cap)
    so.c.num_blocks = st.region.num_blocks
    live_before = bitmap_ids(st.region.live, st.cap)
    so.set_live(live_before)
    table_h = st.table.cpu().numpy().copy()
    sums_before = {l: st.block_sums(l, live_before) for l in (0, cfg.num_layers - 1)}
    rc_h, remap_h, res_h = so.resize(B_new, [table_h], [st.used.cpu().numpy()])
    remap_d = torch.full((st.region.num_blocks,), -9, dtype=torch.int32, device="cuda")
    rc_d, res_d = P.pipelive_kv_resize(st.region, B_new, [st.table], [st.used], remap_out=remap_d)
    assert rc_h == oracle.OK and rc_d == P.OK, (rc_h, rc_d)
    st.region.sync_block_list()   # a per-block pool had its block list permuted on the device
    assert (res_d.n_live, res_d.n_moved, res_d.old_num_blocks, res_d.new_num_blocks) == tuple(int(x) for x in res_h)
    assert np.array_equal(remap_d.cpu().numpy(), remap_h)
    assert np.array_equal(st.table.cpu().numpy(), table_h)
    assert np.array_equal(bitmap_ids(st.region.live, st.cap), so.live_ids())
    new_ids = remap_h[live_before]
    assert new_ids.min() >= 0 and new_ids.max() < B_new
    for l, before in sums_before.items():            # every live block, on the device
        assert torch.equal(st.block_sums(l, new_ids), before)
    moved = live_before[remap_h[live_before] != live_before]
    for b in moved[:: max(1, len(moved) // 6)][:6] if check_content else []:     # sampled moved blocks against numpy regeneration
        l = int(b) % cfg.num_layers
        got = st.region.block(l, int(remap_h[b])).cpu().numpy().view(np.uint16)
        exp = pin.kv_block_bits(cfg, SEED, st.cap, 0, l, int(b))   # content is keyed by the id it was written at
        assert np.array_equal(got, exp) or _tail_ok(cfg, batch, b, got, exp), (l, int(b))
    log(f"  {tag}: B {int(res_h[2])} -> {int(res_h[3])}, live {int(res_h[0])}, moved {int(res_h[1])}")
    return table_h, remap_h


def _tail_ok(cfg, batch, b, got, exp):
    """A sequence's last block carries NaN in the slots past its length."""
    for s in range(cfg.num_seqs):
        u = int(batch.used[s])
        if u and int(batch.table[s, u - 1]) == int(b):
            valid = int(batch.ctx_lens[s]) - (u - 1) * cfg.block_tokens
            m = pin.token_slot_mask(cfg.layout, cfg.num_kv_heads, cfg.block_tokens, cfg.head_dim, valid)
            return np.array_equal(got[~m], exp[~m]) and (got[m] == pin.BF16_NAN).all()
    return False


def _free_gb():
    free, _ = torch.cuda.mem_get_info()
    return free / 2**30


def test_stage8b_decode_in_bench_configuration():
    """Workload 2: pool = 85 % of the HBM left after the stage weights."""
    cfg = pin.CONFIGS["stage8b"]
    torch.cuda.empty_cache()
    weights = torch.empty(7 * 2**30, dtype=torch.uint8, device="cuda")
    free, _ = torch.cuda.mem_get_info()
    B = int(0.85 * free // (cfg.num_layers * cfg.blk_bytes))
    log(f"stage8b: pool {B} blocks/layer ({B * cfg.num_layers * cfg.blk_bytes / 2**30:.1f} GiB)")
    st = Stage(cfg, B)
    st.check_attention(64, salt=2)
    del st, weights
    torch.cuda.empty_cache()


def test_resize8b_shrink_decode_with_appends_grow_shrink():
    """Workload 3: tight pool, the stage grows 16 -> 20 layers so every pool shrinks by 20 % while the batch
    keeps decoding: decode -> shrink -> decode (bit-identical) -> 16 decode steps that append a token per
    sequence in every layer (new blocks take the lowest free id) -> grow back -> decode -> shrink again ->
    decode; attention after the appends against the oracle on 64 sampled (layer, sequence) pairs."""
    cfg = pin.CONFIGS["resize8b"]
    ctx = pin.draw_ctx_lens(cfg, SEED)
    n_live = int(((ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens).sum())
    B = int(math.ceil(n_live / 0.75))
    B_new = int(B * 16 // 20)
    assert n_live <= B_new
    log(f"resize8b: B {B} -> {B_new}, live {n_live}")
    st = Stage(cfg, B, stride_pad=2)
    batch0 = st.batch
    before = st.check_attention(64, salt=3)
    table_h, _ = _resize_and_check(st, B_new, "shrink")
    after = {l: st.decode(l).cpu().numpy() for l in before}
    for l in before:                                   # attention unchanged bit for bit
        assert np.array_equal(before[l].view(np.uint32), after[l].view(np.uint32)), l
    # 16 decode steps on the shrunken pool
    bm = pin.BlockManager(batch0, B)
    bm.set_num_blocks(B_new)
    bm.adopt(table_h, bitmap_ids(st.region.live, st.cap))
    steps, n_new = 16, 0
    for k in range(steps):
        _, new_entries = st.append_step(bm, k, count_layer=-1, mark=False)
        assert all(b < B_new for _, _, b in new_entries)
        n_new += len(new_entries)
    torch.cuda.synchronize()
    assert n_new > 0 and np.array_equal(st.table.cpu().numpy(), bm.table)
    assert np.array_equal(bitmap_ids(st.region.live, st.cap), bm.live_ids())
    log(f"  {steps} decode steps appended {steps * cfg.num_seqs} tokens per layer into {n_new} new blocks")
    # grow back (nothing moves): decode against the oracle on sampled pairs
    rc, res = P.pipelive_kv_resize(st.region, B, [st.table], [st.used])
    assert rc == P.OK and res.n_moved == 0 and st.region.num_blocks == B
    pairs = _sample_pairs(cfg, 64, 33)
    outs = {l: st.decode(l).cpu().numpy() for l in sorted({l for l, _ in pairs})}
    oracle.lib()
    with ThreadPoolExecutor(max_workers=12) as ex:
        refs = list(ex.map(lambda ls: _oracle_pair_after_appends(cfg, batch0, st.cap, ls[0], ls[1], steps), pairs))
    worst = (0.0, 0.0)
    for (l, s), ref in zip(pairs, refs):
        ma, rl = attn_errors(outs[l][s], ref)
        assert ma <= MAX_ABS and rl <= REL_L2, (l, s, ma, rl)
        worst = (max(worst[0], ma), max(worst[1], rl))
    log(f"  attention after the appends: {len(pairs)} pairs, worst max_abs {worst[0]:.2e} rel_l2 {worst[1]:.2e}")
    # shrink again: tables, remap and bitmaps against the oracle, attention bit-identical
    table_h2, _ = _resize_and_check(st, B_new, "second shrink", check_content=False)
    again = {l: st.decode(l).cpu().numpy() for l in outs}
    for l in outs:
        assert np.array_equal(outs[l].view(np.uint32), again[l].view(np.uint32)), l
    # infeasible request: nothing changes
    rc, res = P.pipelive_kv_resize(st.region, n_live - 1, [st.table], [st.used])
    assert rc == P.E_INFEASIBLE and st.region.num_blocks == B_new
    assert np.array_equal(st.table.cpu().numpy(), table_h2)
    assert P.pipelive_kv_read_state(st.region).status == 0
    del st
    torch.cuda.empty_cache()


def test_stage70b_incremental_patching_six_rounds():
    """Workload 4: round 0 (pre-copy) + 6 rounds, dirty fraction 20 % -> 1 % geometrically."""
    cfg = pin.CONFIGS["stage70b"]
    ctx = pin.draw_ctx_lens(cfg, SEED)
    n_live = int(((ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens).sum())
    B = int(math.ceil(1.25 * n_live))
    L = cfg.num_layers
    log(f"stage70b: source and target {B} blocks/layer x {L} layers ({B * L * cfg.blk_bytes / 2**30:.1f} GiB each), free {_free_gb():.0f} GiB")
    st = Stage(cfg, B, stride_pad=2)
    st.check_attention(64, salt=4)
    bm = pin.BlockManager(st.batch, B)
    touched = set()
    tgt = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B, arenas=3)
    so = _state_oracle(B)
    so_t = _state_oracle(B)
    live = st.batch.live_ids
    layers = list(range(L))
    fr = pin.geometric_fractions(0.20, 0.01, 6)
    n_r1 = len(pin.draw_dirty_ids(st.batch, SEED, 1, fr[0]))
    cap_small = 64 + 256 + (n_r1 + 8) * (4 + L * cfg.blk_bytes)     # sized for patch round 1; the pre-copy round is clipped
    patch = torch.empty(cap_small, dtype=torch.uint8, device="cuda")
    patch_h = np.zeros(64 + 256 + (n_r1 + 8) * (4 + so.blk_bytes) + 8 * B, dtype=np.uint8)
    max_blocks = P.pipelive_patch_max_blocks(st.region, L, cap_small)
    hdr = torch.zeros(64, dtype=torch.uint8).pin_memory()
    sched, applied_ids = 0, set()
    for rnd in range(7):
        if rnd == 0:
            ids, ntok = live, 0
        else:
            # the decode step between two rounds: every sequence appends one token in every layer (fused
            # dirty mark; layer 0 counts the tokens); the state oracle mirrors bits and count with its own append
            pos, _ = st.append_step(bm, rnd - 1)
            so.set_live(bm.live_ids())
            z = np.zeros((cfg.num_seqs, 1, 8), dtype=np.uint16)
            assert so.append(0, z, z, bm.table, pos, mark=True, count_tokens=True) == oracle.OK
            touched |= set(bm.last_block_ids().tolist())
            ntok = cfg.num_seqs
            # ... and a seeded sample of live blocks is rewritten (sampled layers get new content) and marked
            ids = pin.draw_dirty_ids(st.batch, SEED, rnd, fr[rnd - 1], include_last=False)
            for l in (0, 7, L - 1):
                data = pin.kv_blocks_bits_torch(cfg, SEED, B, rnd, l, ids[:256], "cuda")
                st.region.write_blocks(l, ids[:256], data)
        sched += ntok
        ids32 = torch.from_numpy(np.asarray(ids, dtype=np.int32)).cuda()
        assert so.mark_dirty(ids, 0) == oracle.OK
        P.pipelive_kv_mark_dirty(st.region, ids32, 0)
        drains = 0
        while True:
            # the state oracle drains with the same id capacity
            cap_h = 64 + 256 + max_blocks * (4 + so.blk_bytes)
            assert so.patch_max_blocks(1, cap_h) == max_blocks
            assert so.patch_collect([0], patch_h[:cap_h]) == oracle.OK
            P.pipelive_kv_patch_collect(st.region, layers, patch, hdr_host=hdr)
            torch.cuda.synchronize()
            h = oracle.parse_patch_header(patch_h)
            g = oracle.parse_patch_header(hdr.numpy())
            for k in ("magic", "version", "n_blocks", "n_acc_tokens", "more_pending", "max_blocks"):
                assert g[k] == h[k], (rnd, k, g[k], h[k])
            assert g["n_layers"] == L and g["block_bytes"] == cfg.blk_bytes
            nb = g["n_blocks"]
            ids_d = patch[64:64 + 4 * nb].view(torch.int32)
            ids_h = np.frombuffer(patch_h[64:64 + 4 * nb].tobytes(), dtype=np.int32)
            assert np.array_equal(ids_d.cpu().numpy(), ids_h)
            assert np.array_equal(bitmap_ids(st.region.dirty, B), so.dirty_ids())
            # payload == the source blocks, every byte, compared on the device
            pay = patch[g["payload_offset"]:g["payload_offset"] + nb * L * cfg.blk_bytes].view(torch.int16)
            pay = pay.view(nb, L, cfg.blk_elems)
            for l in (0, 7, L - 1) if rnd else range(0, L, 5):
                assert torch.equal(pay[:, l, :], st.region.read_blocks(l, ids_h)), (rnd, l)
            assert so_t.patch_apply([0], patch_h[:cap_h]) == oracle.OK
            P.pipelive_kv_patch_apply(tgt, layers, patch)
            applied_ids |= set(ids_h.tolist())
            drains += 1
            if not g["more_pending"]:
                break
        log(f"  round {rnd}: {len(ids)} sampled/live blocks marked (+ appends), {drains} drain(s), n_acc {ntok}")
    live = bm.live_ids()
    assert applied_ids == set(live.tolist())
    stt = P.pipelive_kv_read_state(tgt)
    assert stt.t_applied == sched == so_t.t_applied and stt.status == 0
    assert len(bitmap_ids(st.region.dirty, B)) == 0
    for l in range(L):                                  # target == source on every live block, every layer
        assert torch.equal(tgt.read_blocks(l, live), st.region.read_blocks(l, live)), l
    for b in live[:: max(1, len(live) // 5)][:5]:       # sampled blocks against numpy regeneration
        l = int(b) % L
        got = tgt.block(l, int(b)).cpu().numpy().view(np.uint16)
        exp = pin.kv_block_bits(cfg, SEED, B, 0, l, int(b))
        assert np.array_equal(got, exp) or _tail_ok(cfg, st.batch, b, got, exp) or l in (0, 7, L - 1) or int(b) in touched
    del st, tgt, patch
    torch.cuda.empty_cache()


def test_stage70b_placed_by_the_arena_as_the_bench_places_it():
    """Workload 4 with its pools and patch buffer carved out of a probed region-aware arena the way bench.py
    does it (layer l in the zone of class l mod n, the patch buffer in the spread zone): decode against the
    oracle on 64 sampled pairs, a 20 % patch round whose target equals the source, and the 20 % shrink with all
    state compared with the oracle's.  The placement changes addresses only; every result must be what it is
    on torch allocations."""
    cfg = pin.CONFIGS["stage70b"]
    ctx = pin.draw_ctx_lens(cfg, SEED)
    n_live = int(((ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens).sum())
    B = int(math.ceil(1.25 * n_live))
    L = cfg.num_layers
    ids = pin.draw_dirty_ids(pin.draw_batch(cfg, SEED, num_blocks=B, stride_pad=2), SEED, 1, 0.20)
    cap = 64 + 256 + (len(ids) + 8) * (4 + L * cfg.blk_bytes)
    pool_bytes = B * L * cfg.blk_bytes
    arena = P.Arena(2 * pool_bytes + cap + (16 << 30))
    info = arena.info()
    log(f"stage70b on an arena of {arena.nbytes >> 30} GiB: classes {info['class_pieces']}, probe {info['probe_ms']:.0f} ms")
    arena.layout(cap + (256 << 20))
    st = Stage(cfg, B, stride_pad=2, allocator=arena.placer(4))
    lo, hi = arena.base + arena.zones[1][0], arena.base + arena.nbytes
    assert all(lo <= t.data_ptr() < hi for t in st.region.arenas)          # every pool arena in a class zone
    for g in range(L):                                                     # a layer's arenas share one zone
        zs = {z for t in st.region.arenas[4 * g:4 * g + 4] for z in range(1, len(arena.zones))
              if arena.zones[z][0] <= t.data_ptr() - arena.base < arena.zones[z][0] + arena.zones[z][1]}
        assert len(zs) == 1, (g, zs)
    st.check_attention(64, salt=14)
    tgt = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B, arenas=3,
                     allocator=arena.placer(3))
    patch = arena.empty(cap)
    ids32 = torch.from_numpy(np.asarray(ids, dtype=np.int32)).cuda()
    P.pipelive_kv_mark_dirty(st.region, ids32, 7)
    hdr = torch.zeros(64, dtype=torch.uint8).pin_memory()
    P.pipelive_kv_patch_collect(st.region, list(range(L)), patch, hdr_host=hdr)
    P.pipelive_kv_patch_apply(tgt, list(range(L)), patch)
    torch.cuda.synchronize()
    g = oracle.parse_patch_header(hdr.numpy())
    assert g["n_blocks"] == len(ids) and g["n_acc_tokens"] == 7 and not g["more_pending"]
    assert np.array_equal(patch[64:64 + 4 * len(ids)].view(torch.int32).cpu().numpy(), np.sort(ids).astype(np.int32))
    for l in range(L):
        assert torch.equal(tgt.read_blocks(l, ids), st.region.read_blocks(l, ids)), l
    assert P.pipelive_kv_read_state(tgt).t_applied == 7 and len(bitmap_ids(st.region.dirty, B)) == 0
    _resize_and_check(st, int(B * 0.8), "20 % shrink on arena memory")
    assert P.pipelive_kv_read_state(st.region).status == 0
    del st, tgt, patch
    arena.close()
    torch.cuda.empty_cache()


def test_longctx8b_split_decode_resize_and_final_patch():
    """Workload 5: 16 sequences of 16k-32k tokens, block 32; shrink 25 %; final patch round at 2 %."""
    cfg = pin.CONFIGS["longctx8b"]
    ctx = pin.draw_ctx_lens(cfg, SEED)
    n_live = int(((ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens).sum())
    B = int(math.ceil(n_live / 0.70))
    B_new = int(B * 0.75)
    assert n_live <= B_new
    log(f"longctx8b: B {B} -> {B_new}, live {n_live}, free {_free_gb():.0f} GiB")
    st = Stage(cfg, B)
    before = st.check_attention(64, salt=5)
    table_h, remap_h = _resize_and_check(st, B_new, "shrink 25 %")
    after = {l: st.decode(l).cpu().numpy() for l in before}
    for l in before:
        assert np.array_equal(before[l].view(np.uint32), after[l].view(np.uint32)), l
    # round 0 + final round with 2 % dirty blocks into a compact target through a block map
    L = cfg.num_layers
    live = bitmap_ids(st.region.live, st.cap)
    bt = pin.Batch(cfg, SEED, B_new, st.batch.ctx_lens, table_h, st.batch.used, live)
    tgt = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, len(live), arenas=2)
    dmap = torch.full((B_new,), -1, dtype=torch.int32)
    dmap[torch.from_numpy(live)] = torch.arange(len(live), dtype=torch.int32)
    dmap = dmap.cuda()
    cap = 64 + 256 + len(live) * (4 + L * cfg.blk_bytes)
    patch = torch.empty(cap, dtype=torch.uint8, device="cuda")
    hdr = torch.zeros(64, dtype=torch.uint8).pin_memory()
    for rnd, ids in enumerate([live, pin.draw_dirty_ids(bt, SEED, 1, 0.02)]):
        P.pipelive_kv_mark_dirty(st.region, torch.from_numpy(np.asarray(ids, dtype=np.int32)).cuda(), rnd * cfg.num_seqs)
        P.pipelive_kv_patch_collect(st.region, list(range(L)), patch, hdr_host=hdr)
        P.pipelive_kv_patch_apply(tgt, list(range(L)), patch, dst_block_map=dmap)
        torch.cuda.synchronize()
        g = oracle.parse_patch_header(hdr.numpy())
        assert g["n_blocks"] == len(ids) and g["more_pending"] == 0 and g["n_acc_tokens"] == rnd * cfg.num_seqs
        assert np.array_equal(patch[64:64 + 4 * len(ids)].view(torch.int32).cpu().numpy(), np.asarray(ids, dtype=np.int32))
        log(f"  patch round {rnd}: {len(ids)} blocks")
    assert P.pipelive_kv_read_state(tgt).t_applied == cfg.num_seqs
    compact = np.arange(len(live))
    for l in range(L):
        assert torch.equal(tgt.read_blocks(l, compact), st.region.read_blocks(l, live)), l
    del st, tgt, patch
    torch.cuda.empty_cache()


def test_stage8b_stacked_per_block_pool_decode_shrink_release():
    """The 8B stage's batch over independently allocated 2 MiB blocks (k = 4 layers x 128 tokens), as in
    bench.py's stacked leg: sampled attention against the oracle, a 20 % shrink that copies nothing and leaves
    the outputs bit-identical, then the freed blocks really go back to the device."""
    base = pin.CONFIGS["stage8b"]
    cfg = pin.StageConfig("stage8b-stacked", base.num_layers, base.num_q_heads, base.num_kv_heads, base.head_dim,
                          128, base.num_seqs, base.ctx_lo, base.ctx_hi)
    ctx = pin.draw_ctx_lens(cfg, SEED)
    n_live = int(((ctx.astype(np.int64) + 127) // 128).sum())
    B = int(n_live * 1.5)
    B_new = int(B * 0.8)
    torch.cuda.empty_cache()
    log(f"stage8b-stacked: B {B} -> {B_new}, live {n_live}, {B * 4 * 2 / 1024:.1f} GiB in 2 MiB blocks")
    st = Stage(cfg, B, stack_k=4, backing="vmm")
    assert st.region.phys_bytes == 2 << 20 and st.region.pool.allocated == 4 * B
    before = st.check_attention(32, salt=6)
    _resize_and_check(st, B_new, "pointer-only shrink")
    after = {l: st.decode(l).cpu().numpy() for l in before}
    for l in before:
        assert np.array_equal(before[l].view(np.uint32), after[l].view(np.uint32)), l
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    assert st.region.release_tail(B) == 4 * (B - B_new)
    gained = torch.cuda.mem_get_info()[0] - free0
    assert abs(gained - 4 * (B - B_new) * (2 << 20)) <= 64 << 20, gained
    again = {l: st.decode(l).cpu().numpy() for l in before}
    for l in before:
        assert np.array_equal(before[l].view(np.uint32), again[l].view(np.uint32)), l
    assert P.pipelive_kv_read_state(st.region).status == 0
    del st
    torch.cuda.empty_cache()


@pytest.mark.parametrize("case", [("chunk512_of_4096", 16, 4096, 512), ("prompt512", 64, 512, 512)])
def test_prefill_in_bench_configuration(case):
    """bench.py's prefill cases with the 8B stage's heads: a 512-token chunk on 4096 cached tokens (16
    sequences) and 64 prompts of 512 tokens.  A prefill row is the decode of its token over the context it
    may see, so sampled rows are checked against the oracle's *decode* attention on a context truncated at
    the row's position."""
    base = pin.CONFIGS["stage8b"]
    tag, S, ctx_len, q_len = case
    cfg = pin.StageConfig(tag, 1, base.num_q_heads, base.num_kv_heads, base.head_dim,
                          base.block_tokens, S, ctx_len, ctx_len)
    batch = pin.draw_batch(cfg, SEED, pool_factor=1.25)
    cap = batch.num_blocks
    region = P.KVRegion(1, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, cap, arenas=3)
    fill_live_blocks(region, cfg, batch, SEED, cap, poison_tail=False)
    tq = S * q_len
    qb = pin.bf16_normal(pin.stream_key(SEED, pin.STREAM_Q), 0, tq * cfg.num_q_heads * cfg.head_dim)
    qb = qb.reshape(tq, cfg.num_q_heads, cfg.head_dim)
    q_d = torch.from_numpy(qb.view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.full((tq, cfg.num_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")
    qo = torch.arange(0, (S + 1) * q_len, q_len, dtype=torch.int32, device="cuda")
    P.pipelive_paged_attn_prefill(region, 0, q_d, out, torch.from_numpy(batch.table).cuda(),
                                  torch.from_numpy(batch.ctx_lens).cuda(), qo, tq)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    out16 = torch.full((tq, cfg.num_q_heads, cfg.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    P.pipelive_paged_attn_prefill(region, 0, q_d, out16, torch.from_numpy(batch.table).cuda(),
                                  torch.from_numpy(batch.ctx_lens).cuda(), qo, tq)
    torch.cuda.synchronize()
    got16 = out16.float().cpu().numpy()
    assert np.isfinite(got16).all()
    worst = (0.0, 0.0)
    worst16 = (0.0, 0.0)
    for s in (0, 5, 11, S - 1):
        u = int(batch.used[s])
        host = oracle.HostKV(1, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, u,
                             layout=cfg.layout, arenas=2, fill_bits=pin.BF16_NAN)
        for j in range(u):
            host.block(0, j)[:] = pin.kv_block_bits(cfg, SEED, cap, 0, 0, int(batch.table[s, j]))
        tab = np.arange(u, dtype=np.int32)[None, :]
        for i in (0, 1, 31, 32, 255, 300, 510, 511):          # rows of the chunk, incl. both ends
            pos = ctx_len - q_len + i                          # the row sees positions 0 .. pos
            ref = host.attn_decode(0, qb[s * q_len + i][None], tab, np.array([pos + 1], dtype=np.int32))[0]
            ma, rl = attn_errors(got[s * q_len + i], ref)
            assert ma <= MAX_ABS and rl <= REL_L2, (s, i, ma, rl)
            worst = (max(worst[0], ma), max(worst[1], rl))
            ma, rl = attn_errors(got16[s * q_len + i], ref)
            assert ma <= BF16_MAX_ABS and rl <= BF16_REL_L2, ("bf16 out", s, i, ma, rl)
            worst16 = (max(worst16[0], ma), max(worst16[1], rl))
    log(f"  prefill: 32 sampled rows, worst max_abs {worst[0]:.2e} rel_l2 {worst[1]:.2e}; "
        f"bf16 output: {worst16[0]:.2e} {worst16[1]:.2e}")
    assert P.pipelive_kv_read_state(region).status == 0
    del region
    torch.cuda.empty_cache()
