"""GPU parity of chunked-prefill paged attention against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import BF16_MAX_ABS, BF16_REL_L2, MAX_ABS, REL_L2, attn_errors, fill_pair, make_pair

pytestmark = pytest.mark.gpu
SEED = 99


def _batch(cfg, ctx, pad=2, extra=5, seed=SEED):
    ctx = np.asarray(ctx, dtype=np.int32)
    used = (ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens
    B = int(used.sum()) + extra
    perm = pin.permutation(pin.stream_key(seed, pin.STREAM_PERM), B)
    table = np.full((len(ctx), max(int(used.max()), 1) + pad), pin.TABLE_FILL, dtype=np.int32)
    off = 0
    for s, u in enumerate(used):
        table[s, :u] = perm[off:off + u]
        off += int(u)
    return pin.Batch(cfg, seed, B, ctx, table, used.astype(np.int32), np.sort(perm[:off]))


CASES = [
    # ctx, q_len
    ([70, 70], [70, 70]),                    # full prefill
    ([1, 17, 33, 200, 64, 5], [1, 17, 8, 50, 64, 0]),   # mixed: single token, chunked, a sequence without queries
    ([300, 129, 45], [1, 1, 1]),             # decode as the one-query case
    ([515], [515]),                          # several address batches and many query blocks
]


@pytest.mark.parametrize("shape", [(4, 2, 64, 16), (32, 8, 128, 16), (64, 8, 128, 16), (16, 1, 128, 32),
                                   (8, 8, 64, 32), (6, 2, 128, 16), (32, 8, 128, 128), (4, 2, 64, 64),
                                   (32, 16, 64, 16)])     # 16 KV heads: two heads per work list
@pytest.mark.parametrize("case", range(len(CASES)))
def test_prefill_matches_oracle(shape, case):
    Hq, Hkv, D, bs = shape
    ctx, qlen = CASES[case]
    cfg = pin.StageConfig("pf", 2, Hq, Hkv, D, bs, len(ctx), 0, 0)
    batch = _batch(cfg, ctx)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    qo = np.concatenate([[0], np.cumsum(qlen)]).astype(np.int32)
    total_q = int(qo[-1])
    rng = np.random.default_rng(case)
    q = pin.f32_to_bf16_bits(rng.standard_normal((total_q, Hq, D)).astype(np.float32))
    q_d = torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16)
    for layer in range(2):
        out = torch.full((total_q, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
        P.pipelive_paged_attn_prefill(dev, layer, q_d, out, torch.from_numpy(batch.table).cuda(),
                                      torch.from_numpy(batch.ctx_lens).cuda(), torch.from_numpy(qo).cuda(), total_q)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        ref = host.attn_prefill(layer, q, batch.table, batch.ctx_lens, qo, nthreads=8)
        assert np.isfinite(got).all()
        ma, rl = attn_errors(got, ref)
        assert ma <= MAX_ABS and rl <= REL_L2, (ma, rl)
        for s in range(len(ctx)):
            if qlen[s]:
                ma, rl = attn_errors(got[qo[s]:qo[s + 1]], ref[qo[s]:qo[s + 1]])
                assert ma <= MAX_ABS and rl <= REL_L2, (s, ma, rl)
        # bf16 output (the form with single-bf16 softmax weights): its own, derived tolerance
        out16 = torch.full((total_q, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        P.pipelive_paged_attn_prefill(dev, layer, q_d, out16, torch.from_numpy(batch.table).cuda(),
                                      torch.from_numpy(batch.ctx_lens).cuda(), torch.from_numpy(qo).cuda(), total_q)
        torch.cuda.synchronize()
        got16 = out16.float().cpu().numpy()
        assert np.isfinite(got16).all()
        ma, rl = attn_errors(got16, ref)
        assert ma <= BF16_MAX_ABS and rl <= BF16_REL_L2, ("bf16 out", ma, rl)
    assert P.pipelive_kv_read_state(dev).status == 0


def test_prefill_single_query_agrees_with_decode_kernel_and_bf16_out():
    ctx = [257, 40, 1000]
    cfg = pin.StageConfig("pf", 1, 32, 8, 128, 16, 3, 0, 0)
    batch = _batch(cfg, ctx)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    q = pin.q_bits(cfg, SEED, 0)
    q_d = torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16)
    t, c = torch.from_numpy(batch.table).cuda(), torch.from_numpy(batch.ctx_lens).cuda()
    qo = torch.arange(4, dtype=torch.int32, device="cuda")
    a = torch.empty((3, 32, 128), dtype=torch.float32, device="cuda")
    b = torch.empty((3, 32, 128), dtype=torch.float32, device="cuda")
    P.pipelive_paged_attn_prefill(dev, 0, q_d, a, t, c, qo, 3)
    P.pipelive_paged_attn_decode(dev, 0, q_d, b, t, c)
    ma, rl = attn_errors(a.cpu().numpy(), b.cpu().numpy())
    assert ma < 1e-5 and rl < 1e-5                      # same mathematics, other tiling
    h = torch.empty((3, 32, 128), dtype=torch.bfloat16, device="cuda")
    P.pipelive_paged_attn_prefill(dev, 0, q_d, h, t, c, qo, 3)
    ma, rl = attn_errors(h.float().cpu().numpy(), a.cpu().numpy())
    assert ma <= BF16_MAX_ABS and rl <= BF16_REL_L2, (ma, rl)


def test_prefill_many_sequences_multi_chunk_unit_search():
    """More than 64 sequences (the unit search scans them 64 at a time), among them sequences without
    queries and one-token chunks."""
    rng = np.random.default_rng(5)
    S = 150
    ctx = rng.integers(1, 90, size=S)
    qlen = np.minimum(ctx, rng.integers(0, 40, size=S))
    qlen[::7] = 0
    qlen[3::11] = 1
    cfg = pin.StageConfig("pf", 1, 4, 2, 64, 16, S, 0, 0)
    batch = _batch(cfg, ctx)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    qo = np.concatenate([[0], np.cumsum(qlen)]).astype(np.int32)
    total_q = int(qo[-1])
    q = pin.f32_to_bf16_bits(rng.standard_normal((total_q, 4, 64)).astype(np.float32))
    q_d = torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.full((total_q, 4, 64), float("nan"), dtype=torch.float32, device="cuda")
    P.pipelive_paged_attn_prefill(dev, 0, q_d, out, torch.from_numpy(batch.table).cuda(),
                                  torch.from_numpy(batch.ctx_lens).cuda(), torch.from_numpy(qo).cuda(), total_q)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ref = host.attn_prefill(0, q, batch.table, batch.ctx_lens, qo, nthreads=8)
    assert np.isfinite(got).all()
    for s in range(S):
        if qlen[s]:
            ma, rl = attn_errors(got[qo[s]:qo[s + 1]], ref[qo[s]:qo[s + 1]])
            assert ma <= MAX_ABS and rl <= REL_L2, (s, ma, rl)
    assert P.pipelive_kv_read_state(dev).status == 0


@pytest.mark.parametrize("Hkv", [4, 8])                    # one work list for all / one per XCD, dealt by KV head
def test_prefill_more_units_than_resident_workgroups_and_relaunch(Hkv):
    """Enough (sequence, head, query block) units that every resident workgroup has to draw further
    ones from the ticket counters (ragged lengths, chunks and full prompts); a second launch must find
    the counters re-armed and give the same bits."""
    rng = np.random.default_rng(11)
    S, Hq, D, bs = 100, 16, 64, 16                        # more than 64 sequences: the drawn units' search spans chunks
    ctx = rng.integers(60, 260, size=S)
    qlen = np.where(rng.random(S) < 0.5, ctx, np.minimum(ctx, rng.integers(1, 120, size=S)))
    qlen[5::17] = 0
    cfg = pin.StageConfig("pf", 1, Hq, Hkv, D, bs, S, 0, 0)
    batch = _batch(cfg, ctx)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    qo = np.concatenate([[0], np.cumsum(qlen)]).astype(np.int32)
    total_q = int(qo[-1])
    wb = 4 * (32 // (Hq // Hkv))                          # query tokens per unit
    units = Hkv * int(np.sum((qlen + wb - 1) // wb))
    assert units > 2 * 256 * 2                            # more than two per resident workgroup
    q = pin.f32_to_bf16_bits(rng.standard_normal((total_q, Hq, D)).astype(np.float32))
    q_d = torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16)
    t, c, o = torch.from_numpy(batch.table).cuda(), torch.from_numpy(batch.ctx_lens).cuda(), torch.from_numpy(qo).cuda()
    outs = []
    for _ in range(2):
        out = torch.full((total_q, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
        P.pipelive_paged_attn_prefill(dev, 0, q_d, out, t, c, o, total_q)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])
    got = outs[0]
    assert np.isfinite(got).all()
    ref = host.attn_prefill(0, q, batch.table, batch.ctx_lens, qo, nthreads=8)
    for s in range(S):
        ma, rl = attn_errors(got[qo[s]:qo[s + 1]], ref[qo[s]:qo[s + 1]])
        assert ma <= MAX_ABS and rl <= REL_L2, (s, ma, rl)
    assert P.pipelive_kv_read_state(dev).status == 0


def test_clear_status_re_arms_the_prefill_work_counters():
    """Counters left non-zero (as after a launch that was cut short) would make every workgroup stop after
    its first unit; pipelive_kv_clear_status() zeroes them together with the status word."""
    ctx = [300, 260]
    cfg = pin.StageConfig("pf", 1, 8, 2, 64, 16, 2, 0, 0)
    batch = _batch(cfg, ctx)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    qo = np.array([0, 300, 560], dtype=np.int32)
    rng = np.random.default_rng(3)
    q = pin.f32_to_bf16_bits(rng.standard_normal((560, 8, 64)).astype(np.float32))
    q_d = torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16)
    dev.state[24:28] = 77                                  # workgroups that have left ...
    dev.state[64:96] = 77                                  # ... and the ticket counters of the eight work lists
    P.pipelive_kv_clear_status(dev)
    out = torch.full((560, 8, 64), float("nan"), dtype=torch.float32, device="cuda")
    P.pipelive_paged_attn_prefill(dev, 0, q_d, out, torch.from_numpy(batch.table).cuda(),
                                  torch.from_numpy(batch.ctx_lens).cuda(), torch.from_numpy(qo).cuda(), 560)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ref = host.attn_prefill(0, q, batch.table, batch.ctx_lens, qo, nthreads=8)
    assert np.isfinite(got).all()
    ma, rl = attn_errors(got, ref)
    assert ma <= MAX_ABS and rl <= REL_L2, (ma, rl)
    assert int(dev.state[24:28].sum()) + int(dev.state[64:96].sum()) == 0   # re-armed again by the launch itself


def test_prefill_bad_table_entry_sets_status_and_spares_the_others():
    ctx, qlen = [100, 64, 200], [100, 10, 50]
    cfg = pin.StageConfig("pf", 1, 8, 2, 128, 16, 3, 0, 0)
    batch = _batch(cfg, ctx)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    qo = np.concatenate([[0], np.cumsum(qlen)]).astype(np.int32)
    total_q = int(qo[-1])
    rng = np.random.default_rng(8)
    q = pin.f32_to_bf16_bits(rng.standard_normal((total_q, 8, 128)).astype(np.float32))
    q_d = torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16)
    table = batch.table.copy()
    table[1, 2] = 10 ** 6        # beyond the pool
    table[1, 0] = -3             # negative
    out = torch.full((total_q, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
    P.pipelive_paged_attn_prefill(dev, 0, q_d, out, torch.from_numpy(table).cuda(),
                                  torch.from_numpy(batch.ctx_lens).cuda(), torch.from_numpy(qo).cuda(), total_q)
    torch.cuda.synchronize()
    assert P.pipelive_kv_read_state(dev).status == P.E_RANGE
    got = out.cpu().numpy()
    ref = host.attn_prefill(0, q, batch.table, batch.ctx_lens, qo, nthreads=8)
    for s in (0, 2):             # the sequences with valid tables are unaffected
        ma, rl = attn_errors(got[qo[s]:qo[s + 1]], ref[qo[s]:qo[s + 1]])
        assert ma <= MAX_ABS and rl <= REL_L2, (s, ma, rl)


def test_prefill_errors():
    cfg = pin.StageConfig("pf", 1, 4, 2, 64, 16, 1, 0, 0)
    batch = _batch(cfg, [10])
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    q = torch.zeros((12, 4, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((12, 4, 64), dtype=torch.float32, device="cuda")
    t, c = torch.from_numpy(batch.table).cuda(), torch.from_numpy(batch.ctx_lens).cuda()
    qo = torch.tensor([0, 12], dtype=torch.int32, device="cuda")      # 12 queries, 10 cached tokens
    P.pipelive_paged_attn_prefill(dev, 0, q, out, t, c, qo, 12)
    assert P.pipelive_kv_read_state(dev).status == P.E_INVAL
    assert P.pipelive_paged_attn_prefill(dev, 3, q, out, t, c, qo, 12, check=False) == P.E_RANGE


@pytest.mark.parametrize("gran", [0, 1])
@pytest.mark.parametrize("shape", [(4, 2, 64, 16), (32, 8, 128, 16), (16, 8, 128, 32), (16, 8, 128, 128), (8, 2, 64, 64)])
def test_chunk_append_matches_oracle_and_feeds_prefill(shape, gran):
    """The write side of a chunk: ragged starts and ends, whole windows and partial ones, then the prefill
    attention over what was written; every byte of both pools, the dirty bitmap and n_acc are compared."""
    import oracle
    from gpu_common import assert_pools_equal, bitmap_ids
    Hq, Hkv, D, bs = shape
    L, B = 2, 60
    rng = np.random.default_rng(31)
    host = oracle.HostKV(L, Hq, Hkv, D, bs, B, dirty_gran=gran, fill_bits=pin.BF16_NAN)
    dev = P.KVRegion(L, Hq, Hkv, D, bs, B, dirty_granularity=gran, fill_bits=pin.BF16_NAN, arenas=4)
    S = 6
    per_seq = B // S
    table = rng.permutation(B)[: S * per_seq].reshape(S, per_seq).astype(np.int32)
    cap_tokens = per_seq * bs
    done = np.zeros(S, dtype=np.int32)
    table_d = torch.from_numpy(table).cuda()
    for rnd, want in enumerate([[33, 1, 0, 64, 17, 31], [32, 40, 5, 1, 15, 70], [7, 90, 64, 3, 0, 33]]):
        qlen = np.minimum(np.asarray(want, dtype=np.int32), cap_tokens - done)
        ctx = done + qlen
        qo = np.concatenate([[0], np.cumsum(qlen)]).astype(np.int32)
        tq = int(qo[-1])
        for layer in range(L):
            k = pin.f32_to_bf16_bits(rng.standard_normal((tq, Hkv, D)).astype(np.float32))
            v = pin.f32_to_bf16_bits(rng.standard_normal((tq, Hkv, D)).astype(np.float32))
            assert host.append_chunk(layer, k, v, table, ctx, qo, mark=True, count_tokens=(layer == 0)) == oracle.OK
            P.pipelive_kv_append_chunk(dev, layer, torch.from_numpy(k.view(np.int16)).cuda().view(torch.bfloat16),
                                       torch.from_numpy(v.view(np.int16)).cuda().view(torch.bfloat16), table_d,
                                       torch.from_numpy(ctx).cuda(), torch.from_numpy(qo).cuda(), tq,
                                       mark=True, count_tokens=(layer == 0))
        torch.cuda.synchronize()
        units = B * (bs if gran else 1)
        assert np.array_equal(bitmap_ids(dev.dirty, units), host.dirty_ids()), rnd
        st = P.pipelive_kv_read_state(dev)
        assert st.n_acc == host.n_acc and st.status == 0
        assert_pools_equal(host, dev, range(L), range(B))
        # prefill attention of the chunk over the cache it just extended
        q = pin.f32_to_bf16_bits(rng.standard_normal((tq, Hq, D)).astype(np.float32))
        out = torch.full((tq, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
        P.pipelive_paged_attn_prefill(dev, 1, torch.from_numpy(q.view(np.int16)).cuda().view(torch.bfloat16), out,
                                      table_d, torch.from_numpy(ctx).cuda(), torch.from_numpy(qo).cuda(), tq)
        torch.cuda.synchronize()
        ref = host.attn_prefill(1, q, table, ctx, qo, nthreads=8)
        ma, rl = attn_errors(out.cpu().numpy(), ref)
        assert ma <= MAX_ABS and rl <= REL_L2, (rnd, ma, rl)
        done = ctx


def test_chunk_append_flags_bad_input_and_skips_it():
    dev = P.KVRegion(1, 4, 2, 64, 16, 12, fill_bits=pin.BF16_NAN)
    k = torch.zeros((40, 2, 64), dtype=torch.bfloat16, device="cuda")
    table = torch.tensor([[1, 99, 3]], dtype=torch.int32, device="cuda")      # second block id out of range
    qo = torch.tensor([0, 40], dtype=torch.int32, device="cuda")
    P.pipelive_kv_append_chunk(dev, 0, k, k, table, torch.tensor([40], dtype=torch.int32, device="cuda"), qo, 40)
    assert P.pipelive_kv_read_state(dev).status == P.E_RANGE
    assert (dev.block(0, 1).cpu().numpy().view(np.uint16) == pin.BF16_NAN).all()      # shares a window with the bad id
    assert (dev.block(0, 3).cpu().numpy().view(np.uint16) == 0).any()                 # the next window was written
    P.pipelive_kv_clear_status(dev)
    P.pipelive_kv_append_chunk(dev, 0, k, k, table, torch.tensor([30], dtype=torch.int32, device="cuda"), qo, 40)
    assert P.pipelive_kv_read_state(dev).status == P.E_INVAL                       # chunk longer than its context
