"""GPU parity of paged decode attention on small shapes that still span
several tiles, splits and a ragged tail; invariances the method guarantees."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import MAX_ABS, REL_L2, attn_errors, fill_pair, make_pair

pytestmark = pytest.mark.gpu
SEED = 77


def _cfg(Hq, Hkv, D, bs, ctx):
    return pin.StageConfig("case", 2, Hq, Hkv, D, bs, len(ctx), 0, 0)


def _batch(cfg, ctx, pad=3, extra=7, seed=SEED):
    """Block tables over a shuffled pool for explicit context lengths."""
    ctx = np.asarray(ctx, dtype=np.int32)
    used = (ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens
    B = int(used.sum()) + extra
    perm = pin.permutation(pin.stream_key(seed, pin.STREAM_PERM), B)
    table = np.full((len(ctx), int(used.max()) + pad), pin.TABLE_FILL, dtype=np.int32)
    off = 0
    for s, u in enumerate(used):
        table[s, :u] = perm[off:off + u]
        off += int(u)
    return pin.Batch(cfg, seed, B, ctx, table, used.astype(np.int32), np.sort(perm[:off]))


def _run(cfg, batch, dev, layer, split, out_dtype=torch.float32, scale=0.0):
    q = torch.from_numpy(pin.q_bits(cfg, SEED, layer).view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.full((cfg.num_seqs, cfg.num_q_heads, cfg.head_dim), float("nan"), dtype=out_dtype, device="cuda")
    P.pipelive_paged_attn_decode(dev, layer, q, out, torch.from_numpy(batch.table).cuda(),
                                 torch.from_numpy(batch.ctx_lens).cuda(), split_tokens=split, scale=scale)
    torch.cuda.synchronize()
    return out


RAGGED = [0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 0, 257, 700, 1029, 2100]


@pytest.mark.parametrize("shape", [(4, 2, 64, 16), (32, 8, 128, 16), (64, 8, 128, 16), (32, 8, 128, 32),
                                   (8, 8, 128, 16), (16, 1, 64, 32), (32, 8, 128, 64), (32, 8, 128, 128),
                                   (4, 2, 64, 128), (8, 1, 64, 64)])
@pytest.mark.parametrize("split", [0, 32, 64, 256, 1024, 4096])
def test_attention_matches_oracle(shape, split):
    Hq, Hkv, D, bs = shape
    cfg = _cfg(Hq, Hkv, D, bs, RAGGED)
    batch = _batch(cfg, RAGGED)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    for layer in range(2):
        got = _run(cfg, batch, dev, layer, split).cpu().numpy()
        ref = host.attn_decode(layer, pin.q_bits(cfg, SEED, layer), batch.table, batch.ctx_lens, nthreads=8)
        assert np.isfinite(got).all()
        assert (got[0] == 0).all()                       # ctx 0 -> zero row
        ma, rl = attn_errors(got, ref)
        assert ma <= MAX_ABS and rl <= REL_L2, (ma, rl)
        for s in range(cfg.num_seqs):                    # per sequence as well
            ma, rl = attn_errors(got[s], ref[s])
            assert ma <= MAX_ABS and rl <= REL_L2, (s, ma, rl)
    assert P.pipelive_kv_read_state(dev).status == 0


def test_single_token_is_exactly_v():
    cfg = _cfg(8, 2, 128, 16, [1, 1, 1])
    batch = _batch(cfg, [1, 1, 1])
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    got = _run(cfg, batch, dev, 0, 0).cpu().numpy()
    ref = host.attn_decode(0, pin.q_bits(cfg, SEED, 0), batch.table, batch.ctx_lens)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_placement_stride_and_split_invariance():
    ctx = [700, 33, 512, 129]
    cfg = _cfg(32, 8, 128, 16, ctx)
    a = _batch(cfg, ctx, pad=0, extra=0, seed=1)
    b = _batch(cfg, ctx, pad=11, extra=40, seed=2)      # other ids, padded table, larger pool
    outs = []
    for bt in (a, b):
        host, dev = make_pair(cfg, bt, SEED, arenas=2 if bt is a else 5)
        # same logical content at different physical ids: regenerate by logical position
        for layer in range(2):
            for s in range(cfg.num_seqs):
                for j in range(int(bt.used[s])):
                    bits = pin.kv_block_bits(cfg, SEED, 4096, 0, layer, s * 64 + j)
                    dev.write_blocks(layer, [int(bt.table[s, j])],
                                     torch.from_numpy(bits.view(np.int16)[None]).cuda())
        outs.append([_run(cfg, bt, dev, 0, sp).cpu().numpy() for sp in (128, 256)])
    assert np.array_equal(outs[0][0].view(np.uint32), outs[1][0].view(np.uint32))
    assert np.array_equal(outs[0][1].view(np.uint32), outs[1][1].view(np.uint32))
    ma, rl = attn_errors(outs[0][0], outs[0][1])         # split size changes rounding only
    assert ma < 1e-5 and rl < 1e-5


def test_bf16_output_and_scale():
    ctx = [200, 40]
    cfg = _cfg(32, 8, 128, 16, ctx)
    batch = _batch(cfg, ctx)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    ref = host.attn_decode(1, pin.q_bits(cfg, SEED, 1), batch.table, batch.ctx_lens, scale=0.05)
    got32 = _run(cfg, batch, dev, 1, 64, scale=0.05).cpu().numpy()
    ma, rl = attn_errors(got32, ref)
    assert ma <= MAX_ABS and rl <= REL_L2
    got16 = _run(cfg, batch, dev, 1, 64, out_dtype=torch.bfloat16, scale=0.05)
    expect = torch.from_numpy(got32).to(torch.bfloat16)   # round-to-nearest-even of the fp32 result
    assert torch.equal(got16.cpu(), expect)


def test_bad_table_entry_sets_status_and_touches_nothing_else():
    ctx = [100, 50]
    cfg = _cfg(4, 2, 64, 16, ctx)
    batch = _batch(cfg, ctx)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    bad = batch.table.copy()
    bad[0, 2] = batch.num_blocks + 5
    b2 = pin.Batch(cfg, SEED, batch.num_blocks, batch.ctx_lens, bad, batch.used, batch.live_ids)
    out = _run(cfg, b2, dev, 0, 64).cpu().numpy()
    assert P.pipelive_kv_read_state(dev).status == P.E_RANGE
    ref = host.attn_decode(0, pin.q_bits(cfg, SEED, 0), batch.table, batch.ctx_lens)
    assert np.abs(out[1] - ref[1]).max() < 1e-4           # the other sequence is unaffected
    assert np.isfinite(out).all()


def test_argument_errors():
    cfg = _cfg(4, 2, 64, 16, [10])
    batch = _batch(cfg, [10])
    host, dev = make_pair(cfg, batch, SEED)
    q = torch.zeros((1, 4, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((1, 4, 64), dtype=torch.float32, device="cuda")
    t = torch.from_numpy(batch.table).cuda()
    c = torch.from_numpy(batch.ctx_lens).cuda()
    assert P.pipelive_paged_attn_decode(dev, 2, q, out, t, c, check=False) == P.E_RANGE
    ws = dev.attn_workspace(1, 64, 64)
    assert P.pipelive_paged_attn_decode(dev, 0, q, out, t, c, split_tokens=100, workspace=ws, check=False) == P.E_INVAL
    assert P.pipelive_paged_attn_decode(dev, 0, q, out, t, c, split_tokens=64, workspace=ws[:16], check=False) == P.E_NOSPACE
    with pytest.raises(P.PipeliveError):
        P.KVRegion(2, 4, 2, 96, 16, 8)                     # head_dim not supported


@pytest.mark.parametrize("n_seqs", [200, 300])
def test_many_sequences_multi_chunk_scan_and_all_empty(n_seqs):
    """More than 64 sequences (the wave-wide prefix sums run in several chunks), many of them empty or a
    single token; then a batch with no tokens at all."""
    rng = np.random.default_rng(5)
    ctx = rng.integers(0, 90, n_seqs).astype(np.int32)
    ctx[::7] = 0
    ctx[3::11] = 1
    ctx[150] = 1500
    cfg = _cfg(16, 2, 128, 16, ctx.tolist())
    batch = _batch(cfg, ctx.tolist())
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    for split in (0, 32, 512):
        got = _run(cfg, batch, dev, 1, split).cpu().numpy()
        ref = host.attn_decode(1, pin.q_bits(cfg, SEED, 1), batch.table, batch.ctx_lens, nthreads=8)
        assert np.isfinite(got).all()
        ma, rl = attn_errors(got, ref)
        assert ma <= MAX_ABS and rl <= REL_L2, (split, ma, rl)
        assert (got[ctx == 0] == 0).all()
    zero = pin.Batch(cfg, SEED, batch.num_blocks, np.zeros_like(batch.ctx_lens), batch.table, batch.used, batch.live_ids)
    out = _run(cfg, zero, dev, 0, 0).cpu().numpy()
    assert (out == 0).all()
    assert P.pipelive_kv_read_state(dev).status == 0


def test_context_longer_than_max_ctx_is_truncated_and_flagged():
    ctx = [300, 40]
    cfg = _cfg(4, 2, 64, 16, ctx)
    batch = _batch(cfg, ctx)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    q = torch.from_numpy(pin.q_bits(cfg, SEED, 0).view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.full((2, 4, 64), float("nan"), dtype=torch.float32, device="cuda")
    P.pipelive_paged_attn_decode(dev, 0, q, out, torch.from_numpy(batch.table).cuda(),
                                 torch.from_numpy(batch.ctx_lens).cuda(), max_ctx=128)
    torch.cuda.synchronize()
    assert P.pipelive_kv_read_state(dev).status == P.E_RANGE
    ref = host.attn_decode(0, pin.q_bits(cfg, SEED, 0), batch.table, np.array([128, 40], dtype=np.int32))
    ma, rl = attn_errors(out.cpu().numpy(), ref)
    assert ma <= MAX_ABS and rl <= REL_L2           # sequence 0 is attended over its first 128 tokens only
