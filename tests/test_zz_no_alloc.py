"""The decode entry point that allocates nothing, through the C ABI: same result, bit for bit, as
pipelive_paged_attn_decode with a caller's workspace; two calls in a row on the one built-in scratch
buffer, the second on a smaller input; a launch shape that does not fit is refused."""
import numpy as np
import pytest
import torch

import pipelive_inputs as pin
import paper_2604_12171_amd as P
from pipelive_inputs.device_fill import fill_live_blocks

pytestmark = pytest.mark.gpu
SEED = pin.MASTER_SEED


def _case(cfg, pool_factor):
    batch = pin.draw_batch(cfg, SEED, pool_factor=pool_factor)
    region = P.KVRegion(cfg.num_layers, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens,
                        batch.num_blocks, arenas=3)
    fill_live_blocks(region, cfg, batch, SEED, batch.num_blocks, poison_tail=True)
    table = torch.from_numpy(batch.table).cuda()
    ctx = torch.from_numpy(batch.ctx_lens).cuda()
    q = torch.from_numpy(pin.q_bits(cfg, SEED, 0).view(np.int16)).cuda().view(torch.bfloat16)
    return batch, region, table, ctx, q


def _both(case, layer, split):
    batch, region, table, ctx, q = case
    cfg = batch.cfg
    shape = (cfg.num_seqs, cfg.num_q_heads, cfg.head_dim)
    mc = int(batch.ctx_lens.max())
    ref = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    P.pipelive_paged_attn_decode(region, layer, q, ref, table, ctx, max_ctx=mc, split_tokens=split)
    P.pipelive_paged_attn_decode_noalloc(region, layer, q, got, table, ctx, max_ctx=mc, split_tokens=split)
    torch.cuda.synchronize()
    assert torch.isfinite(ref).all()
    assert torch.equal(ref.view(torch.int32), got.view(torch.int32))
    return got


def test_decode_without_allocation_matches_the_workspace_entry_point():
    big = _case(pin.scaled(pin.CONFIGS["stage70b"], num_layers=2, num_seqs=24, ctx_lo=700, ctx_hi=3000), 1.2)
    small = _case(pin.scaled(pin.CONFIGS["stage8b"], num_layers=1, num_seqs=5, ctx_lo=1, ctx_hi=300), 1.5)
    assert P.load().pipelive_noalloc_scratch_bytes() == 16 << 20
    for split in (0, 1024):
        _both(big, 1, split)          # first call: many cut pairs, records all over the scratch buffer
        _both(small, 0, split)        # second call, smaller: must not be disturbed by what the first left behind
        _both(big, 0, split)
    # device memory in use does not move across calls (outputs allocated beforehand)
    batch, region, table, ctx, q = big
    out = torch.zeros((batch.cfg.num_seqs, batch.cfg.num_q_heads, batch.cfg.head_dim), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    for layer in (0, 1, 0):
        P.pipelive_paged_attn_decode_noalloc(region, layer, q, out, table, ctx, max_ctx=int(batch.ctx_lens.max()))
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0
    assert P.pipelive_kv_read_state(big[1]).status == 0 and P.pipelive_kv_read_state(small[1]).status == 0
    # a launch shape whose records do not fit the built-in buffer is refused, nothing is launched
    out.zero_()
    need = P.load().pipelive_paged_attn_workspace_bytes(region.handle, batch.cfg.num_seqs, int(batch.ctx_lens.max()), 32)
    assert need > 16 << 20
    rc = P.pipelive_paged_attn_decode_noalloc(region, 0, q, out, table, ctx, max_ctx=int(batch.ctx_lens.max()),
                                              split_tokens=32, check=False)
    assert rc == P.E_NOSPACE and not out.any()
