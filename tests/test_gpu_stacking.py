"""Layer stacking (paper Sec. 5.2): k layers share one physical block; layer l
lives at byte offset (l mod k) * blk of block_list[l / k][id].  Attention,
resize (which moves whole physical blocks) and patching (which addresses one
layer's part) are checked against the oracle for k = 2 and k = 4."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import MAX_ABS, REL_L2, assert_pools_equal, attn_errors, bitmap_ids, fill_pair, make_pair

pytestmark = pytest.mark.gpu
SEED = 4242


@pytest.mark.parametrize("stack_k,layers", [(2, 4), (4, 8), (4, 6)])
def test_stacked_region_matches_oracle(stack_k, layers):
    cfg = pin.StageConfig("stacked", layers, 8, 2, 128, 16, 6, 1, 400)
    batch = pin.draw_batch(cfg, SEED, pool_factor=1.6)
    B = batch.num_blocks
    host, dev = make_pair(cfg, batch, SEED, stack_k=stack_k)
    assert dev.groups == (layers + stack_k - 1) // stack_k == host.groups
    fill_pair(cfg, batch, SEED, host, dev)
    table_h = batch.table.copy()
    table_d = torch.from_numpy(batch.table).cuda()
    ctx_d = torch.from_numpy(batch.ctx_lens).cuda()
    used_d = torch.from_numpy(batch.used).cuda()

    def decode(layer):
        q = torch.from_numpy(pin.q_bits(cfg, SEED, layer).view(np.int16)).cuda().view(torch.bfloat16)
        out = torch.full((cfg.num_seqs, cfg.num_q_heads, cfg.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        P.pipelive_paged_attn_decode(dev, layer, q, out, table_d, ctx_d)
        return out.cpu().numpy()

    before = []
    for layer in range(layers):
        got = decode(layer)
        ref = host.attn_decode(layer, pin.q_bits(cfg, SEED, layer), table_h, batch.ctx_lens)
        ma, rl = attn_errors(got, ref)
        assert ma <= MAX_ABS and rl <= REL_L2, (layer, ma, rl)
        before.append(got)

    # shrink: physical blocks (all k layers of a group) move together
    n_live = len(batch.live_ids)
    B_new = n_live + 2
    rc_h, remap_h, res_h = host.resize(B_new, [table_h], [batch.used])
    remap_d = torch.zeros(B, dtype=torch.int32, device="cuda")
    rc_d, res_d = P.pipelive_kv_resize(dev, B_new, [table_d], [used_d], remap_out=remap_d)
    assert rc_h == oracle.OK == rc_d and res_d.n_moved == res_h[1] > 0
    assert np.array_equal(remap_d.cpu().numpy(), remap_h) and np.array_equal(table_d.cpu().numpy(), table_h)
    assert_pools_equal(host, dev, range(layers), range(B_new))
    for layer in range(layers):
        assert np.array_equal(decode(layer).view(np.uint32), before[layer].view(np.uint32))

    # patch two layers that share a physical block with layers that do not migrate
    src_layers = [layers - 1, 1]
    tgt_h = oracle.HostKV(2, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B_new,
                          stack_k=2, fill_bits=pin.BF16_NAN)
    tgt_d = P.KVRegion(2, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B_new,
                       stack_k=2, fill_bits=pin.BF16_NAN)
    live = host.live_ids()
    cap = 64 + 256 + len(live) * (4 + 2 * host.blk_bytes)
    patch_h = np.zeros(cap, dtype=np.uint8)
    patch_d = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    host.mark_dirty(live, 3)
    P.pipelive_kv_mark_dirty(dev, torch.from_numpy(live.astype(np.int32)).cuda(), 3)
    assert host.patch_collect(src_layers, patch_h) == oracle.OK
    P.pipelive_kv_patch_collect(dev, src_layers, patch_d)
    h = oracle.parse_patch_header(patch_h)
    end = h["payload_offset"] + h["n_blocks"] * 2 * host.blk_bytes
    g = patch_d.cpu().numpy()
    assert np.array_equal(g[:64 + 4 * h["n_blocks"]], patch_h[:64 + 4 * h["n_blocks"]])
    assert np.array_equal(g[h["payload_offset"]:end], patch_h[h["payload_offset"]:end])
    assert tgt_h.patch_apply([1, 0], patch_h) == oracle.OK
    P.pipelive_kv_patch_apply(tgt_d, [1, 0], patch_d)
    assert_pools_equal(tgt_h, tgt_d, range(2), range(B_new))
    assert_pools_equal(host, dev, range(layers), range(B_new))     # the source is untouched
    assert P.pipelive_kv_read_state(tgt_d).t_applied == 3
    assert len(bitmap_ids(dev.dirty, B_new)) == 0
