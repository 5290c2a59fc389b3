"""GPU parity of chunked-prefill paged attention against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import MAX_ABS, REL_L2, attn_errors, fill_pair, make_pair

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
                                   (8, 8, 64, 32), (6, 2, 128, 16), (32, 8, 128, 128), (4, 2, 64, 64)])
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
    assert torch.equal(h.cpu(), a.cpu().to(torch.bfloat16))


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
