"""The paper's worked example (Sec. 4.1: six layers on three GPUs, <[1,2],[3,4],[5,6]> ->
<[1],[2,3],[4,5,6]>) driven through Alg. 1 with the library's primitives, the three pipeline
stages simulated as three KV regions on the one GPU:

  phase 1  plan (intermediate sets, B_shrink, feasibility)            pipelive_plan_reconfig
  phase 2  every stage shrinks its pool to B_shrink                   pipelive_kv_resize
  phase 3  KV of the migrating layers streams to the stages that add them while decode steps keep
           appending tokens under the current configuration           append / collect / apply
  phase 4  stop when every destination is within tau tokens           pipelive_converged
  phase 5  commit, drop the layers of M_del, resize to B_new          pipelive_kv_resize

An oracle mirror performs every step on host regions; patches, pools, tables and counters are compared
with it, and after the commit each layer's attention on its new owner equals, bit for bit, what the old
owner computes from its own copy."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import MAX_ABS, REL_L2, assert_pools_equal, attn_errors, bitmap_ids

pytestmark = pytest.mark.gpu
SEED = 20260412
Hq, Hkv, D, bs = 8, 2, 64, 16
BLK = 2 * Hkv * bs * D * 2          # bytes of one (layer, block)
SLOT = P.binding.DIRTY_SLOT


def _bits(rng, shape):
    return pin.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def _dev16(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)


class Stage:
    """One simulated GPU: the layers of its intermediate configuration, local index = rank in that set."""

    def __init__(self, layers, B):
        self.layers = sorted(layers)
        n = len(self.layers)
        self.host = oracle.HostKV(n, Hq, Hkv, D, bs, B, dirty_gran=1, fill_bits=pin.BF16_NAN)
        self.dev = P.KVRegion(n, Hq, Hkv, D, bs, B, dirty_granularity=SLOT, fill_bits=pin.BF16_NAN, arenas=3)

    def local(self, layer):
        return self.layers.index(layer)


def test_worked_example_end_to_end():
    rng = np.random.default_rng(5)
    cur = [(0, 1), (2, 3), (4, 5)]
    tgt = [(0, 0), (1, 2), (3, 5)]
    S, B = 6, 64
    ctx = np.array([40, 7, 16, 33, 90, 1], dtype=np.int32)
    used = (ctx + bs - 1) // bs
    per_seq = 8                                              # room for 128 tokens per sequence
    table = rng.permutation(B)[: S * per_seq].reshape(S, per_seq).astype(np.int32)
    live = np.sort(table.reshape(-1))                        # the block manager reserved all of them
    n_live = len(live)                                       # 48 of 64

    # ---- phase 1: plan.  Memory figures chosen so that three layers leave room for 48 blocks
    W, util = 1.0e6, 0.9
    mem = [(48.5 * 3 * BLK + 3 * W) / util] * 3
    rc, plan, mig, dele = P.pipelive_plan_reconfig(cur, tgt, mem, util, W, float(BLK), n_live, B)
    assert rc == P.OK and plan.feasible and plan.need_shrink
    assert plan.b_shrink == 48 == oracle.max_blocks(mem[0], util, 3, W, BLK) and plan.b_new == 48
    assert sorted(mig) == [(0, 1, 1), (1, 2, 3)]             # layer 2 of the paper -> GPU 2, layer 4 -> GPU 3
    assert sorted(dele) == [(0, 1), (1, 3)]
    tmp = [set(range(a, b + 1)) | set(range(c, d + 1)) for (a, b), (c, d) in zip(cur, tgt)]
    assert tmp == [{0, 1}, {1, 2, 3}, {3, 4, 5}]             # the intermediate configuration of the text
    rc_o, po = oracle.plan_reconfig([set(range(a, b + 1)) for a, b in cur], [set(range(a, b + 1)) for a, b in tgt],
                                    6, mem, util, W, BLK, n_live, B)
    assert rc_o == oracle.OK and po["b_shrink"] == plan.b_shrink and po["tmp"] == tmp

    stages = [Stage(t, B) for t in tmp]
    owner = {l: i for i, (a, b) in enumerate(cur) for l in range(a, b + 1)}
    new_owner = {l: i for i, (a, b) in enumerate(tgt) for l in range(a, b + 1)}
    tables_h = [table.copy() for _ in stages]
    tables_d = [torch.from_numpy(table).cuda() for _ in stages]
    used_d = torch.from_numpy(used.astype(np.int32)).cuda()
    for st in stages:
        st.host.set_live(live)
        st.dev.set_live(live)
    # the cache under the current configuration: every layer on its owner
    lens = np.zeros(S, dtype=np.int32)

    sources = {m[0] for m in mig}                            # only a stage that sends KV tracks what it writes

    def decode_step(pos, count_on=None):
        """one token per sequence (pos < 0 skips) in every layer, on the layer's current owner"""
        for l in range(6):
            st = stages[owner[l]]
            k, v = _bits(rng, (S, Hkv, D)), _bits(rng, (S, Hkv, D))
            mark = owner[l] in sources
            cnt = mark and count_on is not None and l == count_on[owner[l]]
            assert st.host.append(st.local(l), k, v, tables_h[owner[l]], pos, mark=mark, count_tokens=cnt) == oracle.OK
            P.pipelive_kv_append(st.dev, st.local(l), _dev16(k), _dev16(v), tables_d[owner[l]],
                                 torch.from_numpy(pos).cuda(), mark=mark, count_tokens=cnt)

    for t in range(int(ctx.max())):                          # build the prompts token by token
        decode_step(np.where(t < ctx, t, -1).astype(np.int32))
    lens = ctx.copy()
    for st in stages:                                        # nothing is pending before the reconfiguration starts
        buf_h = np.zeros(64 + 256 + B * bs * (4 + 3 * st.host.unit_bytes), dtype=np.uint8)
        buf_d = torch.zeros(len(buf_h), dtype=torch.uint8, device="cuda")
        lay = list(range(len(st.layers)))
        assert st.host.patch_collect(lay, buf_h) == oracle.OK
        P.pipelive_kv_patch_collect(st.dev, lay, buf_d)
        st.buf_h, st.buf_d = buf_h, buf_d
    torch.cuda.synchronize()

    # ---- phase 2: every stage shrinks to B_shrink (same ids everywhere: the remaps must agree)
    remaps = []
    for i, st in enumerate(stages):
        rc_h, remap_h, res_h = st.host.resize(plan.b_shrink, [tables_h[i]], [used.astype(np.int32) * 0 + per_seq])
        remap_d = torch.full((B,), -5, dtype=torch.int32, device="cuda")
        full = torch.full((S,), per_seq, dtype=torch.int32, device="cuda")
        rc_d, res_d = P.pipelive_kv_resize(st.dev, plan.b_shrink, [tables_d[i]], [full], remap_out=remap_d)
        assert rc_h == oracle.OK and rc_d == P.OK and res_d.n_moved == int(res_h[1]) > 0
        assert np.array_equal(remap_d.cpu().numpy(), remap_h) and np.array_equal(tables_d[i].cpu().numpy(), tables_h[i])
        remaps.append(remap_h)
    assert all(np.array_equal(remaps[0], r) for r in remaps)
    live2 = np.sort(remaps[0][live])
    assert live2.max() < plan.b_shrink

    # ---- phase 3 + 4: stream the migrating layers while decode goes on under the current configuration
    count_layer = {0: 1, 1: 3, 2: 5}                         # the layer whose append counts a stage's tokens

    def pump():
        """one collect/apply per migration; bit-exact against the oracle's patches"""
        for (src, dst, layer) in sorted(mig):
            a, b = stages[src], stages[dst]
            assert a.host.patch_collect([a.local(layer)], a.buf_h) == oracle.OK
            P.pipelive_kv_patch_collect(a.dev, [a.local(layer)], a.buf_d)
            torch.cuda.synchronize()
            h = oracle.parse_patch_header(a.buf_h)
            end = h["payload_offset"] + h["n_blocks"] * a.host.unit_bytes
            assert np.array_equal(a.buf_d.cpu().numpy()[:end], a.buf_h[:end])
            assert b.host.patch_apply([b.local(layer)], a.buf_h) == oracle.OK
            P.pipelive_kv_patch_apply(b.dev, [b.local(layer)], a.buf_d)

    # round 0: everything the sources hold is dirty (the pre-copy pass)
    units = np.concatenate([np.arange(int(b) * bs, int(b) * bs + bs) for b in live2]).astype(np.int32)
    for src in sources:
        assert stages[src].host.mark_dirty(units, 0) == oracle.OK
        P.pipelive_kv_mark_dirty(stages[src].dev, torch.from_numpy(units).cuda(), 0)
    pump()
    t_sched, tau, steps = 0, S, 0
    while True:
        decode_step(lens.copy(), count_on=count_layer)       # tokens keep arriving during the migration
        lens += 1
        t_sched += S
        steps += 1
        conv_before = P.pipelive_converged(t_sched, [P.pipelive_kv_read_state(stages[d].dev).t_applied
                                                     for (_, d, _) in sorted(mig)], tau)
        assert not conv_before                               # a whole step is outstanding: S tokens, tau = S
        pump()
        applied = [P.pipelive_kv_read_state(stages[d].dev).t_applied for (_, d, _) in sorted(mig)]
        assert applied == [stages[d].host.t_applied for (_, d, _) in sorted(mig)] == [t_sched, t_sched]
        if steps == 5:
            assert P.pipelive_converged(t_sched, applied, tau)
            break
    # ---- commit: the layers run on their new owners; M_del is dropped (poisoned here to prove it is unused)
    before = {}
    for l in range(6):
        st = stages[owner[l]]
        q = _bits(rng, (S, Hq, D))
        out = torch.full((S, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
        P.pipelive_paged_attn_decode(st.dev, st.local(l), _dev16(q), out, tables_d[owner[l]], torch.from_numpy(lens).cuda())
        ref = st.host.attn_decode(st.local(l), q, tables_h[owner[l]], lens)
        ma, rl = attn_errors(out.cpu().numpy(), ref)
        assert ma <= MAX_ABS and rl <= REL_L2, (l, ma, rl)
        before[l] = (q, out.cpu().numpy())
    for (gpu, layer) in dele:
        st = stages[gpu]
        nan = torch.full((len(live2), st.dev.blk_elems), pin.BF16_NAN - 65536, dtype=torch.int16, device="cuda")
        st.dev.write_blocks(st.local(layer), live2, nan)
    for i, st in enumerate(stages):                          # phase 5: ResizeKV(B_new) everywhere
        full = torch.full((S,), per_seq, dtype=torch.int32, device="cuda")
        rc_d, res_d = P.pipelive_kv_resize(st.dev, plan.b_new, [tables_d[i]], [full])
        rc_h, _, _ = st.host.resize(plan.b_new, [tables_h[i]], [np.full(S, per_seq, np.int32)])
        assert rc_d == P.OK and rc_h == oracle.OK and res_d.n_moved == 0 and st.dev.num_blocks == plan.b_new
    for l in range(6):                                       # every layer on its new owner, same bits as before
        st = stages[new_owner[l]]
        q, prev = before[l]
        out = torch.full((S, Hq, D), float("nan"), dtype=torch.float32, device="cuda")
        P.pipelive_paged_attn_decode(st.dev, st.local(l), _dev16(q), out, tables_d[new_owner[l]],
                                     torch.from_numpy(lens).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint32), prev.view(np.uint32)), l
        assert P.pipelive_kv_read_state(st.dev).status == 0
    for (src, dst, layer) in mig:                            # the migrated layers, byte for byte, and the oracle's
        a, b = stages[src], stages[dst]
        assert_pools_equal(b.host, b.dev, [b.local(layer)], live2)
