"""The asynchronous entry points (append, decode, prefill, mark, collect, apply) allocate nothing
and never synchronise, so a serving step can be captured into a HIP graph.  One decode step of
every layer plus a slot-granular patch cycle is captured once and replayed; between replays the
program does ordinary eager work (advance positions, new K/V, synchronise), and after every replay
the outputs, both pools, the patch buffer, the target pool and the counters are compared with an
eager twin that ran the same calls directly."""
import numpy as np
import pytest
import torch

import pipelive_inputs as pin
import paper_2604_12171_amd as P

pytestmark = pytest.mark.gpu


def _bits(rng, shape):
    return pin.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


class _Side:
    """source + target region, static input/output buffers of one step"""

    def __init__(self, L, Hq, Hkv, D, bs, B, S):
        gran = P.binding.DIRTY_SLOT
        self.src = P.KVRegion(L, Hq, Hkv, D, bs, B, dirty_granularity=gran, fill_bits=pin.BF16_NAN, arenas=3)
        self.tgt = P.KVRegion(L, Hq, Hkv, D, bs, B, dirty_granularity=gran, fill_bits=pin.BF16_NAN, arenas=2)
        self.k = torch.zeros((L, S, Hkv, D), dtype=torch.bfloat16, device="cuda")
        self.v = torch.zeros((L, S, Hkv, D), dtype=torch.bfloat16, device="cuda")
        self.q = torch.zeros((L, S, Hq, D), dtype=torch.bfloat16, device="cuda")
        self.out = torch.zeros((L, S, Hq, D), dtype=torch.float32, device="cuda")
        self.pf_out = torch.zeros((S, Hq, D), dtype=torch.float32, device="cuda")
        self.q_off = torch.arange(S + 1, dtype=torch.int32, device="cuda")   # one query row per sequence
        self.pos = torch.zeros(S, dtype=torch.int32, device="cuda")
        self.ctx = torch.zeros(S, dtype=torch.int32, device="cuda")
        cap = 64 + 256 + S * (4 + L * self.src.unit_bytes) + 64
        self.patch = torch.zeros(cap, dtype=torch.uint8, device="cuda")
        self.ws = self.src.attn_workspace(S, 6 * bs, 0)
        self.L = L

    def step(self, table):
        layers = list(range(self.L))
        for l in layers:
            P.pipelive_kv_append(self.src, l, self.k[l], self.v[l], table, self.pos, mark=True, count_tokens=(l == 0))
            P.pipelive_paged_attn_decode(self.src, l, self.q[l], self.out[l], table, self.ctx, max_ctx=int(table.shape[1]) * self.src.bs,
                                         workspace=self.ws)
        # the persistent prefill kernel re-arms its work counters itself: it must replay as well
        P.pipelive_paged_attn_prefill(self.src, 0, self.q[0], self.pf_out, table, self.ctx, self.q_off, self.q.shape[1],
                                      max_ctx=int(table.shape[1]) * self.src.bs)
        P.pipelive_kv_patch_collect(self.src, layers, self.patch)
        P.pipelive_kv_patch_apply(self.tgt, layers, self.patch)


def test_decode_step_and_patch_cycle_replay_from_a_graph():
    L, Hq, Hkv, D, bs, B, S = 3, 8, 2, 128, 16, 40, 5
    rng = np.random.default_rng(23)
    table = torch.from_numpy(rng.permutation(B)[: S * 6].reshape(S, 6).astype(np.int32)).cuda()
    a, b = _Side(L, Hq, Hkv, D, bs, B, S), _Side(L, Hq, Hkv, D, bs, B, S)
    live = np.sort(table.cpu().numpy().reshape(-1))
    for side in (a, b):
        side.src.set_live(live)
        side.tgt.set_live(live)

    def feed(step):
        """eager work between replays: new K/V/q, positions, context lengths"""
        k, v, q = _bits(rng, (L, S, Hkv, D)), _bits(rng, (L, S, Hkv, D)), _bits(rng, (L, S, Hq, D))
        pos = np.full(S, step, dtype=np.int32)          # every sequence appends its token number `step`
        ctx = np.full(S, step + 1, dtype=np.int32)
        for side in (a, b):
            side.k.copy_(torch.from_numpy(k.view(np.int16)).view(torch.bfloat16))
            side.v.copy_(torch.from_numpy(v.view(np.int16)).view(torch.bfloat16))
            side.q.copy_(torch.from_numpy(q.view(np.int16)).view(torch.bfloat16))
            side.pos.copy_(torch.from_numpy(pos))
            side.ctx.copy_(torch.from_numpy(ctx))

    feed(0)
    a.step(table)                                         # warm-up outside the capture (lazy module loads)
    b.step(table)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    feed(1)
    with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
        a.step(table)
    graph.replay()                                        # capture does not execute: run step 1 now
    b.step(table)
    torch.cuda.synchronize()
    for step in range(2, 9):
        feed(step)
        torch.cuda.synchronize()
        graph.replay()
        b.step(table)
        torch.cuda.synchronize()
        assert torch.equal(a.out, b.out), step
        assert torch.equal(a.pf_out, b.pf_out), step
        assert torch.allclose(a.pf_out, a.out[0], atol=1e-5, rtol=1e-5), step    # one-query prefill = decode
        assert torch.isfinite(a.out).all()
        assert torch.equal(a.patch, b.patch), step
        for l in range(L):
            assert torch.equal(a.src.read_blocks(l, live), b.src.read_blocks(l, live)), (step, l)
            assert torch.equal(a.tgt.read_blocks(l, live), b.tgt.read_blocks(l, live)), (step, l)
        assert torch.equal(a.src.dirty, b.src.dirty) and int(a.src.dirty.sum()) == 0
        sa, sb = P.pipelive_kv_read_state(a.tgt), P.pipelive_kv_read_state(b.tgt)
        assert (sa.t_applied, sa.status) == (sb.t_applied, sb.status) and sa.status == 0 and sa.t_applied > 0
        sa, sb = P.pipelive_kv_read_state(a.src), P.pipelive_kv_read_state(b.src)
        assert (sa.n_acc, sa.status) == (sb.n_acc, sb.status) == (0, 0)
    # the target holds what the source holds: the patches carried every appended token
    for l in range(L):
        assert torch.equal(a.tgt.read_blocks(l, live), a.src.read_blocks(l, live)), l
