#!/usr/bin/env python3
"""Benchmark of the PipeLive hot path on one MI355X.

Headline workload: the Llama-3-70B-shaped pipeline stage (20 layers, 64 query /
8 KV heads, head_dim 128, 16-token blocks, bf16, 128 sequences with context
lengths uniform in [1024, 8192]) - the largest of the five workload shapes.
One *step* is one pass of the whole hot path over that batch:

  1. decode attention over all layers (one launch per layer, own q per layer),
  2. one patch cycle: mark every sequence's last block dirty, collect
     (drain + gather) the dirty blocks of all layers into the patch buffer,
     apply (scatter) them into the target region,
  3. ResizeKV: shrink the pool by 20 % (plan, move, remap) - followed by a
     restore (grow back + reset of table and live bitmap, no bytes counted) so
     that every step performs the same moves.

`value` is the algorithmic bytes of the whole step divided by the step time;
`roofline` is the decode-attention launch against the 8 TB/s HBM peak;
`cpu_baseline` is the CPU oracle timed on the host cores on a bounded sample.

After the timed steps the same run executes, once each, the procedure of every
workload shape (object `configs`): the six patch rounds of the 70B stage with
the dirty fraction decaying from 20 % to 1 %, the 8B stage (decode, patch
cycle, shrink, bulk patch, slot-granular patches, prefill, stacked per-block
pool), the resize stress (tight pool, shrink - decode with appends - grow -
shrink), the long-context stage (split decode, 25 % shrink, 2 % patch round)
and the tiny shape (checked byte for byte against the oracle).

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak
MFMA_PEAK_TFLOPS = 2500.0
HEADLINE = "stage70b"
ALL_CONFIGS = ["stage70b", "stage8b", "resize8b", "longctx8b", "tiny"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="all",
                    help="'all' (headline on stage70b, then every workload's procedure) or one workload name, "
                         "which then carries the headline")
    ap.add_argument("--split-tokens", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=1, help="layers in the CPU oracle's attention sample")
    ap.add_argument("--decode-only", action="store_true",
                    help="profiling aid: the steps run decode attention only, followed by one plain copy of known size")
    ap.add_argument("--prefill-only", action="store_true",
                    help="profiling aid: run only the prefill cases of the 8B stage's heads")
    ap.add_argument("--prefill-case", default="both", choices=["both", "prompt512", "chunk512_of_4096"],
                    help="with --prefill-only: which of the two cases")
    ap.add_argument("--decode-iters", type=int, default=50)
    ap.add_argument("--arena-gib", type=int, default=-1,
                    help="size of the region-aware arena the pools and patch buffers are carved out of "
                         "(-1: the free device memory less --arena-reserve-gib; 0: no arena, torch allocations)")
    ap.add_argument("--arena-reserve-gib", type=int, default=20,
                    help="device memory left outside the arena (tables, queries, workspaces, the stacked pool)")
    ap.add_argument("--arena-piece-mib", type=int, default=64, help="piece size of the arena")
    ap.add_argument("--arena-settle-s", type=int, default=24,
                    help="longest pause (in steps of 12 s, memory released meanwhile) before the arena is taken again "
                         "when the driver's hand-out is mixed, as it is right after another process's exit; 0: never")
    ap.add_argument("--arena-probe-mib", type=int, default=1024, help="size of the stretches the arena's probe times")
    ap.add_argument("--core-only", action="store_true",
                    help="profiling aid: skip the legs outside decode, patch and resize (slot patches, prefill, "
                         "stacked pool, 4-layer rounds, sparse pool)")
    return ap.parse_args()


def stage_weight_bytes(cfg) -> int:
    """fp16 weights of the stage's layers (Llama shapes: hidden = Hq*D, 3.5x MLP)."""
    hidden = cfg.num_q_heads * cfg.head_dim
    kvdim = cfg.num_kv_heads * cfg.head_dim
    inter = {4096: 14336, 8192: 28672}.get(hidden, 4 * hidden)
    per_layer = hidden * hidden * 2 + 2 * hidden * kvdim + 3 * hidden * inter
    return 2 * per_layer * cfg.num_layers


def read_traffic(kernel_tag: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if any."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].strip())
    except OSError:
        pass
    return None


def stats(ms_list):
    v = sorted(ms_list)
    return sum(v) / len(v), v[len(v) // 2], v[0]


class Ctx:
    """imports and small helpers shared by the legs"""

    def __init__(self, args):
        import numpy as np
        import torch
        import pipelive_inputs as pin
        from pipelive_inputs.device_fill import fill_live_blocks
        import paper_2604_12171_amd as P
        self.np, self.torch, self.pin, self.P, self.fill = np, torch, pin, P, fill_live_blocks
        self.args = args
        self.seed = pin.MASTER_SEED
        self.dev_name = torch.cuda.get_device_name(0)

    def ev(self):
        return self.torch.cuda.Event(enable_timing=True)

    def sync(self):
        self.torch.cuda.synchronize()

    def free_all(self):
        import gc
        gc.collect()
        self.torch.cuda.empty_cache()

    # ---- Placement: pools and patch buffers are carved out of one region-aware arena (pieces of 64 MiB that
    # the library sorts by the region of the device memory they lie in).  The KV blocks of a layer go into one
    # region, consecutive layers into different ones: a decode launch then reads one region, and the copies,
    # which work on all layers at once, use all of them.  Patch buffers go into the spread zone, whose pieces
    # take the regions in turn.  (--arena-gib 0: every buffer is a torch allocation of its own.)
    arena = None

    def arena_open(self):
        gib = int(self.args.arena_gib)
        if gib == 0:
            return {"arena_GiB": 0}
        free_b = self.torch.cuda.mem_get_info()[0]
        if gib < 0:
            gib = max(1, (free_b >> 30) - int(self.args.arena_reserve_gib))
        # A process that starts within seconds of another one's exit is handed memory in which the regions
        # alternate at a grain finer than the probe resolves (it then sees hundreds of runs of equal class instead of a handful) and
        # which no placement can sort out; about ten seconds after the last big release the driver hands out
        # region by region again.  So: if the hand-out looks mixed, give the memory back, wait and take it again.
        waited = 0
        while True:
            try:
                self.arena = self.P.Arena(gib << 30, piece_bytes=int(self.args.arena_piece_mib) << 20,
                                          probe_bytes=int(self.args.arena_probe_mib) << 20)
            except self.P.PipeliveError as e:   # placement only: the run goes on with torch allocations
                log(f"[arena] not created ({e}); torch allocations instead")
                return {"arena_GiB": 0, "note": f"arena of {gib} GiB could not be created: {e}"}
            info = self.arena.info()
            n_stretches = info["n_pieces"] * int(self.args.arena_piece_mib) // int(self.args.arena_probe_mib)
            if info["n_runs"] <= max(8, n_stretches // 8) or waited + 12 > int(self.args.arena_settle_s):
                break
            log(f"[arena] mixed hand-out ({info['n_runs']} runs of equal class in {info['n_pieces']} pieces): "
                f"memory released, 12 s pause, then taken again")
            self.arena.close()
            self.arena = None
            time.sleep(12)
            waited += 12
        info = self.arena.info()
        log(f"[arena] {gib} GiB in {info['n_pieces']} pieces, classes {info['class_pieces']} in {info['n_runs']} runs, probe {info['probe_ms']:.0f} ms, "
            f"pair copy {info['rate_same_GBps']:.0f} (same region) / {info['rate_other_GBps']:.0f} GB/s")
        return {"arena_GiB": gib, "piece_MiB": int(self.args.arena_piece_mib), "probe_MiB": int(self.args.arena_probe_mib), **info,
                "settle_s": waited,
                "policy": "layer l of a pool in region l mod n_classes; patch buffers in the spread zone"}

    def arena_layout(self, spread_bytes):
        """start of a workload: nothing carved out of the arena is in use any more; `spread_bytes` of it
        (plus a margin) become the spread zone, the rest the per-region zones"""
        if self.arena is not None:
            self.sync()
            self.arena.layout(int(spread_bytes) + (256 << 20))

    def alloc(self, numel, dtype, group=None):
        """1-D device tensor for a large buffer: the arenas of a pool's layer group from a region zone, anything
        else from the spread zone; a torch allocation when there is no arena or it has no room"""
        if self.arena is not None:
            try:
                if group is None:
                    return self.arena.empty(numel, dtype)
                return self.arena.empty_in_class(numel, dtype, prefer=group)
            except self.P.PipeliveError:
                pass
        return self.torch.empty(int(numel), dtype=dtype, device="cuda")

    def big_u8(self, n):
        return self.alloc(n, self.torch.uint8)

    def placer(self, arenas_per_layer):
        """allocator for a pool: all arenas of a layer in one region zone (None without an arena)"""
        if self.arena is None:
            return None
        inner = self.arena.placer(arenas_per_layer)

        def alloc(numel, dtype, group):
            try:
                return inner(numel, dtype, group)
            except self.P.PipeliveError:
                return self.torch.empty(int(numel), dtype=dtype, device="cuda")
        return alloc

    def free_bytes(self):
        """(memory the workload definitions count as free, memory a pool can really take): without an arena both
        are the device's free memory; with one, the first adds what the arena has left and the second is that"""
        free_b = self.torch.cuda.mem_get_info()[0]
        if self.arena is None:
            return free_b, free_b
        room = self.arena.total_room()
        return free_b + room, room


class Stage:
    """Device side of one workload: region, batch, tables, per-layer q and outputs."""

    def __init__(self, c: Ctx, cfg, B, arenas=4, stride_pad=0, capacity=None, poison=True):
        np, torch, pin, P = c.np, c.torch, c.pin, c.P
        self.c, self.cfg, self.B = c, cfg, int(B)
        self.cap = int(capacity or B)
        L, S = cfg.num_layers, cfg.num_seqs
        t0 = time.time()
        self.region = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens,
                                 self.B, capacity_blocks=self.cap, arenas=arenas, allocator=c.placer(arenas))
        self.batch = pin.draw_batch(cfg, c.seed, num_blocks=self.B, stride_pad=stride_pad)
        c.fill(self.region, cfg, self.batch, c.seed, self.cap, poison_tail=poison)
        c.sync()
        self.n_live = len(self.batch.live_ids)
        log(f"[{cfg.name}] pool {self.B} blocks/layer x {L} layers = {self.B * L * cfg.blk_bytes / 2**30:.1f} GiB, "
            f"live {self.n_live} blocks/layer, tokens {self.batch.total_tokens}, filled in {time.time() - t0:.1f}s")
        self.table = torch.from_numpy(self.batch.table).cuda()
        self.table_saved = self.table.clone()
        self.ctx = torch.from_numpy(self.batch.ctx_lens).cuda()
        self.used = torch.from_numpy(self.batch.used).cuda()
        self.live_saved = self.region.live.clone()
        self.max_ctx = int(self.batch.ctx_lens.max())
        self.split = c.args.split_tokens
        self.ws = self.region.attn_workspace(S, self.max_ctx + 64, self.split)
        self.qs = [torch.from_numpy(pin.q_bits(cfg, c.seed, l).view(np.int16)).cuda().view(torch.bfloat16)
                   for l in range(L)]
        self.outs = [torch.empty((S, cfg.num_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
                     for _ in range(L)]
        self.rws = self.region.resize_workspace()
        self.set_tokens(self.batch.total_tokens, int(self.batch.used.sum()))

    def set_tokens(self, tokens, table_entries):
        cfg = self.cfg
        S = cfg.num_seqs
        self.tokens = int(tokens)
        self.q_bytes = S * cfg.num_q_heads * cfg.head_dim * 2
        self.out_bytes = S * cfg.num_q_heads * cfg.head_dim * 4
        self.attn_bytes_layer = self.tokens * cfg.token_bytes + self.q_bytes + self.out_bytes + 4 * int(table_entries)

    def decode_pass(self, max_ctx=None):
        P = self.c.P
        for l in range(self.cfg.num_layers):
            P.pipelive_paged_attn_decode(self.region, l, self.qs[l], self.outs[l], self.table, self.ctx,
                                         max_ctx=max_ctx or self.max_ctx, split_tokens=self.split, workspace=self.ws)

    def time_decode(self, warm, iters, max_ctx=None):
        c = self.c
        for _ in range(warm):
            self.decode_pass(max_ctx)
        evs = [(c.ev(), c.ev()) for _ in range(iters)]
        for a, b in evs:
            a.record()
            self.decode_pass(max_ctx)
            b.record()
        c.sync()
        avg, med, mn = stats([a.elapsed_time(b) for a, b in evs])
        L = self.cfg.num_layers
        bytes_pass = self.attn_bytes_layer * L
        return {"GBps": round(bytes_pass / avg / 1e6, 1), "frac_of_peak": round(bytes_pass / avg / 1e6 / HBM_PEAK_GBPS, 4),
                "ms_avg": round(avg, 4), "ms_median": round(med, 4), "ms_min": round(mn, 4),
                "us_per_launch": round(avg * 1e3 / L, 2), "bytes_per_launch": int(self.attn_bytes_layer),
                "launches_per_pass": L, "timing": f"{warm} warm-up + {iters} timed passes over all layers",
                "traffic_bytes_per_launch": read_traffic(f"attn_decode_{self.cfg.name}")}

    def shrink(self, B_new):
        P = self.c.P
        rc, res = P.pipelive_kv_resize(self.region, B_new, [self.table], [self.used], workspace=self.rws)
        if rc != P.OK:
            raise RuntimeError(f"[{self.cfg.name}] resize to {B_new} failed: rc={rc}")
        return res

    def restore(self, B):
        P = self.c.P
        rc, _ = P.pipelive_kv_resize(self.region, B, [], [], workspace=self.rws)
        if rc != P.OK:
            raise RuntimeError(f"[{self.cfg.name}] grow failed: {rc}")
        self.table.copy_(self.table_saved)
        self.region.live.copy_(self.live_saved)

    def time_shrink(self, B_new, iters, warm=2):
        """shrink B -> B_new (plan, table check, move, finish) timed by events; restore untimed"""
        c, cfg = self.c, self.cfg
        n_moved_expect = int((self.batch.live_ids >= B_new).sum())
        ts = []
        for it in range(warm + iters):
            e0, e1 = c.ev(), c.ev()
            e0.record()
            res = self.shrink(B_new)
            e1.record()
            if res.n_moved != n_moved_expect:
                raise RuntimeError(f"moved {res.n_moved}, expected {n_moved_expect}")
            self.restore(self.B)
            c.sync()
            if it >= warm:
                ts.append(e0.elapsed_time(e1))
        avg, med, mn = stats(ts)
        nbytes = 2 * n_moved_expect * cfg.num_layers * cfg.blk_bytes
        return {"from": self.B, "to": int(B_new), "n_moved": n_moved_expect, "bytes": int(nbytes),
                "us": round(med * 1e3, 1), "us_avg": round(avg * 1e3, 1), "us_min": round(mn * 1e3, 1),
                "GBps": round(nbytes / med / 1e6, 1), "frac_of_peak": round(nbytes / med / 1e6 / HBM_PEAK_GBPS, 4),
                "timing": f"median of {iters} (whole call: plan, table check, move, table + bitmap update; one host wait on the plan)"}

    def status_ok(self):
        return self.c.P.pipelive_kv_read_state(self.region).status == 0


def parse_hdr(c: Ctx, hdr_tensor):
    """the 64-byte patch header (pinned host copy) as the binding's ctypes struct"""
    return c.P.binding.PatchHdr.from_buffer_copy(hdr_tensor.numpy().tobytes())


def patch_capacity(n_blocks, n_layers, blk_bytes):
    return 64 + 256 + int(n_blocks) * (4 + n_layers * blk_bytes) + 4096


def time_patch_round(c: Ctx, src, tgt, ids32, n_tokens, layers, patch, dst_map, reps, blk_bytes, B):
    """mark -> collect -> apply, once for real (first_*), then `reps` repeats with the same set re-marked
    (apply is idempotent); medians of the repeats"""
    P, torch = c.P, c.torch
    hdr = torch.zeros(64, dtype=torch.uint8).pin_memory()
    tc, ta = [], []
    first = None
    for it in range(reps + 1):
        P.pipelive_kv_mark_dirty(src, ids32, n_tokens if it == 0 else 0)
        e0, e1, e2 = c.ev(), c.ev(), c.ev()
        e0.record()
        P.pipelive_kv_patch_collect(src, layers, patch, hdr_host=hdr if it == 0 else None)
        e1.record()
        P.pipelive_kv_patch_apply(tgt, layers, patch, dst_block_map=dst_map)
        e2.record()
        c.sync()
        if it == 0:
            h = parse_hdr(c, hdr)
            if h.more_pending:
                raise RuntimeError("patch buffer too small for the round")
            nb = int(h.n_blocks)
            first = (e0.elapsed_time(e1), e1.elapsed_time(e2))
            if nb != ids32.numel():   # appends had marked blocks beside the sample: re-mark what the drain listed
                ids32 = patch[64:64 + 4 * nb].view(torch.int32).clone()
        else:
            tc.append(e0.elapsed_time(e1))
            ta.append(e1.elapsed_time(e2))
    payload = nb * len(layers) * blk_bytes
    tcm, tam = stats(tc)[1], stats(ta)[1]
    cb, ab = 2 * payload + 2 * (B // 8), 2 * payload
    return {"dirty_blocks": int(nb), "layers": len(layers), "payload_bytes": int(payload),
            "collect_us": round(tcm * 1e3, 1), "collect_GBps": round(cb / tcm / 1e6, 1),
            "collect_frac_of_peak": round(cb / tcm / 1e6 / HBM_PEAK_GBPS, 4),
            "apply_us": round(tam * 1e3, 1), "apply_GBps": round(ab / tam / 1e6, 1),
            "apply_frac_of_peak": round(ab / tam / 1e6 / HBM_PEAK_GBPS, 4),
            "first_collect_us": round(first[0] * 1e3, 1), "first_apply_us": round(first[1] * 1e3, 1),
            "timing": f"median of {reps} repeats (same dirty set re-marked); first_* = the round itself, single shot"}


def decode_step_with_appends(c: Ctx, st: Stage, bm, step_idx, count_layer=0, mark=True, attend=False):
    """One decode step: the block manager hands out slots, every layer appends its token (fused dirty
    mark) and, if `attend`, runs decode attention over the grown context."""
    torch, pin, P, np = c.torch, c.pin, c.P, c.np
    cfg = st.cfg
    pos, new_entries = bm.step()
    for s, col, b in new_entries:
        st.table[s, col] = b
    if new_entries:
        st.region.set_live(bm.live_ids())
        st.used.copy_(torch.from_numpy(bm.used))
    pos_d = torch.from_numpy(pos).cuda()
    n = cfg.num_seqs * cfg.num_kv_heads * cfg.head_dim
    key = pin.stream_key(c.seed, pin.STREAM_NEWTOK)
    shape = (cfg.num_seqs, cfg.num_kv_heads, cfg.head_dim)
    st.ctx.copy_(torch.from_numpy(bm.ctx))
    mc = int(bm.ctx.max())
    for l in range(cfg.num_layers):
        base = (step_idx * cfg.num_layers + l) * 2 * n
        k = pin.bf16_normal_torch(key, base, n, "cuda").view(torch.bfloat16).view(shape)
        v = pin.bf16_normal_torch(key, base + n, n, "cuda").view(torch.bfloat16).view(shape)
        P.pipelive_kv_append(st.region, l, k, v, st.table, pos_d, mark=mark, count_tokens=(l == count_layer))
        if attend:
            P.pipelive_paged_attn_decode(st.region, l, st.qs[l], st.outs[l], st.table, st.ctx, max_ctx=mc,
                                         split_tokens=st.split, workspace=st.ws)
    return mc


# --------------------------------------------------------------------------- workloads

def run_stage70b(c: Ctx, headline: bool):
    """Workload 4.  Source and target pools of ceil(1.25 n_live) blocks per layer."""
    np, torch, pin, P, args = c.np, c.torch, c.pin, c.P, c.args
    cfg = pin.CONFIGS["stage70b"]
    L, S = cfg.num_layers, cfg.num_seqs
    ctx = pin.draw_ctx_lens(cfg, c.seed)
    n_live = int(((ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens).sum())
    B = int(math.ceil(1.25 * n_live))
    c.arena_layout(0 if args.decode_only else patch_capacity(int(0.21 * n_live) + S + 8, L, cfg.blk_bytes))
    st = Stage(c, cfg, B, arenas=4, stride_pad=2)
    res = {"workload": _wl_name(cfg), "pool_blocks_per_layer": B, "pool_GiB": round(B * L * cfg.blk_bytes / 2**30, 1),
           "live_blocks_per_layer": n_live, "tokens": st.tokens}
    head = None
    if args.decode_only:
        head = timed_steps(c, st, None, None, None, None, decode_only=True)
        res["decode"] = head["decode"]
        return res, head, st
    tgt = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B, arenas=3,
                     allocator=c.placer(3))
    fr = pin.geometric_fractions(0.20, 0.01, 6)
    n_r1 = len(pin.draw_dirty_ids(st.batch, c.seed, 1, fr[0]))
    layers = list(range(L))
    patch = c.big_u8(patch_capacity(n_r1 + S + 8, L, cfg.blk_bytes))
    B_new = int(B * 0.8)
    if headline:
        head = timed_steps(c, st, tgt, layers, patch, B_new)
        res.update({k: head[k] for k in ("decode", "patch", "resize", "switch_us")})
        maybe_cpu_baseline(c, st, head)
    else:
        res["decode"] = st.time_decode(10, args.decode_iters)
        res["resize"] = st.time_shrink(B_new, 10)

    # ---- the migration: round 0 (pre-copy of every live block, in as many drains as the buffer sized for
    # patch round 1 needs), then six patch rounds; between rounds every sequence decodes one token (append in every
    # layer, fused dirty mark) and a seeded sample of live blocks is rewritten-and-marked
    bm = pin.BlockManager(st.batch, B)
    t_applied0 = P.pipelive_kv_read_state(tgt).t_applied
    hdr = torch.zeros(64, dtype=torch.uint8).pin_memory()
    live32 = torch.from_numpy(st.batch.live_ids.astype(np.int32)).cuda()
    P.pipelive_kv_mark_dirty(st.region, live32, 0)
    e0, e1 = c.ev(), c.ev()
    drains, blocks0 = 0, 0
    e0.record()
    while True:
        P.pipelive_kv_patch_collect(st.region, layers, patch, hdr_host=hdr)
        P.pipelive_kv_patch_apply(tgt, layers, patch)
        c.sync()
        h = parse_hdr(c, hdr)
        drains += 1
        blocks0 += int(h.n_blocks)
        if not h.more_pending:
            break
    e1.record()
    c.sync()
    ms0 = e0.elapsed_time(e1)
    pay0 = blocks0 * L * cfg.blk_bytes
    res["round0"] = {"dirty_blocks": blocks0, "drains": drains, "payload_bytes": int(pay0), "ms": round(ms0, 3),
                     "collect_plus_apply_GBps": round(4 * pay0 / ms0 / 1e6, 1),
                     "note": "buffer sized for patch round 1, so the pre-copy takes several clipped drains with a host "
                             "read of the header between them"}
    rounds, sched = [], 0
    for r in range(1, 7):
        decode_step_with_appends(c, st, bm, r)
        sched += S
        sample = pin.draw_dirty_ids(st.batch, c.seed, r, fr[r - 1], include_last=False)
        ids32 = torch.from_numpy(sample.astype(np.int32)).cuda()
        out = time_patch_round(c, st.region, tgt, ids32, 0, layers, patch, None, 5, cfg.blk_bytes, B)
        out["round"] = r
        out["dirty_fraction_of_live"] = round(out["dirty_blocks"] / n_live, 4)
        rounds.append(out)
    stt = P.pipelive_kv_read_state(tgt)
    if stt.t_applied - t_applied0 != sched or stt.status != 0 or not st.status_ok():
        raise RuntimeError(f"stage70b migration: t_applied grew by {stt.t_applied - t_applied0}, scheduled {sched}, "
                           f"or status set")
    live_now = bm.live_ids()
    for l in (0, L // 2, L - 1):   # the migrated state: target == source on every live block of sampled layers
        if not torch.equal(tgt.read_blocks(l, live_now), st.region.read_blocks(l, live_now)):
            raise RuntimeError(f"stage70b: target differs from source in layer {l}")
    res["patch_rounds"] = rounds
    res["switch_us"] = round(rounds[-1]["collect_us"] + rounds[-1]["apply_us"], 1)
    res["switch_note"] = "collect + apply of the final (1 %) round, all 20 layers"
    # ---- the same decay with 4 migrating layers (secondary)
    lay4 = list(range(L - 4, L))
    r4 = []
    for r in (() if args.core_only else (1, 6)):
        sample = pin.draw_dirty_ids(st.batch, c.seed, r, fr[r - 1], include_last=True)
        ids32 = torch.from_numpy(sample.astype(np.int32)).cuda()
        out = time_patch_round(c, st.region, tgt, ids32, 0, lay4, patch, None, 5, cfg.blk_bytes, B)
        out["round"] = r
        r4.append(out)
    res["patch_rounds_4_layers"] = r4
    del tgt, patch
    return res, head, st


def timed_steps(c: Ctx, st: Stage, tgt, mig_layers, patch, B_new, decode_only=False, dst_map=None):
    """The headline loop: W warm-up + K timed steps of the whole hot path on `st`."""
    P, torch, np, pin, args = c.P, c.torch, c.np, c.pin, c.args
    cfg = st.cfg
    L, S = cfg.num_layers, cfg.num_seqs
    B = st.B
    if not decode_only:
        last_ids = torch.from_numpy(pin.last_block_ids(st.batch).astype(np.int32)).cuda()
        n_dirty = int(last_ids.numel())
        n_moved_expect = int((st.batch.live_ids >= B_new).sum())
        Lm = len(mig_layers)
    decode_bytes = st.attn_bytes_layer * L
    if decode_only:
        step_bytes = decode_bytes
    else:
        payload = n_dirty * Lm * cfg.blk_bytes
        collect_bytes = 2 * payload + 2 * (B // 8)
        apply_bytes = 2 * payload
        resize_bytes = 2 * n_moved_expect * L * cfg.blk_bytes
        step_bytes = decode_bytes + collect_bytes + apply_bytes + resize_bytes

    def one_step(events=None):
        if events:
            events[0].record()
        st.decode_pass()
        if events:
            events[1].record()
        if decode_only:
            return
        P.pipelive_kv_mark_dirty(st.region, last_ids, S)
        P.pipelive_kv_patch_collect(st.region, mig_layers, patch)
        if events:
            events[2].record()
        P.pipelive_kv_patch_apply(tgt, mig_layers, patch, dst_block_map=dst_map)
        if events:
            events[3].record()
        r = st.shrink(B_new)
        if r.n_moved != n_moved_expect:
            raise RuntimeError(f"resize moved {r.n_moved}, expected {n_moved_expect}")
        if events:
            events[4].record()
        st.restore(B)

    for _ in range(args.warmup):
        one_step()
    c.sync()
    all_events = [[c.ev() for _ in range(5)] for _ in range(args.steps)]
    c.sync()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(all_events[k])
    c.sync()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    def phase(a, b):
        return stats([e[a].elapsed_time(e[b]) for e in all_events])

    dec_avg, dec_med, dec_min = phase(0, 1)
    launch_us = dec_avg * 1e3 / L
    head = {
        "ms_per_step": ms_per_step, "step_bytes": int(step_bytes),
        "decode": {"GBps": round(decode_bytes / dec_avg / 1e6, 1),
                   "frac_of_peak": round(decode_bytes / dec_avg / 1e6 / HBM_PEAK_GBPS, 4),
                   "ms_avg": round(dec_avg, 4), "ms_median": round(dec_med, 4), "ms_min": round(dec_min, 4),
                   "us_per_launch": round(launch_us, 2), "bytes_per_launch": int(st.attn_bytes_layer),
                   "bytes": int(decode_bytes), "timing": f"{args.steps} timed steps (HIP events around the {L} launches)"},
        "roofline": {
            "bound": "hbm",
            "kernel": f"attn_decode_kernel<{cfg.head_dim},{cfg.block_tokens}> (+ its merge), one launch per layer, {cfg.name}",
            "achieved": round(st.attn_bytes_layer / launch_us / 1e3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(st.attn_bytes_layer / launch_us / 1e3 / HBM_PEAK_GBPS, 4),
            "traffic": read_traffic(f"attn_decode_{cfg.name}"),
            "bytes_per_launch": int(st.attn_bytes_layer), "us_per_launch": round(launch_us, 2)},
    }
    if decode_only:
        # calibration for PMC runs: one plain device-to-device copy of known size
        n = 1 << 30
        a = torch.empty(n, dtype=torch.uint8, device="cuda")
        b = torch.empty(n, dtype=torch.uint8, device="cuda")
        b.copy_(a)
        c.sync()
        head["calibration_copy_bytes"] = n
        del a, b
        return head
    col_avg = phase(1, 2)[0]
    app_avg = phase(2, 3)[0]
    rsz_avg = phase(3, 4)[0]
    head["patch"] = {
        "dirty_blocks": n_dirty, "layers": Lm, "payload_bytes": int(payload),
        "collect_us": round(col_avg * 1e3, 1), "collect_GBps": round(collect_bytes / col_avg / 1e6, 1),
        "apply_us": round(app_avg * 1e3, 1), "apply_GBps": round(apply_bytes / app_avg / 1e6, 1),
        "note": "the per-step cycle: last block of every sequence"}
    head["resize"] = {
        "from": B, "to": int(B_new), "n_moved": n_moved_expect, "bytes": int(resize_bytes),
        "us": round(rsz_avg * 1e3, 1), "GBps": round(resize_bytes / rsz_avg / 1e6, 1),
        "frac_of_peak": round(resize_bytes / rsz_avg / 1e6 / HBM_PEAK_GBPS, 4)}
    head["switch_us"] = round((col_avg + app_avg + rsz_avg) * 1e3, 1)
    return head


def maybe_cpu_baseline(c: Ctx, st: Stage, head):
    if head is not None and not c.args.no_cpu_baseline and not c.args.decode_only:
        t0 = time.time()
        head["cpu_baseline"] = cpu_baseline(c, st)
        log(f"[cpu_baseline] {time.time() - t0:.1f}s")


def _wl_name(cfg):
    return (f"{cfg.name}: {cfg.num_layers} layers, {cfg.num_q_heads}q/{cfg.num_kv_heads}kv heads, D{cfg.head_dim}, "
            f"block {cfg.block_tokens}, batch {cfg.num_seqs}, ctx U[{cfg.ctx_lo},{cfg.ctx_hi}]")


def run_stage8b(c: Ctx, headline: bool):
    """Workload 2: pool = 85 % of the HBM left after the stage's fp16 weights."""
    np, torch, pin, P, args = c.np, c.torch, c.pin, c.P, c.args
    cfg = pin.CONFIGS["stage8b"]
    L, S = cfg.num_layers, cfg.num_seqs
    ctx = pin.draw_ctx_lens(cfg, c.seed)
    n_live = int(((ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens).sum())
    bulk_fraction = 0.20
    c.arena_layout(stage_weight_bytes(cfg) + patch_capacity(int((bulk_fraction + 0.01) * n_live) + 2 * S, L, cfg.blk_bytes))
    weights = c.big_u8(stage_weight_bytes(cfg))
    free, room = c.free_bytes()
    B = int(0.85 * free // (L * cfg.blk_bytes))
    if not args.decode_only:
        # the migration target, the patch buffers and the stacked leg must fit beside the pool
        extra = n_live * L * cfg.blk_bytes * (1.0 + bulk_fraction + 0.05) + ((8 << 30) if c.arena is None else (1 << 30))
        B = min(B, int((room - extra) // (L * cfg.blk_bytes)))
    else:
        B = min(B, int((room - (1 << 30)) // (L * cfg.blk_bytes)))
    B = max(B, int(math.ceil(n_live * 1.3)))
    st = Stage(c, cfg, B, arenas=4)
    res = {"workload": _wl_name(cfg), "pool_blocks_per_layer": B, "pool_GiB": round(B * L * cfg.blk_bytes / 2**30, 1),
           "free_after_weights_GiB": round(free / 2**30, 1), "live_blocks_per_layer": n_live, "tokens": st.tokens}
    if args.decode_only:
        head = timed_steps(c, st, None, None, None, None, decode_only=True)
        res["decode"] = head["decode"]
        return res, head, st
    Lm = 4
    mig_layers = list(range(L - Lm, L))
    target = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, n_live, arenas=2,
                        allocator=c.placer(2))
    dst_map = torch.full((B,), -1, dtype=torch.int32)
    dst_map[torch.from_numpy(st.batch.live_ids)] = torch.arange(n_live, dtype=torch.int32)
    dst_map = dst_map.cuda()
    B_new = int(B * 0.8)
    head = None
    patch = c.big_u8(patch_capacity(S, Lm, cfg.blk_bytes))
    if headline:
        head = timed_steps(c, st, target, mig_layers, patch, B_new, dst_map=dst_map)
        res.update({k: head[k] for k in ("decode", "patch", "resize", "switch_us")})
        maybe_cpu_baseline(c, st, head)
    else:
        res["decode"] = st.time_decode(10, args.decode_iters)
        last32 = torch.from_numpy(pin.last_block_ids(st.batch).astype(np.int32)).cuda()
        res["patch"] = time_patch_round(c, st.region, target, last32, S, mig_layers, patch, dst_map, 10, cfg.blk_bytes, B)
        res["resize"] = st.time_shrink(B_new, 10)
        res["switch_us"] = round(res["patch"]["collect_us"] + res["patch"]["apply_us"] + res["resize"]["us"], 1)
    del patch

    # ---- bulk patch round: 20 % of the live blocks, all layers
    bulk_ids = torch.from_numpy(pin.draw_dirty_ids(st.batch, c.seed, 1, bulk_fraction).astype(np.int32)).cuda()
    all_layers = list(range(L))
    bulk_patch = c.big_u8(patch_capacity(bulk_ids.numel(), L, cfg.blk_bytes))
    res["patch_bulk"] = time_patch_round(c, st.region, target, bulk_ids, 0, all_layers, bulk_patch, dst_map, 10,
                                         cfg.blk_bytes, B)
    # context: what torch's own device-to-device copy reaches inside that buffer (read + write counted)
    half = (bulk_patch.numel() // 2) & ~0xFFF
    tcp = []
    for it in range(11):
        e0, e1 = c.ev(), c.ev()
        e0.record()
        bulk_patch[half:2 * half].copy_(bulk_patch[:half])
        e1.record()
        c.sync()
        if it:
            tcp.append(e0.elapsed_time(e1))
    tcpm = stats(tcp)[1]
    res["copy_ceiling"] = {"kind": "torch device-to-device copy, read + write", "bytes": int(half),
                           "us": round(tcpm * 1e3, 1), "GBps": round(2 * half / tcpm / 1e6, 1),
                           "frac_of_peak": round(2 * half / tcpm / 1e6 / HBM_PEAK_GBPS, 4)}
    del bulk_patch
    if P.pipelive_kv_read_state(target).status != 0 or not st.status_ok():
        raise RuntimeError("device status word set during the 8B-stage legs")
    if args.core_only:
        return res, head, None

    # ---- steady-state decode at slot granularity (the paper's own unit): every layer appends one token
    # per sequence, the written slots are drained and applied
    sreg = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B,
                      dirty_granularity=P.binding.DIRTY_SLOT, share_pool_of=st.region)
    stgt = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, n_live,
                      dirty_granularity=P.binding.DIRTY_SLOT, share_pool_of=target)
    knew = torch.zeros((S, cfg.num_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    room = st.batch.ctx_lens < st.batch.used.astype(np.int64) * cfg.block_tokens   # a free slot in the last block
    pos_d = torch.from_numpy(np.where(room, st.batch.ctx_lens, -1).astype(np.int32)).cuda()
    n_tok = int(room.sum())
    spatch = torch.empty(64 + 256 + S * (4 + L * cfg.token_bytes) + 4096, dtype=torch.uint8, device="cuda")
    tapp, tcol, tapl = [], [], []
    for it in range(11):
        e0, e1, e2, e3 = c.ev(), c.ev(), c.ev(), c.ev()
        e0.record()
        for l in range(L):
            P.pipelive_kv_append(sreg, l, knew, knew, st.table, pos_d, mark=True, count_tokens=(l == 0))
        e1.record()
        P.pipelive_kv_patch_collect(sreg, all_layers, spatch)
        e2.record()
        P.pipelive_kv_patch_apply(stgt, all_layers, spatch, dst_block_map=dst_map)
        e3.record()
        c.sync()
        if it:
            tapp.append(e0.elapsed_time(e1)); tcol.append(e1.elapsed_time(e2)); tapl.append(e2.elapsed_time(e3))
    if P.pipelive_kv_read_state(stgt).t_applied != 11 * n_tok or P.pipelive_kv_read_state(sreg).status != 0:
        raise RuntimeError("slot-granular cycle lost tokens")
    res["slot_patch"] = {
        "tokens_per_step": n_tok, "layers": L, "payload_bytes": n_tok * L * cfg.token_bytes,
        "append_all_layers_us": round(stats(tapp)[1] * 1e3, 1), "collect_us": round(stats(tcol)[1] * 1e3, 1),
        "apply_us": round(stats(tapl)[1] * 1e3, 1),
        "note": "block-granular patch of the same step carries %d bytes" % (S * L * cfg.blk_bytes)}
    del sreg, stgt, spatch, target, dst_map
    ctx_lens = st.batch.ctx_lens.copy()
    del st, weights
    c.free_all()
    # the memory-bound leg first: the prefill launches leave the part at a lower clock for a while
    res["stacked_vmm"] = run_stacked(c, cfg, ctx_lens)
    if getattr(c, "defer_prefill", False):
        c.prefill_pending = True          # the all-workload run times it behind the last memory-bound leg
    else:
        res["prefill"] = run_prefill(c, cfg)
    return res, head, None


def run_prefill(c: Ctx, cfg):
    """Prefill attention with the 8B stage's heads: 64 prompts of 512 tokens (the paper's prefill-heavy
    pattern) and a 512-token chunk on top of 4096 cached tokens; plus the chunk's write side."""
    np, torch, pin, P = c.np, c.torch, c.pin, c.P
    pres = {}
    for tag, Sp, ctxp, qlp in (("prompt512", 64, 512, 512), ("chunk512_of_4096", 16, 4096, 512)):
        if c.args.prefill_only and c.args.prefill_case not in ("both", tag):
            continue
        pcfg = pin.StageConfig(tag, 1, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens,
                               Sp, ctxp, ctxp)
        pb = pin.draw_batch(pcfg, c.seed, pool_factor=1.25)
        preg = P.KVRegion(1, pcfg.num_q_heads, pcfg.num_kv_heads, pcfg.head_dim, pcfg.block_tokens,
                          pb.num_blocks, arenas=3)
        c.fill(preg, pcfg, pb, c.seed, pb.num_blocks, poison_tail=False)
        qo_d = torch.arange(0, (Sp + 1) * qlp, qlp, dtype=torch.int32, device="cuda")
        tq = Sp * qlp
        pq = torch.from_numpy(pin.bf16_normal(pin.stream_key(c.seed, pin.STREAM_Q), 0, tq * pcfg.num_q_heads *
                                              pcfg.head_dim).view(np.int16)).cuda().view(torch.bfloat16)
        pq = pq.view(tq, pcfg.num_q_heads, pcfg.head_dim)
        pt, pc = torch.from_numpy(pb.table).cuda(), torch.from_numpy(pb.ctx_lens).cuda()
        ptimes = {}
        for odt in (torch.float32, torch.bfloat16):
            pout = torch.empty((tq, pcfg.num_q_heads, pcfg.head_dim), dtype=odt, device="cuda")
            for _ in range(2):
                P.pipelive_paged_attn_prefill(preg, 0, pq, pout, pt, pc, qo_d, tq)
            e0, e1 = c.ev(), c.ev()
            e0.record()
            for _ in range(10):
                P.pipelive_paged_attn_prefill(preg, 0, pq, pout, pt, pc, qo_d, tq)
            e1.record()
            c.sync()
            ptimes[odt] = e0.elapsed_time(e1) / 10
        pms, pms16 = ptimes[torch.float32], ptimes[torch.bfloat16]
        pk = pq[:, :pcfg.num_kv_heads, :].contiguous()
        for _ in range(2):
            P.pipelive_kv_append_chunk(preg, 0, pk, pk, pt, pc, qo_d, tq, mark=False)
        e2, e3 = c.ev(), c.ev()
        e2.record()
        for _ in range(10):
            P.pipelive_kv_append_chunk(preg, 0, pk, pk, pt, pc, qo_d, tq, mark=False)
        e3.record()
        c.sync()
        ams = e2.elapsed_time(e3) / 10
        abytes = 2 * 2 * tq * pcfg.num_kv_heads * pcfg.head_dim * 2   # K and V, read + write
        pairs = Sp * sum(ctxp - qlp + i + 1 for i in range(qlp))     # (query, visible key) pairs per head
        flops = pairs * pcfg.num_q_heads * 4 * pcfg.head_dim          # QK^T and PV, 2 flop per MAC
        pres[tag] = {"seqs": Sp, "ctx": ctxp, "q_len": qlp, "us": round(pms * 1e3, 1),
                     "TFLOPs": round(flops / pms / 1e9, 1),
                     "frac_of_mfma_peak": round(flops / pms / 1e9 / MFMA_PEAK_TFLOPS, 4),
                     "bf16_out_us": round(pms16 * 1e3, 1), "bf16_out_TFLOPs": round(flops / pms16 / 1e9, 1),
                     "bf16_out_frac_of_mfma_peak": round(flops / pms16 / 1e9 / MFMA_PEAK_TFLOPS, 4),
                     "append_chunk_us": round(ams * 1e3, 1), "append_chunk_GBps": round(abytes / ams / 1e6, 1),
                     "append_chunk_note": "same buffers every launch: they fit the last-level cache, not an HBM figure"}
        del preg, pq, pout
    return {"bound": "mfma", "peak_TFLOPs": MFMA_PEAK_TFLOPS, "dtype": "bf16",
            "note": "fp32 output: softmax weights as bf16 pairs (three MFMA passes per tile); "
                    "bf16 output: single bf16 weights (two passes)", **pres}


def run_stacked(c: Ctx, cfg, ctx):
    """Independently allocated, layer-stacked blocks: the 8B stage's batch over a pool of 2 MiB physical
    blocks (k = 4 layers x 128 tokens): decode, pointer-only shrink, real release."""
    np, torch, pin, P = c.np, c.torch, c.pin, c.P
    L, S = cfg.num_layers, cfg.num_seqs
    k_stack, bs_v = 4, 128
    vcfg = pin.StageConfig(cfg.name + "-stacked", L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, bs_v,
                           S, cfg.ctx_lo, cfg.ctx_hi)
    v_live = int(((ctx.astype(np.int64) + bs_v - 1) // bs_v).sum())
    Bv = int(v_live * 1.5)
    t0 = time.perf_counter()
    vreg = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, bs_v, Bv, stack_k=k_stack, backing="vmm")
    t_alloc = time.perf_counter() - t0
    vb = pin.draw_batch(vcfg, c.seed, num_blocks=Bv)
    c.fill(vreg, vcfg, vb, c.seed, Bv, poison_tail=True)
    vt, vc, vu = (torch.from_numpy(x).cuda() for x in (vb.table, vb.ctx_lens, vb.used))
    vq = torch.from_numpy(pin.q_bits(vcfg, c.seed, 0).view(np.int16)).cuda().view(torch.bfloat16)
    vout = torch.empty((S, cfg.num_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
    vmax = int(vb.ctx_lens.max())
    vws = vreg.attn_workspace(S, vmax, 0)

    def vdecode():
        for l in range(L):
            P.pipelive_paged_attn_decode(vreg, l, vq, vout, vt, vc, max_ctx=vmax, workspace=vws)
    for _ in range(5):
        vdecode()
    e0, e1 = c.ev(), c.ev()
    e0.record()
    for _ in range(20):
        vdecode()
    e1.record()
    c.sync()
    v_ms = e0.elapsed_time(e1) / 20
    q_bytes = S * cfg.num_q_heads * cfg.head_dim * 2
    v_bytes = L * (vb.total_tokens * cfg.token_bytes + 3 * q_bytes + 4 * int(vb.used.sum()))
    ref_out = vout.clone()
    Bv_new = int(Bv * 0.8)
    v_moved = int((vb.live_ids >= Bv_new).sum())
    vrws = vreg.resize_workspace()
    c.sync()
    t0 = time.perf_counter()
    rc, r = P.pipelive_kv_resize(vreg, Bv_new, [vt], [vu], workspace=vrws)
    c.sync()
    t_shrink = time.perf_counter() - t0
    if rc != P.OK or r.n_moved != v_moved:
        raise RuntimeError(f"stacked shrink failed: rc={rc} moved={r.n_moved} expected={v_moved}")
    free_a = torch.cuda.mem_get_info()[0]
    t0 = time.perf_counter()
    n_rel = vreg.release_tail(Bv)
    t_rel = time.perf_counter() - t0
    free_b = torch.cuda.mem_get_info()[0]
    vdecode()
    c.sync()
    if not torch.equal(vout, ref_out):
        raise RuntimeError("decode changed after the pointer-only shrink")
    tok = cfg.token_bytes
    util = {str(k): round(P.pipelive_kv_utilization(ctx, P.pipelive_stacked_block_tokens(2 << 20, k, tok)), 4)
            for k in (1, 2, 4, 8, 16)}
    out = {"stack_k": k_stack, "block_tokens": bs_v, "phys_block_bytes": vreg.phys_bytes,
           "pool_blocks": Bv, "groups": vreg.groups, "alloc_ms": round(t_alloc * 1e3, 1),
           "decode_GBps": round(v_bytes / v_ms / 1e6, 1), "decode_frac_of_peak": round(v_bytes / v_ms / 1e6 / 8000.0, 4),
           "shrink_to": Bv_new, "ids_remapped": v_moved, "bytes_copied": 0,
           "shrink_us": round(t_shrink * 1e6, 1), "released_blocks": n_rel,
           "release_ms": round(t_rel * 1e3, 1), "returned_GiB": round((free_b - free_a) / 2**30, 2),
           "effective_kv_utilization_vs_k": util,
           "note": "shrink_us is host wall time of pipelive_kv_resize incl. its one sync; release is driver time"}
    del vreg
    return out


def run_resize8b(c: Ctx, headline: bool):
    """Workload 3: the stage grows from 16 to 20 layers, every pool shrinks by 20 % while decoding goes on.
    Primary reading: a tight pool, B = ceil(n_live / 0.75)."""
    np, torch, pin, P, args = c.np, c.torch, c.pin, c.P, c.args
    cfg = pin.CONFIGS["resize8b"]
    L, S = cfg.num_layers, cfg.num_seqs
    ctx = pin.draw_ctx_lens(cfg, c.seed)
    n_live = int(((ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens).sum())
    B = int(math.ceil(n_live / 0.75))
    B_new = B * 16 // 20
    c.arena_layout(patch_capacity(S, L, cfg.blk_bytes))
    st = Stage(c, cfg, B, arenas=4, stride_pad=2)
    res = {"workload": _wl_name(cfg), "pool_blocks_per_layer": B, "pool_GiB": round(B * L * cfg.blk_bytes / 2**30, 1),
           "live_blocks_per_layer": n_live, "tokens": st.tokens, "pool_reading": "tight pool: B = ceil(n_live / 0.75)"}
    head = None
    if args.decode_only:
        head = timed_steps(c, st, None, None, None, None, decode_only=True)
        res["decode"] = head["decode"]
        return res, head, st
    if headline:
        tgt = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B, arenas=2,
                         allocator=c.placer(2))
        patch = c.big_u8(patch_capacity(S, L, cfg.blk_bytes))
        head = timed_steps(c, st, tgt, list(range(L)), patch, B_new)
        maybe_cpu_baseline(c, st, head)
        del tgt, patch
    res["decode"] = st.time_decode(10, args.decode_iters)
    res["resize"] = st.time_shrink(B_new, 20)
    # ---- the procedure: shrink, decode (must not change), 16 decode steps with appends, grow, shrink again
    st.decode_pass()
    before = [o.clone() for o in st.outs]
    r1 = st.shrink(B_new)
    st.decode_pass()
    c.sync()
    same = all(torch.equal(a, b) for a, b in zip(before, st.outs))
    bm = pin.BlockManager(st.batch, B)
    bm.set_num_blocks(B_new)
    bm.adopt(st.table.cpu().numpy(), np.nonzero(np.unpackbits(st.region.live.cpu().numpy(), bitorder="little")[:B_new])[0])
    e0, e1 = c.ev(), c.ev()
    e0.record()
    for k in range(16):
        decode_step_with_appends(c, st, bm, k, count_layer=-1, mark=False, attend=True)
    e1.record()
    c.sync()
    step_ms = e0.elapsed_time(e1) / 16
    st.set_tokens(int(bm.ctx.sum()), int(bm.used.sum()))
    st.max_ctx = int(bm.ctx.max())
    rc, _ = P.pipelive_kv_resize(st.region, B, [], [], workspace=st.rws)      # the stage shrinks back: grow
    if rc != P.OK:
        raise RuntimeError(f"grow failed: {rc}")
    dec_grown = st.time_decode(3, 20)
    r2 = st.shrink(B_new)
    dec_again = st.time_decode(3, 20)
    if not st.status_ok():
        raise RuntimeError("device status word set during the resize stress")
    res["procedure"] = {
        "shrink_n_moved": int(r1.n_moved), "decode_bit_identical_after_shrink": bool(same),
        "decode_steps_with_appends": 16, "ms_per_decode_step_with_appends": round(step_ms, 4),
        "note_steps": "host block manager + 16 appends + 16 attention launches per step, not a bandwidth figure",
        "decode_after_grow": {k: dec_grown[k] for k in ("GBps", "frac_of_peak", "us_per_launch")},
        "second_shrink_n_moved": int(r2.n_moved),
        "decode_after_second_shrink": {k: dec_again[k] for k in ("GBps", "frac_of_peak", "us_per_launch")}}
    if not same:
        raise RuntimeError("resize8b: decode changed after the shrink")
    return res, head, None


def run_resize8b_sparse(c: Ctx):
    """Secondary reading of workload 3: the same batch in a pool sized like the 8B stage's (85 % of HBM)."""
    np, torch, pin, P, args = c.np, c.torch, c.pin, c.P, c.args
    cfg = pin.CONFIGS["resize8b"]
    L = cfg.num_layers
    c.arena_layout(stage_weight_bytes(cfg))
    weights = c.big_u8(stage_weight_bytes(cfg))
    free, room = c.free_bytes()
    B = min(int(0.85 * free // (L * cfg.blk_bytes)), int((room - (1 << 30)) // (L * cfg.blk_bytes)))
    st = Stage(c, cfg, B, arenas=4)
    out = {"pool_blocks_per_layer": B, "pool_GiB": round(B * L * cfg.blk_bytes / 2**30, 1),
           "decode": st.time_decode(10, args.decode_iters), "resize": st.time_shrink(int(B * 0.8), 5)}
    del st, weights
    return out


def run_longctx8b(c: Ctx, headline: bool):
    """Workload 5: 16 sequences of 16k-32k tokens, 32-token blocks; split decode, 25 % shrink, 2 % patch."""
    np, torch, pin, P, args = c.np, c.torch, c.pin, c.P, c.args
    cfg = pin.CONFIGS["longctx8b"]
    L, S = cfg.num_layers, cfg.num_seqs
    ctx = pin.draw_ctx_lens(cfg, c.seed)
    n_live = int(((ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens).sum())
    B = int(math.ceil(n_live / 0.70))
    B_new = int(B * 0.75)
    c.arena_layout(0 if args.decode_only else patch_capacity(n_live + S, L, cfg.blk_bytes) + patch_capacity(S, L, cfg.blk_bytes))
    st = Stage(c, cfg, B, arenas=4)
    res = {"workload": _wl_name(cfg), "pool_blocks_per_layer": B, "pool_GiB": round(B * L * cfg.blk_bytes / 2**30, 1),
           "live_blocks_per_layer": n_live, "tokens": st.tokens}
    head = None
    if args.decode_only:
        head = timed_steps(c, st, None, None, None, None, decode_only=True)
        res["decode"] = head["decode"]
        return res, head, st
    layers = list(range(L))
    tgt = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, n_live, arenas=2,
                     allocator=c.placer(2))
    if headline:
        patch = c.big_u8(patch_capacity(S, L, cfg.blk_bytes))
        dm = torch.full((B,), -1, dtype=torch.int32)
        dm[torch.from_numpy(st.batch.live_ids)] = torch.arange(n_live, dtype=torch.int32)
        head = timed_steps(c, st, tgt, layers, patch, B_new, dst_map=dm.cuda())
        maybe_cpu_baseline(c, st, head)
        del patch
    res["decode"] = st.time_decode(10, args.decode_iters)
    res["decode"]["note"] = "16 x 8 (sequence, KV head) pairs cut into 1024 equal shares (split-K), merged per launch"
    res["resize"] = st.time_shrink(B_new, 10)
    st.decode_pass()
    before = [o.clone() for o in st.outs]
    st.shrink(B_new)
    st.decode_pass()
    c.sync()
    same = all(torch.equal(a, b) for a, b in zip(before, st.outs))
    res["decode_bit_identical_after_shrink"] = bool(same)
    if not same:
        raise RuntimeError("longctx8b: decode changed after the shrink")
    # round 0 + the final round at 2 % into a compact target through a block map
    live = np.nonzero(np.unpackbits(st.region.live.cpu().numpy(), bitorder="little")[:B_new])[0]
    table_h = st.table.cpu().numpy()
    bt = pin.Batch(cfg, c.seed, B_new, st.batch.ctx_lens, table_h, st.batch.used, live)
    dmap = torch.full((B_new,), -1, dtype=torch.int32)
    dmap[torch.from_numpy(live)] = torch.arange(len(live), dtype=torch.int32)
    dmap = dmap.cuda()
    patch = c.big_u8(patch_capacity(len(live), L, cfg.blk_bytes))
    live32 = torch.from_numpy(live.astype(np.int32)).cuda()
    applied0 = P.pipelive_kv_read_state(tgt).t_applied
    res["round0"] = time_patch_round(c, st.region, tgt, live32, 0, layers, patch, dmap, 2, cfg.blk_bytes, B_new)
    ids = pin.draw_dirty_ids(bt, c.seed, 1, 0.02)
    ids32 = torch.from_numpy(ids.astype(np.int32)).cuda()
    res["patch_final"] = time_patch_round(c, st.region, tgt, ids32, S, layers, patch, dmap, 10, cfg.blk_bytes, B_new)
    res["switch_us"] = round(res["patch_final"]["collect_us"] + res["patch_final"]["apply_us"] + res["resize"]["us"], 1)
    res["switch_note"] = "collect + apply of the 2 % round plus the 25 % shrink"
    compact = np.arange(len(live))
    for l in (0, L - 1):
        if not torch.equal(tgt.read_blocks(l, compact), st.region.read_blocks(l, live)):
            raise RuntimeError(f"longctx8b: target differs from source in layer {l}")
    if P.pipelive_kv_read_state(tgt).t_applied - applied0 != S or not st.status_ok():
        raise RuntimeError("longctx8b: counters or status wrong")
    del tgt, patch
    return res, head, None


def run_tiny(c: Ctx):
    """Workload 1, every byte against the oracle: decode, resize 128 -> 96, decode, round 0 + 3 rounds."""
    np, torch, pin, P = c.np, c.torch, c.pin, c.P
    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from gpu_common import attn_errors, fill_pair, make_pair
    cfg = pin.CONFIGS["tiny"]
    seed = c.seed
    batch = pin.draw_batch(cfg, seed, num_blocks=128)
    host, dev = make_pair(cfg, batch, seed)
    fill_pair(cfg, batch, seed, host, dev)
    table_h = batch.table.copy()
    table_d = torch.from_numpy(batch.table).cuda()
    ctx_d = torch.from_numpy(batch.ctx_lens).cuda()
    used_d = torch.from_numpy(batch.used).cuda()
    worst = [0.0, 0.0]
    t_dec = []

    def decode_all():
        outs = []
        for l in range(cfg.num_layers):
            q = torch.from_numpy(pin.q_bits(cfg, seed, l).view(np.int16)).cuda().view(torch.bfloat16)
            out = torch.empty((cfg.num_seqs, cfg.num_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
            e0, e1 = c.ev(), c.ev()
            e0.record()
            P.pipelive_paged_attn_decode(dev, l, q, out, table_d, ctx_d)
            e1.record()
            c.sync()
            t_dec.append(e0.elapsed_time(e1))
            ref = host.attn_decode(l, pin.q_bits(cfg, seed, l), table_h, batch.ctx_lens)
            ma, rl = attn_errors(out.cpu().numpy(), ref)
            worst[0], worst[1] = max(worst[0], ma), max(worst[1], rl)
            outs.append(out.cpu().numpy())
        return outs
    o1 = decode_all()
    rc_h, remap_h, res_h = host.resize(96, [table_h], [batch.used])
    r0, r1 = c.ev(), c.ev()
    r0.record()
    rc_d, res_d = P.pipelive_kv_resize(dev, 96, [table_d], [used_d])
    r1.record()
    c.sync()
    ok = rc_h == 0 and rc_d == 0 and res_d.n_moved == res_h[1] and np.array_equal(table_d.cpu().numpy(), table_h)
    o2 = decode_all()
    ok = ok and all(np.array_equal(a.view(np.uint32), b.view(np.uint32)) for a, b in zip(o1, o2))
    live = host.live_ids()
    tgt_h = oracle.HostKV(cfg.num_layers, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, 96,
                          layout=cfg.layout, arenas=2, fill_bits=0)
    tgt_d = P.KVRegion(cfg.num_layers, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, 96,
                       fill_bits=0)
    cap = 64 + 256 + len(live) * (4 + cfg.num_layers * host.blk_bytes)
    patch_h = np.zeros(cap, dtype=np.uint8)
    patch_d = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    layers = list(range(cfg.num_layers))
    bt = pin.Batch(cfg, seed, 96, batch.ctx_lens, table_h, batch.used, live)
    t_cyc = []
    for rnd in range(4):
        ids = live if rnd == 0 else pin.draw_dirty_ids(bt, seed, rnd, 0.10)
        if rnd:
            for l in layers:    # the round's writes: new content for the dirty blocks, on both sides
                for b in ids:
                    bits = pin.kv_block_bits(cfg, seed, 128, rnd, l, int(b))
                    host.block(l, int(b))[:] = bits
                dev.write_blocks(l, ids, torch.from_numpy(np.stack([host.block(l, int(b)) for b in ids]).view(np.int16)).cuda())
        host.mark_dirty(ids, cfg.num_seqs if rnd else 0)
        P.pipelive_kv_mark_dirty(dev, torch.from_numpy(ids.astype(np.int32)).cuda(), cfg.num_seqs if rnd else 0)
        ok = ok and host.patch_collect(layers, patch_h) == 0 and host_apply(tgt_h, layers, patch_h)
        e0, e1 = c.ev(), c.ev()
        e0.record()
        P.pipelive_kv_patch_collect(dev, layers, patch_d)
        P.pipelive_kv_patch_apply(tgt_d, layers, patch_d)
        e1.record()
        c.sync()
        t_cyc.append(e0.elapsed_time(e1))
        h = oracle.parse_patch_header(patch_h)
        end = h["payload_offset"] + h["n_blocks"] * cfg.num_layers * host.blk_bytes
        g = patch_d.cpu().numpy()
        ok = ok and np.array_equal(g[:64 + 4 * h["n_blocks"]], patch_h[:64 + 4 * h["n_blocks"]])
        ok = ok and np.array_equal(g[h["payload_offset"]:end], patch_h[h["payload_offset"]:end])
    for l in layers:
        got = tgt_d.read_blocks(l, live).cpu().numpy().view(np.uint16)
        for k, b in enumerate(live):
            ok = ok and np.array_equal(got[k], tgt_h.block(l, int(b))) and np.array_equal(got[k], host.block(l, int(b)))
    ok = ok and P.pipelive_kv_read_state(tgt_d).t_applied == 3 * cfg.num_seqs == tgt_h.t_applied
    ok = ok and worst[0] <= 1e-2 and worst[1] <= 2e-3
    if not ok:
        raise RuntimeError("tiny workload: GPU and oracle disagree")
    return {"workload": _wl_name(cfg), "parity": "every byte of tables, patches, pools and counters equal to the oracle's; "
            "attention within tolerance", "attn_max_abs": worst[0], "attn_rel_l2": worst[1],
            "decode_us_per_launch": round(stats(t_dec)[1] * 1e3, 1), "resize_us": round(r0.elapsed_time(r1) * 1e3, 1),
            "patch_cycle_us": round(stats(t_cyc)[1] * 1e3, 1), "moved": int(res_d.n_moved),
            "note": "latency-sized: no bandwidth figure applies"}


def host_apply(tgt_h, layers, patch_h):
    return tgt_h.patch_apply(layers, patch_h) == 0


def cpu_baseline(c: Ctx, st: Stage):
    """The oracle on the host cores, on a bounded sample of the headline workload (attention), and its copy
    paths (resize, patch collect / apply) on a host region of the resize-stress shape."""
    np, torch, pin, args = c.np, c.torch, c.pin, c.args
    import oracle
    cfg, batch = st.cfg, st.batch
    L, S, B = cfg.num_layers, cfg.num_seqs, st.B
    ncores = min(16, os.cpu_count() or 1)
    Lc = max(1, min(L, args.cpu_layers))
    ids = batch.live_ids
    compact = np.full(B, -1, dtype=np.int32)
    compact[ids] = np.arange(len(ids), dtype=np.int32)
    n_ar = 3
    host = oracle.HostKV(Lc, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens,
                         len(ids), layout=cfg.layout, arenas=n_ar)
    for l in range(Lc):
        for i in range(0, len(ids), 8192):     # the inputs, copied back in pieces
            part = ids[i:i + 8192]
            data = st.region.read_blocks(l, part).cpu().numpy().view(np.uint16)
            for a in range(n_ar):
                sel = (np.arange(i, i + len(part)) % n_ar) == a
                rows = np.arange(i, i + len(part))[sel] // n_ar
                host.arenas[l * n_ar + a][rows] = data[sel]
    tab = np.where(batch.table == pin.TABLE_FILL, pin.TABLE_FILL, compact[np.minimum(batch.table, B - 1)])
    tab = np.ascontiguousarray(tab, dtype=np.int32)
    tc, err, num, den = 0.0, 0.0, 0.0, 0.0
    st.decode_pass()
    c.sync()
    for l in range(Lc):
        qh = pin.q_bits(cfg, c.seed, l)
        tc0 = time.perf_counter()
        ref = host.attn_decode(l, qh, tab, batch.ctx_lens, nthreads=ncores)
        tc += time.perf_counter() - tc0
        got = st.outs[l].cpu().numpy().astype(np.float64)
        err = max(err, float(np.abs(got - ref).max()))
        num += float(((got - ref) ** 2).sum())
        den += float((ref.astype(np.float64) ** 2).sum())
    cpu_bytes = Lc * batch.total_tokens * cfg.token_bytes
    short = np.argsort(batch.ctx_lens)[:8]
    tc1 = time.perf_counter()
    host.attn_decode(0, pin.q_bits(cfg, c.seed, 0)[short], tab[short], batch.ctx_lens[short], nthreads=1)
    tc1 = time.perf_counter() - tc1
    one_bytes = int(batch.ctx_lens[short].sum()) * cfg.token_bytes
    out = {"value": round(cpu_bytes / tc / 1e9, 4), "unit": "GB/s", "cores": ncores, "kind": "oracle",
           "sample": f"decode attention of layer(s) 0..{Lc - 1} of {L} of {cfg.name} (all {S} sequences, all "
                     f"{cfg.num_q_heads} heads, {Lc * batch.total_tokens} token-layers), {tc:.2f} s wall on {ncores} threads",
           "single_thread": {"value": round(one_bytes / tc1 / 1e9, 4), "unit": "GB/s",
                             "sample": f"layer 0, the 8 shortest sequences ({int(batch.ctx_lens[short].sum())} tokens), {tc1:.2f} s"},
           "gpu_vs_oracle_max_abs": err, "gpu_vs_oracle_rel_l2": math.sqrt(num / den)}
    del host
    # ---- copy paths: the resize-stress shape on the host, 4 of its 16 layers (per-layer work is identical)
    rcfg = pin.CONFIGS["resize8b"]
    Lh = 4
    rb = pin.draw_batch(rcfg, c.seed, pool_factor=1.0 / 0.75)
    Bh = rb.num_blocks
    hk = oracle.HostKV(Lh, rcfg.num_q_heads, rcfg.num_kv_heads, rcfg.head_dim, rcfg.block_tokens, Bh,
                       layout=rcfg.layout, arenas=3, fill_bits=0x3C00)
    hk.set_live(rb.live_ids)
    tgt = oracle.HostKV(Lh, rcfg.num_q_heads, rcfg.num_kv_heads, rcfg.head_dim, rcfg.block_tokens, Bh,
                        layout=rcfg.layout, arenas=2, fill_bits=0)
    dirty = pin.draw_dirty_ids(rb, c.seed, 1, 0.20)
    pbuf = np.zeros(64 + 256 + len(dirty) * (4 + Lh * hk.blk_bytes) + 4096, dtype=np.uint8)
    hk.mark_dirty(dirty, 0)
    t0 = time.perf_counter()
    rc1 = hk.patch_collect(list(range(Lh)), pbuf)
    t_col = time.perf_counter() - t0
    t0 = time.perf_counter()
    rc2 = tgt.patch_apply(list(range(Lh)), pbuf)
    t_app = time.perf_counter() - t0
    table_h = rb.table.copy()
    B_new = Bh * 16 // 20
    n_moved = int((rb.live_ids >= B_new).sum())
    t0 = time.perf_counter()
    rc3, _, rres = hk.resize(B_new, [table_h], [rb.used])
    t_rsz = time.perf_counter() - t0
    if rc1 or rc2 or rc3 or int(rres[1]) != n_moved:
        raise RuntimeError("oracle copy-path sample failed")
    pay = len(dirty) * Lh * hk.blk_bytes
    mv = n_moved * Lh * hk.blk_bytes
    out["copy_paths"] = {
        "cores": 1, "kind": "oracle", "shape": f"{rcfg.name}, {Lh} of {rcfg.num_layers} layers, tight pool of {Bh} blocks",
        "resize": {"n_moved": n_moved, "bytes": 2 * mv, "s": round(t_rsz, 4), "GBps": round(2 * mv / t_rsz / 1e9, 3)},
        "patch_collect": {"dirty_blocks": int(len(dirty)), "bytes": 2 * pay, "s": round(t_col, 4),
                          "GBps": round(2 * pay / t_col / 1e9, 3)},
        "patch_apply": {"bytes": 2 * pay, "s": round(t_app, 4), "GBps": round(2 * pay / t_app / 1e9, 3)}}
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
            f"--gpus {args.gpus} is not supported.")
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the hot path has no CPU fallback.")
        sys.exit(3)
    torch.cuda.set_device(0)
    c = Ctx(args)
    c.P.load()
    if args.prefill_only:
        print(json.dumps({"prefill": run_prefill(c, c.pin.CONFIGS["stage8b"])}), flush=True)
        return
    placement = c.arena_open()
    runners = {"stage70b": run_stage70b, "stage8b": run_stage8b, "resize8b": run_resize8b, "longctx8b": run_longctx8b}
    headline_name = HEADLINE if args.config == "all" else args.config
    if headline_name not in runners:
        log(f"bench.py: unknown workload {headline_name!r}")
        sys.exit(2)
    t_all = time.time()
    configs = {}
    c.defer_prefill = args.config == "all" and not args.decode_only
    res, head, st = runners[headline_name](c, True)
    configs[headline_name] = res
    cfg = c.pin.CONFIGS[headline_name]
    result = {
        "metric": "hot-path HBM GB/s per step (decode paged attention over all layers + KV patch cycle + KV resize)",
        "value": round(head["step_bytes"] / (head["ms_per_step"] * 1e-3) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": _wl_name(cfg), "pool_blocks_per_layer": res["pool_blocks_per_layer"],
                   "pool_GiB": res["pool_GiB"], "live_blocks_per_layer": res["live_blocks_per_layer"],
                   "tokens": res["tokens"], "split_tokens": int(args.split_tokens), "device": c.dev_name,
                   "decode_only": bool(args.decode_only), "placement": placement},
        "step_bytes": head["step_bytes"],
        "roofline": head["roofline"],
    }
    if args.decode_only and "calibration_copy_bytes" in head:
        result["calibration_copy_bytes"] = head["calibration_copy_bytes"]
    if "cpu_baseline" in head:
        result["cpu_baseline"] = head["cpu_baseline"]
    del st
    c.free_all()
    if args.config == "all" and not args.decode_only:
        for name in ALL_CONFIGS:
            if name == headline_name:
                continue
            t0 = time.time()
            if name == "tiny":
                if args.no_cpu_baseline:      # the tiny shape is a byte-for-byte comparison with the oracle:
                    continue                  # it belongs to the oracle leg of the run
                configs[name] = run_tiny(c)
                result.setdefault("cpu_baseline", {})["tiny_parity"] = "configs.tiny: full comparison with the oracle"
            else:
                r, _, s2 = runners[name](c, False)
                configs[name] = r
                del s2
            c.free_all()
            if name == "resize8b" and not args.core_only:
                configs[name]["sparse_pool"] = run_resize8b_sparse(c)
                c.free_all()
            log(f"[{name}] done in {time.time() - t0:.1f}s")
    if getattr(c, "prefill_pending", False):
        configs["stage8b"]["prefill"] = run_prefill(c, c.pin.CONFIGS["stage8b"])
        c.free_all()
    result["configs"] = configs
    bar = {}
    for name, r in configs.items():
        if "decode" in r:
            bar[name + ".decode"] = r["decode"]["frac_of_peak"]
        if "resize" in r and r["resize"]:
            bar[name + ".resize"] = r["resize"]["frac_of_peak"]
        if "patch_rounds" in r:
            for pr in r["patch_rounds"]:
                bar[f"{name}.round{pr['round']}.collect"] = pr["collect_frac_of_peak"]
                bar[f"{name}.round{pr['round']}.apply"] = pr["apply_frac_of_peak"]
        for key in ("patch_bulk", "patch_final"):
            if key in r:
                bar[f"{name}.{key}.collect"] = r[key]["collect_frac_of_peak"]
                bar[f"{name}.{key}.apply"] = r[key]["apply_frac_of_peak"]
    result["hbm_fraction_summary"] = bar
    result["below_60_percent"] = sorted(k for k, v in bar.items() if v < 0.60)
    log(f"[bench] total {time.time() - t_all:.1f}s")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
