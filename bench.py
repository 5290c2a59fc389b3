#!/usr/bin/env python3
"""Benchmark of the PipeLive hot path on one MI355X.

Workload (default): the Llama-3-8B-shaped pipeline stage - 16 layers, 32 query
/ 8 KV heads, head_dim 128, block 16 tokens, bf16, 64 sequences with context
lengths uniform in [512, 4096], block pool sized to 85 % of the HBM left after
the stage's fp16 weights.  One *step* is one pass of the whole hot path on that
batch:

  1. decode attention over all layers (one launch per layer, own q per layer),
  2. one patch cycle: mark every sequence's last block dirty, collect
     (drain + gather) the dirty blocks of the migrating layers into the patch
     buffer, apply (scatter) them into the target region,
  3. ResizeKV: shrink the pool by 20 % (plan, move, remap) - followed by an
     untimed-in-bytes restore (grow back + reset of table and live bitmap) so
     that every step performs the same moves.

`value` is the algorithmic bytes of the whole step divided by the step time.
The per-phase figures (HIP events on the launch stream) and the roofline of the
dominant kernel (decode attention) are reported beside it, and the CPU oracle is
timed on the host cores on a bounded sample of the same workload.

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


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="stage8b", help="workload name (see pipelive_inputs.CONFIGS)")
    ap.add_argument("--split-tokens", type=int, default=0)
    ap.add_argument("--mig-layers", type=int, default=4, help="layers carried by each patch")
    ap.add_argument("--pool-blocks", type=int, default=0, help="override the pool size (blocks per layer)")
    ap.add_argument("--shrink", type=float, default=0.20)
    ap.add_argument("--bulk-fraction", type=float, default=0.20, help="dirty fraction of the bulk patch round")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=6, help="layers in the CPU oracle sample")
    ap.add_argument("--decode-only", action="store_true", help="profiling aid: steps run phase 1 only")
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


def main():
    args = parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
            f"--gpus {args.gpus} is not supported.")
        sys.exit(2)

    import numpy as np
    import torch

    import pipelive_inputs as pin
    from pipelive_inputs.device_fill import fill_live_blocks
    import paper_2604_12171_amd as P

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the hot path has no CPU fallback.")
        sys.exit(3)
    torch.cuda.set_device(0)
    lib = P.load()
    dev_name = torch.cuda.get_device_name(0)
    cfg = pin.CONFIGS[args.config]
    seed = pin.MASTER_SEED
    L, S = cfg.num_layers, cfg.num_seqs

    # ---------------- pool sizing: 85 % of the HBM left after the stage weights
    t_setup = time.time()
    weights = torch.empty(stage_weight_bytes(cfg), dtype=torch.uint8, device="cuda")
    free, total = torch.cuda.mem_get_info()
    ctx = pin.draw_ctx_lens(cfg, seed)
    n_live = int(((ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens).sum())
    B = args.pool_blocks or int(0.85 * free // (L * cfg.blk_bytes))
    if not args.decode_only and not args.pool_blocks:
        # the migration target, the patch buffers and the oracle sample must fit beside the pool
        extra = n_live * L * cfg.blk_bytes * (1.0 + args.bulk_fraction + 0.05) + (8 << 30)
        B = min(B, int((free - extra) // (L * cfg.blk_bytes)))
    B = max(B, int(math.ceil(n_live * 1.3)))
    region = None
    while region is None:
        try:
            region = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens,
                                B, arenas=4)
        except torch.OutOfMemoryError:
            log(f"pool of {B} blocks/layer does not fit; halving")
            torch.cuda.empty_cache()
            B //= 2
    batch = pin.draw_batch(cfg, seed, num_blocks=B)
    log(f"[setup] {dev_name}: pool {B} blocks/layer x {L} layers = {B * L * cfg.blk_bytes / 2**30:.1f} GiB "
        f"(free after weights {free / 2**30:.1f} GiB), live {n_live} blocks/layer, "
        f"tokens {batch.total_tokens}")
    fill_live_blocks(region, cfg, batch, seed, B, poison_tail=True)
    torch.cuda.synchronize()
    log(f"[setup] pool filled in {time.time() - t_setup:.1f}s")

    table_d = torch.from_numpy(batch.table).cuda()
    table_saved = table_d.clone()
    ctx_d = torch.from_numpy(batch.ctx_lens).cuda()
    used_d = torch.from_numpy(batch.used).cuda()
    live_saved = region.live.clone()
    max_ctx = int(batch.ctx_lens.max())
    split = args.split_tokens
    ws = region.attn_workspace(S, max_ctx, split)
    qs = [torch.from_numpy(pin.q_bits(cfg, seed, l).view(np.int16)).cuda().view(torch.bfloat16)
          for l in range(L)]
    outs = [torch.empty((S, cfg.num_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
            for _ in range(L)]

    # migration target: a compact region reached through a block map
    Lm = min(args.mig_layers, L)
    mig_layers = list(range(L - Lm, L))
    target = None if args.decode_only else P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                                                      cfg.block_tokens, n_live, arenas=2)
    dst_map = torch.full((B,), -1, dtype=torch.int32)
    dst_map[torch.from_numpy(batch.live_ids)] = torch.arange(n_live, dtype=torch.int32)
    dst_map = dst_map.cuda()
    last_ids = torch.from_numpy(pin.last_block_ids(batch).astype(np.int32)).cuda()
    n_dirty = int(last_ids.numel())
    patch_cap = 64 + 256 + n_dirty * (4 + Lm * cfg.blk_bytes) + 4096
    patch = torch.empty(patch_cap, dtype=torch.uint8, device="cuda")
    B_new = int(B * (1.0 - args.shrink))
    n_moved_expect = int((batch.live_ids >= B_new).sum())
    rws = region.resize_workspace()

    # ---------------- algorithmic bytes
    kv_bytes_layer = batch.total_tokens * cfg.token_bytes
    q_bytes = S * cfg.num_q_heads * cfg.head_dim * 2
    out_bytes = S * cfg.num_q_heads * cfg.head_dim * 4
    tab_bytes = 4 * int(batch.used.sum())
    attn_bytes_layer = kv_bytes_layer + q_bytes + out_bytes + tab_bytes
    decode_bytes = attn_bytes_layer * L
    patch_payload = n_dirty * Lm * cfg.blk_bytes
    collect_bytes = 2 * patch_payload + 2 * (B // 8)
    apply_bytes = 2 * patch_payload
    resize_bytes = 2 * n_moved_expect * L * cfg.blk_bytes
    step_bytes = decode_bytes if args.decode_only else decode_bytes + collect_bytes + apply_bytes + resize_bytes

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def one_step(events=None):
        if events:
            events[0].record()
        for l in range(L):
            P.pipelive_paged_attn_decode(region, l, qs[l], outs[l], table_d, ctx_d, max_ctx=max_ctx,
                                         split_tokens=split, workspace=ws)
        if events:
            events[1].record()
        if args.decode_only:
            return
        P.pipelive_kv_mark_dirty(region, last_ids, S)
        P.pipelive_kv_patch_collect(region, mig_layers, patch)
        if events:
            events[2].record()
        P.pipelive_kv_patch_apply(target, mig_layers, patch, dst_block_map=dst_map)
        if events:
            events[3].record()
        rc, res = P.pipelive_kv_resize(region, B_new, [table_d], [used_d], workspace=rws)
        if rc != P.OK or res.n_moved != n_moved_expect:
            raise RuntimeError(f"resize failed: rc={rc} moved={res.n_moved} expected={n_moved_expect}")
        if events:
            events[4].record()
        # restore (not counted in bytes): grow back, put table and live bitmap back
        rc, _ = P.pipelive_kv_resize(region, B, [], [], workspace=rws)
        if rc != P.OK:
            raise RuntimeError(f"grow failed: {rc}")
        table_d.copy_(table_saved)
        region.live.copy_(live_saved)

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    all_events = [[ev() for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(all_events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    def phase_ms(a, b):
        v = sorted(e[a].elapsed_time(e[b]) for e in all_events)
        return sum(v) / len(v), v[len(v) // 2], v[0]

    dec_avg, dec_med, dec_min = phase_ms(0, 1)
    result = {
        "metric": "hot-path HBM GB/s per step (decode paged attention over all layers + KV patch cycle + KV resize)",
        "value": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {L} layers, {cfg.num_q_heads}q/{cfg.num_kv_heads}kv heads, "
                               f"D{cfg.head_dim}, block {cfg.block_tokens}, batch {S}, ctx U[{cfg.ctx_lo},{cfg.ctx_hi}]",
                   "pool_blocks_per_layer": B, "pool_GiB": round(B * L * cfg.blk_bytes / 2**30, 1),
                   "live_blocks_per_layer": n_live, "tokens": batch.total_tokens,
                   "split_tokens": int(split), "mig_layers": Lm, "device": dev_name,
                   "decode_only": bool(args.decode_only)},
        "step_bytes": int(step_bytes),
        "decode": {"GBps": round(decode_bytes / (dec_avg * 1e-3) / 1e9, 1),
                   "frac_of_peak": round(decode_bytes / (dec_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                   "ms_avg": round(dec_avg, 4), "ms_median": round(dec_med, 4), "ms_min": round(dec_min, 4),
                   "bytes": int(decode_bytes)},
    }
    launch_us = dec_avg * 1e3 / L
    result["roofline"] = {
        "bound": "hbm", "kernel": f"attn_decode_kernel<{cfg.head_dim},{cfg.block_tokens}> + attn_merge_kernel, one launch per layer",
        "achieved": round(attn_bytes_layer / (launch_us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBPS,
        "unit": "GB/s", "frac": round(attn_bytes_layer / (launch_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "traffic": read_traffic(f"attn_decode_{cfg.name}"),
        "bytes_per_launch": int(attn_bytes_layer), "us_per_launch": round(launch_us, 2),
    }
    if not args.decode_only:
        col_avg, _, col_min = phase_ms(1, 2)
        app_avg, _, app_min = phase_ms(2, 3)
        rsz_avg, _, rsz_min = phase_ms(3, 4)
        result["patch"] = {
            "dirty_blocks": n_dirty, "payload_bytes": int(patch_payload),
            "collect_us": round(col_avg * 1e3, 1), "collect_GBps": round(collect_bytes / (col_avg * 1e-3) / 1e9, 1),
            "apply_us": round(app_avg * 1e3, 1), "apply_GBps": round(apply_bytes / (app_avg * 1e-3) / 1e9, 1)}
        result["resize"] = {
            "shrink_to": B_new, "n_moved": n_moved_expect, "bytes": int(resize_bytes),
            "us": round(rsz_avg * 1e3, 1), "GBps": round(resize_bytes / (rsz_avg * 1e-3) / 1e9, 1),
            "frac_of_peak": round(resize_bytes / (rsz_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        result["switch_us"] = round((col_avg + app_avg + rsz_avg) * 1e3, 1)

    # ---------------- bulk patch round (the patch GB/s figure): 20 % of the live blocks, all layers
    if not args.decode_only:
        bulk_ids_np = pin.draw_dirty_ids(batch, seed, 1, args.bulk_fraction)
        bulk_ids = torch.from_numpy(bulk_ids_np.astype(np.int32)).cuda()
        nb = int(bulk_ids.numel())
        all_layers = list(range(L))
        bulk_cap = 64 + 256 + nb * (4 + L * cfg.blk_bytes) + 4096
        bulk_patch = torch.empty(bulk_cap, dtype=torch.uint8, device="cuda")
        bulk_payload = nb * L * cfg.blk_bytes
        tc, ta = [], []
        for it in range(11):
            e0, e1, e2 = ev(), ev(), ev()
            P.pipelive_kv_mark_dirty(region, bulk_ids, 0)
            e0.record()
            P.pipelive_kv_patch_collect(region, all_layers, bulk_patch)
            e1.record()
            P.pipelive_kv_patch_apply(target, all_layers, bulk_patch, dst_block_map=dst_map)
            e2.record()
            torch.cuda.synchronize()
            if it:
                tc.append(e0.elapsed_time(e1))
                ta.append(e1.elapsed_time(e2))
        tcm, tam = sorted(tc)[len(tc) // 2], sorted(ta)[len(ta) // 2]   # medians of 10
        result["patch_bulk"] = {
            "dirty_blocks": nb, "layers": L, "payload_bytes": int(bulk_payload),
            "timing": "median of 10",
            "collect_us": round(tcm * 1e3, 1), "collect_GBps": round(2 * bulk_payload / (tcm * 1e-3) / 1e9, 1),
            "collect_frac_of_peak": round(2 * bulk_payload / (tcm * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "apply_us": round(tam * 1e3, 1), "apply_GBps": round(2 * bulk_payload / (tam * 1e-3) / 1e9, 1),
            "apply_frac_of_peak": round(2 * bulk_payload / (tam * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        st = P.pipelive_kv_read_state(target)
        if st.status != 0 or P.pipelive_kv_read_state(region).status != 0:
            raise RuntimeError("device status word set during the bench")
        # context for the HBM fractions above: what a plain device-to-device copy of the same size class
        # reaches on this part (torch's copy kernel over the patch buffer; read + write bytes counted)
        half = (bulk_cap // 2) & ~0xFFF
        tcp = []
        for it in range(11):
            e0, e1 = ev(), ev()
            e0.record()
            bulk_patch[half:2 * half].copy_(bulk_patch[:half])
            e1.record()
            torch.cuda.synchronize()
            if it:
                tcp.append(e0.elapsed_time(e1))
        tcpm = sorted(tcp)[len(tcp) // 2]
        result["copy_ceiling"] = {"kind": "torch device-to-device copy, read + write", "bytes": int(half),
                                  "us": round(tcpm * 1e3, 1), "GBps": round(2 * half / (tcpm * 1e-3) / 1e9, 1),
                                  "frac_of_peak": round(2 * half / (tcpm * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        del bulk_patch

    # ---------------- steady-state decode at slot granularity (the paper's own unit): every layer
    # appends one token per sequence, the written slots are drained and applied
    if not args.decode_only:
        sreg = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B,
                          dirty_granularity=P.binding.DIRTY_SLOT, share_pool_of=region)
        stgt = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, n_live,
                          dirty_granularity=P.binding.DIRTY_SLOT, share_pool_of=target)
        knew = torch.zeros((S, cfg.num_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
        room = batch.ctx_lens < batch.used.astype(np.int64) * cfg.block_tokens   # a free slot in the last block
        pos_d = torch.from_numpy(np.where(room, batch.ctx_lens, -1).astype(np.int32)).cuda()
        n_tok = int(room.sum())
        spatch = torch.empty(64 + 256 + S * (4 + L * cfg.token_bytes) + 4096, dtype=torch.uint8, device="cuda")
        tapp, tcol, tapl = [], [], []
        for it in range(11):
            e0, e1, e2, e3 = ev(), ev(), ev(), ev()
            e0.record()
            for l in range(L):
                P.pipelive_kv_append(sreg, l, knew, knew, table_d, pos_d, mark=True, count_tokens=(l == 0))
            e1.record()
            P.pipelive_kv_patch_collect(sreg, all_layers, spatch)
            e2.record()
            P.pipelive_kv_patch_apply(stgt, all_layers, spatch, dst_block_map=dst_map)
            e3.record()
            torch.cuda.synchronize()
            if it:
                tapp.append(e0.elapsed_time(e1)); tcol.append(e1.elapsed_time(e2)); tapl.append(e2.elapsed_time(e3))
        med = lambda v: sorted(v)[len(v) // 2]
        if P.pipelive_kv_read_state(stgt).t_applied != 11 * n_tok or P.pipelive_kv_read_state(sreg).status != 0:
            raise RuntimeError("slot-granular cycle lost tokens")
        result["slot_patch"] = {
            "tokens_per_step": n_tok, "layers": L, "payload_bytes": n_tok * L * cfg.token_bytes,
            "append_all_layers_us": round(med(tapp) * 1e3, 1), "collect_us": round(med(tcol) * 1e3, 1),
            "apply_us": round(med(tapl) * 1e3, 1),
            "note": "block-granular patch of the same step carries %d bytes" % (n_dirty * L * cfg.blk_bytes)}

    # ---------------- prefill attention (the compute-bound neighbour of the decode path): the
    # prefill-heavy pattern, 512-token prompts, and a 512-token chunk on top of 4096 cached tokens
    if not args.decode_only:
        MFMA_PEAK_TFLOPS = 2500.0
        pres = {}
        for tag, Sp, ctxp, qlp in (("prompt512", 64, 512, 512), ("chunk512_of_4096", 16, 4096, 512)):
            pcfg = pin.StageConfig(tag, 1, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens,
                                   Sp, ctxp, ctxp)
            pb = pin.draw_batch(pcfg, seed, pool_factor=1.25)
            preg = P.KVRegion(1, pcfg.num_q_heads, pcfg.num_kv_heads, pcfg.head_dim, pcfg.block_tokens,
                              pb.num_blocks, arenas=3)
            fill_live_blocks(preg, pcfg, pb, seed, pb.num_blocks, poison_tail=False)
            qo_d = torch.arange(0, (Sp + 1) * qlp, qlp, dtype=torch.int32, device="cuda")
            tq = Sp * qlp
            pq = torch.from_numpy(pin.bf16_normal(pin.stream_key(seed, pin.STREAM_Q), 0, tq * pcfg.num_q_heads *
                                                  pcfg.head_dim).view(np.int16)).cuda().view(torch.bfloat16)
            pq = pq.view(tq, pcfg.num_q_heads, pcfg.head_dim)
            pt, pc = torch.from_numpy(pb.table).cuda(), torch.from_numpy(pb.ctx_lens).cuda()
            ptimes = {}
            for odt in (torch.float32, torch.bfloat16):
                pout = torch.empty((tq, pcfg.num_q_heads, pcfg.head_dim), dtype=odt, device="cuda")
                for _ in range(2):
                    P.pipelive_paged_attn_prefill(preg, 0, pq, pout, pt, pc, qo_d, tq)
                e0, e1 = ev(), ev()
                e0.record()
                for _ in range(10):
                    P.pipelive_paged_attn_prefill(preg, 0, pq, pout, pt, pc, qo_d, tq)
                e1.record()
                torch.cuda.synchronize()
                ptimes[odt] = e0.elapsed_time(e1) / 10
            pms, pms16 = ptimes[torch.float32], ptimes[torch.bfloat16]
            # the chunk's write side (token-major K/V rows -> in-block layout), same launch pattern
            pk = pq[:, :pcfg.num_kv_heads, :].contiguous()
            for _ in range(2):
                P.pipelive_kv_append_chunk(preg, 0, pk, pk, pt, pc, qo_d, tq, mark=False)
            e2, e3 = ev(), ev()
            e2.record()
            for _ in range(10):
                P.pipelive_kv_append_chunk(preg, 0, pk, pk, pt, pc, qo_d, tq, mark=False)
            e3.record()
            torch.cuda.synchronize()
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
        result["prefill"] = {"bound": "mfma", "peak_TFLOPs": MFMA_PEAK_TFLOPS, "dtype": "bf16",
                             "note": "fp32 output: softmax weights as bf16 pairs (three MFMA passes per tile); "
                                     "bf16 output: single bf16 weights (two passes)", **pres}

    # ---------------- CPU oracle on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        import oracle
        ncores = min(16, os.cpu_count() or 1)
        Lc = max(1, min(L, args.cpu_layers))
        ids = batch.live_ids
        compact = np.full(B, -1, dtype=np.int32)
        compact[ids] = np.arange(len(ids), dtype=np.int32)
        n_ar = 3
        host = oracle.HostKV(Lc, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens,
                             len(ids), layout=cfg.layout, arenas=n_ar)
        for l in range(Lc):
            data = region.read_blocks(l, ids).cpu().numpy().view(np.uint16)   # the inputs, copied back
            for a in range(n_ar):
                host.arenas[l * n_ar + a][:] = data[a::n_ar]
        tab = np.where(batch.table == pin.TABLE_FILL, pin.TABLE_FILL, compact[np.minimum(batch.table, B - 1)])
        tab = np.ascontiguousarray(tab, dtype=np.int32)
        tc, err, num, den = 0.0, 0.0, 0.0, 0.0
        for l in range(Lc):
            qh = pin.q_bits(cfg, seed, l)
            tc0 = time.perf_counter()
            ref = host.attn_decode(l, qh, tab, batch.ctx_lens, nthreads=ncores)
            tc += time.perf_counter() - tc0
            got = outs[l].cpu().numpy().astype(np.float64)
            err = max(err, float(np.abs(got - ref).max()))
            num += float(((got - ref) ** 2).sum())
            den += float((ref.astype(np.float64) ** 2).sum())
        cpu_bytes = Lc * batch.total_tokens * cfg.token_bytes
        # the same oracle on one thread, on the 16 shortest sequences of layer 0
        short = np.argsort(batch.ctx_lens)[:16]
        tc1 = time.perf_counter()
        host.attn_decode(0, pin.q_bits(cfg, seed, 0)[short], tab[short], batch.ctx_lens[short], nthreads=1)
        tc1 = time.perf_counter() - tc1
        one_bytes = int(batch.ctx_lens[short].sum()) * cfg.token_bytes
        result["cpu_baseline"] = {
            "value": round(cpu_bytes / tc / 1e9, 4), "unit": "GB/s", "cores": ncores, "kind": "oracle",
            "sample": f"decode attention of layers 0..{Lc - 1} of {L} (all {S} sequences, all "
                      f"{cfg.num_q_heads} heads, {Lc * batch.total_tokens} token-layers), {tc:.2f} s wall on "
                      f"{ncores} threads",
            "single_thread": {"value": round(one_bytes / tc1 / 1e9, 4), "unit": "GB/s",
                              "sample": f"layer 0, the 16 shortest sequences ({int(batch.ctx_lens[short].sum())} tokens), "
                                        f"{tc1:.2f} s"},
            "gpu_vs_oracle_max_abs": err, "gpu_vs_oracle_rel_l2": math.sqrt(num / den)}
    # ---------------- independently allocated, layer-stacked blocks: the same batch over a pool of
    # 2 MiB physical blocks (k = 4 layers x 128 tokens), decode, pointer-only shrink, real release
    if not args.decode_only:
        sreg = stgt = None      # second handles over the same pools
        del region, target, patch, ws, qs
        torch.cuda.empty_cache()
        k_stack, bs_v = 4, 128
        vcfg = pin.StageConfig(cfg.name + "-stacked", L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, bs_v,
                               S, cfg.ctx_lo, cfg.ctx_hi)
        v_live = int(((ctx.astype(np.int64) + bs_v - 1) // bs_v).sum())
        Bv = int(v_live * 1.5)
        t0 = time.perf_counter()
        vreg = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, bs_v, Bv, stack_k=k_stack,
                          backing="vmm")
        t_alloc = time.perf_counter() - t0
        vb = pin.draw_batch(vcfg, seed, num_blocks=Bv)
        fill_live_blocks(vreg, vcfg, vb, seed, Bv, poison_tail=True)
        vt, vc, vu = (torch.from_numpy(x).cuda() for x in (vb.table, vb.ctx_lens, vb.used))
        vq = torch.from_numpy(pin.q_bits(vcfg, seed, 0).view(np.int16)).cuda().view(torch.bfloat16)
        vout = torch.empty((S, cfg.num_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda")
        vmax = int(vb.ctx_lens.max())
        vws = vreg.attn_workspace(S, vmax, 0)

        def vdecode():
            for l in range(L):
                P.pipelive_paged_attn_decode(vreg, l, vq, vout, vt, vc, max_ctx=vmax, workspace=vws)
        for _ in range(3):
            vdecode()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(10):
            vdecode()
        e1.record()
        torch.cuda.synchronize()
        v_ms = e0.elapsed_time(e1) / 10
        v_bytes = L * (vb.total_tokens * cfg.token_bytes + q_bytes + out_bytes + 4 * int(vb.used.sum()))
        ref_out = vout.clone()
        Bv_new = int(Bv * 0.8)
        v_moved = int((vb.live_ids >= Bv_new).sum())
        vrws = vreg.resize_workspace()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rc, res = P.pipelive_kv_resize(vreg, Bv_new, [vt], [vu], workspace=vrws)
        torch.cuda.synchronize()
        t_shrink = time.perf_counter() - t0
        if rc != P.OK or res.n_moved != v_moved:
            raise RuntimeError(f"stacked shrink failed: rc={rc} moved={res.n_moved} expected={v_moved}")
        free_a = torch.cuda.mem_get_info()[0]
        t0 = time.perf_counter()
        n_rel = vreg.release_tail(Bv)
        t_rel = time.perf_counter() - t0
        free_b = torch.cuda.mem_get_info()[0]
        vdecode()
        torch.cuda.synchronize()
        if not torch.equal(vout, ref_out):
            raise RuntimeError("decode changed after the pointer-only shrink")
        tok = cfg.token_bytes
        util = {str(k): round(P.pipelive_kv_utilization(ctx, P.pipelive_stacked_block_tokens(2 << 20, k, tok)), 4)
                for k in (1, 2, 4, 8, 16)}
        result["stacked_vmm"] = {
            "stack_k": k_stack, "block_tokens": bs_v, "phys_block_bytes": vreg.phys_bytes,
            "pool_blocks": Bv, "groups": vreg.groups, "alloc_ms": round(t_alloc * 1e3, 1),
            "decode_GBps": round(v_bytes / v_ms / 1e6, 1), "decode_frac_of_peak": round(v_bytes / v_ms / 1e6 / 8000.0, 4),
            "shrink_to": Bv_new, "ids_remapped": v_moved, "bytes_copied": 0,
            "shrink_us": round(t_shrink * 1e6, 1), "released_blocks": n_rel,
            "release_ms": round(t_rel * 1e3, 1), "returned_GiB": round((free_b - free_a) / 2**30, 2),
            "effective_kv_utilization_vs_k": util,
            "note": "shrink_us is host wall time of pipelive_kv_resize incl. its one sync; release is driver time"}
        del vreg

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
