"""Helpers for the GPU parity tests: build a host region (oracle) and a device
region (HIP library) with identical logical contents from the seeded inputs."""
import numpy as np
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P


def live_block_bits(cfg, batch, seed, capacity, epoch, layer):
    """dict block_id -> uint16[blk_elems] for every live block of `layer`;
    slots past the context length are poisoned with NaN."""
    out = {}
    for s in range(cfg.num_seqs):
        n = int(batch.ctx_lens[s])
        for j in range(int(batch.used[s])):
            b = int(batch.table[s, j])
            bits = pin.kv_block_bits(cfg, seed, capacity, epoch, layer, b)
            valid = min(cfg.block_tokens, n - j * cfg.block_tokens)
            if valid < cfg.block_tokens:
                bits = bits.copy()
                bits[pin.token_slot_mask(cfg.layout, cfg.num_kv_heads, cfg.block_tokens,
                                         cfg.head_dim, valid)] = pin.BF16_NAN
            out[b] = bits
    return out


def make_pair(cfg, batch, seed, capacity=None, num_layers=None, stack_k=1, arenas=3, backing="arena"):
    """(HostKV, KVRegion) holding the same blocks; everything else is NaN.  backing="vmm": every
    device block is an allocation of its own and the oracle resizes by block-list exchange."""
    L = num_layers or cfg.num_layers
    cap = capacity or batch.num_blocks
    host = oracle.HostKV(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens,
                         batch.num_blocks, capacity_blocks=cap, layout=cfg.layout, stack_k=stack_k,
                         arenas=arenas, fill_bits=pin.BF16_NAN, per_block=backing == "vmm")
    dev = P.KVRegion(L, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens,
                     batch.num_blocks, capacity_blocks=cap, stack_k=stack_k, arenas=arenas + 1,
                     fill_bits=pin.BF16_NAN, backing=backing)
    return host, dev


def fill_pair(cfg, batch, seed, host, dev, layers=None, epoch=0, capacity=None):
    cap = capacity or host.capacity
    for layer in (layers if layers is not None else range(cfg.num_layers)):
        blocks = live_block_bits(cfg, batch, seed, cap, epoch, layer)
        ids = sorted(blocks)
        arr = np.stack([blocks[b] for b in ids])
        for b, row in zip(ids, arr):
            host.block(layer, b)[:] = row
        dev.write_blocks(layer, ids, torch.from_numpy(arr.view(np.int16)).cuda())
    host.set_live(batch.live_ids)
    dev.set_live(batch.live_ids)


def dev_block(dev, layer, b) -> np.ndarray:
    return dev.block(layer, b).cpu().numpy().view(np.uint16)


def assert_pools_equal(host, dev, layers, ids):
    for layer in layers:
        got = dev.read_blocks(layer, list(ids)).cpu().numpy().view(np.uint16)
        for k, b in enumerate(ids):
            assert np.array_equal(got[k], host.block(layer, int(b))), (layer, int(b))


def bitmap_ids(t: torch.Tensor, n: int) -> np.ndarray:
    bits = np.unpackbits(t.cpu().numpy(), bitorder="little")[:n]
    return np.nonzero(bits)[0]


def attn_errors(got: np.ndarray, ref: np.ndarray):
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    max_abs = float(np.abs(got - ref).max()) if got.size else 0.0
    den = np.sqrt((ref * ref).sum())
    rel = float(np.sqrt(((got - ref) ** 2).sum()) / (den if den > 0 else 1.0))
    return max_abs, rel


MAX_ABS, REL_L2 = 1e-2, 2e-3  # tolerance of the attention output (bf16 in, fp32 accumulate)

# Prefill attention with bf16 output: the output is rounded to bf16 (relative error <= 2^-9 per element)
# and the kernel then also rounds each softmax weight p_j to one bf16 before the PV product (<= 2^-9
# relative per weight, in numerator and denominator).  Per element |err| <= 2^-9 (2 |o| + max|v|): with
# the generator's |v| <= 4.4 and |o| <= max|v| that is < 2.6e-2; in the L2 norm the output rounding alone
# is <= 2^-9 = 1.95e-3 and the independent weight roundings add about 2^-9 / sqrt(3).
BF16_MAX_ABS, BF16_REL_L2 = 3e-2, 4e-3
