"""Fill a device KV region with the seeded synthetic content (torch ops only).

Duck-typed on the region: it needs ``write_blocks(layer, ids, int16 tensor)``
and ``set_live(ids)``; this module imports neither the HIP binding nor the
oracle."""
from __future__ import annotations

import numpy as np

from . import BF16_NAN, StageConfig, kv_blocks_bits_torch, token_slot_mask


def fill_live_blocks(region, cfg: StageConfig, batch, seed: int, capacity_blocks: int,
                     layers=None, epoch: int = 0, chunk_blocks: int = 512, poison_tail: bool = True,
                     device="cuda") -> None:
    """Write block content for every live block of every layer in ``layers``.

    Content of (layer, block id) is the pure function kv_block_bits(...); the
    slots of a sequence's last block past its context length are poisoned
    with NaN when ``poison_tail``."""
    import torch

    ids = np.asarray(batch.live_ids, dtype=np.int64)
    tails = {}
    if poison_tail:
        for s in range(cfg.num_seqs):
            n, u = int(batch.ctx_lens[s]), int(batch.used[s])
            if u and n < u * cfg.block_tokens:
                tails[int(batch.table[s, u - 1])] = n - (u - 1) * cfg.block_tokens
    for layer in (layers if layers is not None else range(cfg.num_layers)):
        for i in range(0, len(ids), chunk_blocks):
            part = ids[i:i + chunk_blocks]
            data = kv_blocks_bits_torch(cfg, seed, capacity_blocks, epoch, layer, part, device)
            for k, b in enumerate(part):
                valid = tails.get(int(b))
                if valid is not None:
                    m = token_slot_mask(cfg.layout, cfg.num_kv_heads, cfg.block_tokens,
                                        cfg.head_dim, valid)
                    data[k, torch.from_numpy(m).to(device)] = BF16_NAN - 65536
            region.write_blocks(layer, part, data)
    region.set_live(ids)
