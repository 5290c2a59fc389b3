"""Seeded synthetic inputs shared by the tests, the bench and the smoke check.

This module only *draws inputs*: integers from a counter-based generator,
bf16 bit patterns from a normal-quantile table, block-id permutations and the
five workload shapes.  It contains none of the method's arithmetic (no
attention, no resize planning, no patch encoding) and it imports neither the
HIP binding nor the oracle, so both sides can be fed from it.

Generator: splitmix64's output function applied to ``key + (counter+1)*GOLD``
where ``key`` is derived from (seed, stream).  Every draw is a pure function
of (seed, stream, counter), so the CPU (numpy, uint64) and the GPU (torch,
int64 with wrap-around) regenerate identical values without copying pools.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from functools import lru_cache

import numpy as np

MASTER_SEED = 20260412

_GOLD = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK = (1 << 64) - 1

# stream ids (one per purpose)
STREAM_LENGTHS = 1
STREAM_PERM = 2
STREAM_KV = 3
STREAM_Q = 4
STREAM_DIRTY = 5
STREAM_MISC = 6


def _mix_int(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


def stream_key(seed: int, stream: int) -> int:
    """64-bit key of one (seed, stream) pair (python int)."""
    return _mix_int(_mix_int(seed * _GOLD + 0x1234567) + stream * _GOLD)


def hash_u64(key: int, counters) -> np.ndarray:
    """splitmix64 output function at ``counters`` (any integer array) -> uint64."""
    c = np.asarray(counters).astype(np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(key) + (c + np.uint64(1)) * np.uint64(_GOLD)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
        z = z ^ (z >> np.uint64(31))
    return z


def _signed(x: int) -> int:
    x &= _MASK
    return x - (1 << 64) if x >= (1 << 63) else x


def hash_i64_torch(key: int, counters):
    """Same function as :func:`hash_u64` on a torch int64 tensor (any device).

    int64 multiplication wraps like uint64; right shifts are made logical by
    masking off the sign-extension bits."""
    import torch

    def lsr(z, k):
        return (z >> k) & ((1 << (64 - k)) - 1)

    z = (counters + 1) * _signed(_GOLD) + _signed(key)
    z = (z ^ lsr(z, 30)) * _signed(_M1)
    z = (z ^ lsr(z, 27)) * _signed(_M2)
    z = z ^ lsr(z, 31)
    return z


@lru_cache(maxsize=1)
def bf16_normal_table() -> np.ndarray:
    """65536 bf16 bit patterns: entry i is the N(0,1) quantile at (i+0.5)/65536,
    rounded to nearest-even bf16.  Indexing it with 16 uniform bits gives
    bf16 ~ N(0,1) (clipped at about +-4.3 sigma)."""
    from scipy.special import ndtri

    p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    f = ndtri(p).astype(np.float32)
    u = f.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_normal(key: int, start: int, count: int) -> np.ndarray:
    """``count`` bf16 bit patterns (uint16) for counters start..start+count-1."""
    h = hash_u64(key, np.arange(start, start + count, dtype=np.uint64))
    return bf16_normal_table()[(h >> np.uint64(48)).astype(np.int64)]


def bf16_normal_torch(key: int, start: int, count: int, device):
    """Device twin of :func:`bf16_normal`; returns an int16 tensor of bit patterns."""
    import torch

    tab = _table_torch(str(device))
    c = torch.arange(start, start + count, dtype=torch.int64, device=device)
    h = hash_i64_torch(key, c)
    idx = (h >> 48) & 0xFFFF
    return tab[idx]


_TABLE_CACHE: dict = {}


def _table_torch(device: str):
    import torch

    if device not in _TABLE_CACHE:
        t = torch.from_numpy(bf16_normal_table().view(np.int16).copy())
        _TABLE_CACHE[device] = t.to(device)
    return _TABLE_CACHE[device]


def uniform_ints(key: int, start: int, count: int, lo: int, hi: int) -> np.ndarray:
    """Integers on the closed range [lo, hi] (int64)."""
    h = hash_u64(key, np.arange(start, start + count, dtype=np.uint64))
    return (lo + (h % np.uint64(hi - lo + 1)).astype(np.int64)).astype(np.int64)


def permutation(key: int, n: int) -> np.ndarray:
    """A seeded permutation of range(n): indices sorted by their hash."""
    h = hash_u64(key, np.arange(n, dtype=np.uint64))
    return np.argsort(h, kind="stable").astype(np.int64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit pattern (uint16). Inputs finite."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    u = np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


BF16_NAN = 0xFFFF  # poison pattern for unused slots and free blocks

# --------------------------------------------------------------------------
# in-block layouts (byte placement only; both consumers document the same
# formulas independently)
LAYOUT_D8 = 0   # runs of min(bs, 32) tokens, each K[Hkv][D/8][run][8] then V[Hkv][D][run]
LAYOUT_ROW = 1  # K[Hkv][bs][D]      then V[Hkv][bs][D]


def block_elems(num_kv_heads: int, block_tokens: int, head_dim: int) -> int:
    """bf16 elements of one (layer, block): K and V for all KV heads."""
    return 2 * num_kv_heads * block_tokens * head_dim


def token_slot_mask(layout: int, num_kv_heads: int, block_tokens: int, head_dim: int,
                    n_valid: int) -> np.ndarray:
    """Boolean mask over the elements of one block: True where the element
    belongs to a token slot >= n_valid (to be poisoned)."""
    hkv, bs, d = num_kv_heads, block_tokens, head_dim
    tok_bad = np.arange(bs) >= n_valid
    if layout == LAYOUT_D8:
        # sub-blocks of min(bs, 32) tokens, each K[Hkv][D/8][sb][8] then V[Hkv][D][sb]
        sb = min(bs, 32)
        parts = []
        for u in range(bs // sb):
            bad = tok_bad[u * sb:(u + 1) * sb]
            parts.append(np.broadcast_to(bad[None, None, :, None], (hkv, d // 8, sb, 8)).reshape(-1))
            parts.append(np.broadcast_to(bad[None, None, :], (hkv, d, sb)).reshape(-1))
        return np.concatenate(parts)
    elif layout == LAYOUT_ROW:
        k = np.broadcast_to(tok_bad[None, :, None], (hkv, bs, d))
        v = k
    else:
        raise ValueError("layout")
    return np.concatenate([k.reshape(-1), v.reshape(-1)])


# --------------------------------------------------------------------------
@dataclass(frozen=True)
class StageConfig:
    """One of the workload shapes (a pipeline stage's attention + KV pool)."""
    name: str
    num_layers: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_tokens: int
    num_seqs: int
    ctx_lo: int
    ctx_hi: int
    layout: int = LAYOUT_D8

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def blk_elems(self) -> int:
        return block_elems(self.num_kv_heads, self.block_tokens, self.head_dim)

    @property
    def blk_bytes(self) -> int:
        return 2 * self.blk_elems

    @property
    def token_bytes(self) -> int:
        """K+V bytes of one token in one layer."""
        return 2 * self.num_kv_heads * self.head_dim * 2


CONFIGS = {
    "tiny": StageConfig("tiny", 2, 4, 2, 64, 16, 8, 1, 256),
    "stage8b": StageConfig("stage8b", 16, 32, 8, 128, 16, 64, 512, 4096),
    "resize8b": StageConfig("resize8b", 16, 32, 8, 128, 16, 64, 256, 2048),
    "stage70b": StageConfig("stage70b", 20, 64, 8, 128, 16, 128, 1024, 8192),
    "longctx8b": StageConfig("longctx8b", 16, 32, 8, 128, 32, 16, 16384, 32768),
}


def scaled(cfg: StageConfig, **kw) -> StageConfig:
    """A copy of ``cfg`` with some fields replaced (reduced parity cases)."""
    return replace(cfg, **kw)


@dataclass
class Batch:
    """A drawn decode batch: context lengths and block tables over a pool."""
    cfg: StageConfig
    seed: int
    num_blocks: int                 # pool size B (ids 0..B-1)
    ctx_lens: np.ndarray            # int32 [S]
    table: np.ndarray               # int32 [S][stride]; unused entries = TABLE_FILL
    used: np.ndarray                # int32 [S]: ceil(ctx/bs)
    live_ids: np.ndarray            # int64 sorted unique block ids referenced

    @property
    def stride(self) -> int:
        return int(self.table.shape[1])

    @property
    def total_tokens(self) -> int:
        return int(self.ctx_lens.sum())


TABLE_FILL = 0x7FFFFFF0  # an id far out of any pool: must never be dereferenced


def draw_ctx_lens(cfg: StageConfig, seed: int) -> np.ndarray:
    key = stream_key(seed, STREAM_LENGTHS)
    return uniform_ints(key, 0, cfg.num_seqs, cfg.ctx_lo, cfg.ctx_hi).astype(np.int32)


def draw_batch(cfg: StageConfig, seed: int = MASTER_SEED, num_blocks: int | None = None,
               pool_factor: float | None = None, stride_pad: int = 0) -> Batch:
    """Draw context lengths, then deal the leading entries of a seeded
    permutation of [0, B) to the sequences in order.

    ``num_blocks`` fixes the pool size; else ``pool_factor`` sizes it as
    ceil(n_live * pool_factor); else it is exactly n_live."""
    ctx = draw_ctx_lens(cfg, seed)
    used = (ctx.astype(np.int64) + cfg.block_tokens - 1) // cfg.block_tokens
    n_live = int(used.sum())
    if num_blocks is None:
        num_blocks = int(math.ceil(n_live * pool_factor)) if pool_factor else n_live
    if n_live > num_blocks:
        raise ValueError(f"draw needs {n_live} blocks, pool has {num_blocks}")
    perm = permutation(stream_key(seed, STREAM_PERM), num_blocks)
    stride = int(used.max()) + stride_pad if len(used) else stride_pad
    table = np.full((cfg.num_seqs, max(stride, 1)), TABLE_FILL, dtype=np.int32)
    off = 0
    for s in range(cfg.num_seqs):
        u = int(used[s])
        table[s, :u] = perm[off:off + u]
        off += u
    live = np.sort(perm[:n_live])
    return Batch(cfg, seed, num_blocks, ctx, table, used.astype(np.int32), live)


def kv_counter_base(cfg: StageConfig, capacity_blocks: int, epoch: int, layer: int,
                    block_id: int) -> int:
    """First generator counter of the bf16 elements of (epoch, layer, block)."""
    return ((epoch * cfg.num_layers + layer) * capacity_blocks + block_id) * cfg.blk_elems


def kv_block_bits(cfg: StageConfig, seed: int, capacity_blocks: int, epoch: int, layer: int,
                  block_id: int) -> np.ndarray:
    """uint16 [blk_elems]: the synthetic content of one (layer, block), in
    storage order (the values are i.i.d., so storage order == draw order)."""
    key = stream_key(seed, STREAM_KV)
    base = kv_counter_base(cfg, capacity_blocks, epoch, layer, block_id)
    return bf16_normal(key, base, cfg.blk_elems)


def kv_blocks_bits_torch(cfg: StageConfig, seed: int, capacity_blocks: int, epoch: int,
                         layer: int, block_ids, device):
    """Device twin of :func:`kv_block_bits` for many blocks: int16 [n][blk_elems]."""
    import torch

    key = stream_key(seed, STREAM_KV)
    tab = _table_torch(str(device))
    ids = torch.as_tensor(np.asarray(block_ids, dtype=np.int64), device=device)
    e = torch.arange(cfg.blk_elems, dtype=torch.int64, device=device)
    base = ((epoch * cfg.num_layers + layer) * capacity_blocks + ids) * cfg.blk_elems
    c = base[:, None] + e[None, :]
    h = hash_i64_torch(key, c)
    return tab[(h >> 48) & 0xFFFF]


def q_bits(cfg: StageConfig, seed: int, layer: int) -> np.ndarray:
    """uint16 [S][Hq][D] query bit patterns for one layer."""
    key = stream_key(seed, STREAM_Q)
    n = cfg.num_seqs * cfg.num_q_heads * cfg.head_dim
    return bf16_normal(key, layer * n, n).reshape(cfg.num_seqs, cfg.num_q_heads, cfg.head_dim)


def last_block_ids(batch: Batch) -> np.ndarray:
    """Block id holding the newest token of every non-empty sequence."""
    out = []
    for s in range(batch.cfg.num_seqs):
        u = int(batch.used[s])
        if u:
            out.append(int(batch.table[s, u - 1]))
    return np.asarray(out, dtype=np.int64)


def draw_dirty_ids(batch: Batch, seed: int, round_idx: int, fraction: float,
                   include_last: bool = True) -> np.ndarray:
    """Sorted ids of the blocks written in one round: a seeded sample of
    ``ceil(fraction * n_live)`` live blocks, united with every sequence's last
    block (decode appends there)."""
    live = batch.live_ids
    k = int(math.ceil(fraction * len(live)))
    key = stream_key(seed, STREAM_DIRTY) ^ _mix_int(round_idx + 1)
    perm = permutation(key, len(live))
    pick = live[perm[:k]]
    if include_last:
        pick = np.union1d(pick, last_block_ids(batch))
    return np.sort(np.unique(pick)).astype(np.int64)


def geometric_fractions(first: float, last: float, rounds: int) -> list[float]:
    """Dirty fractions decaying geometrically from ``first`` to ``last``."""
    if rounds == 1:
        return [first]
    r = (last / first) ** (1.0 / (rounds - 1))
    return [first * r ** i for i in range(rounds)]


# --------------------------------------------------------------------------
# decode steps: the caller's block manager and the new tokens' K/V
STREAM_NEWTOK = 7


def new_token_bits(cfg: StageConfig, seed: int, step: int, layer: int):
    """(k, v) uint16 [S][Hkv][D] each: K/V of the token every sequence appends in
    decode step ``step`` at ``layer``."""
    key = stream_key(seed, STREAM_NEWTOK)
    n = cfg.num_seqs * cfg.num_kv_heads * cfg.head_dim
    base = (step * cfg.num_layers + layer) * 2 * n
    shape = (cfg.num_seqs, cfg.num_kv_heads, cfg.head_dim)
    return bf16_normal(key, base, n).reshape(shape), bf16_normal(key, base + n, n).reshape(shape)


class BlockManager:
    """The serving engine's side of a decode batch (an *input* of the library, which is
    told liveness and tables and never allocates ids itself): context lengths, block
    table and the set of live ids, advanced one token per sequence per step.  A sequence
    that fills its last block takes the lowest free id below the current pool size."""

    def __init__(self, batch: Batch, capacity_blocks: int | None = None):
        self.cfg = batch.cfg
        self.num_blocks = int(batch.num_blocks)
        cap = int(capacity_blocks or batch.num_blocks)
        self.ctx = batch.ctx_lens.astype(np.int32).copy()
        self.used = batch.used.astype(np.int32).copy()
        self.table = batch.table.copy()
        self.live = np.zeros(cap, dtype=bool)
        self.live[batch.live_ids] = True

    def set_num_blocks(self, n: int) -> None:
        self.num_blocks = int(n)

    def adopt(self, table: np.ndarray, live_ids) -> None:
        """take over tables and liveness as a resize left them"""
        self.table = table.copy()
        self.live[:] = False
        self.live[np.asarray(live_ids, dtype=np.int64)] = True

    def live_ids(self) -> np.ndarray:
        return np.nonzero(self.live)[0]

    def step(self):
        """Advance every sequence by one token.  Returns (positions int32 [S], the position
        the new token is written at; new_entries [(seq, table column, block id)])."""
        bs = self.cfg.block_tokens
        pos = self.ctx.copy()
        new_entries = []
        free = None
        for s in range(len(self.ctx)):
            if int(pos[s]) == int(self.used[s]) * bs:        # last block full (or no block yet)
                if int(self.used[s]) >= self.table.shape[1]:
                    raise ValueError("block table row is full: draw the batch with stride_pad")
                if free is None:
                    free = iter(np.nonzero(~self.live[: self.num_blocks])[0])
                try:
                    b = int(next(free))
                except StopIteration:
                    raise ValueError("pool exhausted") from None
                self.live[b] = True
                self.table[s, self.used[s]] = b
                new_entries.append((s, int(self.used[s]), b))
                self.used[s] += 1
        self.ctx = (self.ctx + 1).astype(np.int32)
        return pos.astype(np.int32), new_entries

    def last_block_ids(self) -> np.ndarray:
        return np.asarray([int(self.table[s, self.used[s] - 1]) for s in range(len(self.ctx)) if self.used[s]],
                          dtype=np.int64)
