"""Python face of the CPU oracle (test infrastructure, never the product path).

Loads ``liboracle.so`` (built from ``pipelive_oracle.c`` with gcc) through
ctypes and offers :class:`HostKV`, a KV region in host memory whose blocks
live in several separate numpy arenas and are reached through a block list of
host addresses, exactly as the device region is reached through device
addresses.  Nothing here imports the HIP binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pipelive_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

OK, E_INVAL, E_INFEASIBLE, E_NOSPACE, E_BUSY, E_RANGE = 0, -1, -2, -3, -4, -5
PATCH_MAGIC = 0x564B4C50
PATCH_HDR_BYTES = 64


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP only parallelises independent outer loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _KV(C.Structure):
    _fields_ = [
        ("num_layers", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("block_tokens", C.c_int32), ("stack_k", C.c_int32),
        ("layout", C.c_int32), ("dirty_gran", C.c_int32),
        ("num_blocks", C.c_int64), ("capacity_blocks", C.c_int64),
        ("block_list", C.c_void_p), ("live_bitmap", C.c_void_p), ("dirty_bitmap", C.c_void_p),
        ("n_acc", C.c_uint64), ("t_applied", C.c_uint64),
        ("per_block", C.c_int32), ("pad_", C.c_int32),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.orc_struct_bytes.restype = C.c_int32
        assert L.orc_struct_bytes() == C.sizeof(_KV)
        L.orc_paged_attn_decode.restype = C.c_int32
        L.orc_paged_attn_decode.argtypes = [C.POINTER(_KV), C.c_int32, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                            C.c_double, C.c_int32]
        L.orc_kv_resize.restype = C.c_int32
        L.orc_kv_resize.argtypes = [C.POINTER(_KV), C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.orc_kv_mark_dirty.restype = C.c_int32
        L.orc_kv_mark_dirty.argtypes = [C.POINTER(_KV), C.c_void_p, C.c_int32, C.c_int64]
        L.orc_patch_max_blocks.restype = C.c_int64
        L.orc_patch_max_blocks.argtypes = [C.POINTER(_KV), C.c_int32, C.c_uint64]
        L.orc_kv_patch_collect.restype = C.c_int32
        L.orc_kv_patch_collect.argtypes = [C.POINTER(_KV), C.c_void_p, C.c_int32, C.c_void_p,
                                           C.c_uint64]
        L.orc_kv_patch_apply.restype = C.c_int32
        L.orc_kv_patch_apply.argtypes = [C.POINTER(_KV), C.c_void_p, C.c_int32, C.c_void_p,
                                         C.c_void_p]
        L.orc_max_blocks.restype = C.c_int64
        L.orc_max_blocks.argtypes = [C.c_double, C.c_double, C.c_int64, C.c_double, C.c_double]
        L.orc_kv_append_chunk.restype = C.c_int32
        L.orc_kv_append_chunk.argtypes = [C.POINTER(_KV), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                          C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
        L.orc_kv_utilization.restype = C.c_double
        L.orc_kv_utilization.argtypes = [C.c_void_p, C.c_int64, C.c_int32]
        L.orc_stacked_block_tokens.restype = C.c_int64
        L.orc_stacked_block_tokens.argtypes = [C.c_uint64, C.c_int32, C.c_uint64]
        L.orc_paged_attn_prefill.restype = C.c_int32
        L.orc_paged_attn_prefill.argtypes = [C.POINTER(_KV), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_double, C.c_int32]
        L.orc_kv_append.restype = C.c_int32
        L.orc_kv_append.argtypes = [C.POINTER(_KV), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                    C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
        L.orc_plan_reconfig.restype = C.c_int32
        L.orc_plan_reconfig.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double,
                                        C.c_double, C.c_double, C.c_int64, C.c_int64, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data


class HostKV:
    """A KV region in host memory.

    ``arenas`` separate numpy allocations hold the physical blocks (block id
    ``b`` of a group sits in arena ``b % arenas``), so nothing may assume
    ``address = base + id * stride``."""

    def __init__(self, num_layers, num_q_heads, num_kv_heads, head_dim, block_tokens,
                 num_blocks, capacity_blocks=None, layout=0, stack_k=1, arenas=3,
                 fill_bits=0xFFFF, dirty_gran=0, per_block=False):
        self.L, self.Hq, self.Hkv, self.D, self.bs = num_layers, num_q_heads, num_kv_heads, head_dim, block_tokens
        self.layout, self.stack_k = layout, stack_k
        self.capacity = int(capacity_blocks if capacity_blocks is not None else num_blocks)
        self.blk_elems = 2 * num_kv_heads * block_tokens * head_dim
        self.blk_bytes = 2 * self.blk_elems
        self.groups = (num_layers + stack_k - 1) // stack_k
        phys_elems = self.blk_elems * stack_k
        self.arenas = []
        self.block_list = np.zeros((self.groups, self.capacity), dtype=np.uint64)
        n_ar = self._n_ar = max(1, min(arenas, self.capacity))
        for g in range(self.groups):
            for a in range(n_ar):
                ids = np.arange(a, self.capacity, n_ar)
                arr = np.full((len(ids), phys_elems), fill_bits, dtype=np.uint16)
                self.arenas.append(arr)  # arena (g, a) is self.arenas[g * n_ar + a]
                self.block_list[g, ids] = arr.ctypes.data + np.arange(len(ids), dtype=np.uint64) * np.uint64(phys_elems * 2)
        nbytes = (self.capacity + 63) // 64 * 8
        self.dirty_gran = dirty_gran
        self.units_per_block = block_tokens if dirty_gran else 1
        self.unit_bytes = 2 * num_kv_heads * head_dim * 2 if dirty_gran else self.blk_bytes
        self.live = np.zeros(nbytes, dtype=np.uint8)
        self.dirty = np.zeros((self.capacity * self.units_per_block + 63) // 64 * 8, dtype=np.uint8)
        self.c = _KV(num_layers, num_q_heads, num_kv_heads, head_dim, block_tokens, stack_k,
                     layout, dirty_gran, int(num_blocks), self.capacity,
                     self.block_list.ctypes.data, self.live.ctypes.data, self.dirty.ctypes.data,
                     0, 0, int(bool(per_block)), 0)
        self.per_block = bool(per_block)
        self._arena_base = np.array([a.ctypes.data for a in self.arenas], dtype=np.uint64)

    # ---- state access
    @property
    def num_blocks(self) -> int:
        return int(self.c.num_blocks)

    @property
    def n_acc(self) -> int:
        return int(self.c.n_acc)

    @property
    def t_applied(self) -> int:
        return int(self.c.t_applied)

    def block(self, layer: int, block_id: int) -> np.ndarray:
        """uint16 view [blk_elems] of (layer, block)."""
        g = layer // self.stack_k
        addr = int(self.block_list[g, int(block_id)])  # follows the block list: a shrink may permute it
        phys = self.blk_bytes * self.stack_k
        for a in range(g * self._n_ar, (g + 1) * self._n_ar):
            off = addr - int(self._arena_base[a])
            if 0 <= off < self.arenas[a].nbytes:
                o = (layer % self.stack_k) * self.blk_elems
                return self.arenas[a][off // phys, o:o + self.blk_elems]
        raise IndexError(f"block {block_id} of layer {layer} has no memory")

    def set_live(self, ids) -> None:
        self.live[:] = 0
        ids = np.asarray(ids, dtype=np.int64)
        np.bitwise_or.at(self.live, ids >> 3, (1 << (ids & 7)).astype(np.uint8))

    def live_ids(self) -> np.ndarray:
        bits = np.unpackbits(self.live, bitorder="little")[: self.num_blocks]
        return np.nonzero(bits)[0]

    def dirty_ids(self) -> np.ndarray:
        bits = np.unpackbits(self.dirty, bitorder="little")[: self.num_blocks * self.units_per_block]
        return np.nonzero(bits)[0]

    # ---- the four operations
    def attn_decode(self, layer, q_bits, table, ctx_lens, scale=0.0, nthreads=1) -> np.ndarray:
        q = np.ascontiguousarray(q_bits, dtype=np.uint16)
        table = np.ascontiguousarray(table, dtype=np.int32)
        ctx = np.ascontiguousarray(ctx_lens, dtype=np.int32)
        S = len(ctx)
        out = np.empty((S, self.Hq, self.D), dtype=np.float32)
        rc = lib().orc_paged_attn_decode(C.byref(self.c), layer, _ptr(q), _ptr(out), _ptr(table),
                                         table.shape[1], _ptr(ctx), S, float(scale), nthreads)
        if rc != OK:
            raise OracleError(rc)
        return out

    def attn_prefill(self, layer, q_bits, table, ctx_lens, q_offsets, scale=0.0, nthreads=1) -> np.ndarray:
        """q_bits uint16 [total_q][Hq][D]; q_offsets int32 [S+1]; returns float32 [total_q][Hq][D]."""
        q = np.ascontiguousarray(q_bits, dtype=np.uint16)
        table = np.ascontiguousarray(table, dtype=np.int32)
        ctx = np.ascontiguousarray(ctx_lens, dtype=np.int32)
        qo = np.ascontiguousarray(q_offsets, dtype=np.int32)
        out = np.empty((int(qo[-1]), self.Hq, self.D), dtype=np.float32)
        rc = lib().orc_paged_attn_prefill(C.byref(self.c), layer, _ptr(q), _ptr(out), _ptr(table), table.shape[1],
                                          _ptr(ctx), _ptr(qo), len(ctx), float(scale), nthreads)
        if rc != OK:
            raise OracleError(rc)
        return out

    def resize(self, new_num_blocks, tables=(), used=()):
        """Returns (rc, remap[int32 old B], result[int64 4]); tables are remapped in place."""
        tabs = [t for t in tables]
        for t in tabs:
            assert t.dtype == np.int32 and t.flags.c_contiguous
        useds = [np.ascontiguousarray(u, dtype=np.int32) for u in used]
        n = len(tabs)
        tp = (C.c_void_p * max(n, 1))(*[t.ctypes.data for t in tabs])
        up = (C.c_void_p * max(n, 1))(*[u.ctypes.data for u in useds])
        rows = np.asarray([t.shape[0] for t in tabs], dtype=np.int32)
        strides = np.asarray([t.shape[1] for t in tabs], dtype=np.int32)
        remap = np.full(max(self.num_blocks, 1), -2, dtype=np.int32)
        result = np.zeros(4, dtype=np.int64)
        rc = lib().orc_kv_resize(C.byref(self.c), int(new_num_blocks), tp, _ptr(rows), _ptr(strides),
                                 up, n, _ptr(remap), _ptr(result))
        return rc, remap, result

    def append(self, layer, k_new, v_new, table, positions, mark=True, count_tokens=False) -> int:
        """k_new, v_new: uint16 [S][Hkv][D]; positions int32 [S] (-1 = skip)."""
        k = np.ascontiguousarray(k_new, dtype=np.uint16)
        v = np.ascontiguousarray(v_new, dtype=np.uint16)
        table = np.ascontiguousarray(table, dtype=np.int32)
        pos = np.ascontiguousarray(positions, dtype=np.int32)
        return lib().orc_kv_append(C.byref(self.c), int(layer), _ptr(k), _ptr(v), _ptr(table), table.shape[1],
                                   _ptr(pos), len(pos), int(bool(mark)), int(bool(count_tokens)))

    def append_chunk(self, layer, k_new, v_new, table, ctx_lens, q_offsets, mark=True, count_tokens=False) -> int:
        """k_new, v_new: uint16 [total_q][Hkv][D]; ctx_lens int32 [S] (chunk included); q_offsets int32 [S+1]."""
        k = np.ascontiguousarray(k_new, dtype=np.uint16)
        v = np.ascontiguousarray(v_new, dtype=np.uint16)
        table = np.ascontiguousarray(table, dtype=np.int32)
        ctx = np.ascontiguousarray(ctx_lens, dtype=np.int32)
        qo = np.ascontiguousarray(q_offsets, dtype=np.int32)
        return lib().orc_kv_append_chunk(C.byref(self.c), int(layer), _ptr(k), _ptr(v), _ptr(table), table.shape[1],
                                         _ptr(ctx), _ptr(qo), len(ctx), int(bool(mark)), int(bool(count_tokens)))

    def mark_dirty(self, ids, n_tokens) -> int:
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        return lib().orc_kv_mark_dirty(C.byref(self.c), _ptr(ids), len(ids), int(n_tokens))

    def patch_max_blocks(self, n_layers, capacity) -> int:
        return int(lib().orc_patch_max_blocks(C.byref(self.c), n_layers, int(capacity)))

    def patch_collect(self, layers, patch: np.ndarray) -> int:
        layers = np.ascontiguousarray(layers, dtype=np.int32)
        assert patch.dtype == np.uint8
        return lib().orc_kv_patch_collect(C.byref(self.c), _ptr(layers), len(layers), _ptr(patch),
                                          patch.nbytes)

    def patch_apply(self, dst_layers, patch: np.ndarray, dst_map=None) -> int:
        dst_layers = np.ascontiguousarray(dst_layers, dtype=np.int32)
        m = None if dst_map is None else np.ascontiguousarray(dst_map, dtype=np.int32)
        return lib().orc_kv_patch_apply(C.byref(self.c), _ptr(dst_layers), len(dst_layers),
                                        _ptr(patch), _ptr(m))


class OracleError(RuntimeError):
    def __init__(self, rc):
        super().__init__(f"oracle returned {rc}")
        self.rc = rc


def parse_patch_header(patch: np.ndarray) -> dict:
    """Decode the 64-byte patch header (little endian)."""
    h = np.frombuffer(patch[:64].tobytes(), dtype=np.uint32)
    q = np.frombuffer(patch[:64].tobytes(), dtype=np.uint64)
    return dict(magic=int(h[0]), version=int(h[1]), n_blocks=int(h[2]), n_layers=int(h[3]),
                block_bytes=int(q[2]), n_acc_tokens=int(q[3]), payload_offset=int(q[4]),
                max_blocks=int(h[10]), more_pending=int(h[11]), unit_tokens=int(h[12]))


def max_blocks(mem_bytes, util, layers, weight_bytes_per_layer, block_bytes_per_layer) -> int:
    return int(lib().orc_max_blocks(mem_bytes, util, layers, weight_bytes_per_layer,
                                    block_bytes_per_layer))


def kv_utilization(ctx_lens, block_tokens) -> float:
    c = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    return float(lib().orc_kv_utilization(c.ctypes.data, len(c), int(block_tokens)))


def stacked_block_tokens(phys_bytes, k, token_bytes_per_layer) -> int:
    return int(lib().orc_stacked_block_tokens(int(phys_bytes), int(k), int(token_bytes_per_layer)))


def plan_reconfig(cur_sets, tgt_sets, num_layers, mem_bytes, util, weight_bytes_per_layer,
                  block_bytes_per_layer, blocks_in_use, cur_blocks):
    """cur_sets / tgt_sets: one set of layer ids (0-based) per GPU.  Returns
    (rc, dict) with the intermediate sets, M_mig as {(src, dst): set}, M_del and the scalars."""
    n = len(cur_sets)
    cur = np.zeros((n, num_layers), dtype=np.uint8)
    tgt = np.zeros((n, num_layers), dtype=np.uint8)
    for i in range(n):
        cur[i, sorted(cur_sets[i])] = 1
        tgt[i, sorted(tgt_sets[i])] = 1
    tmp = np.zeros((n, num_layers), dtype=np.uint8)
    mig = np.zeros((n, n, num_layers), dtype=np.uint8)
    dele = np.zeros((n, num_layers), dtype=np.uint8)
    sc = np.zeros(4, dtype=np.int64)
    mem = np.ascontiguousarray(mem_bytes, dtype=np.float64)
    rc = lib().orc_plan_reconfig(n, num_layers, _ptr(cur), _ptr(tgt), _ptr(mem), float(util),
                                 float(weight_bytes_per_layer), float(block_bytes_per_layer),
                                 int(blocks_in_use), int(cur_blocks), _ptr(tmp), _ptr(mig), _ptr(dele), _ptr(sc))
    out = dict(
        tmp=[set(np.nonzero(tmp[i])[0].tolist()) for i in range(n)],
        mig={(a, b): set(np.nonzero(mig[a, b])[0].tolist()) for a in range(n) for b in range(n) if mig[a, b].any()},
        dele=[set(np.nonzero(dele[i])[0].tolist()) for i in range(n)],
        feasible=bool(sc[0]), need_shrink=bool(sc[1]), b_shrink=int(sc[2]), b_new=int(sc[3]))
    return rc, out
