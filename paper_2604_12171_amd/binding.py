"""Thin ctypes binding of libpipelive.so: argument marshalling only.

Every function has the name of the C entry point it calls (without the
``pipelive_`` prefix being dropped: ``pipelive_paged_attn_decode`` etc.).
Tensors are passed as raw device addresses, the stream as the current torch
stream's handle.  :class:`KVRegion` is plumbing: it owns the torch
allocations of one KV region (block arenas, block list, bitmaps, device
state) and the library handle.  Nothing here computes: if the HIP library
cannot be loaded the import fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

OK, E_INVAL, E_INFEASIBLE, E_NOSPACE, E_BUSY, E_RANGE, E_HIP = 0, -1, -2, -3, -4, -5, -6
LAYOUT_D8 = 0
DIRTY_BLOCK, DIRTY_SLOT = 0, 1
BACKING_ARENA, BACKING_PER_BLOCK = 0, 1
OUT_F32, OUT_BF16 = 0, 1
MAX_PATCH_LAYERS = 128
MAX_TABLES = 8
PATCH_MAGIC = 0x564B4C50

EXPORTS = [
    "pipelive_bitmap_bytes", "pipelive_kv_dirty_units", "pipelive_kv_append", "pipelive_kv_append_chunk", "pipelive_kv_state_bytes", "pipelive_kv_create", "pipelive_kv_destroy",
    "pipelive_kv_num_blocks", "pipelive_paged_attn_decode", "pipelive_paged_attn_prefill", "pipelive_paged_attn_workspace_bytes",
    "pipelive_paged_attn_decode_noalloc", "pipelive_noalloc_scratch_bytes",
    "pipelive_kv_resize", "pipelive_kv_resize_workspace_bytes",
    "pipelive_max_blocks", "pipelive_kv_mark_dirty", "pipelive_patch_max_blocks",
    "pipelive_kv_patch_collect", "pipelive_kv_patch_apply", "pipelive_kv_read_state", "pipelive_kv_tokens_applied",
    "pipelive_vmm_backing_bytes", "pipelive_vmm_pool_create", "pipelive_vmm_pool_destroy", "pipelive_vmm_pool_alloc",
    "pipelive_vmm_pool_free", "pipelive_vmm_pool_allocated", "pipelive_vmm_pool_base",
    "pipelive_arena_create", "pipelive_arena_layout", "pipelive_arena_destroy", "pipelive_arena_base",
    "pipelive_arena_bytes", "pipelive_arena_info", "pipelive_arena_zone", "pipelive_arena_piece_class", "pipelive_kv_utilization", "pipelive_stacked_block_tokens",
    "pipelive_kv_clear_status", "pipelive_plan_reconfig", "pipelive_converged", "pipelive_strerror", "pipelive_last_hip_error", "pipelive_device_ok",
]


class KVDesc(C.Structure):
    _fields_ = [
        ("num_layers", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("block_tokens", C.c_int32), ("stack_k", C.c_int32),
        ("dtype", C.c_int32), ("in_block_layout", C.c_int32),
        ("dirty_granularity", C.c_int32), ("block_backing", C.c_int32),
        ("num_blocks", C.c_int64), ("capacity_blocks", C.c_int64),
        ("block_list", C.c_void_p), ("live_bitmap", C.c_void_p), ("dirty_bitmap", C.c_void_p),
        ("dev_state", C.c_void_p),
    ]


class ResizeResult(C.Structure):
    _fields_ = [("n_live", C.c_int64), ("n_moved", C.c_int64), ("old_num_blocks", C.c_int64),
                ("new_num_blocks", C.c_int64), ("status", C.c_int32), ("reserved", C.c_int32)]


class PatchHdr(C.Structure):
    _fields_ = [("magic", C.c_uint32), ("version", C.c_uint32), ("n_blocks", C.c_uint32),
                ("n_layers", C.c_uint32), ("block_bytes", C.c_uint64), ("n_acc_tokens", C.c_uint64),
                ("payload_offset", C.c_uint64), ("max_blocks", C.c_uint32),
                ("more_pending", C.c_uint32), ("unit_tokens", C.c_uint32), ("pad", C.c_uint8 * 12)]


class ReconfigPlan(C.Structure):
    _fields_ = [("feasible", C.c_int32), ("need_shrink", C.c_int32), ("b_shrink", C.c_int64),
                ("b_new", C.c_int64), ("n_mig", C.c_int32), ("n_del", C.c_int32)]


class ArenaInfo(C.Structure):
    _fields_ = [("n_pieces", C.c_int32), ("n_classes", C.c_int32), ("class_pieces", C.c_int32 * 4),
                ("n_runs", C.c_int32), ("probe_ms", C.c_float), ("rate_same_GBps", C.c_float), ("rate_other_GBps", C.c_float)]


class KVState(C.Structure):
    _fields_ = [("n_acc", C.c_uint64), ("t_applied", C.c_uint64), ("status", C.c_int32),
                ("reserved", C.c_int32)]


assert C.sizeof(PatchHdr) == 64

_lib = None


def load(path: str | None = None):
    """dlopen the HIP library (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or _build.LIB
    if not os.path.exists(path):
        _build.build_lib()
    L = C.CDLL(path)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.pipelive_bitmap_bytes.restype = sz
    L.pipelive_bitmap_bytes.argtypes = [i64]
    L.pipelive_kv_dirty_units.restype = i64
    L.pipelive_kv_dirty_units.argtypes = [i64, i32, i32]
    L.pipelive_kv_append.restype = i32
    L.pipelive_kv_append.argtypes = [vp, i32, vp, vp, vp, i32, vp, i32, i32, i32, vp]
    L.pipelive_kv_append_chunk.restype = i32
    L.pipelive_kv_append_chunk.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, vp]
    L.pipelive_kv_state_bytes.restype = sz
    L.pipelive_kv_state_bytes.argtypes = [i64]
    L.pipelive_kv_create.restype = i32
    L.pipelive_kv_create.argtypes = [C.POINTER(KVDesc), C.POINTER(vp)]
    L.pipelive_kv_destroy.restype = None
    L.pipelive_kv_destroy.argtypes = [vp]
    L.pipelive_kv_num_blocks.restype = i64
    L.pipelive_kv_num_blocks.argtypes = [vp]
    L.pipelive_paged_attn_decode.restype = i32
    L.pipelive_paged_attn_decode.argtypes = [vp, i32, vp, vp, i32, vp, i32, vp, i32, i32, C.c_float,
                                             i32, vp, sz, vp]
    L.pipelive_paged_attn_decode_noalloc.restype = i32
    L.pipelive_paged_attn_decode_noalloc.argtypes = [vp, i32, vp, vp, i32, vp, i32, vp, i32, i32, C.c_float, i32, vp]
    L.pipelive_noalloc_scratch_bytes.restype = sz
    L.pipelive_noalloc_scratch_bytes.argtypes = []
    L.pipelive_paged_attn_prefill.restype = i32
    L.pipelive_paged_attn_prefill.argtypes = [vp, i32, vp, vp, i32, vp, i32, vp, vp, i32, i32, i32,
                                              C.c_float, vp]
    L.pipelive_paged_attn_workspace_bytes.restype = sz
    L.pipelive_paged_attn_workspace_bytes.argtypes = [vp, i32, i32, i32]
    L.pipelive_kv_resize.restype = i32
    L.pipelive_kv_resize.argtypes = [vp, i64, vp, vp, vp, vp, i32, vp, C.POINTER(ResizeResult), vp,
                                     sz, vp]
    L.pipelive_kv_resize_workspace_bytes.restype = sz
    L.pipelive_kv_resize_workspace_bytes.argtypes = [vp]
    L.pipelive_max_blocks.restype = i64
    L.pipelive_max_blocks.argtypes = [C.c_double, C.c_double, i64, C.c_double, C.c_double]
    L.pipelive_kv_mark_dirty.restype = i32
    L.pipelive_kv_mark_dirty.argtypes = [vp, vp, i32, i64, vp]
    L.pipelive_patch_max_blocks.restype = i64
    L.pipelive_patch_max_blocks.argtypes = [vp, i32, sz]
    L.pipelive_kv_patch_collect.restype = i32
    L.pipelive_kv_patch_collect.argtypes = [vp, vp, i32, vp, sz, vp, vp]
    L.pipelive_kv_patch_apply.restype = i32
    L.pipelive_kv_patch_apply.argtypes = [vp, vp, i32, vp, sz, vp, i64, vp]
    L.pipelive_kv_tokens_applied.restype = i64
    L.pipelive_kv_tokens_applied.argtypes = [vp]
    L.pipelive_kv_read_state.restype = i32
    L.pipelive_kv_read_state.argtypes = [vp, C.POINTER(KVState), vp]
    L.pipelive_kv_clear_status.restype = i32
    L.pipelive_kv_clear_status.argtypes = [vp, vp]
    L.pipelive_plan_reconfig.restype = i32
    L.pipelive_plan_reconfig.argtypes = [i32, vp, vp, vp, vp, vp, C.c_double, C.c_double, C.c_double, i64,
                                         i64, C.POINTER(ReconfigPlan), vp, i32, vp, i32]
    L.pipelive_converged.restype = i32
    L.pipelive_converged.argtypes = [i64, vp, i32, i64]
    L.pipelive_vmm_backing_bytes.restype = sz
    L.pipelive_vmm_backing_bytes.argtypes = [sz]
    L.pipelive_vmm_pool_create.restype = i32
    L.pipelive_vmm_pool_create.argtypes = [sz, i64, C.POINTER(vp)]
    L.pipelive_vmm_pool_destroy.restype = None
    L.pipelive_vmm_pool_destroy.argtypes = [vp]
    L.pipelive_vmm_pool_alloc.restype = i32
    L.pipelive_vmm_pool_alloc.argtypes = [vp, i64, vp]
    L.pipelive_vmm_pool_free.restype = i32
    L.pipelive_vmm_pool_free.argtypes = [vp, i64, vp]
    L.pipelive_vmm_pool_allocated.restype = i64
    L.pipelive_vmm_pool_allocated.argtypes = [vp]
    L.pipelive_vmm_pool_base.restype = C.c_uint64
    L.pipelive_vmm_pool_base.argtypes = [vp]
    L.pipelive_arena_create.restype = i32
    L.pipelive_arena_create.argtypes = [sz, sz, sz, C.POINTER(vp)]
    L.pipelive_arena_layout.restype = i32
    L.pipelive_arena_layout.argtypes = [vp, sz]
    L.pipelive_arena_zone.restype = i32
    L.pipelive_arena_zone.argtypes = [vp, i32, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
    L.pipelive_arena_destroy.restype = None
    L.pipelive_arena_destroy.argtypes = [vp]
    L.pipelive_arena_base.restype = C.c_uint64
    L.pipelive_arena_base.argtypes = [vp]
    L.pipelive_arena_bytes.restype = sz
    L.pipelive_arena_bytes.argtypes = [vp]
    L.pipelive_arena_info.restype = i32
    L.pipelive_arena_info.argtypes = [vp, C.POINTER(ArenaInfo)]
    L.pipelive_arena_piece_class.restype = i32
    L.pipelive_arena_piece_class.argtypes = [vp, i64]
    L.pipelive_kv_utilization.restype = C.c_double
    L.pipelive_kv_utilization.argtypes = [vp, i64, i32]
    L.pipelive_stacked_block_tokens.restype = i64
    L.pipelive_stacked_block_tokens.argtypes = [sz, i32, sz]
    L.pipelive_strerror.restype = C.c_char_p
    L.pipelive_strerror.argtypes = [i32]
    L.pipelive_last_hip_error.restype = C.c_char_p
    L.pipelive_device_ok.restype = i32
    _lib = L
    return L


class PipeliveError(RuntimeError):
    def __init__(self, rc: int):
        L = load()
        msg = L.pipelive_strerror(rc).decode()
        if rc == E_HIP:
            msg += ": " + L.pipelive_last_hip_error().decode()
        super().__init__(f"pipelive error {rc}: {msg}")
        self.rc = rc


def _check(rc: int) -> int:
    if rc != OK:
        raise PipeliveError(rc)
    return rc


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _p(t) -> int | None:
    return None if t is None else t.data_ptr()


def _i32_array(vals):
    vals = [int(v) for v in vals]
    return (C.c_int32 * max(len(vals), 1))(*vals)


# ---- the entry points, same names as the C ABI ---------------------------------

def pipelive_paged_attn_decode(kv: "KVRegion", layer, q, out, block_table, ctx_lens, max_ctx=0,
                               scale=0.0, split_tokens=0, workspace=None, check=True):
    """q bf16 [S][Hq][D]; out fp32 or bf16 [S][Hq][D]; block_table int32 [S][stride]; ctx_lens int32 [S]."""
    L = load()
    S = int(ctx_lens.shape[0])
    out_dtype = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
    stride = int(block_table.shape[1])
    if workspace is None:
        workspace = kv.attn_workspace(S, max_ctx if max_ctx > 0 else stride * kv.bs, split_tokens)
    rc = L.pipelive_paged_attn_decode(kv.handle, int(layer), _p(q), _p(out), out_dtype,
                                      _p(block_table), stride, _p(ctx_lens), S, int(max_ctx),
                                      float(scale), int(split_tokens), _p(workspace),
                                      workspace.numel() * workspace.element_size(), _stream())
    return _check(rc) if check else rc


def pipelive_paged_attn_decode_noalloc(kv: "KVRegion", layer, q, out, block_table, ctx_lens, max_ctx=0,
                                       scale=0.0, split_tokens=0, check=True):
    """As pipelive_paged_attn_decode, on the library's built-in scratch buffer (the call allocates nothing)."""
    out_dtype = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
    rc = load().pipelive_paged_attn_decode_noalloc(kv.handle, int(layer), _p(q), _p(out), out_dtype,
                                                   _p(block_table), int(block_table.shape[1]), _p(ctx_lens),
                                                   int(ctx_lens.shape[0]), int(max_ctx), float(scale),
                                                   int(split_tokens), _stream())
    return _check(rc) if check else rc


def pipelive_paged_attn_prefill(kv: "KVRegion", layer, q, out, block_table, ctx_lens, q_offsets, total_q,
                                max_ctx=0, scale=0.0, check=True):
    """q bf16 [total_q][Hq][D]; out fp32|bf16 same shape; q_offsets int32 [S+1] on the device."""
    out_dtype = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
    rc = load().pipelive_paged_attn_prefill(kv.handle, int(layer), _p(q), _p(out), out_dtype, _p(block_table),
                                            int(block_table.shape[1]), _p(ctx_lens), _p(q_offsets),
                                            int(ctx_lens.shape[0]), int(total_q), int(max_ctx), float(scale),
                                            _stream())
    return _check(rc) if check else rc


def pipelive_kv_resize(kv: "KVRegion", new_num_blocks, tables=(), used=(), remap_out=None,
                       workspace=None):
    """Returns (rc, ResizeResult).  tables: int32 device tensors [rows][stride], remapped in place."""
    L = load()
    n = len(tables)
    tp = (C.c_void_p * max(n, 1))(*[t.data_ptr() for t in tables])
    up = (C.c_void_p * max(n, 1))(*[u.data_ptr() for u in used])
    rows = _i32_array([t.shape[0] for t in tables])
    strides = _i32_array([t.shape[1] for t in tables])
    if workspace is None:
        workspace = kv.resize_workspace()
    res = ResizeResult()
    rc = L.pipelive_kv_resize(kv.handle, int(new_num_blocks), tp, rows, strides, up, n,
                              _p(remap_out), C.byref(res), _p(workspace), workspace.numel(),
                              _stream())
    return rc, res


def pipelive_kv_append(kv: "KVRegion", layer, k_new, v_new, block_table, positions, mark=True,
                       count_tokens=False, check=True):
    """k_new, v_new bf16 [S][Hkv][D]; positions int32 [S] (-1 skips a sequence)."""
    rc = load().pipelive_kv_append(kv.handle, int(layer), _p(k_new), _p(v_new), _p(block_table),
                                   int(block_table.shape[1]), _p(positions), int(positions.numel()),
                                   int(bool(mark)), int(bool(count_tokens)), _stream())
    return _check(rc) if check else rc


def pipelive_kv_append_chunk(kv: "KVRegion", layer, k_new, v_new, block_table, ctx_lens, q_offsets, total_q,
                             mark=True, count_tokens=False, check=True):
    """k_new, v_new bf16 [total_q][Hkv][D]; ctx_lens int32 [S] (chunk included); q_offsets int32 [S+1] (device)."""
    rc = load().pipelive_kv_append_chunk(kv.handle, int(layer), _p(k_new), _p(v_new), _p(block_table),
                                         int(block_table.shape[1]), _p(ctx_lens), _p(q_offsets),
                                         int(ctx_lens.shape[0]), int(total_q), int(bool(mark)),
                                         int(bool(count_tokens)), _stream())
    return _check(rc) if check else rc


def pipelive_kv_mark_dirty(kv: "KVRegion", block_ids, n_tokens, check=True):
    L = load()
    rc = L.pipelive_kv_mark_dirty(kv.handle, _p(block_ids), int(block_ids.numel()), int(n_tokens),
                                  _stream())
    return _check(rc) if check else rc


def pipelive_kv_patch_collect(src: "KVRegion", layers, patch_buf, hdr_host=None, check=True):
    L = load()
    la = _i32_array(layers)
    rc = L.pipelive_kv_patch_collect(src.handle, la, len(layers), _p(patch_buf), patch_buf.numel(),
                                     _p(hdr_host), _stream())
    return _check(rc) if check else rc


def pipelive_kv_patch_apply(dst: "KVRegion", dst_layers, patch_buf, dst_block_map=None, check=True):
    L = load()
    la = _i32_array(dst_layers)
    rc = L.pipelive_kv_patch_apply(dst.handle, la, len(dst_layers), _p(patch_buf),
                                   patch_buf.numel() * patch_buf.element_size(), _p(dst_block_map),
                                   0 if dst_block_map is None else dst_block_map.numel(), _stream())
    return _check(rc) if check else rc


def pipelive_kv_tokens_applied(dst: "KVRegion") -> int:
    """T_applied; the caller has synchronised the stream of the applies."""
    v = int(load().pipelive_kv_tokens_applied(dst.handle))
    if v < 0:
        raise PipeliveError(v)
    return v


def pipelive_patch_max_blocks(kv: "KVRegion", n_layers, capacity) -> int:
    return int(load().pipelive_patch_max_blocks(kv.handle, int(n_layers), int(capacity)))


def pipelive_kv_read_state(kv: "KVRegion") -> KVState:
    st = KVState()
    _check(load().pipelive_kv_read_state(kv.handle, C.byref(st), _stream()))
    return st


def pipelive_kv_clear_status(kv: "KVRegion"):
    return _check(load().pipelive_kv_clear_status(kv.handle, _stream()))


def pipelive_max_blocks(mem_bytes, util, layers, weight_bytes_per_layer, block_bytes_per_layer) -> int:
    return int(load().pipelive_max_blocks(mem_bytes, util, layers, weight_bytes_per_layer,
                                          block_bytes_per_layer))


def pipelive_plan_reconfig(cur, tgt, mem_bytes, util, weight_bytes_per_layer, block_bytes_per_layer,
                           blocks_in_use, cur_blocks):
    """cur, tgt: lists of inclusive (first, last) layer ranges per GPU.
    Returns (rc, ReconfigPlan, mig [(src, dst, layer)], del [(gpu, layer)])."""
    L = load()
    n = len(cur)
    cf, cl = _i32_array([c[0] for c in cur]), _i32_array([c[1] for c in cur])
    tf, tl = _i32_array([t[0] for t in tgt]), _i32_array([t[1] for t in tgt])
    mem = (C.c_double * n)(*[float(m) for m in mem_bytes])
    cap = sum(max(0, t[1] - t[0] + 1) for t in tgt) + sum(max(0, c[1] - c[0] + 1) for c in cur) + 1
    mig = (C.c_int32 * (3 * cap))()
    dele = (C.c_int32 * (2 * cap))()
    plan = ReconfigPlan()
    rc = L.pipelive_plan_reconfig(n, cf, cl, tf, tl, mem, float(util), float(weight_bytes_per_layer),
                                  float(block_bytes_per_layer), int(blocks_in_use), int(cur_blocks),
                                  C.byref(plan), mig, cap, dele, cap)
    m = [(mig[3 * k], mig[3 * k + 1], mig[3 * k + 2]) for k in range(min(plan.n_mig, cap))] if rc in (OK, E_NOSPACE) else []
    d = [(dele[2 * k], dele[2 * k + 1]) for k in range(min(plan.n_del, cap))] if rc in (OK, E_NOSPACE) else []
    return rc, plan, m, d


def pipelive_converged(t_sched, t_applied, tau) -> bool:
    arr = (C.c_int64 * max(len(t_applied), 1))(*[int(t) for t in t_applied])
    return bool(load().pipelive_converged(int(t_sched), arr, len(t_applied), int(tau)))


def pipelive_kv_utilization(ctx_lens, block_tokens) -> float:
    arr = _i32_array(ctx_lens)
    return float(load().pipelive_kv_utilization(arr, len(ctx_lens), int(block_tokens)))


def pipelive_stacked_block_tokens(phys_block_bytes, stack_k, token_bytes_per_layer) -> int:
    return int(load().pipelive_stacked_block_tokens(int(phys_block_bytes), int(stack_k),
                                                    int(token_bytes_per_layer)))


def pipelive_vmm_backing_bytes(block_bytes) -> int:
    return int(load().pipelive_vmm_backing_bytes(int(block_bytes)))


class VmmPool:
    """Handle of one pipelive_vmm_pool: blocks of device memory allocated and released one by one."""

    def __init__(self, block_bytes: int, max_blocks: int):
        h = C.c_void_p()
        _check(load().pipelive_vmm_pool_create(int(block_bytes), int(max_blocks), C.byref(h)))
        self.handle, self.block_bytes, self.max_blocks = h, int(block_bytes), int(max_blocks)

    def alloc(self, n: int) -> list[int]:
        out = (C.c_uint64 * max(int(n), 1))()
        _check(load().pipelive_vmm_pool_alloc(self.handle, int(n), out))
        return [int(out[i]) for i in range(int(n))]

    def free(self, addrs) -> None:
        arr = (C.c_uint64 * max(len(addrs), 1))(*[int(a) for a in addrs])
        _check(load().pipelive_vmm_pool_free(self.handle, len(addrs), arr))

    @property
    def allocated(self) -> int:
        return int(load().pipelive_vmm_pool_allocated(self.handle))

    def close(self) -> None:
        if self.handle:
            load().pipelive_vmm_pool_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class _DeviceSpan:
    """Presents a range of device addresses to torch (no copy, no ownership)."""

    def __init__(self, addr: int, nbytes: int):
        self.__cuda_array_interface__ = {"shape": (int(nbytes) // 2,), "typestr": "<i2",
                                         "data": (int(addr), False), "version": 2}


class Arena:
    """One pipelive_arena and a bump allocator per zone: tensors carved out of a range whose pieces
    are sorted by the region of the device memory they lie in (zone 0: the regions in turn; zone
    1 + c: region c only).  The tensors are views without ownership: keep the arena alive, and do
    not call :meth:`layout` again, as long as they are in use."""

    def __init__(self, nbytes: int, piece_bytes: int = 64 << 20, probe_bytes: int = 1 << 30):
        h = C.c_void_p()
        _check(load().pipelive_arena_create(int(nbytes), int(piece_bytes), int(probe_bytes), C.byref(h)))
        self.handle = h
        self.piece_bytes = int(piece_bytes)
        self.base = int(load().pipelive_arena_base(h))
        self.nbytes = int(load().pipelive_arena_bytes(h))
        self.n_classes = self.info()["n_classes"]
        self._read_zones()

    def info(self) -> dict:
        i = ArenaInfo()
        _check(load().pipelive_arena_info(self.handle, C.byref(i)))
        return {"n_pieces": i.n_pieces, "n_classes": i.n_classes,
                "class_pieces": [int(x) for x in i.class_pieces][:max(1, i.n_classes)], "n_runs": i.n_runs,
                "probe_ms": round(float(i.probe_ms), 1), "rate_same_GBps": round(float(i.rate_same_GBps), 1),
                "rate_other_GBps": round(float(i.rate_other_GBps), 1)}

    def _read_zones(self) -> None:
        self.zones = []   # [offset, bytes, used] per zone
        for z in range(self.n_classes + 1):
            off, n = C.c_uint64(), C.c_uint64()
            _check(load().pipelive_arena_zone(self.handle, z, C.byref(off), C.byref(n)))
            self.zones.append([int(off.value), int(n.value), 0])

    def layout(self, spread_bytes: int) -> None:
        """size of the spread zone; everything carved out so far is given up (contents undefined)"""
        torch.cuda.synchronize()
        _check(load().pipelive_arena_layout(self.handle, int(spread_bytes)))
        self._read_zones()

    def piece_class(self, piece: int) -> int:
        rc = int(load().pipelive_arena_piece_class(self.handle, int(piece)))
        if rc < 0:
            raise PipeliveError(rc)
        return rc

    def room(self, zone: int = 0, align: int = 4096) -> int:
        _, n, used = self.zones[zone]
        return n - (used + align - 1) // align * align

    def total_room(self) -> int:
        return sum(max(0, self.room(z)) for z in range(len(self.zones)))

    def empty(self, numel: int, dtype=torch.uint8, zone: int = 0, align: int = 4096):
        """1-D tensor of `numel` elements at the next `align`-byte boundary of the zone"""
        itemsize = torch.empty(0, dtype=dtype).element_size()
        off, n, used = self.zones[zone]
        at = (used + align - 1) // align * align
        nbytes = int(numel) * itemsize
        if nbytes == 0:
            return torch.empty(0, dtype=dtype, device="cuda")
        if at + nbytes > n:
            raise PipeliveError(E_NOSPACE)
        self.zones[zone][2] = at + nbytes
        t = torch.as_tensor(_DeviceSpan(self.base + off + at, (nbytes + 1) // 2 * 2), device="cuda")
        return t.view(torch.uint8)[:nbytes].view(dtype)

    def empty_in_class(self, numel: int, dtype=torch.uint8, prefer: int = 0):
        """like :meth:`empty`, from the zone of class ``prefer % n_classes`` if it has room, else from the
        class zone with the most room, else from the spread zone"""
        nbytes = int(numel) * torch.empty(0, dtype=dtype).element_size()
        first = 1 + int(prefer) % self.n_classes
        rest = sorted((z for z in range(1, self.n_classes + 1) if z != first), key=lambda z: -self.room(z))
        for z in [first] + rest + [0]:
            if self.room(z) >= nbytes:
                return self.empty(numel, dtype, zone=z)
        raise PipeliveError(E_NOSPACE)

    def placer(self, arenas_per_group: int):
        """An ``allocator`` for :class:`KVRegion`: all arenas of a layer group in one class zone, so that
        a kernel that reads one layer reads one region of the memory.  Group g goes to class g mod
        n_classes if that zone can hold the whole group, else to the class zone with the most room that
        can; a group is only split over zones when none can."""
        chosen = {}

        def alloc(numel, dtype, group):
            nbytes = int(numel) * torch.empty(0, dtype=dtype).element_size()
            z = chosen.get(group)
            if z is None:
                need = int(arenas_per_group) * (nbytes + 4096)
                first = 1 + int(group) % self.n_classes
                rest = sorted((c for c in range(1, self.n_classes + 1) if c != first), key=lambda c: -self.room(c))
                z = next((c for c in [first] + rest if self.room(c) >= need), None)
                if z is None:
                    z = max(range(1, self.n_classes + 1), key=self.room)
                chosen[group] = z
            if self.room(z) >= nbytes:
                return self.empty(numel, dtype, zone=z)
            return self.empty_in_class(numel, dtype, prefer=group)
        return alloc

    def close(self) -> None:
        if self.handle:
            load().pipelive_arena_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- device memory plumbing ------------------------------------------------------

class KVRegion:
    """Torch allocations + library handle of one KV region on the current device.

    ``backing="arena"``: physical blocks are spread over ``arenas`` separate torch
    allocations per layer group (block ``b`` in arena ``b % arenas``) so that no
    address is ``base + id * stride``; all ``capacity`` ids are backed.
    ``backing="vmm"``: every physical block is an allocation of its own from a
    :class:`VmmPool` (shuffled positions); only ids below ``num_blocks`` are
    backed, :meth:`grow_backing` and :meth:`release_tail` follow a resize.
    ``allocator`` (arena backing only): ``allocator(numel, dtype, group)`` returns the 1-D device
    tensor one arena of layer group ``group`` is laid in (e.g. :meth:`Arena.placer`); default: torch
    allocations."""

    def __init__(self, num_layers, num_q_heads, num_kv_heads, head_dim, block_tokens, num_blocks,
                 capacity_blocks=None, stack_k=1, arenas=3, fill_bits=None, device="cuda",
                 dirty_granularity=DIRTY_BLOCK, share_pool_of: "KVRegion | None" = None,
                 backing="arena", allocator=None):
        import numpy as np
        L = load()
        if not torch.cuda.is_available():
            raise RuntimeError("pipelive needs a GPU: no CPU fallback exists")
        self.L_, self.Hq, self.Hkv, self.D, self.bs = num_layers, num_q_heads, num_kv_heads, head_dim, block_tokens
        self.stack_k = stack_k
        self.capacity = int(capacity_blocks if capacity_blocks is not None else num_blocks)
        self.blk_elems = 2 * num_kv_heads * block_tokens * head_dim
        self.blk_bytes = 2 * self.blk_elems
        self.groups = (num_layers + stack_k - 1) // stack_k
        self.device = torch.device(device)
        self.backing = backing
        self.pool = None
        self._bl_host = None
        self._fill = None if fill_bits is None else (fill_bits - 65536 if fill_bits >= 32768 else fill_bits)
        phys = self.blk_elems * stack_k
        self.phys_bytes = 2 * phys
        if share_pool_of is not None:
            # a second handle over the same physical blocks (own dirty bitmap and state),
            # e.g. to track the same pool at another dirty granularity
            o = share_pool_of
            assert (o.L_, o.Hkv, o.D, o.bs, o.stack_k, o.capacity) == (num_layers, num_kv_heads, head_dim,
                                                                      block_tokens, stack_k, self.capacity)
            assert o.backing == "arena" and backing == "arena"
            self._n_ar, self.arenas, self.block_list = o._n_ar, o.arenas, o.block_list
        elif backing == "vmm":
            slots = self.groups * self.capacity
            self.pool = VmmPool(self.phys_bytes, slots)
            self._pool_base = int(L.pipelive_vmm_pool_base(self.pool.handle))
            self._pool_view = None  # made at the first allocation: torch wants a mapped first byte
            self._bl_host = np.zeros((self.groups, self.capacity), dtype=np.int64)
            self.block_list = torch.zeros((self.groups, self.capacity), dtype=torch.int64, device=self.device)
            self._back(0, int(num_blocks))
        else:
            assert backing == "arena"
            self._n_ar = n_ar = max(1, min(arenas, self.capacity))
            self.arenas = []
            bl = torch.zeros((self.groups, self.capacity), dtype=torch.int64)
            for g in range(self.groups):
                for a in range(n_ar):
                    cnt = len(range(a, self.capacity, n_ar))
                    if allocator is not None:
                        t = allocator(cnt * phys, torch.int16, g).view(cnt, phys)
                    else:
                        t = torch.empty((cnt, phys), dtype=torch.int16, device=self.device)
                    if self._fill is not None:
                        t.fill_(self._fill)
                    self.arenas.append(t)
                    bl[g, a::n_ar] = t.data_ptr() + torch.arange(cnt, dtype=torch.int64) * (phys * 2)
            self.block_list = bl.to(self.device)
        nb = L.pipelive_bitmap_bytes(self.capacity)
        self.dirty_granularity = dirty_granularity
        self.units_per_block = block_tokens if dirty_granularity == DIRTY_SLOT else 1
        self.unit_bytes = 2 * num_kv_heads * head_dim * 2 if dirty_granularity == DIRTY_SLOT else self.blk_bytes
        units = L.pipelive_kv_dirty_units(self.capacity, block_tokens, dirty_granularity)
        self.live = torch.zeros(nb, dtype=torch.uint8, device=self.device)
        self.dirty = torch.zeros(L.pipelive_bitmap_bytes(units), dtype=torch.uint8, device=self.device)
        self.state = torch.zeros(L.pipelive_kv_state_bytes(units), dtype=torch.uint8, device=self.device)
        d = KVDesc(num_layers, num_q_heads, num_kv_heads, head_dim, block_tokens, stack_k, 0,
                   LAYOUT_D8, dirty_granularity, BACKING_PER_BLOCK if backing == "vmm" else BACKING_ARENA,
                   int(num_blocks), self.capacity, self.block_list.data_ptr(),
                   self.live.data_ptr(), self.dirty.data_ptr(), self.state.data_ptr())
        h = C.c_void_p()
        torch.cuda.synchronize()
        _check(L.pipelive_kv_create(C.byref(d), C.byref(h)))
        self.handle = h
        self._ws = {}

    def __del__(self):
        try:
            if getattr(self, "handle", None):
                load().pipelive_kv_destroy(self.handle)
                self.handle = None
            if getattr(self, "pool", None) is not None:
                torch.cuda.synchronize()
                self._pool_view = None
                self.pool.close()
        except Exception:
            pass

    @property
    def num_blocks(self) -> int:
        return int(load().pipelive_kv_num_blocks(self.handle))

    # ---- per-block backing: allocate for a grow, release after a shrink
    def _back(self, lo: int, hi: int) -> None:
        """allocate physical blocks for ids [lo, hi) of every group and enter them in the block list"""
        import numpy as np
        if hi <= lo:
            return
        n = (hi - lo) * self.groups
        addrs = np.array(self.pool.alloc(n), dtype=np.int64)
        if self._pool_view is None:
            # one view over the whole address range; only rows with physical memory are ever indexed
            slots = self.groups * self.capacity
            self._pool_view = torch.as_tensor(_DeviceSpan(self._pool_base, slots * self.phys_bytes),
                                              device=self.device).view(slots, self.phys_bytes // 2)
        addrs = addrs[np.random.default_rng(lo * 7919 + hi).permutation(n)]  # no address = base + id * stride
        if self._fill is not None:
            rows = torch.from_numpy((addrs - self._pool_base) // self.phys_bytes).to(self.device)
            self._pool_view[rows] = self._fill
        self._bl_host[:, lo:hi] = addrs.reshape(self.groups, hi - lo)
        self.block_list[:, lo:hi] = torch.from_numpy(self._bl_host[:, lo:hi]).to(self.device)

    def grow_backing(self, new_num_blocks: int) -> None:
        """before a grow: back ids [num_blocks, new_num_blocks)"""
        assert self.backing == "vmm" and new_num_blocks <= self.capacity
        self._back(self.num_blocks, int(new_num_blocks))

    def release_tail(self, old_num_blocks: int) -> int:
        """after a shrink: return the physical blocks left at ids [num_blocks, old_num_blocks) to the
        device; returns how many were released"""
        assert self.backing == "vmm"
        lo, hi = self.num_blocks, int(old_num_blocks)
        if hi <= lo:
            return 0
        torch.cuda.synchronize()
        self._bl_host = self.block_list.cpu().numpy().copy()  # the resize permuted it on the device
        tail = self._bl_host[:, lo:hi].reshape(-1)
        self.pool.free([int(a) for a in tail])
        self._bl_host[:, lo:hi] = 0
        self.block_list[:, lo:hi] = 0
        return int(tail.size)

    def _where(self, layer: int, ids):
        """[(tensor, selector over ids, rows)]: where the physical blocks of `ids` lie"""
        g = layer // self.stack_k
        if self.backing == "vmm":
            if self._bl_host is None:
                self._bl_host = self.block_list.cpu().numpy().copy()
            rows = (self._bl_host[g, ids.numpy()] - self._pool_base) // self.phys_bytes
            assert (rows >= 0).all(), "block id without physical memory"
            return [(self._pool_view, torch.ones(len(ids), dtype=torch.bool), torch.from_numpy(rows))]
        out = []
        for a in range(self._n_ar):
            sel = (ids % self._n_ar) == a
            if sel.any():
                out.append((self.arenas[g * self._n_ar + a], sel, ids[sel] // self._n_ar))
        return out

    def sync_block_list(self) -> None:
        """re-read the block list after the library permuted it (per-block backing, shrink)"""
        if self.backing == "vmm":
            torch.cuda.synchronize()
            self._bl_host = self.block_list.cpu().numpy().copy()

    def block(self, layer: int, block_id: int) -> torch.Tensor:
        """int16 view [blk_elems] of (layer, block) in device memory."""
        t, _, rows = self._where(layer, torch.tensor([int(block_id)], dtype=torch.int64))[0]
        o = (layer % self.stack_k) * self.blk_elems
        return t[int(rows[0]), o:o + self.blk_elems]

    def write_blocks(self, layer: int, block_ids, data: torch.Tensor) -> None:
        """data: int16 [n][blk_elems] on the device -> blocks ``block_ids`` of ``layer``."""
        ids = torch.tensor([int(b) for b in block_ids], dtype=torch.int64)
        o = (layer % self.stack_k) * self.blk_elems
        for t, sel, rows in self._where(layer, ids):
            t[rows.to(self.device), o:o + self.blk_elems] = data[sel.to(data.device)]

    def read_blocks(self, layer: int, block_ids) -> torch.Tensor:
        ids = torch.tensor([int(b) for b in block_ids], dtype=torch.int64)
        out = torch.empty((len(ids), self.blk_elems), dtype=torch.int16, device=self.device)
        o = (layer % self.stack_k) * self.blk_elems
        for t, sel, rows in self._where(layer, ids):
            out[sel.to(self.device)] = t[rows.to(self.device), o:o + self.blk_elems]
        return out

    def set_live(self, ids) -> None:
        import numpy as np
        bm = np.zeros(self.live.numel(), dtype=np.uint8)
        ids = np.asarray(ids, dtype=np.int64)
        np.bitwise_or.at(bm, ids >> 3, (1 << (ids & 7)).astype(np.uint8))
        self.live.copy_(torch.from_numpy(bm))

    def attn_workspace(self, num_seqs, max_ctx, split_tokens=0) -> torch.Tensor:
        n = load().pipelive_paged_attn_workspace_bytes(self.handle, int(num_seqs), int(max_ctx),
                                                       int(split_tokens))
        if n == 0:
            raise PipeliveError(E_INVAL)
        key = ("attn", n)
        if key not in self._ws:
            self._ws = {k: v for k, v in self._ws.items() if k[0] != "attn"}
            self._ws[key] = torch.zeros(n, dtype=torch.uint8, device=self.device)  # zeroed once
        return self._ws[key]

    def resize_workspace(self) -> torch.Tensor:
        n = load().pipelive_kv_resize_workspace_bytes(self.handle)
        key = ("resize", n)
        if key not in self._ws:
            self._ws[key] = torch.empty(n, dtype=torch.uint8, device=self.device)
        return self._ws[key]
