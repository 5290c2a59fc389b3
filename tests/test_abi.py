"""The C-ABI library loads without a GPU and exports every function that
include/pipelive.h declares; host-only helpers behave."""
import ctypes as C
import os
import re

import paper_2604_12171_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "pipelive.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pipelive_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert "pipelive_paged_attn_decode" in names and "pipelive_kv_resize" in names
    assert "pipelive_kv_patch_collect" in names and "pipelive_kv_patch_apply" in names
    lib = P.load()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(P.binding.EXPORTS) == names


def test_host_only_helpers():
    lib = P.load()
    assert lib.pipelive_bitmap_bytes(1) == 8 and lib.pipelive_bitmap_bytes(64) == 8
    assert lib.pipelive_bitmap_bytes(65) == 16
    assert lib.pipelive_kv_state_bytes(1000) % 256 == 0
    assert P.pipelive_max_blocks(80e9, 0.9, 16, 0.4e9, 65536) == int((80e9 * 0.9 - 16 * 0.4e9) // (16 * 65536))
    assert lib.pipelive_strerror(P.E_BUSY).decode().startswith("busy")
    assert C.sizeof(P.binding.PatchHdr) == 64


def test_create_rejects_bad_descriptors_without_a_gpu():
    lib = P.load()
    h = C.c_void_p()
    d = P.binding.KVDesc(2, 4, 2, 64, 16, 1, 0, 0, 0, 0, 8, 8, None, None, None, None)
    assert lib.pipelive_kv_create(C.byref(d), C.byref(h)) == P.E_INVAL   # null device pointers
    d = P.binding.KVDesc(2, 4, 3, 64, 16, 1, 0, 0, 0, 0, 8, 8, 256, 256, 256, 256)
    assert lib.pipelive_kv_create(C.byref(d), C.byref(h)) == P.E_INVAL   # Hq % Hkv != 0
    d = P.binding.KVDesc(2, 4, 2, 64, 16, 1, 0, 0, 0, 0, 9, 8, 256, 256, 256, 256)
    assert lib.pipelive_kv_create(C.byref(d), C.byref(h)) == P.E_INVAL   # B > capacity
