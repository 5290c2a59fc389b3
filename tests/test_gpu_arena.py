"""GPU tests of the region-aware device arena: the range is backed, every layout maps every piece
exactly once and sorts the class zones by class, data holds across every piece boundary, and a
patch round whose buffer and target pool lie in it equals the oracle's byte for byte."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
import paper_2604_12171_amd as P
from gpu_common import assert_pools_equal, fill_pair, make_pair

pytestmark = pytest.mark.gpu
SEED = 777
MiB = 1 << 20


def _free() -> int:
    torch.cuda.synchronize()
    torch.cuda.empty_cache()   # what torch's own allocator has cached is not the arena's
    return torch.cuda.mem_get_info()[0]


@pytest.mark.parametrize("probe", [False, True])
def test_arena_is_backed_whole_and_holds_data_across_pieces(probe):
    w = P.Arena(2 * MiB, piece_bytes=2 * MiB, probe_bytes=0)        # first mapping of the process: not counted
    w.close()
    (torch.arange(16, dtype=torch.int64, device="cuda") * 3).cpu()   # nor the first load of torch's kernels
    free0 = _free()
    a = P.Arena(23 * MiB, piece_bytes=4 * MiB, probe_bytes=4 * MiB if probe else 0)
    assert a.nbytes == 24 * MiB and a.base % (2 * MiB) == 0      # rounded up to whole pieces
    assert abs(free0 - _free() - 24 * MiB) <= 2 * MiB            # all of it backed
    info = a.info()
    assert info["n_pieces"] == 6 and 1 <= info["n_classes"] <= 4
    assert sum(info["class_pieces"]) == 6 and all(n > 0 for n in info["class_pieces"])
    assert info["n_classes"] <= info["n_runs"] <= 6
    if not probe:
        assert info["n_classes"] == 1 and info["probe_ms"] == 0.0
    classes = [a.piece_class(j) for j in range(6)]                 # every class as often as the probe counted it
    assert [classes.count(c) for c in range(info["n_classes"])] == info["class_pieces"]
    for bad in (-1, 6):
        with pytest.raises(P.PipeliveError) as e:
            a.piece_class(bad)
        assert e.value.rc == P.E_INVAL
    t = a.empty(24 * MiB // 8, torch.int64)
    assert t.data_ptr() == a.base and a.room() == 0
    # distinct contents everywhere: a physical piece mapped twice, or not at all, would show
    t.copy_(torch.arange(t.numel(), dtype=torch.int64, device="cuda") * 2654435761)
    assert np.array_equal(t.cpu().numpy(), np.arange(t.numel(), dtype=np.int64) * 2654435761)
    with pytest.raises(P.PipeliveError) as e:
        a.empty(1)
    assert e.value.rc == P.E_NOSPACE
    del t
    # 9 MiB (3 pieces) stay in the spread zone, the other three pieces go to the zones of their classes
    a.layout(9 * MiB)
    assert a.zones[0][:2] == [0, 12 * MiB] and a.room() == 12 * MiB
    assert sum(z[1] for z in a.zones) == 24 * MiB
    at = 12 * MiB
    for c in range(info["n_classes"]):
        off, n, _ = a.zones[1 + c]
        assert off == at and n % (4 * MiB) == 0                    # zones follow each other, whole pieces
        assert all(a.piece_class(j) == c for j in range(off // (4 * MiB), (off + n) // (4 * MiB)))
        at += n
    assert at == 24 * MiB
    classes = [a.piece_class(j) for j in range(6)]
    assert [classes.count(c) for c in range(info["n_classes"])] == info["class_pieces"]
    with pytest.raises(P.PipeliveError) as e:
        P.binding._check(P.load().pipelive_arena_zone(a.handle, info["n_classes"] + 1, None, None))
    assert e.value.rc == P.E_INVAL
    parts = [a.empty(a.room(z) // 8, torch.int64, zone=z) for z in range(len(a.zones)) if a.room(z) > 0]
    assert sum(p.numel() for p in parts) * 8 == 24 * MiB and a.total_room() == 0
    for k, part in enumerate(parts):                               # again distinct contents everywhere
        part.copy_(torch.arange(part.numel(), dtype=torch.int64, device="cuda") * 2654435761 + k)
    for k, part in enumerate(parts):
        assert np.array_equal(part.cpu().numpy(), np.arange(part.numel(), dtype=np.int64) * 2654435761 + k)
    t = a.empty_in_class(0, torch.int16, prefer=5)
    assert t.numel() == 0
    with pytest.raises(P.PipeliveError) as e:
        a.empty_in_class(8, torch.int16, prefer=1)
    assert e.value.rc == P.E_NOSPACE
    del parts, part
    a.layout(24 * MiB)                                             # back to one zone
    assert a.room() == 24 * MiB and a.total_room() == 24 * MiB
    a.close()
    assert abs(free0 - _free()) <= 8 * MiB                         # everything returned (up to the runtime's own)


def test_create_rejects_bad_geometry():
    for kw in (dict(nbytes=4 * MiB, piece_bytes=3 * MiB // 2), dict(nbytes=4 * MiB, piece_bytes=0), dict(nbytes=0)):
        kw.setdefault("piece_bytes", 2 * MiB)
        with pytest.raises(P.PipeliveError) as e:
            P.Arena(**kw)
        assert e.value.rc == P.E_INVAL
    h = P.binding.C.c_void_p()
    assert P.load().pipelive_arena_create(8 * MiB, 2 * MiB, 3 * MiB, P.binding.C.byref(h)) == P.E_INVAL   # not whole pieces
    assert P.load().pipelive_arena_create(4 * MiB, 2 * MiB, 2 * MiB, None) == P.E_INVAL


def test_probe_on_large_pieces_interleaves_what_it_finds():
    """3 GiB in pieces of 64 MiB, probed in stretches of 256 MiB: whatever classes the probe finds on this machine,
    the four pieces of a stretch share one, and consecutive pieces of the spread zone take the classes in turn
    (a class is only placed while no other has a larger share left)"""
    a = P.Arena(3 << 30, piece_bytes=64 * MiB, probe_bytes=256 * MiB)
    info = a.info()
    assert info["n_pieces"] == 48 and info["probe_ms"] > 0
    assert all(n % 4 == 0 for n in info["class_pieces"])
    classes = [a.piece_class(j) for j in range(48)]
    assert [classes.count(c) for c in range(info["n_classes"])] == info["class_pieces"]
    if info["n_classes"] > 1:
        assert info["rate_other_GBps"] > info["rate_same_GBps"] > 0
        left = list(info["class_pieces"])
        for c in classes:                                         # the rule the header states, replayed
            share = [left[k] / info["class_pieces"][k] for k in range(info["n_classes"])]
            assert share[c] >= max(share) - 1e-9
            left[c] -= 1
    a.close()


@pytest.mark.parametrize("offset", [2 * MiB - 96 * 1024, 4 * MiB - 512 * 1024 + 4096])
def test_patch_round_through_arena_memory_equals_oracle(offset):
    """the bulk round of the tiny configuration with the target pool and the patch buffer inside a probed
    arena, the buffer starting shortly before a piece boundary"""
    cfg = pin.CONFIGS["tiny"]
    B = 128
    batch = pin.draw_batch(cfg, SEED, num_blocks=B)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    live = host.live_ids()
    a = P.Arena(12 * MiB, piece_bytes=2 * MiB, probe_bytes=2 * MiB)
    cap = 64 + 256 + len(live) * (4 + 2 * host.blk_bytes)
    assert offset + cap > (offset // (2 * MiB) + 1) * 2 * MiB              # really crosses into the next piece
    a.layout(6 * MiB)
    a.empty(offset)
    patch_d = a.empty(cap)
    patch_d.zero_()
    tgt_h = oracle.HostKV(2, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B,
                          fill_bits=pin.BF16_NAN)
    tgt_d = P.KVRegion(2, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B,
                       arenas=2, fill_bits=pin.BF16_NAN,
                       allocator=a.placer(2))
    assert all(a.base + 6 * MiB <= t.data_ptr() < a.base + a.nbytes for t in tgt_d.arenas)   # in the class zones
    patch_h = np.zeros(cap, dtype=np.uint8)
    layers, dst_layers = [0, 1], [1, 0]
    assert host.mark_dirty(live, 5) == oracle.OK
    P.pipelive_kv_mark_dirty(dev, torch.from_numpy(np.asarray(live, dtype=np.int32)).cuda(), 5)
    assert host.patch_collect(layers, patch_h) == oracle.OK
    P.pipelive_kv_patch_collect(dev, layers, patch_d)
    torch.cuda.synchronize()
    h = oracle.parse_patch_header(patch_h)
    end = h["payload_offset"] + h["n_blocks"] * 2 * host.blk_bytes
    got = patch_d.cpu().numpy()
    assert h["n_blocks"] == len(live)
    assert np.array_equal(got[:64 + 4 * h["n_blocks"]], patch_h[:64 + 4 * h["n_blocks"]])
    assert np.array_equal(got[h["payload_offset"]:end], patch_h[h["payload_offset"]:end])
    assert tgt_h.patch_apply(dst_layers, patch_h) == oracle.OK
    P.pipelive_kv_patch_apply(tgt_d, dst_layers, patch_d)
    assert P.pipelive_kv_read_state(tgt_d).t_applied == 5 == tgt_h.t_applied
    assert_pools_equal(tgt_h, tgt_d, range(2), range(B))
    del patch_d, tgt_d
    a.close()
