"""GPU tests of the striped device range: pieces of one virtual range backed part by part, data
intact across every piece boundary, and a patch round whose buffer straddles the parts equal to
the oracle's byte for byte."""
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
    torch.cuda.empty_cache()   # what torch's own allocator has cached is not the range's
    return torch.cuda.mem_get_info()[0]


def test_parts_are_backed_one_by_one_and_hold_data_across_pieces():
    w = P.StripedRange(2 * MiB, ways=1, piece_bytes=2 * MiB)       # first mapping of the process: not counted
    w.close()
    (torch.arange(16, dtype=torch.int64, device="cuda") * 3).cpu()   # nor the first load of torch's kernels
    free0 = _free()
    r = P.StripedRange(11 * MiB, ways=3, piece_bytes=2 * MiB, back_now=False)
    assert r.nbytes == 12 * MiB and r.base % (2 * MiB) == 0       # rounded up to whole pieces
    assert abs(free0 - _free()) <= MiB                             # an address range only
    with pytest.raises(P.PipeliveError) as e:
        r.empty(16)                                                # nothing may be carved before every part is backed
    assert e.value.rc == P.E_INVAL
    for part in range(3):
        r.back(part)
        assert abs(free0 - _free() - (part + 1) * 4 * MiB) <= MiB  # two pieces per part
    r.back(1)                                                      # backed already: left alone
    assert abs(free0 - _free() - 12 * MiB) <= MiB
    for bad in (-1, 3):
        with pytest.raises(P.PipeliveError) as e:
            r.back(bad)
        assert e.value.rc == P.E_INVAL
    t = r.empty(12 * MiB // 8, torch.int64)
    assert t.data_ptr() == r.base and r.room() == 0
    t.copy_(torch.arange(t.numel(), dtype=torch.int64, device="cuda") * 2654435761)
    back = t.cpu().numpy()
    assert np.array_equal(back, np.arange(t.numel(), dtype=np.int64) * 2654435761)
    with pytest.raises(P.PipeliveError) as e:
        r.empty(1)
    assert e.value.rc == P.E_NOSPACE
    del t
    r.close()
    assert abs(free0 - _free()) <= 8 * MiB                         # everything returned (up to the runtime's own)


def test_create_rejects_bad_geometry():
    for kw in (dict(nbytes=4 * MiB, piece_bytes=3 * MiB // 2), dict(nbytes=4 * MiB, piece_bytes=0),
               dict(nbytes=0), dict(nbytes=4 * MiB, ways=0), dict(nbytes=4 * MiB, ways=65)):
        kw.setdefault("piece_bytes", 2 * MiB)
        with pytest.raises(P.PipeliveError) as e:
            P.StripedRange(**kw)
        assert e.value.rc == P.E_INVAL


@pytest.mark.parametrize("offset", [2 * MiB - 96 * 1024, 4 * MiB - 512 * 1024 + 4096])
def test_patch_round_through_a_striped_buffer_equals_oracle(offset):
    """the bulk round of the tiny configuration gathered into and scattered from a buffer that
    starts shortly before a piece boundary, so that header, ids and payload lie in different parts"""
    cfg = pin.CONFIGS["tiny"]
    B = 128
    batch = pin.draw_batch(cfg, SEED, num_blocks=B)
    host, dev = make_pair(cfg, batch, SEED)
    fill_pair(cfg, batch, SEED, host, dev)
    live = host.live_ids()
    r = P.StripedRange(8 * MiB, ways=3, piece_bytes=2 * MiB, back_now=False)
    r.back(0)
    tgt_h = oracle.HostKV(2, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B,
                          fill_bits=pin.BF16_NAN)
    tgt_d = P.KVRegion(2, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_tokens, B,
                       arenas=2, fill_bits=pin.BF16_NAN)                    # allocated between the parts
    r.back(1)
    r.back(2)
    cap = 64 + 256 + len(live) * (4 + 2 * host.blk_bytes)
    assert offset + cap > (offset // (2 * MiB) + 1) * 2 * MiB              # really crosses into the next piece
    r.empty(offset)
    patch_d = r.empty(cap)
    patch_d.zero_()
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
    del patch_d
    r.close()
