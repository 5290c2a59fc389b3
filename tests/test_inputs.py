import numpy as np
import torch

import pipelive_inputs as pin


def test_hash_numpy_equals_torch():
    key = pin.stream_key(pin.MASTER_SEED, pin.STREAM_KV)
    c = np.array([0, 1, 2, 12345, 2**40 + 17, 2**62 + 5], dtype=np.uint64)
    a = pin.hash_u64(key, c)
    b = pin.hash_i64_torch(key, torch.from_numpy(c.astype(np.int64)))
    assert np.array_equal(a, b.numpy().view(np.uint64))
    # the reference splitmix64 stream: seed 0 -> first output (published test vector)
    assert pin._mix_int(0x9E3779B97F4A7C15) == 0xE220A8397B1DCDAF


def test_bf16_normal_twins_and_moments():
    key = pin.stream_key(7, pin.STREAM_KV)
    a = pin.bf16_normal(key, 1000, 50000)
    b = pin.bf16_normal_torch(key, 1000, 50000, "cpu").numpy().view(np.uint16)
    assert np.array_equal(a, b)
    x = pin.bf16_bits_to_f64(a)
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1.0) < 0.02
    assert np.isfinite(x).all()


def test_table_is_monotone_and_symmetric():
    t = pin.bf16_bits_to_f64(pin.bf16_normal_table())
    assert (np.diff(t) >= 0).all()
    assert np.allclose(t, -t[::-1])


def test_f32_to_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.0 + 2**-8, 1.0 + 2**-8 + 2**-16, 1.0 + 3 * 2**-8], dtype=np.float32)
    b = pin.f32_to_bf16_bits(x)
    assert list(b) == [0x3F80, 0x3F80, 0x3F81, 0x3F82]


def test_draw_batch_structure():
    cfg = pin.CONFIGS["tiny"]
    bt = pin.draw_batch(cfg, pin.MASTER_SEED, num_blocks=128)
    assert bt.ctx_lens.min() >= 1 and bt.ctx_lens.max() <= 256
    used_ids = np.concatenate([bt.table[s, :bt.used[s]] for s in range(cfg.num_seqs)])
    assert len(np.unique(used_ids)) == len(used_ids) == len(bt.live_ids)
    assert used_ids.max() < 128
    assert (bt.table[0, bt.used[0]:] == pin.TABLE_FILL).all()
    bt2 = pin.draw_batch(cfg, pin.MASTER_SEED, num_blocks=128)
    assert np.array_equal(bt.table, bt2.table)


def test_kv_block_twins():
    cfg = pin.CONFIGS["tiny"]
    ids = [3, 77]
    a = np.stack([pin.kv_block_bits(cfg, 5, 128, 1, 1, b) for b in ids])
    b = pin.kv_blocks_bits_torch(cfg, 5, 128, 1, 1, ids, "cpu").numpy().view(np.uint16)
    assert np.array_equal(a, b)


def test_slot_mask_counts():
    for layout in (0, 1):
        m = pin.token_slot_mask(layout, 2, 16, 64, 5)
        assert m.sum() == 2 * 2 * 64 * (16 - 5)


def test_dirty_ids_include_last_blocks():
    cfg = pin.CONFIGS["tiny"]
    bt = pin.draw_batch(cfg, pin.MASTER_SEED, num_blocks=128)
    d = pin.draw_dirty_ids(bt, 1, 0, 0.10)
    assert set(pin.last_block_ids(bt)).issubset(set(d))
    assert set(d).issubset(set(bt.live_ids))
    f = pin.geometric_fractions(0.20, 0.01, 6)
    assert abs(f[0] - 0.2) < 1e-12 and abs(f[-1] - 0.01) < 1e-12


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: --gpus N with N > 1 exits with a message before it touches a device"""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
