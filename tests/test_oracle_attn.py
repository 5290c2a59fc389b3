"""Pins for the oracle's paged decode attention (CPU only).

The oracle must equal textbook softmax attention over the contiguous KV
(PagedAttention is an addressing scheme: paper Sec. 2 "LLM Inference" and
Sec. 5.1), and reduce to closed forms in special cases."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
from helpers import dense_attention, rel_l2, scatter_dense


def _rand_bits(rng, shape):
    return pin.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def _make(layout, L, Hq, Hkv, D, bs, ctx, seed, B=None, stack_k=1, stride_pad=0):
    rng = np.random.default_rng(seed)
    used = [(n + bs - 1) // bs for n in ctx]
    B = B or (sum(used) + 5)
    kv = oracle.HostKV(L, Hq, Hkv, D, bs, B, layout=layout, stack_k=stack_k)
    perm = rng.permutation(B)
    table = np.full((len(ctx), max(max(used), 1) + stride_pad), pin.TABLE_FILL, dtype=np.int32)
    off = 0
    dense = {}
    for s, n in enumerate(ctx):
        table[s, :used[s]] = perm[off:off + used[s]]
        off += used[s]
        for layer in range(L):
            k = _rand_bits(rng, (n, Hkv, D))
            v = _rand_bits(rng, (n, Hkv, D))
            dense[(layer, s)] = (k, v)
            scatter_dense(kv, layer, table[s], k, v)
    q = _rand_bits(rng, (L, len(ctx), Hq, D))
    return kv, table, np.asarray(ctx, dtype=np.int32), q, dense


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("shape", [(4, 2, 64, 16), (8, 2, 128, 32), (3, 3, 64, 16), (8, 1, 128, 16),
                                   (4, 2, 64, 64), (4, 1, 128, 128)])
def test_paged_equals_dense(layout, shape):
    Hq, Hkv, D, bs = shape
    ctx = [1, 15, 16, 17, 63, 100, 0, 33]
    kv, table, ctxa, q, dense = _make(layout, 2, Hq, Hkv, D, bs, ctx, seed=11)
    for layer in range(2):
        out = kv.attn_decode(layer, q[layer], table, ctxa)
        for s, n in enumerate(ctx):
            if n == 0:
                assert (out[s] == 0).all()
                continue
            k, v = dense[(layer, s)]
            ref = dense_attention(q[layer, s], k, v, Hq // Hkv)
            assert np.abs(out[s] - ref).max() < 2e-6
            assert rel_l2(out[s], ref) < 1e-6


def test_against_library_sdpa():
    """Special case that reduces to a library routine: torch SDPA in float64."""
    Hq, Hkv, D, bs = 4, 2, 64, 16
    ctx = [37, 64]
    kv, table, ctxa, q, dense = _make(0, 1, Hq, Hkv, D, bs, ctx, seed=3)
    out = kv.attn_decode(0, q[0], table, ctxa)
    for s, n in enumerate(ctx):
        k, v = dense[(0, s)]
        kt = torch.from_numpy(pin.bf16_bits_to_f64(k)).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)
        vt = torch.from_numpy(pin.bf16_bits_to_f64(v)).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)
        qt = torch.from_numpy(pin.bf16_bits_to_f64(q[0, s]))[:, None, :]
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt)[:, 0, :].numpy()
        assert np.abs(out[s] - ref).max() < 2e-6


def test_single_token_returns_v_bit_exact():
    kv, table, ctxa, q, dense = _make(0, 1, 4, 2, 64, 16, [1, 1], seed=5)
    out = kv.attn_decode(0, q[0], table, ctxa)
    for s in range(2):
        v = dense[(0, s)][1]
        expect = np.repeat(pin.bf16_bits_to_f64(v[0]), 2, axis=0).astype(np.float32)
        assert np.array_equal(out[s].view(np.uint32), expect.view(np.uint32))


def test_equal_keys_give_mean_of_values():
    Hq, Hkv, D, bs, n = 4, 2, 64, 16, 40
    kv, table, ctxa, q, dense = _make(0, 1, Hq, Hkv, D, bs, [n], seed=6)
    k, v = dense[(0, 0)]
    k[:] = k[0]
    scatter_dense(kv, 0, table[0], k, v)
    out = kv.attn_decode(0, q[0], table, ctxa)
    mean = np.repeat(pin.bf16_bits_to_f64(v).mean(axis=0), Hq // Hkv, axis=0)
    assert np.abs(out[0] - mean).max() < 1e-6


def test_constant_values_give_constant():
    Hq, Hkv, D, bs, n = 4, 2, 64, 16, 50
    kv, table, ctxa, q, dense = _make(1, 1, Hq, Hkv, D, bs, [n], seed=7)
    k, v = dense[(0, 0)]
    v[:] = pin.f32_to_bf16_bits(np.float32(0.75))
    scatter_dense(kv, 0, table[0], k, v)
    out = kv.attn_decode(0, q[0], table, ctxa)
    assert np.abs(out[0] - 0.75).max() < 1e-7


def test_dominant_key_selects_its_value():
    Hq, Hkv, D, bs, n = 2, 2, 64, 16, 30
    kv, table, ctxa, q, dense = _make(0, 1, Hq, Hkv, D, bs, [n], seed=8)
    k, v = dense[(0, 0)]
    j = 21
    # key j = 64 * q (per kv head == per q head here): score >> all others
    k[j] = pin.f32_to_bf16_bits((64.0 * pin.bf16_bits_to_f64(q[0, 0])).astype(np.float32))
    scatter_dense(kv, 0, table[0], k, v)
    out = kv.attn_decode(0, q[0], table, ctxa)
    assert np.abs(out[0] - pin.bf16_bits_to_f64(v[j])).max() < 1e-6


def test_scale_argument():
    Hq, Hkv, D, bs = 4, 2, 64, 16
    kv, table, ctxa, q, dense = _make(0, 1, Hq, Hkv, D, bs, [29], seed=9)
    out = kv.attn_decode(0, q[0], table, ctxa, scale=0.3)
    ref = dense_attention(q[0, 0], *dense[(0, 0)], Hq // Hkv, scale=0.3)
    assert np.abs(out[0] - ref).max() < 2e-6


def test_placement_stride_and_garbage_invariance():
    """Same logical KV at other physical ids, with a padded table and NaN in
    every unused slot and free block -> identical output bits."""
    Hq, Hkv, D, bs = 4, 2, 64, 16
    ctx = [45, 7, 96]
    a = _make(0, 2, Hq, Hkv, D, bs, ctx, seed=21, B=40)
    b = _make(0, 2, Hq, Hkv, D, bs, ctx, seed=21, B=40, stride_pad=9)
    kvb, tableb = b[0], b[1]
    rng = np.random.default_rng(99)
    perm = rng.permutation(40)
    tableb2 = tableb.copy()
    kvb2 = oracle.HostKV(2, Hq, Hkv, D, bs, 40, layout=0)
    off = 0
    for s, n in enumerate(ctx):
        u = (n + bs - 1) // bs
        tableb2[s, :u] = perm[off:off + u]
        off += u
        for layer in range(2):
            scatter_dense(kvb2, layer, tableb2[s], *b[4][(layer, s)])
    for layer in range(2):
        o1 = a[0].attn_decode(layer, a[3][layer], a[1], a[2])
        o2 = kvb2.attn_decode(layer, b[3][layer], tableb2, b[2])
        assert np.array_equal(o1.view(np.uint32), o2.view(np.uint32))
        assert np.isfinite(o1).all()


def test_layer_stacking_addresses():
    """stack_k = 2: layers 2g and 2g+1 share one physical block."""
    Hq, Hkv, D, bs = 4, 2, 64, 16
    ctx = [20, 33]
    kv, table, ctxa, q, dense = _make(0, 4, Hq, Hkv, D, bs, ctx, seed=31, stack_k=2)
    assert kv.groups == 2
    for layer in range(4):
        out = kv.attn_decode(layer, q[layer], table, ctxa)
        for s in range(2):
            ref = dense_attention(q[layer, s], *dense[(layer, s)], Hq // Hkv)
            assert np.abs(out[s] - ref).max() < 2e-6


def test_bad_block_id_is_an_error():
    kv, table, ctxa, q, dense = _make(0, 1, 4, 2, 64, 16, [20], seed=2)
    table[0, 1] = kv.num_blocks
    with pytest.raises(oracle.OracleError):
        kv.attn_decode(0, q[0], table, ctxa)


def test_threads_do_not_change_bits():
    kv, table, ctxa, q, dense = _make(0, 1, 8, 2, 64, 16, [50, 60, 70], seed=4)
    a = kv.attn_decode(0, q[0], table, ctxa, nthreads=1)
    b = kv.attn_decode(0, q[0], table, ctxa, nthreads=4)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
