"""Pins for the oracle's chunked-prefill attention: textbook causal softmax
attention over the contiguous KV, a library SDPA special case, and the decode
oracle as the q_len = 1 case."""
import numpy as np
import pytest
import torch

import oracle
import pipelive_inputs as pin
from helpers import scatter_dense


def _bits(rng, shape):
    return pin.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))


def _setup(layout, Hq, Hkv, D, bs, ctx, qlen, seed=1):
    rng = np.random.default_rng(seed)
    used = [(n + bs - 1) // bs for n in ctx]
    B = sum(used) + 4
    kv = oracle.HostKV(1, Hq, Hkv, D, bs, B, layout=layout)
    perm = rng.permutation(B)
    table = np.full((len(ctx), max(used) + 2), pin.TABLE_FILL, dtype=np.int32)
    dense, off = [], 0
    for s, n in enumerate(ctx):
        table[s, :used[s]] = perm[off:off + used[s]]
        off += used[s]
        k, v = _bits(rng, (n, Hkv, D)), _bits(rng, (n, Hkv, D))
        dense.append((k, v))
        scatter_dense(kv, 0, table[s], k, v)
    qo = np.concatenate([[0], np.cumsum(qlen)]).astype(np.int32)
    q = _bits(rng, (int(qo[-1]), Hq, D))
    return kv, table, np.asarray(ctx, dtype=np.int32), qo, q, dense


def _dense_causal(q_rows, k, v, group, ctx, qlen, scale=None):
    """q_rows uint16 [qlen][Hq][D]; k, v uint16 [ctx][Hkv][D] -> float64 [qlen][Hq][D]."""
    q = pin.bf16_bits_to_f64(q_rows)
    kk = np.repeat(pin.bf16_bits_to_f64(k), group, axis=1)
    vv = np.repeat(pin.bf16_bits_to_f64(v), group, axis=1)
    d = q.shape[-1]
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    x = np.einsum("ihd,jhd->hij", q, kk) * scale                  # [Hq][qlen][ctx]
    pos = ctx - qlen + np.arange(qlen)
    mask = np.arange(ctx)[None, :] <= pos[:, None]
    x = np.where(mask[None], x, -np.inf)
    x = x - x.max(axis=2, keepdims=True)
    p = np.exp(x)
    p /= p.sum(axis=2, keepdims=True)
    return np.einsum("hij,jhd->ihd", p, vv)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("shape", [(4, 2, 64, 16), (8, 1, 128, 32), (2, 2, 64, 16)])
def test_prefill_equals_dense_causal(layout, shape):
    Hq, Hkv, D, bs = shape
    ctx = [5, 40, 33, 64, 17]
    qlen = [5, 7, 33, 1, 0]
    kv, table, ctxa, qo, q, dense = _setup(layout, Hq, Hkv, D, bs, ctx, qlen)
    out = kv.attn_prefill(0, q, table, ctxa, qo)
    for s in range(len(ctx)):
        if qlen[s] == 0:
            continue
        ref = _dense_causal(q[qo[s]:qo[s + 1]], *dense[s], Hq // Hkv, ctx[s], qlen[s])
        assert np.abs(out[qo[s]:qo[s + 1]] - ref).max() < 2e-6


def test_against_library_sdpa_causal():
    Hq, Hkv, D, bs = 4, 2, 64, 16
    kv, table, ctxa, qo, q, dense = _setup(0, Hq, Hkv, D, bs, [48], [48], seed=3)
    out = kv.attn_prefill(0, q, table, ctxa, qo)
    k, v = dense[0]
    kt = torch.from_numpy(pin.bf16_bits_to_f64(k)).permute(1, 0, 2).repeat_interleave(2, 0)
    vt = torch.from_numpy(pin.bf16_bits_to_f64(v)).permute(1, 0, 2).repeat_interleave(2, 0)
    qt = torch.from_numpy(pin.bf16_bits_to_f64(q)).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True).permute(1, 0, 2).numpy()
    assert np.abs(out - ref).max() < 2e-6


def test_decode_is_the_single_query_case_and_first_token_is_v0():
    Hq, Hkv, D, bs = 4, 2, 64, 16
    ctx = [37, 20]
    kv, table, ctxa, qo, q, dense = _setup(0, Hq, Hkv, D, bs, ctx, [1, 1], seed=5)
    a = kv.attn_prefill(0, q, table, ctxa, qo)
    b = kv.attn_decode(0, q, table, ctxa)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    kv2, table2, ctx2, qo2, q2, dense2 = _setup(0, Hq, Hkv, D, bs, [9], [9], seed=6)
    out = kv2.attn_prefill(0, q2, table2, ctx2, qo2)
    v0 = np.repeat(pin.bf16_bits_to_f64(dense2[0][1][0]), 2, axis=0).astype(np.float32)
    assert np.array_equal(out[0].view(np.uint32), v0.view(np.uint32))     # position 0 sees only itself


def test_prefill_argument_errors():
    kv, table, ctxa, qo, q, dense = _setup(0, 4, 2, 64, 16, [10], [4])
    bad = qo.copy(); bad[1] = 11                                           # more queries than context
    with pytest.raises(oracle.OracleError):
        kv.attn_prefill(0, np.zeros((11, 4, 64), np.uint16), table, ctxa, bad)
