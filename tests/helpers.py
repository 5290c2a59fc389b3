"""Test-local helpers: an independent way to place logical K/V into blocks
(numpy reshapes, not index formulas) and textbook dense attention."""
import numpy as np

import pipelive_inputs as pin


def pack_block(layout, k_tok, v_tok):
    """k_tok, v_tok: uint16 [bs][Hkv][D] (token-major logical content of one
    block) -> uint16 [blk_elems] in storage order.
    layout 0: consecutive runs of min(bs, 32) tokens, each stored as K [Hkv][D/8][run][8]
    followed by V [Hkv][D][run];
    layout 1: K and V as [Hkv][bs][D]."""
    bs, hkv, d = k_tok.shape
    if layout == 0:
        run = min(bs, 32)
        out = []
        for lo in range(0, bs, run):
            kk, vv = k_tok[lo:lo + run], v_tok[lo:lo + run]
            out.append(np.ascontiguousarray(kk.reshape(run, hkv, d // 8, 8).transpose(1, 2, 0, 3)).reshape(-1))
            out.append(np.ascontiguousarray(vv.transpose(1, 2, 0)).reshape(-1))
        return np.concatenate(out)
    else:
        k = k_tok.transpose(1, 0, 2)
        v = v_tok.transpose(1, 0, 2)
    return np.concatenate([np.ascontiguousarray(k).reshape(-1), np.ascontiguousarray(v).reshape(-1)])


def unpack_block(layout, blk, bs, hkv, d):
    """Inverse of pack_block -> (k_tok, v_tok) uint16 [bs][Hkv][D]."""
    half = hkv * bs * d
    if layout == 0:
        run = min(bs, 32)
        h = hkv * run * d
        ks, vs = [], []
        for i in range(bs // run):
            part = blk[2 * h * i:2 * h * (i + 1)]
            ks.append(part[:h].reshape(hkv, d // 8, run, 8).transpose(2, 0, 1, 3).reshape(run, hkv, d))
            vs.append(part[h:].reshape(hkv, d, run).transpose(2, 0, 1))
        k, v = np.concatenate(ks), np.concatenate(vs)
    else:
        k = blk[:half].reshape(hkv, bs, d).transpose(1, 0, 2)
        v = blk[half:].reshape(hkv, bs, d).transpose(1, 0, 2)
    return np.ascontiguousarray(k), np.ascontiguousarray(v)


def scatter_dense(kv, layer, table_row, k_dense, v_dense, poison=pin.BF16_NAN):
    """Write logical K/V (uint16 [n][Hkv][D]) of one sequence into a HostKV
    through its block table row; slots past n are poisoned."""
    n = k_dense.shape[0]
    bs = kv.bs
    for b in range((n + bs - 1) // bs):
        kt = np.full((bs, kv.Hkv, kv.D), poison, dtype=np.uint16)
        vt = np.full((bs, kv.Hkv, kv.D), poison, dtype=np.uint16)
        m = min(bs, n - b * bs)
        kt[:m] = k_dense[b * bs:b * bs + m]
        vt[:m] = v_dense[b * bs:b * bs + m]
        kv.block(layer, int(table_row[b]))[:] = pack_block(kv.layout, kt, vt)


def dense_attention(q_bits, k_dense, v_dense, group, scale=None):
    """Textbook softmax attention in float64. q uint16 [Hq][D]; k, v uint16
    [n][Hkv][D] -> float64 [Hq][D]. Query head h uses KV head h // group."""
    q = pin.bf16_bits_to_f64(q_bits)
    k = np.repeat(pin.bf16_bits_to_f64(k_dense), group, axis=1)  # [n][Hq][D]
    v = np.repeat(pin.bf16_bits_to_f64(v_dense), group, axis=1)
    d = q.shape[-1]
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    x = np.einsum("hd,nhd->hn", q, k) * scale
    x = x - x.max(axis=1, keepdims=True)
    p = np.exp(x)
    p /= p.sum(axis=1, keepdims=True)
    return np.einsum("hn,nhd->hd", p, v)


def gather_logical(kv, layer, table_row, n):
    """Read back the logical K/V of a sequence: uint16 [n][Hkv][D] each."""
    ks, vs = [], []
    bs = kv.bs
    for b in range((n + bs - 1) // bs):
        k, v = unpack_block(kv.layout, kv.block(layer, int(table_row[b])), bs, kv.Hkv, kv.D)
        ks.append(k)
        vs.append(v)
    if not ks:
        z = np.zeros((0, kv.Hkv, kv.D), dtype=np.uint16)
        return z, z
    return np.concatenate(ks)[:n], np.concatenate(vs)[:n]


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.sqrt((b * b).sum())
    return float(np.sqrt(((a - b) ** 2).sum()) / (den if den > 0 else 1.0))
