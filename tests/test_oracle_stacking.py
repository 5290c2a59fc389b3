"""Pins for the layer-stacking arithmetic (CPU only).

Paper: Sec. 5.2 (k layers share one physical block of the allocation
granularity, each taking C/k tokens of it); Sec. 7.5 (Effective KV Utilisation =
share of the request-allocated KV slots that hold tokens, which rises with k
because the logical block shrinks)."""
import numpy as np
import pytest

import oracle
import paper_2604_12171_amd.binding as B
import pipelive_inputs as pin


def test_closed_forms():
    assert oracle.kv_utilization([64, 128, 1024], 64) == 1.0          # whole blocks only
    assert oracle.kv_utilization([1], 16) == pytest.approx(1 / 16)
    assert oracle.kv_utilization([528], 512) == pytest.approx(528 / 1024)   # one token over a block: two blocks
    assert oracle.kv_utilization([17, 31], 16) == pytest.approx(48 / 64)
    assert oracle.kv_utilization([0, 0], 16) == 1.0                    # nothing allocated
    assert oracle.kv_utilization([0, 5], 16) == pytest.approx(5 / 16)  # empty sequences occupy nothing


def test_against_numpy_expression():
    rng = np.random.default_rng(5)
    for bs in (16, 32, 64, 128, 512):
        n = rng.integers(0, 5000, 300)
        ref = n.sum() / (np.ceil(n / bs) * bs).sum()
        assert oracle.kv_utilization(n, bs) == pytest.approx(ref, rel=1e-12)


def test_halving_the_block_never_lowers_utilisation():
    rng = np.random.default_rng(6)
    n = rng.integers(1, 3000, 200)
    u = [oracle.kv_utilization(n, bs) for bs in (512, 256, 128, 64, 32, 16)]
    assert all(b >= a for a, b in zip(u, u[1:]))
    assert u[-1] > 0.97 and u[0] < 0.9


def test_uniform_lengths_expectation():
    """Lengths uniform on [1, m*bs]: the last block is half full on average, so U -> E[n] / (E[n] + bs/2 - 1/2)."""
    bs, m = 64, 8
    n = np.arange(1, m * bs + 1)
    exp = n.mean() / (n.mean() + (bs - 1) / 2)
    assert oracle.kv_utilization(n, bs) == pytest.approx(exp, rel=1e-12)


def test_stacked_block_tokens_is_c_over_k():
    tok = 2 * 8 * 128 * 2       # bytes per token per layer, 8 KV heads of 128, bf16 K and V
    C = (2 << 20) // tok        # tokens of one layer that fill a 2 MiB block
    assert C == 512
    for k in (1, 2, 4, 8, 16, 32):
        assert oracle.stacked_block_tokens(2 << 20, k, tok) == C // k
    assert oracle.stacked_block_tokens(2 << 20, 3, tok) == 170          # floor
    assert oracle.stacked_block_tokens(1000, 4, tok) == 0


def test_library_matches_oracle():
    rng = np.random.default_rng(7)
    tok = 4096
    for bs in (16, 32, 128, 512):
        n = rng.integers(0, 9000, 100)
        assert B.pipelive_kv_utilization(n, bs) == pytest.approx(oracle.kv_utilization(n, bs), rel=1e-12)
    for k in (1, 2, 3, 4, 16):
        assert B.pipelive_stacked_block_tokens(2 << 20, k, tok) == oracle.stacked_block_tokens(2 << 20, k, tok)
    assert B.pipelive_kv_utilization([], 16) == 1.0
    assert B.pipelive_vmm_backing_bytes(1) == 2 << 20
    assert B.pipelive_vmm_backing_bytes(2 << 20) == 2 << 20
    assert B.pipelive_vmm_backing_bytes((2 << 20) + 4096) == 4 << 20
    assert B.pipelive_vmm_backing_bytes(512 << 10) == 2 << 20   # a quarter-filled unit: what stacking avoids


def test_stacking_raises_utilisation_on_the_decode_workloads():
    """Same physical block (2 MiB), more layers stacked -> shorter logical block -> higher utilisation."""
    cfg = pin.CONFIGS["stage8b"]
    ctx = pin.draw_ctx_lens(cfg, pin.MASTER_SEED)
    tok = 2 * cfg.num_kv_heads * cfg.head_dim * 2
    u = {k: oracle.kv_utilization(ctx, oracle.stacked_block_tokens(2 << 20, k, tok)) for k in (1, 2, 4, 8, 16)}
    assert u[1] < u[2] < u[4] < u[8] < u[16]
    assert u[1] < 0.92 and u[16] > 0.99
