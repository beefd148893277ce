"""GPU-vs-oracle parity on small shapes: every call goes through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
from harness import Pair, rand_q, rand_tokens

pytestmark = pytest.mark.gpu


def test_tiny_config_prefill_then_decode():
    # workload 1: 8 query / 2 kv heads, d=64, fp32, prefill 512, 16 decode steps, W=64, P=16
    from wgkv_workloads import get_config, unit_rates, draw_scores
    cfg = get_config(0)
    rates = unit_rates(cfg)
    assert ((rates >= 0.10) & (rates <= 0.40)).all()
    pr = Pair(1, 8, 2, 64, wg.F32, 16, 64, 1, 64, 256)
    rng = np.random.default_rng(cfg.seed)
    k, v, _ = rand_tokens(rng, 512, 2, 64, torch.float32)
    g = torch.from_numpy(draw_scores(cfg, 0, 0, 512, rates))
    pr.prefill(0, [0], [512], k, v, g, cfg.tau)
    pr.check_state()
    for step in range(16):
        k1, v1, _ = rand_tokens(rng, 1, 2, 64, torch.float32)
        g1 = torch.from_numpy(draw_scores(cfg, 0, 0, 1, rates, purpose="dec_scores", step=step))
        pr.decode(0, [0], k1, v1, g1, cfg.tau)
        pr.check_state()
        pr.check_attend(0, [0], rand_q(rng, 1, 8, 64, torch.float32))


@pytest.mark.parametrize("dtype,d,Hq,Hk", [(wg.BF16, 128, 8, 2), (wg.BF16, 64, 4, 4), (wg.F32, 128, 4, 2),
                                            (wg.F32, 64, 16, 2), (wg.BF16, 128, 2, 1)])
@pytest.mark.parametrize("P,W", [(16, 64), (32, 64), (4, 24), (1, 5), (8, 1), (64, 64), (16, 40)])
def test_shapes_pages_windows(dtype, d, Hq, Hk, P, W):
    tdt = torch.float32 if dtype == wg.F32 else torch.bfloat16
    pr = Pair(2, Hq, Hk, d, dtype, P, W, 3, 4096 // P + 8, 3 * 2 * Hk * (700 // P + W // P + 4) + 64)
    rng = np.random.default_rng(100 + P + W)
    tau = 0.6
    # ragged multi-sequence prefill in uneven chunks, two layers, one shared pool
    plan = [(0, [0, 2], [37, 300]), (1, [1], [W]), (0, [1, 0], [1, 263]), (1, [2, 0, 1], [5, W + 3, 200]),
            (0, [2], [W - 1 if W > 1 else 1])]
    for layer, seqs, lens in plan:
        n = sum(lens)
        k, v, g = rand_tokens(rng, n, Hk, d, tdt)
        pr.prefill(layer, seqs, lens, k, v, g, tau)
        pr.check_state()
    for step in range(2 * W + 3 if W < 40 else 20):
        for layer in (0, 1):
            k, v, g = rand_tokens(rng, 3, Hk, d, tdt)
            pr.decode(layer, [2, 0, 1], k, v, g, tau)
            pr.check_attend(layer, [2, 0, 1], rand_q(rng, 3, Hq, d, tdt))
        if step % 7 == 0:
            pr.check_state()
    pr.check_state()


def test_admit_all_none_ties_and_nan():
    pr = Pair(1, 4, 2, 128, wg.BF16, 16, 32, 2, 64, 400)
    rng = np.random.default_rng(5)
    k, v, g = rand_tokens(rng, 300, 2, 128, torch.bfloat16)
    g[:, 0] = torch.from_numpy(rng.choice(np.array([0.25, 0.5, 0.75], np.float32), 300))
    g[::7, 1] = float("nan")
    pr.prefill(0, [0], [300], k, v, g, 0.5)       # ties admit, NaN does not
    pr.check_state()
    k, v, g = rand_tokens(rng, 300, 2, 128, torch.bfloat16)
    pr.prefill(0, [1], [300], k, v, g, 0.0)       # tau <= 0 admits everything
    pr.check_state()
    assert pr.orc.global_len(1, 0, 0) == 300 - 32
    q = rand_q(rng, 2, 4, 128, torch.bfloat16)
    pr.check_attend(0, [0, 1], q)
    for _ in range(40):                            # tau > 1 admits nothing
        k, v, g = rand_tokens(rng, 2, 2, 128, torch.bfloat16)
        pr.decode(0, [1, 0], k, v, g, 2.0)
    pr.check_state()
    assert pr.orc.global_len(1, 0, 0) == 300 - 32
    pr.check_attend(0, [1, 0], q)


def test_decode_from_empty_equals_prefill_content():
    # N single-token steps from an empty slot cache the same tokens as one N-token prefill
    Hk, d, W, P, N = 2, 64, 16, 4, 90
    a = Pair(1, 4, Hk, d, wg.BF16, P, W, 1, 64, 200)
    b = Pair(1, 4, Hk, d, wg.BF16, P, W, 1, 64, 200)
    rng = np.random.default_rng(8)
    k, v, g = rand_tokens(rng, N, Hk, d, torch.bfloat16)
    a.prefill(0, [0], [N], k, v, g, 0.5)
    for i in range(N):
        b.decode(0, [0], k[i:i + 1], v[i:i + 1], g[i:i + 1], 0.5)
    a.check_state()
    b.check_state()
    q = rand_q(rng, 1, 4, d, torch.bfloat16)
    oa, _ = a.attend(0, [0], q)
    ob, _ = b.attend(0, [0], q)
    np.testing.assert_allclose(oa, ob, atol=1e-5)


def test_free_seq_returns_pages_in_order():
    pr = Pair(2, 4, 2, 64, wg.BF16, 8, 16, 2, 64, 300)
    rng = np.random.default_rng(9)
    for layer in (0, 1):
        k, v, g = rand_tokens(rng, 150, 2, 64, torch.bfloat16)
        pr.prefill(layer, [0, 1], [100, 50], k, v, g, 0.5)
    pr.pool.free_seq(0)
    pr.orc.free_seq(0)
    pr.touched = {(1, 0), (1, 1)}
    pr.check_state()
    k, v, g = rand_tokens(rng, 60, 2, 64, torch.bfloat16)
    pr.prefill(1, [0], [60], k, v, g, 0.5)        # the slot is usable again, pages are recycled
    pr.check_state()


def test_attend_before_any_token_is_zero():
    pr = Pair(1, 4, 2, 64, wg.F32, 16, 32, 2, 8, 64)
    rng = np.random.default_rng(3)
    k, v, g = rand_tokens(rng, 1, 2, 64, torch.float32)
    pr.decode(0, [1], k, v, g, 0.5)
    out, ref = pr.attend(0, [0, 1], rand_q(rng, 2, 4, 64, torch.float32))
    assert (out[0] == 0).all() and np.abs(out[1] - ref[1]).max() < 1e-5
    np.testing.assert_allclose(out[1], np.repeat(v[0].numpy(), 2, axis=0), atol=1e-6)  # one key: output = its V
