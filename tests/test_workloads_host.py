"""Host-side checks of the synthetic workloads and of bench.py's bookkeeping (no GPU).

The generators hold none of the method's arithmetic; what is pinned here is the input recipe:
the shapes of the five workloads, the score law (P(g >= tau) equals the unit's target rate),
reproducibility of the seeded streams, and the byte count bench.py prices a decode-attention
launch with (K and V rows of the valid tokens, page-table entries, q in, out out)."""
import importlib.util
import os
import subprocess
import sys

import numpy as np

import wgkv_workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_the_five_workload_shapes():
    names = [c.name for c in wl.CONFIGS]
    assert names == ["tiny", "llama8b_1layer_32k", "llama8b_32layer_b8_128k", "qwen3_4b_36layer_b32_64k",
                     "llama8b_chunked_prefill_128k"]
    head = wl.get_config("llama8b_32layer_b8_128k")
    assert (head.batch, head.n_layers, head.n_q_heads, head.n_kv_heads, head.head_dim) == (8, 32, 32, 8, 128)
    assert (head.w_local, head.page_size, head.tau, head.dtype) == (256, 16, 0.5, "bf16")
    assert (head.ctx_min, head.ctx_max, head.decode_steps) == (65536, 131072, 256)
    assert head.seed == 251217000 + 2 and wl.get_config(2) is head
    ragged = wl.get_config(3)
    assert (ragged.batch, ragged.n_layers, ragged.w_local, ragged.page_size) == (32, 36, 128, 32)
    chunked = wl.get_config(4)
    assert (chunked.batch, chunked.chunk, chunked.hidden_dim, chunked.ctx_max) == (4, 4096, 4096, 131072)


def test_contexts_and_rates_follow_the_recipe():
    cfg = wl.get_config(2)
    ctx = wl.context_lengths(cfg)
    assert ctx.shape == (8,) and ctx.min() >= cfg.ctx_min and ctx.max() <= cfg.ctx_max
    assert np.array_equal(ctx, wl.context_lengths(cfg))                 # seeded: the same on every call
    rates = wl.unit_rates(cfg)
    assert rates.shape == (32, 8) and (rates > 0).all() and (rates < 1).all()
    assert abs(rates.mean() - 1.5 / 9.5) < 0.02                          # Beta(1.5, 8): mean 0.158 over 256 draws
    mix = wl.unit_rates(wl.get_config(3))
    assert set(np.round(np.unique(mix), 4)) <= {0.01, 0.0707, 0.9}       # the three kinds of heads
    assert abs(mix.mean() - 0.10) < 0.03


def test_score_law_hits_the_target_rate():
    cfg = wl.get_config(0)
    rates = np.array([[0.05, 0.5]]).repeat(cfg.n_layers, axis=0)[:, :cfg.n_kv_heads]
    if rates.shape[1] < cfg.n_kv_heads:
        rates = np.tile(rates, (1, cfg.n_kv_heads))[:, :cfg.n_kv_heads]
    n = 200_000
    g = wl.draw_scores(cfg, 0, 0, n, rates)
    assert g.dtype == np.float32 and g.shape == (n, cfg.n_kv_heads) and g.min() >= 0.0 and g.max() <= 1.0
    for h in range(cfg.n_kv_heads):
        r = rates[0, h]
        got = float((g[:, h] >= cfg.tau).mean())
        assert abs(got - r) < 4.0 * np.sqrt(r * (1 - r) / n), (h, r, got)   # P(g >= tau) = (1 - tau)^b = r
    assert np.array_equal(g, wl.draw_scores(cfg, 0, 0, n, rates))            # reproducible
    assert not np.array_equal(g[:1000], wl.draw_scores(cfg, 1, 0, 1000, rates))  # another sequence, another stream


def test_decode_attention_byte_count_by_hand():
    bench = _bench_module()
    cfg = wl.get_config(2)                      # bf16, d 128, P 16, W 256, group of 4
    seq_len = np.array([[300], [100]])          # [B, L]: tokens fed so far
    global_len = np.array([[[17, 0]], [[5, 40]]])  # [B, L, H] entries in the global cache
    per_layer = bench.attend_algorithmic_bytes(cfg.scaled(n_kv_heads=2, n_q_heads=8), seq_len, global_len, [0])
    row = 2 * 128 * 2                            # K and V row of one token
    fixed = 4 * 128 * 2 + 4 * 128 * 4            # q rows in, fp32 rows out
    want = 0
    for t, gls in ((300, (17, 0)), (100, (5, 40))):
        for gl in gls:
            want += (min(t, 256) + gl) * row + 4 * (16 + -(-gl // 16)) + fixed
    assert per_layer == [want]


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
