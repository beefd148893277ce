"""Decode attention must give the same bits every time it runs on the same state: partial results
cross workgroups (and XCDs) inside the launch, the split of the work is a fixed function of the
lengths and the fold runs in a fixed order.  Checked at one layer of the two large decode
workloads (64 and 256 (sequence, kv head) units per launch, every share straddling units), together
with parity of sampled sequences against the definition oracle, before and after the split has been tuned to
the machine (wgkv_tune_decode_attention)."""
import math

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
import wgkv_workloads as wl
from oracle import attend_definition

pytestmark = pytest.mark.gpu

MAX_ABS_TOL, MEAN_ABS_TOL = 1e-2, 1e-3
N_REPEATS = 24


@pytest.mark.parametrize("index,layer", [(2, 5), (3, 11)])
def test_decode_attention_repeats_bit_for_bit(index, layer):
    cfg = wl.get_config(index)
    B, Hq, Hk, d, W, P = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.w_local, cfg.page_size
    dev = torch.device("cuda:0")
    ctx = wl.context_lengths(cfg)
    rates = wl.unit_rates(cfg)
    max_ctx = int(ctx.max())
    exp_tokens = sum(float(rates[layer, h]) * int(c) for c in ctx for h in range(Hk))
    n_pages = int(exp_tokens / P * 1.15) + B * Hk * (-(-W // P) + 3) + Hk * (max_ctx // P + 2) + 256
    max_gp = max_ctx // P + 4
    pool = wg.Pool(wg.Config(1, Hq, Hk, d, wg.BF16, P, W, B, max_gp, n_pages), B, max_ctx)
    sampled = sorted({int(np.argmax(ctx)), int(np.argmin(ctx))})
    hist = {}
    for s in range(B):
        n = int(ctx[s])
        k = wl.draw_normal(cfg, "k", (n, Hk, d), device=dev, key=(s, layer))
        v = wl.draw_normal(cfg, "v", (n, Hk, d), device=dev, key=(s, layer))
        g = wl.draw_scores(cfg, s, layer, n, rates, device=dev)
        pool.prefill_admit(0, [s], [n], k, v, g, tau=cfg.tau)
        free, flag = pool.status()
        assert flag == 0
        if s in sampled:
            hist[s] = [k.float().cpu().numpy(), v.float().cpu().numpy(), g.cpu().numpy()]
    seqs = list(range(B))
    k1 = wl.draw_normal(cfg, "dec_k", (B, Hk, d), device=dev, key=(layer, 0))
    v1 = wl.draw_normal(cfg, "dec_v", (B, Hk, d), device=dev, key=(layer, 0))
    q1 = wl.draw_normal(cfg, "q", (B, Hq, d), device=dev, key=(layer, 0))
    g1 = torch.from_numpy(np.concatenate([wl.draw_scores(cfg, s, layer, 1, rates, purpose="dec_scores", step=0)
                                          for s in seqs])).to(dev)
    pool.decode_step(0, seqs, k1, v1, g1, tau=cfg.tau)
    scale = 1.0 / math.sqrt(d)
    outs = []
    for r in range(N_REPEATS):
        out = torch.full((B, Hq, d), float("nan"), dtype=torch.float32, device=dev)
        pool.attend(0, seqs, q1, out, scale)
        outs.append(out)
        if r % 3 == 1:   # other work between the launches moves the timing of the next one
            torch.randn(1 << 20, device=dev).sum().item()
    torch.cuda.synchronize()
    for r in range(1, N_REPEATS):
        assert torch.equal(outs[0], outs[r]), f"launch {r} differs from launch 0"
    o = outs[0].cpu().numpy()
    assert np.isfinite(o).all()
    refs = {}
    for s in sampled:
        K = np.concatenate([hist[s][0], k1[s:s + 1].float().cpu().numpy()])
        V = np.concatenate([hist[s][1], v1[s:s + 1].float().cpu().numpy()])
        G = np.concatenate([hist[s][2], g1[s:s + 1].cpu().numpy()])
        t = K.shape[0]
        refs[s] = attend_definition(K, V, G, q1[s].float().cpu().numpy()[None], np.array([t - 1]), W, cfg.tau, scale)[0]
        err = np.abs(o[s].astype(np.float64) - refs[s])
        assert err.max() <= MAX_ABS_TOL and err.mean() <= MEAN_ABS_TOL, (s, err.max(), err.mean())
    # tuning the split to the machine: one of the candidates is kept, the cache is untouched, and with the
    # kept value the launches repeat bit for bit again and stay within tolerance
    meta_before = pool.meta_buf.cpu().numpy().copy()
    scratch = torch.empty((B, Hq, d), dtype=torch.float32, device=dev)
    kept = pool.tune_decode_attention(seqs, q1, scratch, scale)
    assert kept in (0, 25, 50, 75, 100, 125)
    print(f"workload {index}: split correction kept by the tuning: {kept} per mille", flush=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(pool.meta_buf.cpu().numpy(), meta_before)
    outs = []
    for r in range(6):
        out = torch.full((B, Hq, d), float("nan"), dtype=torch.float32, device=dev)
        pool.attend(0, seqs, q1, out, scale)
        outs.append(out)
    torch.cuda.synchronize()
    for r in range(1, 6):
        assert torch.equal(outs[0], outs[r]), f"after tuning: launch {r} differs from launch 0"
    o = outs[0].cpu().numpy()
    for s in sampled:
        err = np.abs(o[s].astype(np.float64) - refs[s])
        assert err.max() <= MAX_ABS_TOL and err.mean() <= MEAN_ABS_TOL, (s, err.max(), err.mean())
    with pytest.raises(wg.WgkvError) as e:
        pool.tune_decode_attention(seqs + [B], q1, scratch, scale)   # no such sequence slot
    assert e.value.code == -1


def test_tuning_runs_over_every_layer_and_leaves_the_cache_alone():
    from harness import Pair, rand_q, rand_tokens
    L, Hq, Hk, d, P, W, B = 3, 8, 2, 128, 16, 32, 2
    rng = np.random.default_rng(77)
    pr = Pair(L, Hq, Hk, d, wg.BF16, P, W, B, 64, 2000, max_call_seqs=B, max_call_tokens=1024)
    seqs = [1, 0]
    for l in range(L):
        k, v, g = rand_tokens(rng, 900, Hk, d, pr.tdt, rates=[0.5] * Hk)
        pr.prefill(l, seqs, [500, 400], k, v, g, 0.5)
    pr.check_state()
    q = rand_q(rng, B, Hq, d, pr.tdt)
    scratch = torch.empty((B, Hq, d), dtype=torch.float32, device=pr.dev)
    kept = pr.pool.tune_decode_attention(seqs, q.to(pr.dev), scratch, 1.0 / math.sqrt(d))
    assert kept in (0, 25, 50, 75, 100, 125)
    pr.check_state()
    for l in range(L):
        pr.check_attend(l, seqs, rand_q(rng, B, Hq, d, pr.tdt))
