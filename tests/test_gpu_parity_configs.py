"""GPU-vs-oracle parity at the sizes of the named workloads, every call through the
C ABI.  Integer state (admit masks, lengths, page tables, promotions, free stack) is
compared for every (sequence, layer, kv head); attention is compared exhaustively on
the small workloads and, where the dense history does not fit the host, on sampled
(sequence, layer) pairs against the definition oracle, which needs only the dense
K/V/score history of that pair."""
import math
import os

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
import wgkv_workloads as wl
from oracle import Oracle, OracleConfig, attend_definition

pytestmark = pytest.mark.gpu

SCALE = float(os.environ.get("WGKV_TEST_SCALE", "1.0"))  # shrink contexts when iterating
MAX_ABS_TOL, MEAN_ABS_TOL = 1e-2, 1e-3


def _say(*a):
    print(*a, flush=True)


def _dt(cfg):
    return wg.F32 if cfg.dtype == "f32" else wg.BF16


def _compare_meta(pool, orc, cfg, layers=None):
    """Bit-exact comparison of every metadata array with the oracle."""
    free, flag = pool.status()
    assert flag == 0
    m = {k: v.cpu().numpy() for k, v in pool.meta().items()}
    assert int(m["free_top"][0]) == orc.free_top == free
    np.testing.assert_array_equal(m["free_stack"][: orc.free_top], orc.free_stack()[: orc.free_top])
    for s in range(cfg.batch):
        for l in (range(cfg.n_layers) if layers is None else layers):
            assert int(m["seq_len"][s, l]) == orc.seq_len(s, l)
            for h in range(cfg.n_kv_heads):
                lp, gp, rg, _ = orc.head_tables(s, l, h)
                assert int(m["global_len"][s, l, h]) == orc.global_len(s, l, h), (s, l, h)
                np.testing.assert_array_equal(m["local_pt"][s, l, h], lp)
                np.testing.assert_array_equal(m["global_pt"][s, l, h], gp)
                np.testing.assert_array_equal(m["ring_g"][s, l, h].view(np.uint32), rg.view(np.uint32))
    return m


def _check_pages_injective(m, cfg, P):
    used = [m["local_pt"].reshape(-1)]
    gl = m["global_len"].reshape(-1)
    gp = m["global_pt"].reshape(len(gl), -1)
    npg = -(-gl // P)
    mask = np.arange(gp.shape[1])[None, :] < npg[:, None]
    used.append(gp[mask])
    used = np.concatenate(used)
    used = used[used >= 0]
    assert len(np.unique(used)) == len(used)
    assert len(used) + int(m["free_top"][0]) == len(m["free_stack"])


def _err_ok(out, ref, what):
    err = np.abs(out.astype(np.float64) - ref)
    assert np.isfinite(out).all(), what
    assert err.max() <= MAX_ABS_TOL and err.mean() <= MEAN_ABS_TOL, (what, err.max(), err.mean())
    return err.max(), err.mean()


def test_llama8b_single_layer_32k_exhaustive():
    """Workload 2: one layer, prefill 32K then 128 decode steps; everything is compared."""
    cfg = wl.get_config(1)
    n = max(int(cfg.ctx_max * SCALE), cfg.w_local + 1)
    Hq, Hk, d, W, P = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.w_local, cfg.page_size
    dev = torch.device("cuda:0")
    rates = wl.unit_rates(cfg)
    max_gp = (n + cfg.decode_steps) // P + 2
    n_pages = Hk * (max_gp + W // P) + 64
    pool = wg.Pool(wg.Config(1, Hq, Hk, d, _dt(cfg), P, W, 1, max_gp, n_pages), 1, n)
    orc = Oracle(OracleConfig(1, Hq, Hk, d, P, W, 1, max_gp, n_pages, True))
    k = wl.draw_normal(cfg, "k", (n, Hk, d), device=dev, key=(0, 0))
    v = wl.draw_normal(cfg, "v", (n, Hk, d), device=dev, key=(0, 0))
    g = wl.draw_scores(cfg, 0, 0, n, rates)
    mask = torch.zeros((n, Hk), dtype=torch.uint8, device=dev)
    pool.prefill_admit(0, [0], [n], k, v, torch.from_numpy(g).to(dev), tau=cfg.tau, admit_mask_out=mask)
    admit, _ = orc.push_tokens(0, [0], [n], k.float().cpu().numpy(), v.float().cpu().numpy(), g, cfg.tau)
    np.testing.assert_array_equal(mask.cpu().numpy(), admit)
    m = _compare_meta(pool, orc, cfg)
    _check_pages_injective(m, cfg, P)
    rate_seen = admit[: n - W].mean(0)
    assert np.abs(rate_seen - rates[0]).max() < 0.02          # the draw follows the stated per-head rates
    # cached rows, dereferenced through the page tables
    pages = pool.pool_pages()
    for h in range(Hk):
        gk, gv, _, _ = orc.payload(0, 0, h)
        G = orc.global_len(0, 0, h)
        idx = torch.arange(G, device=dev)
        pg = pool.meta()["global_pt"][0, 0, h][idx // P].long()
        assert torch.equal(pages[pg, 0, idx % P].float().cpu(), torch.from_numpy(gk))
        assert torch.equal(pages[pg, 1, idx % P].float().cpu(), torch.from_numpy(gv))
    scale = 1.0 / math.sqrt(d)
    out = torch.empty((1, Hq, d), dtype=torch.float32, device=dev)
    prom = torch.zeros((1, Hk), dtype=torch.uint8, device=dev)
    worst = (0.0, 0.0)
    for step in range(cfg.decode_steps):
        k1 = wl.draw_normal(cfg, "dec_k", (1, Hk, d), device=dev, key=(0, step))
        v1 = wl.draw_normal(cfg, "dec_v", (1, Hk, d), device=dev, key=(0, step))
        q1 = wl.draw_normal(cfg, "q", (1, Hq, d), device=dev, key=(0, step))
        g1 = wl.draw_scores(cfg, 0, 0, 1, rates, purpose="dec_scores", step=step)
        pool.decode_step(0, [0], k1, v1, torch.from_numpy(g1).to(dev), tau=cfg.tau, promoted_out=prom)
        pool.attend(0, [0], q1, out, scale)
        _, oprom = orc.push_tokens(0, [0], [1], k1.float().cpu().numpy(), v1.float().cpu().numpy(), g1, cfg.tau)
        np.testing.assert_array_equal(prom.cpu().numpy(), oprom)
        ref = orc.attend_cached(0, 0, q1[0].float().cpu().numpy(), scale)
        e = _err_ok(out[0].cpu().numpy(), ref, f"step {step}")
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
        if step % 32 == 31:
            _compare_meta(pool, orc, cfg)
    _compare_meta(pool, orc, cfg)
    _say(f"[workload 2] n={n}: attention max abs err {worst[0]:.2e}, worst mean abs err {worst[1]:.2e}")


def _run_multilayer(cfg, n_samples, decode_steps, check_steps):
    """Workloads 3 and 4: full integer-state parity, sampled attention parity."""
    B, L, Hq, Hk, d, W, P = (cfg.batch, cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                            cfg.w_local, cfg.page_size)
    dev = torch.device("cuda:0")
    ctx = wl.context_lengths(cfg)
    if SCALE != 1.0:
        ctx = np.maximum((ctx * SCALE).astype(np.int64), W + 1)
    rates = wl.unit_rates(cfg)
    max_ctx = int(ctx.max())
    exp_tokens = sum(float(rates[l, h]) * int(c) for c in ctx for l in range(L) for h in range(Hk))
    n_pages = int(exp_tokens / P * 1.10) + B * L * Hk * (-(-W // P) + 2 + -(-decode_steps // P)) + \
        Hk * (max_ctx // P + 2) + 1024
    max_gp = (max_ctx + decode_steps) // P + 2
    pool = wg.Pool(wg.Config(L, Hq, Hk, d, _dt(cfg), P, W, B, max_gp, n_pages), B, max_ctx)
    orc = Oracle(OracleConfig(L, Hq, Hk, d, P, W, B, max_gp, n_pages, False))  # integer state only
    _say(f"[{cfg.name}] B={B} L={L} ctx {int(ctx.min())}..{max_ctx}, pool {n_pages} pages "
         f"({pool.pool_buf.numel() / 2**30:.1f} GiB)")
    # sampled (sequence, layer) pairs for attention: longest sequence, densest and emptiest head, then seeded
    rng = np.random.default_rng(cfg.seed + 77)
    dense_l, _ = np.unravel_index(np.argmax(rates), rates.shape)
    empty_l, _ = np.unravel_index(np.argmin(rates), rates.shape)
    pairs = [(int(np.argmax(ctx)), 0), (int(rng.integers(B)), int(dense_l)), (int(rng.integers(B)), int(empty_l))]
    while len(pairs) < n_samples:
        pr = (int(rng.integers(B)), int(rng.integers(L)))
        if pr not in pairs:
            pairs.append(pr)
    hist = {}
    admit_total = np.zeros((L, Hk)); seen_total = np.zeros((L, Hk))
    for l in range(L):
        for s in range(B):
            n = int(ctx[s])
            k = wl.draw_normal(cfg, "k", (n, Hk, d), device=dev, key=(s, l))
            v = wl.draw_normal(cfg, "v", (n, Hk, d), device=dev, key=(s, l))
            g = wl.draw_scores(cfg, s, l, n, rates, device=dev)
            mask = torch.empty((n, Hk), dtype=torch.uint8, device=dev)
            pool.prefill_admit(l, [s], [n], k, v, g, tau=cfg.tau, admit_mask_out=mask)
            gh = g.cpu().numpy()
            admit, _ = orc.push_tokens(l, [s], [n], None, None, gh, cfg.tau)
            assert np.array_equal(mask.cpu().numpy(), admit), (s, l)
            admit_total[l] += admit.sum(0); seen_total[l] += n
            free, flag = pool.status()
            assert flag == 0 and free == orc.free_top, (s, l, free, orc.free_top)
            if (s, l) in pairs:  # dense history of the sampled pairs, with room for the decode tokens
                K = np.empty((n + decode_steps, Hk, d), np.float32)
                V = np.empty((n + decode_steps, Hk, d), np.float32)
                G = np.empty((n + decode_steps, Hk), np.float32)
                K[:n] = k.float().cpu().numpy(); V[:n] = v.float().cpu().numpy(); G[:n] = gh
                hist[(s, l)] = [K, V, G, n]
        if l % 8 == 7 or l == L - 1:
            _say(f"[{cfg.name}] prefilled layers 0..{l}, free pages {free}")
    assert np.abs(admit_total / seen_total - rates).max() < 0.02
    m = _compare_meta(pool, orc, cfg)
    _check_pages_injective(m, cfg, P)
    _say(f"[{cfg.name}] prefill state identical for all {B * L * Hk} (sequence, layer, head) units")
    seqs = list(range(B))
    scale = 1.0 / math.sqrt(d)
    out = torch.empty((L, B, Hq, d), dtype=torch.float32, device=dev)
    prom = torch.zeros((B, Hk), dtype=torch.uint8, device=dev)
    worst = [0.0, 0.0]
    for step in range(decode_steps):
        q_host = {}
        if step % 2 == 1:   # every other token with the promotions of all layers done ahead of the layers' steps
            pool.decode_promote(seqs, tau=cfg.tau)
        for l in range(L):
            k1 = wl.draw_normal(cfg, "dec_k", (B, Hk, d), device=dev, key=(l, step))
            v1 = wl.draw_normal(cfg, "dec_v", (B, Hk, d), device=dev, key=(l, step))
            q1 = wl.draw_normal(cfg, "q", (B, Hq, d), device=dev, key=(l, step))
            g1 = np.concatenate([wl.draw_scores(cfg, s, l, 1, rates, purpose="dec_scores", step=step) for s in seqs])
            pool.decode_step(l, seqs, k1, v1, torch.from_numpy(g1).to(dev), tau=cfg.tau, promoted_out=prom)
            pool.attend(l, seqs, q1, out[l], scale)
            _, oprom = orc.push_tokens(l, seqs, [1] * B, None, None, g1, cfg.tau)
            assert np.array_equal(prom.cpu().numpy(), oprom), (step, l)
            for (s, ll) in pairs:
                if ll == l:
                    h = hist[(s, l)]
                    t = h[3]
                    h[0][t] = k1[s].float().cpu().numpy()
                    h[1][t] = v1[s].float().cpu().numpy()
                    h[2][t] = g1[s]
                    h[3] = t + 1
                    q_host[(s, l)] = q1[s].float().cpu().numpy()
        if step in check_steps:
            o = out.cpu().numpy()
            for (s, l) in pairs:
                K, V, gg, t = hist[(s, l)]
                ref = attend_definition(K[:t], V[:t], gg[:t], q_host[(s, l)][None], np.array([t - 1]), W, cfg.tau, scale)
                e = _err_ok(o[l, s], ref[0], f"step {step} seq {s} layer {l}")
                worst = [max(worst[0], e[0]), max(worst[1], e[1])]
            _say(f"[{cfg.name}] step {step}: attention of {len(pairs)} sampled (seq, layer) pairs within tolerance")
    m = _compare_meta(pool, orc, cfg)
    _check_pages_injective(m, cfg, P)
    _say(f"[{cfg.name}] state identical after {decode_steps} decode steps; attention max abs err "
         f"{worst[0]:.2e}, worst mean abs err {worst[1]:.2e}")


def test_llama8b_32_layers_batch8_128k():
    """Workload 3 (the benchmark's): 32 layers, batch 8, contexts in [64K, 128K], 256 decode steps."""
    cfg = wl.get_config(2)
    steps = cfg.decode_steps if SCALE == 1.0 else 48
    _run_multilayer(cfg, n_samples=8, decode_steps=steps, check_steps={0, 1, 16, steps // 2, steps - 1})


def test_qwen3_4b_36_layers_batch32_64k_ragged():
    """Workload 4: 36 layers, batch 32, 64K contexts, W=128, P=32, heads from near-empty to near-dense."""
    cfg = wl.get_config(3)
    steps = cfg.decode_steps if SCALE == 1.0 else 40
    _run_multilayer(cfg, n_samples=8, decode_steps=steps, check_steps={0, 1, 32, steps // 2, steps - 1})
