"""Drives the GPU library and the CPU oracle side by side on the same inputs and
compares them: integer state bit for bit, attention within the stated tolerance."""
import math

import numpy as np
import torch

import paper_2512_17452_amd as wg
from oracle import Oracle, OracleConfig

MAX_ABS_TOL = 1e-2   # bf16 inputs, fp32 accumulation (stated target)
MEAN_ABS_TOL = 1e-3
F32_MAX_ABS_TOL = 2e-5  # fp32 inputs: rounding of fp32 dot products / exp2 only


def torch_dtype(dt):
    return torch.float32 if dt == wg.F32 else torch.bfloat16


class Pair:
    """One GPU pool and one oracle fed with identical calls."""

    def __init__(self, n_layers, Hq, Hk, d, dtype, P, W, max_seqs, max_gp, n_pages,
                 max_call_seqs=8, max_call_tokens=4096, payload=True):
        self.cfg = wg.Config(n_layers, Hq, Hk, d, dtype, P, W, max_seqs, max_gp, n_pages)
        self.pool = wg.Pool(self.cfg, max_call_seqs, max_call_tokens)
        self.orc = Oracle(OracleConfig(n_layers, Hq, Hk, d, P, W, max_seqs, max_gp, n_pages, payload))
        self.dev = self.pool.device
        self.tdt = torch_dtype(dtype)
        self.touched = set()

    # inputs are torch CPU tensors in the pool dtype (k, v, q) and float32 (g)
    def prefill(self, layer, seq_ids, n_tokens, k, v, g, tau, check_mask=True, max_admitted_per_head=None):
        tot = int(sum(n_tokens))
        Hk = self.cfg.n_kv_heads
        mask = torch.zeros((max(tot, 1), Hk), dtype=torch.uint8, device=self.dev)
        self.pool.prefill_admit(layer, seq_ids, n_tokens, k.to(self.dev), v.to(self.dev),
                                g.to(self.dev), tau=tau, admit_mask_out=mask,
                                max_admitted_per_head=max_admitted_per_head)
        admit, _ = self.orc.push_tokens(layer, seq_ids, n_tokens, k.float().numpy(), v.float().numpy(),
                                        g.numpy(), tau)
        for s, n in zip(seq_ids, n_tokens):
            if n > 0:
                self.touched.add((s, layer))
        if check_mask and tot > 0:
            np.testing.assert_array_equal(mask.cpu().numpy()[:tot], admit)

    def decode(self, layer, seq_ids, k, v, g, tau):
        n = len(seq_ids)
        Hk = self.cfg.n_kv_heads
        prom = torch.zeros((n, Hk), dtype=torch.uint8, device=self.dev)
        self.pool.decode_step(layer, seq_ids, k.to(self.dev), v.to(self.dev), g.to(self.dev), tau=tau,
                              promoted_out=prom)
        _, oprom = self.orc.push_tokens(layer, seq_ids, [1] * n, k.float().numpy(), v.float().numpy(),
                                        g.numpy(), tau)
        for s in seq_ids:
            self.touched.add((s, layer))
        np.testing.assert_array_equal(prom.cpu().numpy(), oprom)

    def evict(self, layer, seq_ids, scores, frac):
        """scores: numpy float32 [len(seq_ids) * Hk, stride]; both sides drop floor(frac * N) per head."""
        n_units = len(seq_ids) * self.cfg.n_kv_heads
        gone = torch.full((n_units,), -1, dtype=torch.int32, device=self.dev)
        self.pool.evict_apply(layer, seq_ids, torch.from_numpy(scores).to(self.dev), frac, n_evicted_out=gone)
        ogone = self.orc.evict_apply(layer, seq_ids, scores, frac)
        np.testing.assert_array_equal(gone.cpu().numpy().astype(np.int64), ogone)
        return ogone

    def attend(self, layer, seq_ids, q, scale=None):
        c = self.cfg
        if scale is None:
            scale = 1.0 / math.sqrt(c.head_dim)
        out = torch.full((len(seq_ids), c.n_q_heads, c.head_dim), float("nan"), dtype=torch.float32, device=self.dev)
        self.pool.attend(layer, seq_ids, q.to(self.dev), out, scale)
        ref = np.stack([self.orc.attend_cached(s, layer, q[i].float().numpy(), scale) for i, s in enumerate(seq_ids)])
        return out.cpu().numpy().astype(np.float64), ref

    def check_attend(self, layer, seq_ids, q, scale=None):
        out, ref = self.attend(layer, seq_ids, q, scale)
        err = np.abs(out - ref)
        assert np.isfinite(out).all()
        if self.cfg.dtype == wg.F32:
            assert err.max() <= F32_MAX_ABS_TOL, err.max()
        else:
            assert err.max() <= MAX_ABS_TOL and err.mean() <= MEAN_ABS_TOL, (err.max(), err.mean())
        return err.max(), err.mean()

    def check_state(self, payload=True):
        """Bit-exact comparison of all metadata and of the cached rows."""
        c = self.cfg
        free, flag = self.pool.status()
        assert flag == 0
        m = {k: v.cpu().numpy() for k, v in self.pool.meta().items()}
        o = self.orc
        assert int(m["free_top"][0]) == o.free_top == free
        np.testing.assert_array_equal(m["free_stack"][: o.free_top], o.free_stack()[: o.free_top])
        pages = self.pool.pool_pages().float().cpu().numpy() if payload else None
        P, W = c.page_size, c.w_local
        for s in range(c.max_seqs):
            for l in range(c.n_layers):
                assert int(m["seq_len"][s, l]) == o.seq_len(s, l)
                for h in range(c.n_kv_heads):
                    lp, gp, rg, rp = o.head_tables(s, l, h)
                    G = o.global_len(s, l, h)
                    assert int(m["global_len"][s, l, h]) == G
                    np.testing.assert_array_equal(m["local_pt"][s, l, h], lp)
                    np.testing.assert_array_equal(m["global_pt"][s, l, h], gp)
                    np.testing.assert_array_equal(m["ring_g"][s, l, h].view(np.uint32), rg.view(np.uint32))
                    if payload and (s, l) in self.touched:
                        gk, gv, rk, rv = o.payload(s, l, h)
                        if G:
                            idx = np.arange(G)
                            pg = m["global_pt"][s, l, h][idx // P]
                            np.testing.assert_array_equal(pages[pg, 0, idx % P], gk)
                            np.testing.assert_array_equal(pages[pg, 1, idx % P], gv)
                        valid = np.nonzero(rp >= 0)[0]
                        if len(valid):
                            pg = m["local_pt"][s, l, h][valid // P]
                            np.testing.assert_array_equal(pages[pg, 0, valid % P], rk[valid])
                            np.testing.assert_array_equal(pages[pg, 1, valid % P], rv[valid])


def rand_tokens(rng, n, Hk, d, tdt, rates=None, tau=0.5):
    """K, V ~ N(0,1) in dtype, scores uniform (or with per-head admission rates)."""
    k = torch.from_numpy(rng.standard_normal((n, Hk, d)).astype(np.float32)).to(tdt)
    v = torch.from_numpy(rng.standard_normal((n, Hk, d)).astype(np.float32)).to(tdt)
    u = rng.random((n, Hk))
    if rates is not None:
        b = np.log(np.asarray(rates)) / math.log(1 - tau)
        u = 1 - np.power(1 - u, 1 / b[None, :])
    return k, v, torch.from_numpy(u.astype(np.float32))


def rand_q(rng, n, Hq, d, tdt):
    return torch.from_numpy(rng.standard_normal((n, Hq, d)).astype(np.float32)).to(tdt)
