"""Removal step of the budgeted eviction (appendix "Eviction policy implementation") on the GPU
against the oracle, through the C ABI: which entries go, in-place compaction of the rows, page
release order, and that the cache keeps working afterwards (attention, promotion, reuse of pages)."""
import math

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
from harness import Pair, rand_tokens

pytestmark = pytest.mark.gpu


def _scores(rng, pair, layer, seq_ids, kind, extra=3):
    Hk = pair.cfg.n_kv_heads
    N = max(pair.orc.global_len(s, layer, h) for s in seq_ids for h in range(Hk))
    shape = (len(seq_ids) * Hk, N + extra)
    if kind == "uniform":
        return rng.random(shape).astype(np.float32)
    if kind == "ties":                       # eight distinct values: every cut falls inside a tie
        return (rng.integers(0, 8, shape) / 8.0).astype(np.float32)
    if kind == "signed":                     # negative numbers, zeros of both signs, an infinity
        x = rng.standard_normal(shape).astype(np.float32)
        x[:, ::7] = 0.0
        x[:, 3::11] = -0.0
        x[:, 5::13] = np.inf
        return x
    raise ValueError(kind)


@pytest.mark.parametrize("dtype,d,P,W,T,frac,kind", [
    (wg.F32, 64, 4, 8, 300, 0.1, "uniform"),
    (wg.BF16, 128, 16, 32, 700, 0.1, "ties"),
    (wg.BF16, 128, 16, 256, 3000, 0.5, "uniform"),     # more than one tile of 1024 entries per head
    (wg.BF16, 64, 8, 16, 500, 0.37, "signed"),
    (wg.F32, 128, 2, 4, 200, 1.0, "uniform"),          # everything goes
    (wg.BF16, 128, 16, 64, 400, 0.0, "uniform"),       # nothing goes
])
def test_evict_apply_state_and_attention(dtype, d, P, W, T, frac, kind):
    rng = np.random.default_rng(T + d)
    Hq, Hk, L, B = 8, 2, 2, 3
    max_gp = T // P + 8
    n_pages = B * L * Hk * (max_gp + -(-W // P)) + 16
    pair = Pair(L, Hq, Hk, d, dtype, P, W, B, max_gp, n_pages, max_call_seqs=B, max_call_tokens=B * T)
    lens = [T, T - 57, T // 2]
    for layer in range(L):
        k, v, g = rand_tokens(rng, sum(lens), Hk, d, pair.tdt, rates=[0.7, 0.35])
        pair.prefill(layer, [0, 1, 2], lens, k, v, g, 0.5)
    pair.check_state()
    used_before = n_pages - pair.orc.free_top
    # evict on layer 1 for two of the sequences, in an order that is not the slot order
    seqs = [2, 0]
    sc = _scores(rng, pair, 1, seqs, kind)
    gone = pair.evict(1, seqs, sc, frac)
    n_before = [g0 + pair.orc.global_len(s, 1, h) for (s, h), g0 in zip([(s, h) for s in seqs for h in range(Hk)], gone)]
    assert list(gone) == [int(math.floor(float(np.float32(frac)) * n)) for n in n_before]
    pair.check_state()
    assert n_pages - pair.orc.free_top <= used_before
    q = torch.from_numpy(rng.standard_normal((3, Hq, d)).astype(np.float32)).to(pair.tdt)
    pair.check_attend(1, [0, 1, 2], q)
    # the cache goes on: decode steps promote into the packed caches and reuse the released pages
    for step in range(2 * P + 3):
        k, v, g = rand_tokens(rng, 3, Hk, d, pair.tdt, rates=[0.9, 0.6])
        pair.decode(1, [0, 1, 2], k, v, g, 0.5)
    pair.check_state()
    pair.check_attend(1, [0, 1, 2], q)
    # a second round on everything, then free a sequence
    sc = _scores(rng, pair, 1, [0, 1, 2], "ties")
    pair.evict(1, [0, 1, 2], sc, 0.25)
    pair.check_state()
    pair.check_attend(1, [1, 2], q[:2])
    pair.pool.free_seq(0)
    pair.orc.free_seq(0)
    pair.check_state()


def test_evict_apply_many_entries_and_units():
    """64 heads of about 10K entries (one layer of a long-context batch), 10 % removed."""
    rng = np.random.default_rng(99)
    Hq, Hk, d, P, W, B, T = 32, 8, 128, 16, 256, 8, 16000
    max_gp = T // P + 4
    n_pages = B * Hk * (max_gp + W // P) + 64
    pair = Pair(1, Hq, Hk, d, wg.BF16, P, W, B, max_gp, n_pages, max_call_seqs=B, max_call_tokens=T)
    for s in range(B):
        k, v, g = rand_tokens(rng, T - 100 * s, Hk, d, pair.tdt, rates=list(np.linspace(0.3, 0.9, Hk)))
        pair.prefill(0, [s], [T - 100 * s], k, v, g, 0.5)
    seqs = list(range(B))
    pair.pool.status()      # exact lengths on the host, so that score rows need not cover the worst case
    sc = _scores(rng, pair, 0, seqs, "uniform")
    gone = pair.evict(0, seqs, sc, 0.1)
    assert gone.min() > 300 and gone.max() > 1200
    pair.check_state()
    q = torch.from_numpy(rng.standard_normal((B, Hq, d)).astype(np.float32)).to(pair.tdt)
    pair.check_attend(0, seqs, q)


def test_evict_apply_rejects_bad_arguments():
    rng = np.random.default_rng(1)
    pair = Pair(1, 4, 2, 64, wg.F32, 4, 8, 2, 64, 400, max_call_seqs=2, max_call_tokens=256)
    k, v, g = rand_tokens(rng, 100, 2, 64, pair.tdt)
    pair.prefill(0, [0], [100], k, v, g, 0.3)
    dev = pair.dev
    good = torch.zeros((2, 128), dtype=torch.float32, device=dev)
    with pytest.raises(wg.WgkvError):
        pair.pool.evict_apply(0, [0], good, 1.5)
    with pytest.raises(wg.WgkvError):
        pair.pool.evict_apply(0, [0], good, float("nan"))
    with pytest.raises(wg.WgkvError):                      # rows shorter than what a head may hold
        pair.pool.evict_apply(0, [0], torch.zeros((2, 8), dtype=torch.float32, device=dev), 0.1)
    with pytest.raises(wg.WgkvError):
        pair.pool.evict_apply(0, [0, 0], torch.zeros((4, 128), dtype=torch.float32, device=dev), 0.1)
    pair.check_state()                                      # nothing happened


# ---- the scoring steps ----
# fp32 products of exactly representable inputs, fp32 exp2 and sums of up to n_obs weights in [0, 1]:
# relative error of a score ~1e-6 per operation; scores are at most n_obs.
SCORE_RTOL = 2e-5


def _check_scores(pair, layer, seqs, q_obs, scale, pool_w):
    Hk = pair.cfg.n_kv_heads
    N = [pair.orc.global_len(s, layer, h) for s in seqs for h in range(Hk)]
    stride = max(N) + 5
    raw, out = pair.pool.evict_scores(layer, seqs, q_obs.to(pair.dev), scale, stride, pool_w=pool_w)
    raw, out = raw.cpu().numpy(), out.cpu().numpy()
    worst = 0.0
    refs = np.zeros_like(out)
    for b, s in enumerate(seqs):
        for h in range(Hk):
            u = b * Hk + h
            r_ref, s_ref = pair.orc.evict_scores(layer, s, h, q_obs[b].float().numpy(), scale, pool_w=pool_w)
            n = N[u]
            assert np.all(raw[u, n:] == 0) and np.all(out[u, n:] == 0)          # rows past the length are left alone
            if n:
                tol = SCORE_RTOL * max(1.0, float(r_ref.max()))
                assert np.abs(raw[u, :n] - r_ref).max() <= tol
                assert np.abs(out[u, :n] - s_ref).max() <= tol
                worst = max(worst, np.abs(out[u, :n] - s_ref).max() / max(1.0, float(r_ref.max())))
                refs[u, :n] = s_ref
    return out, refs, N, worst


@pytest.mark.parametrize("dtype,Hq,Hk,d,P,W,T,n_obs,pool_w", [
    (wg.F32, 8, 2, 64, 4, 8, 300, 16, 5),
    (wg.BF16, 8, 2, 128, 16, 32, 500, 32, 5),
    (wg.BF16, 4, 4, 128, 16, 16, 200, 7, 3),          # group of one, rows not a multiple of the tile
    (wg.BF16, 16, 2, 64, 8, 16, 333, 24, 1),          # group of eight, no pooling
    (wg.F32, 4, 2, 128, 2, 4, 150, 40, 9),
    (wg.BF16, 32, 8, 128, 16, 256, 2500, 256, 5),     # the paper's window of 256 queries, matrix-core path
    (wg.BF16, 8, 2, 128, 16, 8, 140, 8, 5),           # matrix-core path, caches shorter than a block of keys
])
def test_evict_scores_match_fp64(dtype, Hq, Hk, d, P, W, T, n_obs, pool_w):
    rng = np.random.default_rng(T * 3 + n_obs)
    B = 2
    max_gp = T // P + 4
    pair = Pair(1, Hq, Hk, d, dtype, P, W, B, max_gp, B * Hk * (max_gp + -(-W // P)) + 8, max_call_seqs=B,
                max_call_tokens=B * T)
    lens = [T, T // 3]
    k, v, g = rand_tokens(rng, sum(lens), Hk, d, pair.tdt, rates=list(np.linspace(0.8, 0.3, Hk)))
    pair.prefill(0, [0, 1], lens, k, v, g, 0.5)
    pair.pool.status()
    q_obs = torch.from_numpy(rng.standard_normal((B, n_obs, Hq, d)).astype(np.float32)).to(pair.tdt)
    scale = 1.0 / math.sqrt(d)
    _, _, N, worst = _check_scores(pair, 0, [1, 0], q_obs, scale, pool_w)
    assert min(N) > 10
    pair.check_state()          # scoring changes nothing


def test_evict_scores_then_apply():
    """Both steps chained on each side: the GPU removes by its fp32 scores, the oracle by its own fp64
    scores (rounded to fp32, its input format), and the states must then agree bit for bit."""
    rng = np.random.default_rng(2024)
    Hq, Hk, d, P, W, T, n_obs = 8, 2, 128, 16, 64, 900, 48
    max_gp = T // P + 4
    pair = Pair(1, Hq, Hk, d, wg.BF16, P, W, 1, max_gp, Hk * (max_gp + W // P) + 8, max_call_seqs=1, max_call_tokens=T)
    k, v, g = rand_tokens(rng, T, Hk, d, pair.tdt, rates=[0.7, 0.5])
    pair.prefill(0, [0], [T], k, v, g, 0.5)
    pair.pool.status()
    q_obs = torch.from_numpy(rng.standard_normal((1, n_obs, Hq, d)).astype(np.float32)).to(pair.tdt)
    scale = 1.0 / math.sqrt(d)
    out, refs, N, _ = _check_scores(pair, 0, [0], q_obs, scale, 5)
    frac = 0.1
    for u in range(Hk):
        # Max-pooling makes runs of exactly equal scores on both sides (copies of one value), which the
        # common tie rule settles; what could differ is the order of two distinct values closer than the
        # rounding error.  The seeded input must not have that at the cut: the entries that a stable
        # sort of either side's scores puts below the cut are the same.
        n_e = int(math.floor(float(np.float32(frac)) * N[u]))
        low_gpu = set(np.argsort(out[u, :N[u]], kind="stable")[:n_e])
        low_orc = set(np.argsort(refs[u, :N[u]].astype(np.float32), kind="stable")[:n_e])
        assert n_e > 10 and low_gpu == low_orc, "the cut falls into a near-tie of distinct scores: pick another seed"
    gone = torch.zeros((Hk,), dtype=torch.int32, device=pair.dev)
    pair.pool.evict_apply(0, [0], torch.from_numpy(out).to(pair.dev), frac, n_evicted_out=gone)
    ogone = pair.orc.evict_apply(0, [0], refs.astype(np.float32), frac)
    np.testing.assert_array_equal(gone.cpu().numpy(), ogone)
    pair.check_state()
    q = torch.from_numpy(rng.standard_normal((1, Hq, d)).astype(np.float32)).to(pair.tdt)
    pair.check_attend(0, [0], q)
