"""wgkv_decode_promote: steps (1)-(2) of the lazy promotion (Sec. 4.3) of all layers ahead of the layers' own
decode steps.  The cache state, the promotion masks and the attention must be what the plain steps give (the
oracle knows nothing of the split), in eager calls, mixed with plain steps, for part of the sequences only, and
in a replayed HIP graph; the misuses are refused from the host or by the device's sticky flag, every kernel
exiting normally."""
import math

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
from harness import MAX_ABS_TOL, MEAN_ABS_TOL, Pair, rand_q, rand_tokens

pytestmark = pytest.mark.gpu

INVALID, OUT_OF_PAGES, NOT_PROMOTED = -1, -2, -9


def _prefill_all_layers(pr, rng, L, seqs, lens, Hk, d, rate=0.6):
    for l in range(L):
        k, v, g = rand_tokens(rng, sum(lens), Hk, d, pr.tdt, rates=[rate] * Hk)
        pr.prefill(l, seqs, lens, k, v, g, 0.5)


@pytest.mark.parametrize("P,W", [(4, 8), (16, 32), (1, 3)])
def test_promote_ahead_gives_the_state_of_plain_steps(P, W):
    L, Hq, Hk, d, B = 3, 8, 2, 64, 3
    rng = np.random.default_rng(50 + P)
    pr = Pair(L, Hq, Hk, d, wg.BF16, P, W, B, 64, 2000, max_call_seqs=B, max_call_tokens=128)
    seqs = [2, 0, 1]
    _prefill_all_layers(pr, rng, L, seqs, [W + 5, 2, W - 1], Hk, d)   # full ring, nearly empty, one short of full
    pr.check_state()
    for step in range(3 * W + 7):
        mode = step % 4
        if mode in (0, 1):
            pr.pool.decode_promote(seqs, tau=0.5)          # every sequence: the layers' steps only write the ring
            if mode == 1:
                pr.pool.decode_promote(seqs, tau=0.5)      # twice: nothing more happens
        for l in range(L):
            k, v, g = rand_tokens(rng, B, Hk, d, pr.tdt, rates=[0.6] * Hk)
            pr.decode(l, seqs, k, v, g, 0.5)               # compares the promotion mask with the oracle's
        if step % 5 == 0:
            pr.check_state()
    pr.check_state()
    for l in range(L):
        pr.check_attend(l, seqs, rand_q(rng, B, Hq, d, pr.tdt))


@pytest.mark.parametrize("seed", range(8))
def test_promote_ahead_on_seeded_random_shapes(seed):
    """Shapes, window, page size, sequence lengths and the tokens with a promotion ahead all drawn from the seed."""
    rng = np.random.default_rng(700 + seed)
    L = int(rng.integers(1, 4))
    Hk = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 4, 8]))
    d = int(rng.choice([64, 128]))
    dtype = wg.BF16 if rng.random() < 0.7 else wg.F32
    P = int(rng.choice([1, 2, 4, 8, 16, 32]))
    W = int(rng.integers(1, 41))
    B = int(rng.integers(1, 5))
    pr = Pair(L, Hk * G, Hk, d, dtype, P, W, B, 96, 6000, max_call_seqs=B, max_call_tokens=256)
    seqs = [int(x) for x in rng.permutation(B)]
    lens = [int(rng.integers(1, 2 * W + 20)) for _ in seqs]
    _prefill_all_layers(pr, rng, L, seqs, lens, Hk, d, rate=float(rng.uniform(0.2, 0.9)))
    n_steps = 2 * W + 9
    for step in range(n_steps):
        if rng.random() < 0.6:
            pr.pool.decode_promote(seqs, tau=0.5)
        for l in range(L):
            k, v, g = rand_tokens(rng, B, Hk, d, pr.tdt, rates=[0.6] * Hk)
            pr.decode(l, seqs, k, v, g, 0.5)
        if step % 7 == 3 or step == n_steps - 1:
            pr.check_state()
            l = int(rng.integers(L))
            pr.check_attend(l, seqs, rand_q(rng, B, Hk * G, d, pr.tdt))


def test_promote_ahead_for_part_of_the_call():
    """A step whose call holds promoted and unpromoted sequences takes the general kernel, which honours the
    stamps.  One layer and the promoted sequence first in the call: the pages are then taken in the order of
    plain steps and the page tables can be compared bit for bit."""
    L, Hq, Hk, d, B, P, W = 1, 8, 2, 64, 3, 4, 8
    rng = np.random.default_rng(56)
    pr = Pair(L, Hq, Hk, d, wg.BF16, P, W, B, 64, 600, max_call_seqs=B, max_call_tokens=128)
    seqs = [2, 0, 1]
    _prefill_all_layers(pr, rng, L, seqs, [W + 5, W + 1, W - 1], Hk, d)
    for step in range(2 * W + 3):
        if step % 2 == 0:
            pr.pool.decode_promote([2], tau=0.5)
        k, v, g = rand_tokens(rng, B, Hk, d, pr.tdt, rates=[0.6] * Hk)
        pr.decode(0, seqs, k, v, g, 0.5)
        pr.check_state()
    pr.check_attend(0, seqs, rand_q(rng, B, Hq, d, pr.tdt))


def test_promote_ahead_in_a_replayed_graph():
    rng = np.random.default_rng(57)
    L, Hq, Hk, d, P, W, B, T = 2, 32, 8, 128, 16, 32, 2, 150
    max_gp = (T + 64) // P + 4
    pr = Pair(L, Hq, Hk, d, wg.BF16, P, W, B, max_gp, B * L * Hk * (max_gp + W // P) + 16, max_call_seqs=B,
              max_call_tokens=B * T)
    dev, seqs = pr.dev, [0, 1]
    _prefill_all_layers(pr, rng, L, seqs, [T, T], Hk, d)
    pr.pool.decode_promote(seqs, tau=0.5)                  # one eager step first
    for l in range(L):
        k, v, g = rand_tokens(rng, B, Hk, d, pr.tdt, rates=[0.7] * Hk)
        pr.decode(l, seqs, k, v, g, 0.5)
    pr.check_state()
    scale = 1.0 / math.sqrt(d)
    kb = torch.zeros((L, B, Hk, d), dtype=torch.bfloat16, device=dev)
    vb = torch.zeros_like(kb)
    gb = torch.zeros((L, B, Hk), dtype=torch.float32, device=dev)
    qb = torch.zeros((L, B, Hq, d), dtype=torch.bfloat16, device=dev)
    ob = torch.zeros((L, B, Hq, d), dtype=torch.float32, device=dev)
    pm = torch.zeros((L, B, Hk), dtype=torch.uint8, device=dev)
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            pr.pool.decode_promote(seqs, tau=0.5)
            for l in range(L):
                pr.pool.decode_step(l, seqs, kb[l], vb[l], gb[l], tau=0.5, promoted_out=pm[l])
                pr.pool.attend(l, seqs, qb[l], ob[l], scale)
    torch.cuda.current_stream().wait_stream(side)
    for step in range(2 * P + 3):
        ks, vs, gs, qs = [], [], [], []
        for l in range(L):
            k, v, g = rand_tokens(rng, B, Hk, d, pr.tdt, rates=[0.8] * Hk)
            ks.append(k); vs.append(v); gs.append(g)
            qs.append(rand_q(rng, B, Hq, d, pr.tdt))
        kb.copy_(torch.stack(ks)); vb.copy_(torch.stack(vs)); gb.copy_(torch.stack(gs)); qb.copy_(torch.stack(qs))
        ob.fill_(float("nan"))
        pm.fill_(7)
        graph.replay()
        torch.cuda.synchronize()
        out = ob.cpu().numpy().astype(np.float64)
        for l in range(L):
            _, oprom = pr.orc.push_tokens(l, seqs, [1] * B, ks[l].float().numpy(), vs[l].float().numpy(),
                                          gs[l].numpy(), 0.5)
            np.testing.assert_array_equal(pm[l].cpu().numpy(), oprom)
            ref = np.stack([pr.orc.attend_cached(s, l, qs[l][i].float().numpy(), scale) for i, s in enumerate(seqs)])
            err = np.abs(out[l] - ref)
            assert np.isfinite(out[l]).all() and err.max() <= MAX_ABS_TOL and err.mean() <= MEAN_ABS_TOL, (step, l)
    pr.check_state()


def test_replayed_ring_write_without_its_promotion_sets_the_flag():
    rng = np.random.default_rng(58)
    L, Hq, Hk, d, P, W = 1, 8, 2, 64, 4, 8
    pr = Pair(L, Hq, Hk, d, wg.BF16, P, W, 1, 32, 200, max_call_seqs=1, max_call_tokens=64)
    dev = pr.dev
    _prefill_all_layers(pr, rng, L, [0], [W + 3], Hk, d)
    k1, v1, g1 = rand_tokens(rng, 1, Hk, d, pr.tdt, rates=[0.9] * Hk)
    kb, vb, gb = k1.to(dev), v1.to(dev), g1.to(dev)
    pr.pool.decode_promote([0], tau=0.5)        # eager: the promotion of the coming token is done
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            pr.pool.decode_step(0, [0], kb, vb, gb, tau=0.5)    # captured as the ring write alone
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()                               # this token was promoted ahead: a good step
    torch.cuda.synchronize()
    pr.orc.push_tokens(0, [0], [1], k1.float().numpy(), v1.float().numpy(), g1.numpy(), 0.5)
    free, flag = pr.pool.status()
    assert flag == 0
    pr.check_state()
    graph.replay()                               # the next one was not: nothing may change
    torch.cuda.synchronize()
    free, flag = pr.pool.status()
    assert flag == NOT_PROMOTED
    pr.pool.clear_error()
    pr.check_state()
    k2, v2, g2 = rand_tokens(rng, 1, Hk, d, pr.tdt, rates=[0.9] * Hk)
    pr.decode(0, [0], k2, v2, g2, 0.5)           # a plain step goes on from there
    pr.check_state()
    pr.check_attend(0, [0], rand_q(rng, 1, Hq, d, pr.tdt))


def test_promote_ahead_refusals_and_slot_reuse():
    rng = np.random.default_rng(59)
    L, Hq, Hk, d, P, W = 2, 8, 2, 64, 4, 8
    # sequence 0: 12 tokens, all admitted: 4 global entries = 1 full page per head and layer; ring 2 pages
    n_pages = L * Hk * (1 + 2)
    pr = Pair(L, Hq, Hk, d, wg.BF16, P, W, 2, 8, n_pages, max_call_seqs=2, max_call_tokens=64)
    dev = pr.dev
    for l in range(L):
        k, v, g = rand_tokens(rng, 12, Hk, d, pr.tdt)
        g[:] = 0.9
        pr.prefill(l, [0], [12], k, v, g, 0.5)
    pr.check_state()
    assert pr.orc.free_top == 0
    before = pr.pool.meta_buf.cpu().numpy().copy()
    with pytest.raises(wg.WgkvError) as e:       # every head would open a second global page: none left
        pr.pool.decode_promote([0], tau=0.5)
    assert e.value.code == OUT_OF_PAGES
    torch.cuda.synchronize()
    np.testing.assert_array_equal(pr.pool.meta_buf.cpu().numpy(), before)
    # layers out of step: refused
    pr2 = Pair(L, Hq, Hk, d, wg.BF16, P, W, 2, 8, 100, max_call_seqs=2, max_call_tokens=64)
    k, v, g = rand_tokens(rng, 12, Hk, d, pr2.tdt)
    pr2.prefill(0, [0], [12], k, v, g, 0.5)
    pr2.prefill(1, [0], [11], k[:11], v[:11], g[:11], 0.5)
    with pytest.raises(wg.WgkvError) as e:
        pr2.pool.decode_promote([0], tau=0.5)
    assert e.value.code == INVALID
    pr2.prefill(1, [0], [1], k[11:], v[11:], g[11:], 0.5)
    pr2.pool.decode_promote([0], tau=0.5)
    with pytest.raises(wg.WgkvError) as e:       # promoted ahead: only the decode step may follow
        pr2.pool.prefill_admit(0, [0], [1], k[:1].to(pr2.dev), v[:1].to(pr2.dev), g[:1].to(pr2.dev), tau=0.5)
    assert e.value.code == INVALID
    # a freed slot forgets the promotion: the same token count later is a new token
    pr2.pool.free_seq(0)
    pr2.orc.free_seq(0)
    for l in range(L):
        pr2.touched.discard((0, l))
    for l in range(L):
        k, v, g = rand_tokens(rng, 12, Hk, d, pr2.tdt, rates=[0.7] * Hk)
        pr2.prefill(l, [0], [12], k, v, g, 0.5)
    for l in range(L):
        k, v, g = rand_tokens(rng, 1, Hk, d, pr2.tdt, rates=[0.7] * Hk)
        pr2.decode(l, [0], k, v, g, 0.5)
    pr2.check_state()
    for l in range(L):
        pr2.check_attend(l, [0], rand_q(rng, 1, Hq, d, pr2.tdt))
