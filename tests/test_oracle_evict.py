"""Pins of the oracle's budgeted eviction (appendix "Eviction policy implementation"):
importance scores against a library softmax / max-pool composition and hand-computed
cases, the removal against a library sort, page accounting, and attention over the
cache that is left against library attention under an explicit mask."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import Oracle, OracleConfig


def _filled(seed, T, Hq=4, Hk=2, d=8, P=4, W=4, tau=0.4, n_pages=256, max_gp=64):
    """An oracle that has seen T tokens of one sequence; returns it with the inputs."""
    o = Oracle(OracleConfig(1, Hq, Hk, d, P, W, 2, max_gp, n_pages, True))
    r = np.random.default_rng(seed)
    k = r.standard_normal((T, Hk, d)).astype(np.float32)
    v = r.standard_normal((T, Hk, d)).astype(np.float32)
    g = r.random((T, Hk)).astype(np.float32)
    o.push_tokens(0, [0], [T], k, v, g, tau)
    return o, k, v, g, r


def _library_scores(gk, q, scale, pool_w):
    """q [n_obs, G, d] of one group, gk [N, d]: the three steps from torch routines, fp64."""
    a = torch.softmax(torch.einsum("igd,jd->igj", torch.from_numpy(q).double(), torch.from_numpy(gk).double()) * scale, dim=-1)
    raw = a.amax(dim=1).sum(dim=0)
    s = F.max_pool1d(raw[None, None], pool_w, stride=1, padding=pool_w // 2)[0, 0]
    return raw.numpy(), s.numpy()


def test_scores_match_library_composition():
    for seed, (Hq, Hk, pool_w, n_obs) in enumerate([(4, 2, 5, 6), (2, 2, 3, 9), (8, 2, 1, 3), (4, 1, 5, 16)]):
        o, *_, r = _filled(seed, 60, Hq=Hq, Hk=Hk)
        G = Hq // Hk
        q = r.standard_normal((n_obs, Hq, 8)).astype(np.float32)
        for h in range(Hk):
            raw, s = o.evict_scores(0, 0, h, q, 0.3, pool_w=pool_w)
            gk = o.payload(0, 0, h)[0]
            assert len(raw) == o.global_len(0, 0, h) > 10
            raw_ref, s_ref = _library_scores(gk, q[:, h * G:(h + 1) * G], 0.3, pool_w)
            assert np.abs(raw - raw_ref).max() < 1e-14 and np.abs(s - s_ref).max() < 1e-14
            # every query row spreads weight one over the entries; the maximum over the group keeps
            # at least that and at most G times that
            assert n_obs - 1e-9 <= raw.sum() <= n_obs * G + 1e-9
            if G == 1:
                assert abs(raw.sum() - n_obs) < 1e-12
            assert np.all(s >= raw)


def test_scores_by_hand():
    # one-dimensional keys 0 and ln 3, query +1: weights (1/4, 3/4); the group's other head has
    # query -1: weights (3/4, 1/4).  Two observation rows.
    W, P = 2, 2
    o = Oracle(OracleConfig(1, 2, 1, 1, P, W, 1, 8, 16, True))
    k = np.array([0.0, math.log(3.0), 5.0, 5.0], np.float32).reshape(4, 1, 1)    # the last W tokens stay in the ring
    o.push_tokens(0, [0], [4], k, k, np.ones((4, 1), np.float32), 0.5)
    assert o.global_len(0, 0, 0) == 2
    q = np.array([[[1.0], [-1.0]], [[1.0], [-1.0]]], np.float32)                  # [n_obs=2, Hq=2, d=1]
    raw, s = o.evict_scores(0, 0, 0, q, 1.0, pool_w=1)
    assert np.allclose(raw, [1.5, 1.5], atol=1e-7) and np.allclose(s, raw)          # ln 3 is rounded to fp32
    q1 = np.array([[[1.0], [1.0]], [[1.0], [1.0]]], np.float32)                   # both heads +1
    raw, s = o.evict_scores(0, 0, 0, q1, 1.0, pool_w=3)
    assert np.allclose(raw, [0.5, 1.5], atol=1e-7) and np.allclose(s, [1.5, 1.5], atol=1e-7)
    # scale enters the exponent: with scale 2 the weights are (1/10, 9/10)
    raw, _ = o.evict_scores(0, 0, 0, q1[:1], 2.0, pool_w=1)
    assert np.allclose(raw, [0.1, 0.9], atol=1e-7)


def test_max_pool_window_is_centred_and_clipped():
    o, *_, r = _filled(3, 80, Hq=2, Hk=2)
    q = r.standard_normal((4, 2, 8)).astype(np.float32)
    raw, s = o.evict_scores(0, 0, 1, q, 0.5, pool_w=5)
    n = len(raw)
    for j in range(n):
        assert s[j] == raw[max(0, j - 2):min(n, j + 3)].max()


def test_apply_removes_the_lowest_scores_and_keeps_order():
    o, k, v, g, r = _filled(5, 90)
    Hk = 2
    N = [o.global_len(0, 0, h) for h in range(Hk)]
    pos0 = [o.global_pos(0, 0, h).copy() for h in range(Hk)]
    pay0 = [[x.copy() for x in o.payload(0, 0, h)[:2]] for h in range(Hk)]
    used0 = 256 - o.free_top
    sc = r.random((Hk, max(N) + 3)).astype(np.float32)
    sc[0, 5] = sc[0, 9] = sc[0, 2] = 0.0          # ties at the bottom: the older one goes first
    gone = o.evict_apply(0, [0], sc, 0.1)
    for h in range(Hk):
        n_e = int(math.floor(np.float32(0.1).astype(np.float64) * N[h]))
        assert gone[h] == n_e > 0
        keep = np.sort(np.argsort(sc[h, :N[h]], kind="stable")[n_e:])           # library sort, stable = older first
        assert o.global_len(0, 0, h) == N[h] - n_e
        assert np.array_equal(o.global_pos(0, 0, h), pos0[h][keep])
        gk, gv = o.payload(0, 0, h)[:2]
        assert np.array_equal(gk, pay0[h][0][keep]) and np.array_equal(gv, pay0[h][1][keep])
    assert {2, 5}.isdisjoint(set(np.searchsorted(pos0[0], o.global_pos(0, 0, 0))))
    # pages: every page is either in a table or on the free stack, exactly once
    P = 4
    used1 = sum(-(-o.global_len(0, 0, h) // P) + 1 for h in range(Hk))             # global pages + one local page
    assert 256 - o.free_top == used1 <= used0
    seen = list(o.free_stack()[:o.free_top])
    for h in range(Hk):
        lp, gp, _, _ = o.head_tables(0, 0, h)
        n_gp = -(-o.global_len(0, 0, h) // P)
        assert np.all(gp[n_gp:] == -1)
        seen += list(lp) + list(gp[:n_gp])
    assert sorted(seen) == list(range(256))


def test_apply_page_release_order_and_reuse():
    # W = P = 2, one head: 9 admitted tokens then 2 more -> 9 global entries on pages taken in order
    o = Oracle(OracleConfig(1, 1, 1, 1, 2, 2, 1, 8, 10, False))
    o.push_tokens(0, [0], [11], None, None, np.ones((11, 1), np.float32), 0.5)
    lp, gp, _, _ = o.head_tables(0, 0, 0)
    assert o.global_len(0, 0, 0) == 9 and list(lp) == [0] and list(gp[:5]) == [1, 2, 3, 4, 5]
    sc = np.arange(9, dtype=np.float32)[None, :]
    gone = o.evict_apply(0, [0], sc, 0.6)                                       # floor(5.4) = 5 of 9 go
    assert gone[0] == 5 and list(o.global_pos(0, 0, 0)) == [5, 6, 7, 8]
    lp, gp, _, _ = o.head_tables(0, 0, 0)
    assert list(gp[:5]) == [1, 2, -1, -1, -1]
    # released in ascending table index: page 3, then 4, then 5 (on top of the stack)
    assert o.free_top == 7 and list(o.free_stack()[4:7]) == [3, 4, 5]
    # the next promotion that needs a page pops the top: page 5
    o.push_tokens(0, [0], [1], None, None, np.ones((1, 1), np.float32), 0.5)
    lp, gp, _, _ = o.head_tables(0, 0, 0)
    assert o.global_len(0, 0, 0) == 5 and list(gp[:4]) == [1, 2, 5, -1]
    assert list(o.global_pos(0, 0, 0)) == [5, 6, 7, 8, 9]


def test_apply_edge_fractions_and_score_order():
    o, *_ = _filled(8, 50)
    N = [o.global_len(0, 0, h) for h in range(2)]
    pos0 = o.global_pos(0, 0, 0).copy()
    sc = np.zeros((2, max(N)), np.float32)
    assert list(o.evict_apply(0, [0], sc, 0.0)) == [0, 0] and o.global_len(0, 0, 0) == N[0]
    assert list(o.evict_apply(0, [0], sc, 1.0 / (max(N) + 1))) == [0, 0]         # floor(frac N) = 0
    # all scores equal: the cut falls inside the tie and the oldest entries go
    gone = o.evict_apply(0, [0], sc, np.float32(2.5 / N[0]))
    assert gone[0] == 2 and np.array_equal(o.global_pos(0, 0, 0), pos0[2:])
    pos0, N[0] = pos0[2:], N[0] - 2
    # negative below zero below positive below NaN: the order of the bit patterns
    sc[0, :4] = [np.nan, -1.0, 3.0, 0.0]
    sc[0, 4:] = 7.0
    n_e = 3
    gone = o.evict_apply(0, [0], sc, np.float32((n_e + 0.5) / N[0]))
    assert gone[0] == n_e and list(o.global_pos(0, 0, 0)) == [pos0[0]] + list(pos0[4:])
    free_before = o.free_top
    gone = o.evict_apply(0, [0], sc, 1.0)
    assert o.global_len(0, 0, 0) == 0 == o.global_len(0, 0, 1)
    lp, gp, _, _ = o.head_tables(0, 0, 0)
    assert np.all(gp == -1) and o.free_top > free_before
    assert o.free_top == 256 - 2                                                 # only the two local pages are left


def test_attention_after_eviction_is_attention_over_what_is_left():
    o, k, v, g, r = _filled(13, 70, Hq=4, Hk=2, d=8, W=4)
    T, Hq, Hk, d, W = 70, 4, 2, 8, 4
    N = [o.global_len(0, 0, h) for h in range(Hk)]
    sc = r.random((Hk, max(N))).astype(np.float32)
    o.evict_apply(0, [0], sc, 0.3)
    q = r.standard_normal((Hq, d)).astype(np.float32)
    out = o.attend_cached(0, 0, q, 0.4)
    G = Hq // Hk
    for h in range(Hk):
        visible = np.zeros(T, dtype=bool)
        visible[o.global_pos(0, 0, h)] = True
        visible[T - W:] = True
        mask = torch.from_numpy(visible)[None, None, :]
        for gq in range(G):
            qq = torch.from_numpy(q[h * G + gq]).double()[None, None, :]
            ref = F.scaled_dot_product_attention(qq[None], torch.from_numpy(k[:, h]).double()[None, None],
                                                 torch.from_numpy(v[:, h]).double()[None, None],
                                                 attn_mask=mask[None], scale=0.4)[0, 0, 0].numpy()
            assert np.abs(out[h * G + gq] - ref).max() < 1e-13
