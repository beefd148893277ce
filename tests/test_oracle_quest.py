"""Pins of the oracle's read-time page selection (appendix "Synergy with KV Selection"; the
published Quest procedure with per-page minimum / maximum key landmarks): the page score is an
upper bound of every dot product in the page and exact in constructed cases, the selection
against a library sort, attention over a selection against library attention under an
explicit mask, and the full budget against ordinary attention over the cache."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import Oracle, OracleConfig, quest_select


def _filled(seed, T, Hq=4, Hk=2, d=8, P=4, W=4, tau=0.4):
    o = Oracle(OracleConfig(1, Hq, Hk, d, P, W, 1, 64, 256, True))
    r = np.random.default_rng(seed)
    k = r.standard_normal((T, Hk, d)).astype(np.float32)
    v = r.standard_normal((T, Hk, d)).astype(np.float32)
    g = r.random((T, Hk)).astype(np.float32)
    o.push_tokens(0, [0], [T], k, v, g, tau)
    return o, k, v, g, r


def test_page_score_is_an_upper_bound_and_matches_numpy_landmarks():
    partly_filled = 0
    for seed, (Hq, Hk, P) in enumerate([(4, 2, 4), (2, 2, 8), (8, 2, 2), (4, 1, 16)]):
        o, *_, r = _filled(seed, 90, Hq=Hq, Hk=Hk, P=P)
        G = Hq // Hk
        q = r.standard_normal((Hq, 8)).astype(np.float32)
        for h in range(Hk):
            gk = o.payload(0, 0, h)[0].astype(np.float64)
            n = len(gk)
            u = o.quest_page_scores(0, 0, h, q)
            assert len(u) == -(-n // P)
            partly_filled += n % P != 0
            for p in range(len(u)):
                page = gk[p * P:(p + 1) * P]
                lo, hi = page.min(axis=0), page.max(axis=0)      # library min / max as the landmarks
                per_head = [np.maximum(q[h * G + g].astype(np.float64) * lo, q[h * G + g].astype(np.float64) * hi).sum()
                            for g in range(G)]
                assert abs(u[p] - max(per_head)) < 1e-12
                dots = page @ q[h * G:(h + 1) * G].astype(np.float64).T
                assert u[p] >= dots.max() - 1e-12
    assert partly_filled >= 3       # the case of a last page that is not full was really exercised


def test_page_score_exact_cases():
    # a page that holds one key: the bound is the dot product itself; keys that are multiples of
    # one vector c*w with q = w: the bound is max(c) |w|^2
    W, P, d = 2, 2, 4
    o = Oracle(OracleConfig(1, 1, 1, d, P, W, 1, 8, 16, True))
    w = np.array([1.0, -2.0, 0.5, 3.0], np.float32)
    c = np.array([0.5, -1.0, 2.0, 0.25, 1.5], np.float32)           # five admitted keys: pages (0.5,-1), (2,0.25), (1.5)
    k = np.concatenate([c[:, None] * w[None, :], np.zeros((W, d), np.float32)])[:, None, :]
    o.push_tokens(0, [0], [len(k)], k, k, np.ones((len(k), 1), np.float32), 0.5)
    assert o.global_len(0, 0, 0) == 5
    u = o.quest_page_scores(0, 0, 0, w[None, :])
    ww = float(np.dot(w.astype(np.float64), w.astype(np.float64)))
    assert np.allclose(u, [0.5 * ww, 2.0 * ww, 1.5 * ww], atol=1e-12)
    u_neg = o.quest_page_scores(0, 0, 0, -w[None, :])               # q = -w: the bound takes the other landmark
    assert np.allclose(u_neg, [1.0 * ww, -0.25 * ww, -1.5 * ww], atol=1e-12)


def test_select_is_the_top_of_a_stable_sort():
    r = np.random.default_rng(4)
    for n, b in [(50, 7), (7, 50), (33, 33), (20, 0), (0, 5)]:
        s = (r.integers(0, 6, n) / 4.0 - 0.5).astype(np.float32)       # many ties, both signs
        sel = quest_select(s, b)
        want = np.sort(np.argsort(-s, kind="stable")[:min(n, b)])     # largest first, lower index first among equals
        assert np.array_equal(sel, want)
    s = np.array([1.0, np.inf, -0.0, 0.0, np.nan, -np.inf], np.float32)
    assert list(quest_select(s, 3)) == [0, 1, 4]                     # NaN (sign clear) above +inf above 1
    assert list(quest_select(s, 5)) == [0, 1, 2, 3, 4]
    assert list(quest_select(s[2:4], 1)) == [1]                      # +0 above -0 in the order of the bit patterns


def test_attention_over_a_selection_is_masked_library_attention():
    o, k, v, g, r = _filled(9, 120, Hq=4, Hk=2, d=8, P=4, W=4)
    T, Hq, Hk, d, P, W = 120, 4, 2, 8, 4, 4
    q = r.standard_normal((Hq, d)).astype(np.float32)
    n_pages = [-(-o.global_len(0, 0, h) // P) for h in range(Hk)]
    budget = 5
    sel = np.zeros((Hk, budget), np.int32)
    n_sel = np.zeros(Hk, np.int32)
    for h in range(Hk):
        s = quest_select(o.quest_page_scores(0, 0, h, q).astype(np.float32), budget)
        if h == 1:
            s = np.array(sorted(set(s[:-1]) | {n_pages[h] - 1}), np.int32)   # make sure the partly filled page is in
        sel[h, :len(s)] = s
        n_sel[h] = len(s)
    out = o.attend_selected(0, 0, q, sel, n_sel, 0.4)
    G = Hq // Hk
    for h in range(Hk):
        pos = o.global_pos(0, 0, h)
        visible = np.zeros(T, dtype=bool)
        for p in sel[h, :n_sel[h]]:
            visible[pos[p * P:(p + 1) * P]] = True
        visible[T - W:] = True
        mask = torch.from_numpy(visible)[None, None, None, :]
        for gq in range(G):
            qq = torch.from_numpy(q[h * G + gq]).double()[None, None, None, :]
            ref = F.scaled_dot_product_attention(qq, torch.from_numpy(k[:, h]).double()[None, None],
                                                 torch.from_numpy(v[:, h]).double()[None, None], attn_mask=mask,
                                                 scale=0.4)[0, 0, 0].numpy()
            assert np.abs(out[h * G + gq] - ref).max() < 1e-13
    # the whole cache selected: ordinary attention over the cache
    sel_all = np.zeros((Hk, max(n_pages)), np.int32)
    for h in range(Hk):
        sel_all[h, :n_pages[h]] = np.arange(n_pages[h])
    assert np.array_equal(o.attend_selected(0, 0, q, sel_all, n_pages, 0.4), o.attend_cached(0, 0, q, 0.4))
    # nothing selected: the window alone
    out0 = o.attend_selected(0, 0, q, sel, np.zeros(Hk, np.int32), 0.4)
    for h in range(Hk):
        mask = torch.zeros(T, dtype=torch.bool)
        mask[T - W:] = True
        qq = torch.from_numpy(q[h * G]).double()[None, None, None, :]
        ref = F.scaled_dot_product_attention(qq, torch.from_numpy(k[:, h]).double()[None, None],
                                             torch.from_numpy(v[:, h]).double()[None, None],
                                             attn_mask=mask[None, None, None, :], scale=0.4)[0, 0, 0].numpy()
        assert np.abs(out0[h * G] - ref).max() < 1e-13
