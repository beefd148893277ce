"""Pins of the CPU oracle against things that are not the oracle: a library
attention routine under explicitly built masks, closed forms of the cache state,
hand-computable softmax cases and brute force over all admission patterns."""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import Oracle, OracleConfig, attend_definition, attend_soft, linear_gate


def _rand(seed, n, Hq, Hk, d):
    r = np.random.default_rng(seed)
    K = r.standard_normal((n, Hk, d)).astype(np.float32)
    V = r.standard_normal((n, Hk, d)).astype(np.float32)
    Q = r.standard_normal((n, Hq, d)).astype(np.float32)
    g = r.random((n, Hk)).astype(np.float32)
    return K, V, Q, g


def _sdpa(K, V, Q, mask=None, causal=False):
    """Library attention in fp64: heads first, kv heads repeated for the group."""
    n, Hk, d = K.shape
    Hq = Q.shape[1]
    G = Hq // Hk
    k = torch.from_numpy(K).double().permute(1, 0, 2).repeat_interleave(G, dim=0)
    v = torch.from_numpy(V).double().permute(1, 0, 2).repeat_interleave(G, dim=0)
    q = torch.from_numpy(Q).double().permute(1, 0, 2)
    if mask is not None:
        mask = torch.from_numpy(mask).repeat_interleave(G, dim=0)
    o = F.scaled_dot_product_attention(q[None], k[None], v[None], attn_mask=None if mask is None else mask[None],
                                       is_causal=causal)
    return o[0].permute(1, 0, 2).numpy()


def test_tau_admits_all_is_dense_causal_attention():
    # Sec. 2.1 equation: with every token admitted the mask is plain causal
    n, Hq, Hk, d, W = 97, 4, 2, 16, 8
    K, V, Q, g = _rand(1, n, Hq, Hk, d)
    out = attend_definition(K, V, g, Q, np.arange(n), W, tau=0.0, scale=1 / math.sqrt(d))
    ref = _sdpa(K, V, Q, causal=True)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    out2 = attend_definition(K, V, g, Q, np.arange(n), W, tau=-1.0, scale=1 / math.sqrt(d))
    np.testing.assert_allclose(out2, ref, rtol=0, atol=1e-12)


def test_tau_admits_none_is_sliding_window():
    n, Hq, Hk, d, W = 80, 4, 2, 8, 5
    K, V, Q, g = _rand(2, n, Hq, Hk, d)
    i = np.arange(n)[:, None]
    j = np.arange(n)[None, :]
    band = (j <= i) & (i - j < W)
    mask = np.broadcast_to(band, (Hk, n, n)).copy()
    out = attend_definition(K, V, g, Q, np.arange(n), W, tau=2.0, scale=1 / math.sqrt(d))
    np.testing.assert_allclose(out, _sdpa(K, V, Q, mask=mask), rtol=0, atol=1e-12)
    # tau = 1 still admits a score of exactly 1
    g1 = g.copy()
    g1[3, 0] = 1.0
    mask1 = mask.copy()
    mask1[0, 3:, 3] = True
    out1 = attend_definition(K, V, g1, Q, np.arange(n), W, tau=1.0, scale=1 / math.sqrt(d))
    ref1 = _sdpa(K, V, Q, mask=mask1)
    np.testing.assert_allclose(out1, ref1, rtol=0, atol=1e-12)


@pytest.mark.parametrize("W", [1, 3, 16])
def test_general_tau_matches_explicit_vertical_slash_mask(W):
    # Sec. 4.2 mask equation, built by broadcasting
    n, Hq, Hk, d, tau = 70, 6, 3, 8, 0.6
    K, V, Q, g = _rand(3 + W, n, Hq, Hk, d)
    i = np.arange(n)[None, :, None]
    j = np.arange(n)[None, None, :]
    M = ((i - j < W) | (g.T[:, None, :] >= np.float32(tau))) & (i >= j)
    out = attend_definition(K, V, g, Q, np.arange(n), W, tau=tau, scale=1 / math.sqrt(d))
    np.testing.assert_allclose(out, _sdpa(K, V, Q, mask=M), rtol=0, atol=1e-12)


def test_gqa_group_reads_kv_head_hq_div_G():
    # distinct V per kv head, q = 0 so the output is the mean of the visible V rows
    n, Hq, Hk, d = 6, 4, 2, 3
    K = np.zeros((n, Hk, d), np.float32)
    V = np.zeros((n, Hk, d), np.float32)
    V[:, 0, :] = 1.0
    V[:, 1, :] = 5.0
    Q = np.zeros((1, Hq, d), np.float32)
    g = np.ones((n, Hk), np.float32)
    out = attend_definition(K, V, g, Q, np.array([n - 1]), 2, 0.5, 1.0)
    np.testing.assert_allclose(out[0, :, 0], [1, 1, 5, 5])


def test_hand_computed_softmax_weights():
    # two visible keys with scores ln 3 and 0: weights 3/4 and 1/4
    d = 2
    K = np.array([[[math.log(3.0), 0.0]], [[0.0, 0.0]]], np.float32)
    V = np.array([[[8.0, 0.0]], [[0.0, 4.0]]], np.float32)
    Q = np.array([[[1.0, 0.0]]], np.float32)
    g = np.zeros((2, 1), np.float32)
    out = attend_definition(K, V, g, Q, np.array([1]), 2, 0.5, 1.0)
    w0 = math.exp(float(np.float32(math.log(3.0))))
    np.testing.assert_allclose(out[0, 0], [8 * w0 / (w0 + 1), 4 / (w0 + 1)], rtol=1e-14)
    # the older key drops out when the window is 1 and it is not admitted ...
    out = attend_definition(K, V, g, Q, np.array([1]), 1, 0.5, 1.0)
    np.testing.assert_allclose(out[0, 0], [0.0, 4.0], rtol=1e-14)
    # ... and comes back when its score reaches tau exactly (>=)
    g[0, 0] = 0.5
    out = attend_definition(K, V, g, Q, np.array([1]), 1, 0.5, 1.0)
    np.testing.assert_allclose(out[0, 0], [8 * w0 / (w0 + 1), 4 / (w0 + 1)], rtol=1e-14)
    # scale multiplies the logits
    out = attend_definition(K, V, g, Q, np.array([1]), 1, 0.5, 2.0)
    w2 = math.exp(2 * float(np.float32(math.log(3.0))))
    np.testing.assert_allclose(out[0, 0], [8 * w2 / (w2 + 1), 4 / (w2 + 1)], rtol=1e-14)


def test_nan_score_never_admits():
    n, Hq, Hk, d, W = 12, 2, 1, 4, 2
    K, V, Q, g = _rand(5, n, Hq, Hk, d)
    g[:] = np.nan
    a = attend_definition(K, V, g, Q, np.arange(n), W, tau=0.5, scale=0.5)
    g[:] = 0.0
    b = attend_definition(K, V, g, Q, np.arange(n), W, tau=0.5, scale=0.5)
    np.testing.assert_array_equal(a, b)


def test_soft_mask_with_binary_scores_is_the_hard_mask():
    # Sec. 3.2: multiplicative mask m_ij = max(1(i-j<W), g_j), and its log-space form
    n, Hq, Hk, d, W = 50, 4, 2, 8, 4
    K, V, Q, g = _rand(6, n, Hq, Hk, d)
    gb = (g > 0.7).astype(np.float32)
    hard = attend_definition(K, V, gb, Q, np.arange(n), W, tau=0.5, scale=1 / math.sqrt(d))
    soft = attend_soft(K, V, gb, Q, np.arange(n), W, 1 / math.sqrt(d))
    np.testing.assert_allclose(soft, hard, rtol=0, atol=1e-13)
    softlog = attend_soft(K, V, gb, Q, np.arange(n), W, 1 / math.sqrt(d), use_log=True, eps=1e-30)
    np.testing.assert_allclose(softlog, hard, rtol=0, atol=1e-12)
    # g = 1 everywhere: soft form is dense causal attention
    ones = np.ones_like(g)
    np.testing.assert_allclose(attend_soft(K, V, ones, Q, np.arange(n), W, 1 / math.sqrt(d)),
                               _sdpa(K, V, Q, causal=True), rtol=0, atol=1e-12)


# ---------------- mechanism: closed forms of the state ----------------

def _mk(Hq=4, Hk=2, d=8, P=4, W=8, n_pages=400, max_gp=64, L=1, S=1, payload=True):
    return Oracle(OracleConfig(L, Hq, Hk, d, P, W, S, max_gp, n_pages, payload))


def _check_state_closed_form(o, seq, layer, g_hist, tau):
    cfg = o.cfg
    t = g_hist.shape[0]
    W, P = cfg.w_local, cfg.page_size
    assert o.seq_len(seq, layer) == t
    pages = []
    for h in range(cfg.n_kv_heads):
        lp, gp, rg, rp = o.head_tables(seq, layer, h)
        # ring = positions [max(0,t-W), t), position p in slot p mod W, score stored
        exp_pos = np.full(W, -1, np.int64)
        for p in range(max(0, t - W), t):
            exp_pos[p % W] = p
        np.testing.assert_array_equal(rp, exp_pos)
        for s in range(W):
            if exp_pos[s] >= 0:
                assert rg[s] == g_hist[exp_pos[s], h]
        # global = { j < t-W : g_j >= tau } in ascending order (Sec. 4.2 population rule)
        left = np.arange(max(0, t - W))
        exp_glob = left[g_hist[: max(0, t - W), h] >= np.float32(tau)]
        np.testing.assert_array_equal(o.global_pos(seq, layer, h), exp_glob)
        G = o.global_len(seq, layer, h)
        assert G == len(exp_glob)
        ngp = -(-G // P)
        assert (gp[:ngp] >= 0).all() and (gp[ngp:] == -1).all()
        if t > 0:
            pages += list(lp) + list(gp[:ngp])
    return pages


@pytest.mark.parametrize("chunks", [[1] * 40, [40], [3, 17, 1, 19], [8, 8, 8, 8, 8], [39, 1]])
def test_state_closed_form_and_chunking_invariance(chunks):
    Hk, d, W, P, tau = 2, 8, 8, 4, 0.45
    r = np.random.default_rng(7)
    n = sum(chunks)
    K = r.standard_normal((n, Hk, d)).astype(np.float32)
    V = r.standard_normal((n, Hk, d)).astype(np.float32)
    g = r.random((n, Hk)).astype(np.float32)
    o = _mk(Hk=Hk, d=d, W=W, P=P)
    base = 0
    for c in chunks:
        admit, prom = o.push_tokens(0, [0], [c], K[base:base + c], V[base:base + c], g[base:base + c], tau)
        np.testing.assert_array_equal(admit, (g[base:base + c] >= np.float32(tau)).astype(np.uint8))
        # promotion at the push of position p  <=>  p >= W and g[p-W] >= tau  (Sec. 4.3)
        exp_prom = np.zeros((c, Hk), np.uint8)
        for i in range(c):
            p = base + i
            if p >= W:
                exp_prom[i] = g[p - W] >= np.float32(tau)
        np.testing.assert_array_equal(prom, exp_prom)
        base += c
        pages = _check_state_closed_form(o, 0, 0, g[:base], tau)
        assert len(set(pages)) == len(pages)                      # page tables injective
        assert len(pages) + o.free_top == o.cfg.n_pages           # used + free = total
        fs = o.free_stack()[: o.free_top]
        assert not (set(fs.tolist()) & set(pages))
    # content is what the positions say, whatever the chunking
    for h in range(Hk):
        gk, gv, rk, rv = o.payload(0, 0, h)
        pos = o.global_pos(0, 0, h)
        np.testing.assert_array_equal(gk, K[pos, h])
        np.testing.assert_array_equal(gv, V[pos, h])
        _, _, _, rp = o.head_tables(0, 0, h)
        np.testing.assert_array_equal(rk, K[rp, h])
        np.testing.assert_array_equal(rv, V[rp, h])


@pytest.mark.parametrize("W,P", [(1, 1), (4, 4), (8, 2), (16, 16), (6, 4)])
def test_mechanism_attention_equals_definition(W, P):
    Hq, Hk, d, tau, n = 4, 2, 8, 0.5, 60
    K, V, Q, g = _rand(11 + W, n, Hq, Hk, d)
    o = _mk(Hq, Hk, d, P, W)
    scale = 1 / math.sqrt(d)
    ref = attend_definition(K, V, g, Q, np.arange(n), W, tau, scale)
    for p in range(n):
        o.push_tokens(0, [0], [1], K[p:p + 1], V[p:p + 1], g[p:p + 1], tau)
        out = o.attend_cached(0, 0, Q[p], scale)
        np.testing.assert_allclose(out, ref[p], rtol=0, atol=1e-12)
    out_b, _ = o.attend_cached_batch(0, [0], Q[n - 1][None], scale)
    np.testing.assert_array_equal(out_b[0], o.attend_cached(0, 0, Q[n - 1], scale))


def test_batched_decode_attention_on_permuted_sequences_and_layers():
    """orc_attend_cached_batch against library attention under the Sec. 4.2 mask, built from each
    (sequence, layer)'s own history: four sequences of different lengths, two layers with different
    contents, the calls naming the sequences out of order and only some of them.  Reading the wrong
    sequence, the wrong layer, or the batch slot instead of the sequence id fails it."""
    Hq, Hk, d, W, P, tau = 6, 3, 8, 4, 2, 0.55
    S, L = 4, 2
    o = _mk(Hq, Hk, d, P, W, n_pages=600, max_gp=64, L=L, S=S)
    scale = 1 / math.sqrt(d)
    lens = {(s, l): 9 + 7 * s + 5 * l for s in range(S) for l in range(L)}
    hist = {}
    for (s, l), n in lens.items():
        K, V, Q, g = _rand(100 + 10 * s + l, n, Hq, Hk, d)
        hist[(s, l)] = (K, V, Q, g)
        o.push_tokens(l, [s], [n], K, V, g, tau)

    def expected(s, l):
        K, V, Q, g = hist[(s, l)]
        n = K.shape[0]
        j = np.arange(n)
        vis = ((n - 1 - j < W)[None, :] | (g.T >= np.float32(tau)))  # [Hk, n]: what the last position sees
        return _sdpa(K, V, Q[n - 1:n], mask=vis[:, None, :])[0]

    for layer, ids in [(1, [3, 0, 2]), (0, [1, 3, 2, 0]), (1, [1]), (0, [2, 2])]:
        q = np.stack([hist[(s, layer)][2][-1] for s in ids])
        out, threads = o.attend_cached_batch(layer, ids, q, scale)
        assert threads >= 1
        for b, s in enumerate(ids):
            np.testing.assert_allclose(out[b], expected(s, layer), rtol=0, atol=1e-12)
            np.testing.assert_array_equal(out[b], o.attend_cached(s, layer, q[b], scale))


@pytest.mark.parametrize("W,P", [(1, 1), (2, 1), (2, 2), (4, 2), (4, 1)])
def test_brute_force_all_admission_patterns(W, P):
    # every one of the 2^N admit patterns of one head, N <= 10
    N, d = 9, 2
    r = np.random.default_rng(3)
    K = r.standard_normal((N, 1, d)).astype(np.float32)
    V = r.standard_normal((N, 1, d)).astype(np.float32)
    Q = r.standard_normal((N, 1, d)).astype(np.float32)
    for bits in itertools.product([0, 1], repeat=N):
        g = np.array(bits, np.float32)[:, None] * 0.8 + 0.1  # 0.1 or 0.9
        o = _mk(1, 1, d, P, W, n_pages=40, max_gp=16)
        for p in range(N):
            o.push_tokens(0, [0], [1], K[p:p + 1], V[p:p + 1], g[p:p + 1], 0.5)
            # visible set by brute force
            vis = [j for j in range(p + 1) if (p - j < W) or bits[j]]
            s = np.array([float(np.dot(Q[p, 0].astype(np.float64), K[j, 0].astype(np.float64))) for j in vis])
            w = np.exp(s - s.max())
            w /= w.sum()
            exp_out = (w[:, None] * V[vis, 0].astype(np.float64)).sum(0)
            np.testing.assert_allclose(o.attend_cached(0, 0, Q[p], 1.0)[0], exp_out, rtol=0, atol=1e-13)
            cached = sorted(o.global_pos(0, 0, 0).tolist() + [x for x in o.head_tables(0, 0, 0)[3] if x >= 0])
            assert cached == vis                                  # each token in exactly one place
            G = o.global_len(0, 0, 0)
            assert G == sum(bits[: max(0, p + 1 - W)])
            assert o.free_top == 40 - (-(-W // P)) - (-(-G // P))


def test_page_allocation_rule_small_worked_example():
    # project rule (paper silent): LIFO stack handing out 0,1,2,...; units in
    # (sequence position in call, kv head) order; local pages before global pages.
    # W=4, P=2: two local pages per head.  Two heads, one sequence.
    o = _mk(2, 2, 2, P=2, W=4, n_pages=32, max_gp=8, payload=False)
    g = np.zeros((10, 2), np.float32)
    g[[0, 1, 2, 5], 0] = 1.0          # head 0 admits 0,1,2,5
    g[[3], 1] = 1.0                   # head 1 admits 3
    o.push_tokens(0, [0], [10], None, None, g, 0.5)
    # positions leaving the window: 0..5.  head 0: global = [0,1,2,5] -> 2 pages; head 1: [3] -> 1 page
    lp0, gp0, _, _ = o.head_tables(0, 0, 0)
    lp1, gp1, _, _ = o.head_tables(0, 0, 1)
    assert lp0.tolist() == [0, 1] and gp0[:2].tolist() == [2, 3]
    assert lp1.tolist() == [4, 5] and gp1[:1].tolist() == [6]
    assert o.free_top == 32 - 7 and o.free_stack()[o.free_top - 1] == 7
    # a decode step that promotes position 6 on head 1 only (g=1 there): no new page (G=1 -> 2 fits)
    g2 = np.zeros((12, 2), np.float32)
    o2 = _mk(2, 2, 2, P=2, W=4, n_pages=32, max_gp=8, payload=False)
    g2[:10] = g
    g2[6, 1] = 1.0
    o2.push_tokens(0, [0], [10], None, None, g2[:10], 0.5)
    _, prom = o2.push_tokens(0, [0], [1], None, None, g2[10:11], 0.5)
    assert prom.tolist() == [[0, 1]] and o2.global_len(0, 0, 1) == 2 and o2.free_top == 32 - 7
    # freeing gives the pages back: layer asc, head asc, local then global
    o.free_seq(0)
    assert o.free_top == 32
    assert o.free_stack()[25:32].tolist() == [0, 1, 2, 3, 4, 5, 6]
    assert o.seq_len(0, 0) == 0 and o.global_len(0, 0, 0) == 0


def test_multi_sequence_multi_layer_share_one_pool():
    Hk, d, W, P, tau = 2, 4, 4, 2, 0.5
    o = _mk(2, Hk, d, P, W, n_pages=200, max_gp=32, L=2, S=3)
    r = np.random.default_rng(5)
    hist = {}
    for layer, seqs, lens in [(0, [2, 0], [7, 11]), (1, [0, 1, 2], [5, 1, 9]), (0, [0, 1, 2], [1, 1, 1]),
                              (1, [2], [13])]:
        tot = sum(lens)
        K = r.standard_normal((tot, Hk, d)).astype(np.float32)
        V = r.standard_normal((tot, Hk, d)).astype(np.float32)
        g = r.random((tot, Hk)).astype(np.float32)
        o.push_tokens(layer, seqs, lens, K, V, g, tau)
        b = 0
        for s, n in zip(seqs, lens):
            hist[(s, layer)] = np.concatenate([hist.get((s, layer), np.zeros((0, Hk), np.float32)), g[b:b + n]])
            b += n
        pages = []
        for (s, l), gh in hist.items():
            pages += _check_state_closed_form(o, s, l, gh, tau)
        assert len(set(pages)) == len(pages)
        assert len(pages) + o.free_top == 200


def test_out_of_pages_and_table_overflow_are_reported():
    from oracle.wgkv_oracle import OracleError
    o = _mk(1, 1, 2, P=2, W=2, n_pages=2, max_gp=8, payload=False)
    g = np.ones((8, 1), np.float32)
    with pytest.raises(OracleError) as e:
        o.push_tokens(0, [0], [8], None, None, g, 0.5)
    assert e.value.code == -2
    o = _mk(1, 1, 2, P=2, W=2, n_pages=20, max_gp=1, payload=False)
    with pytest.raises(OracleError) as e:
        o.push_tokens(0, [0], [8], None, None, g, 0.5)
    assert e.value.code == -3


def test_linear_gate_against_library_matmul():
    r = np.random.default_rng(9)
    x = r.standard_normal((33, 64)).astype(np.float32)
    w = (0.02 * r.standard_normal((3, 64))).astype(np.float32)
    logit, g = linear_gate(x, w)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    np.testing.assert_allclose(logit, ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(g, torch.sigmoid(torch.from_numpy(ref)).numpy(), rtol=0, atol=1e-15)
    # sigma(0) = 1/2: a zero weight vector sits exactly on tau = 0.5
    _, g0 = linear_gate(x, np.zeros_like(w))
    assert (g0 == 0.5).all()


def test_tie_at_threshold_admits_in_the_mechanism_too():
    # 1(g >= tau): a stored score equal to tau is promoted (Sec. 3.3 last sentence; Sec. 4.3 step (1))
    Hk, d, W, P, tau, n = 2, 4, 4, 2, 0.5, 30
    r = np.random.default_rng(21)
    K = r.standard_normal((n, Hk, d)).astype(np.float32)
    V = r.standard_normal((n, Hk, d)).astype(np.float32)
    Q = r.standard_normal((n, 2 * Hk, d)).astype(np.float32)
    g = r.choice(np.array([0.25, 0.5, 0.75], np.float32), size=(n, Hk))
    assert (g == 0.5).sum() > 5
    o = _mk(2 * Hk, Hk, d, P, W)
    _, prom = o.push_tokens(0, [0], [n], K, V, g, tau)
    _check_state_closed_form(o, 0, 0, g, tau)
    np.testing.assert_array_equal(prom[W:], (g[:-W] >= 0.5).astype(np.uint8))
    ref = attend_definition(K, V, g, Q[-1:], np.array([n - 1]), W, tau, 0.5)
    np.testing.assert_allclose(o.attend_cached(0, 0, Q[-1], 0.5), ref[0], rtol=0, atol=1e-12)
