"""Read-time page selection with key landmarks (appendix "Synergy with KV Selection") on the GPU
against the oracle, through the C ABI: landmarks and their incremental upkeep, page criticality,
the pages picked, and decode attention over window + picked pages."""
import math

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
from harness import Pair, rand_tokens
from oracle import quest_select

pytestmark = pytest.mark.gpu
U_RTOL = 2e-5      # fp32 sum of head_dim products against fp64, relative to the largest |U|


def _landmarks_of(pair, lm, layer, s, h):
    """(lo, hi) rows per page of one head, read back from the landmark buffer: heads in (slot, layer, head) order,
    each with max_global_pages_per_head pages of two rows, in cache order."""
    c = pair.cfg
    es = 4 if c.dtype == wg.F32 else 2
    n = pair.orc.global_len(s, layer, h)
    n_pg = -(-n // c.page_size)
    um = (s * c.n_layers + layer) * c.n_kv_heads + h
    per_head = c.max_global_pages_per_head * 2 * c.head_dim * es
    rows = lm[um * per_head: um * per_head + n_pg * 2 * c.head_dim * es]
    rows = rows.view(torch.float32 if c.dtype == wg.F32 else torch.bfloat16)
    rows = rows.view(n_pg, 2, c.head_dim).float().cpu().numpy()
    return rows[:, 0], rows[:, 1]


def _check_scores(pair, lm, layer, seqs, q, budget):
    c = pair.cfg
    Hk, P = c.n_kv_heads, c.page_size
    n_pg = [-(-pair.orc.global_len(s, layer, h) // P) for s in seqs for h in range(Hk)]
    stride = max(n_pg) + 3
    scores, sel, cnt = pair.pool.quest_select(layer, seqs, q.to(pair.dev), lm, budget, stride)
    scores, sel, cnt = scores.cpu().numpy(), sel.cpu().numpy(), cnt.cpu().numpy()
    sel_ref = np.zeros_like(sel)
    for b, s in enumerate(seqs):
        for h in range(Hk):
            u = b * Hk + h
            ref = pair.orc.quest_page_scores(layer, s, h, q[b].float().numpy())
            gk = pair.orc.payload(s, layer, h)[0]
            lo, hi = _landmarks_of(pair, lm, layer, s, h)
            for p in range(n_pg[u]):                                  # landmarks: exact minimum / maximum rows
                page = gk[p * P:(p + 1) * P]
                assert np.array_equal(lo[p], page.min(axis=0)) and np.array_equal(hi[p], page.max(axis=0))
            if n_pg[u]:
                tol = U_RTOL * max(1.0, float(np.abs(ref).max()))
                assert np.abs(scores[u, :n_pg[u]] - ref).max() <= tol
            assert np.all(scores[u, n_pg[u]:] == 0)
            want = quest_select(ref.astype(np.float32), budget)
            # the seeded inputs must not put two distinct scores closer than the rounding error at the cut
            mine = np.sort(np.argsort(-scores[u, :n_pg[u]], kind="stable")[:min(budget, n_pg[u])])
            assert np.array_equal(mine, want), "near-tie at the cut: pick another seed"
            assert cnt[u] == len(want) and np.array_equal(sel[u, :cnt[u]], want)
            sel_ref[u, :len(want)] = want
    return sel_ref, cnt, n_pg


def _check_attend_selected(pair, layer, seqs, q, sel, cnt, scale):
    c = pair.cfg
    Hk = c.n_kv_heads
    out = torch.full((len(seqs), c.n_q_heads, c.head_dim), float("nan"), dtype=torch.float32, device=pair.dev)
    pair.pool.attend_selected(layer, seqs, q.to(pair.dev), torch.from_numpy(sel).to(pair.dev),
                              torch.from_numpy(cnt.astype(np.int32)).to(pair.dev), out, scale)
    out = out.cpu().numpy().astype(np.float64)
    ref = np.stack([pair.orc.attend_selected(s, layer, q[b].float().numpy(), sel[b * Hk:(b + 1) * Hk],
                                             cnt[b * Hk:(b + 1) * Hk], scale) for b, s in enumerate(seqs)])
    err = np.abs(out - ref)
    assert np.isfinite(out).all()
    if c.dtype == wg.F32:
        assert err.max() <= 2e-5, err.max()
    else:
        assert err.max() <= 1e-2 and err.mean() <= 1e-3, (err.max(), err.mean())
    return out


@pytest.mark.parametrize("dtype,Hq,Hk,d,P,W,T,budget", [
    (wg.F32, 8, 2, 64, 4, 8, 300, 9),
    (wg.BF16, 8, 2, 128, 16, 32, 900, 12),
    (wg.BF16, 32, 8, 128, 16, 256, 6000, 128),      # the paper's budget: 2048 KVs = 128 pages of 16
    (wg.BF16, 4, 4, 64, 32, 64, 700, 5),            # pages larger than a tile, group of one
    (wg.F32, 8, 1, 128, 2, 4, 150, 1000),           # budget larger than the cache: everything is read
    (wg.F32, 8, 2, 64, 1, 4, 3000, 40),             # thousands of pages per head, fp32 scoring kernel
    (wg.BF16, 8, 2, 128, 4, 16, 7000, 33),
    (wg.F32, 8, 2, 64, 1, 4, 6000, 40),             # more than 4096 pages in a head: a second stretch of the selection
    (wg.BF16, 4, 2, 64, 1, 4, 50000, 700),          # 90K pages in the call: several turns per scoring block, a head with
                                                    # more blocks than the plan can name, rows shorter than 16 lanes x 16 bytes
])
def test_quest_select_and_attend(dtype, Hq, Hk, d, P, W, T, budget):
    rng = np.random.default_rng(T + budget)
    B = 2
    max_gp = T // P + 8
    pair = Pair(1, Hq, Hk, d, dtype, P, W, B, max_gp, B * Hk * (max_gp + -(-W // P)) + 8, max_call_seqs=B,
                max_call_tokens=B * T)
    lens = [T, T // 2 + 3]
    k, v, g = rand_tokens(rng, sum(lens), Hk, d, pair.tdt, rates=list(np.linspace(0.8, 0.4, Hk)))
    pair.prefill(0, [0, 1], lens, k, v, g, 0.5)
    pair.pool.status()
    lm = pair.pool.quest_landmarks()
    pair.pool.quest_update(0, [0, 1], lm)
    scale = 1.0 / math.sqrt(d)
    q = torch.from_numpy(rng.standard_normal((B, Hq, d)).astype(np.float32)).to(pair.tdt)
    sel, cnt, n_pg = _check_scores(pair, lm, 0, [1, 0], q, budget)
    out_sel = _check_attend_selected(pair, 0, [1, 0], q, sel, cnt, scale)
    if budget >= max(n_pg):      # the whole cache is selected: the same as ordinary decode attention
        full, _ = pair.attend(0, [1, 0], q, scale)
        assert np.abs(out_sel - full).max() <= 1e-6
    # nothing selected: the window alone
    _check_attend_selected(pair, 0, [1, 0], q, sel, np.zeros_like(cnt), scale)
    # decode steps promote entries into the last pages: an incremental update keeps the landmarks current
    for step in range(P + 3):
        k1, v1, g1 = rand_tokens(rng, B, Hk, d, pair.tdt, rates=[0.9] * Hk)
        pair.decode(0, [0, 1], k1, v1, g1, 0.5)
        if step % 3 == 2:
            pair.pool.quest_update(0, [0, 1], lm)
    pair.pool.quest_update(0, [0, 1], lm)
    pair.pool.status()
    sel, cnt, _ = _check_scores(pair, lm, 0, [0, 1], q, budget)
    _check_attend_selected(pair, 0, [0, 1], q, sel, cnt, scale)
    # eviction moves entries between pages: a full recomputation is asked for
    N = max(pair.orc.global_len(s, 0, h) for s in (0, 1) for h in range(Hk))
    pair.evict(0, [0, 1], rng.random((B * Hk, N + 1)).astype(np.float32), 0.3)
    pair.pool.quest_update(0, [0, 1], lm, reset=True)
    sel, cnt, _ = _check_scores(pair, lm, 0, [0, 1], q, budget)
    _check_attend_selected(pair, 0, [0, 1], q, sel, cnt, scale)
    pair.check_state()


def test_quest_equal_pages_take_the_lower_index_first():
    """Keys that repeat with the page size give every page the same landmarks and so exactly the same
    score on either side: the tie rule alone decides, and it must pick the first pages."""
    rng = np.random.default_rng(7)
    Hq, Hk, d, P, W, T, budget = 8, 2, 128, 16, 16, 16 * 40 + 16, 6
    max_gp = T // P + 2
    pair = Pair(1, Hq, Hk, d, wg.BF16, P, W, 1, max_gp, Hk * (max_gp + 1) + 4, max_call_seqs=1, max_call_tokens=T)
    base = torch.from_numpy(rng.standard_normal((P, Hk, d)).astype(np.float32)).to(torch.bfloat16)
    k = base.repeat(T // P, 1, 1)
    v = torch.from_numpy(rng.standard_normal((T, Hk, d)).astype(np.float32)).to(torch.bfloat16)
    g = torch.ones((T, Hk), dtype=torch.float32)                      # everything is admitted: pages are whole periods
    pair.prefill(0, [0], [T], k, v, g, 0.5)
    pair.pool.status()
    lm = pair.pool.quest_landmarks()
    pair.pool.quest_update(0, [0], lm)
    q = torch.from_numpy(rng.standard_normal((1, Hq, d)).astype(np.float32)).to(torch.bfloat16)
    scores, sel, cnt = pair.pool.quest_select(0, [0], q.to(pair.dev), lm, budget, 64)
    scores, sel, cnt = scores.cpu().numpy(), sel.cpu().numpy(), cnt.cpu().numpy()
    for h in range(Hk):
        ref = pair.orc.quest_page_scores(0, 0, h, q[0].float().numpy())
        assert len(ref) == 40 and np.all(ref == ref[0]) and np.all(scores[h, :40] == scores[h, 0])
        assert cnt[h] == budget and list(sel[h, :budget]) == list(range(budget)) == list(quest_select(ref.astype(np.float32), budget))


def test_quest_rejects_bad_arguments():
    rng = np.random.default_rng(1)
    pair = Pair(1, 4, 2, 64, wg.F32, 4, 8, 2, 64, 400, max_call_seqs=2, max_call_tokens=256)
    k, v, g = rand_tokens(rng, 100, 2, 64, pair.tdt)
    pair.prefill(0, [0], [100], k, v, g, 0.3)
    pair.pool.status()
    lm = pair.pool.quest_landmarks()
    q = torch.zeros((1, 4, 64), dtype=torch.float32, device=pair.dev)
    with pytest.raises(wg.WgkvError):
        pair.pool.quest_update(0, [0], lm[:100])                       # buffer too small
    pair.pool.quest_update(0, [0], lm)
    with pytest.raises(wg.WgkvError):
        pair.pool.quest_select(0, [0], q, lm, 0, 64)                   # no budget
    with pytest.raises(wg.WgkvError):
        pair.pool.quest_select(0, [0], q, lm, 4, 2)                    # score rows shorter than the page count
    q_off = torch.zeros(4 * 64 + 1, dtype=torch.float32, device=pair.dev)[1:].view(1, 4, 64)
    with pytest.raises(wg.WgkvError):
        pair.pool.quest_select(0, [0], q_off, lm, 4, 64)               # queries not 16-byte aligned
    lm_off = torch.zeros(lm.numel() + 16, dtype=torch.uint8, device=pair.dev)[8:]
    with pytest.raises(wg.WgkvError):
        pair.pool.quest_update(0, [0], lm_off)                         # landmarks not 16-byte aligned
    with pytest.raises(wg.WgkvError):
        pair.pool.quest_select(0, [0], q, lm_off, 4, 64)
    # indices outside the table are clamped: garbage in, finite numbers out, nothing outside the pool is read
    sel = torch.tensor([[-5, 3, 10 ** 6], [0, 1, 2]], dtype=torch.int32, device=pair.dev)
    cnt = torch.tensor([3, 99], dtype=torch.int32, device=pair.dev)
    out = torch.zeros((1, 4, 64), dtype=torch.float32, device=pair.dev)
    pair.pool.attend_selected(0, [0], q, sel, cnt, out, 0.1)
    assert torch.isfinite(out).all()
    pair.check_state()


def test_quest_after_replayed_decode_steps_the_host_has_not_seen():
    """Decode steps replayed in a graph grow the caches without the host's bounds moving; scoring sizes its blocks
    from those bounds and must still reach the device's last page (more turns per block), and never write past
    the caller's score row."""
    rng = np.random.default_rng(29)
    Hq, Hk, d, P, W, B, T = 4, 2, 64, 1, 4, 2, 120
    max_gp = T + 400
    pair = Pair(1, Hq, Hk, d, wg.BF16, P, W, B, max_gp, B * Hk * (max_gp + W) + 8, max_call_seqs=B, max_call_tokens=B * T)
    dev, seqs = pair.dev, [0, 1]
    k, v, g = rand_tokens(rng, 2 * T, Hk, d, pair.tdt, rates=[0.7, 0.5])
    pair.prefill(0, seqs, [T, T], k, v, g, 0.5)
    k1, v1, g1 = rand_tokens(rng, B, Hk, d, pair.tdt, rates=[0.9] * Hk)
    pair.decode(0, seqs, k1, v1, g1, 0.5)                    # one eager step: everything is warm before the capture
    pair.pool.status()
    kb = torch.zeros((B, Hk, d), dtype=torch.bfloat16, device=dev)
    vb = torch.zeros_like(kb)
    gb = torch.zeros((B, Hk), dtype=torch.float32, device=dev)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            pair.pool.decode_step(0, seqs, kb, vb, gb, tau=0.5)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(300):                                      # ~270 more pages per head than the host counts
        k1, v1, g1 = rand_tokens(rng, B, Hk, d, pair.tdt, rates=[0.9] * Hk)
        kb.copy_(k1); vb.copy_(v1); gb.copy_(g1)
        graph.replay()
        torch.cuda.synchronize()
        pair.orc.push_tokens(0, seqs, [1] * B, k1.float().numpy(), v1.float().numpy(), g1.numpy(), 0.5)
    lm = pair.pool.quest_landmarks()
    pair.pool.quest_update(0, seqs, lm)
    q = torch.from_numpy(rng.standard_normal((B, Hq, d)).astype(np.float32)).to(pair.tdt)
    n_pg = [pair.orc.global_len(s, 0, h) for s in seqs for h in range(Hk)]      # P = 1: a page per entry
    assert min(n_pg) > 300
    stride = max(n_pg) + 3
    scores, sel, cnt = pair.pool.quest_select(0, seqs, q.to(dev), lm, 20, stride)
    scores, sel, cnt = scores.cpu().numpy(), sel.cpu().numpy(), cnt.cpu().numpy()
    for b, s in enumerate(seqs):
        for h in range(Hk):
            u = b * Hk + h
            ref = pair.orc.quest_page_scores(0, s, h, q[b].float().numpy())
            assert np.abs(scores[u, :n_pg[u]] - ref).max() <= U_RTOL * max(1.0, float(np.abs(ref).max()))
            assert np.all(scores[u, n_pg[u]:] == 0)
            assert cnt[u] == 20 and np.array_equal(sel[u, :20], quest_select(scores[u, :n_pg[u]], 20))
    # a score row shorter than the device's page count: filled to its end and no further, the selection stays inside it
    short = min(n_pg) - 50
    big = torch.full((B * Hk * short + 64,), 7.0, dtype=torch.float32, device=dev)    # 64 guard values behind the rows
    rows = big[:B * Hk * short].view(B * Hk, short)
    sc2, sel2, cnt2 = pair.pool.quest_select(0, seqs, q.to(dev), lm, 20, short, scores=rows)
    assert np.all(big[B * Hk * short:].cpu().numpy() == 7.0)
    assert np.array_equal(sc2.cpu().numpy(), scores[:, :short])       # no row ran over into the next one either
    assert int(sel2.max()) < short and np.all(cnt2.cpu().numpy() == 20)
    pair.check_state()
