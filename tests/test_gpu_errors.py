"""Refusals of the boundary, forced from the host (every kernel that runs exits normally): a pool
a few pages short, a page-table row too narrow, a workspace one byte short, a replayed graph that
runs out of pages (the device-side sticky flag), a recycled page that holds non-finite rows, and
argument limits of the gate form of wgkv_prefill_admit, and the caller's bound on admitted tokens
(wgkv_prefill_admit_bounded) held and broken.  A refused call must leave the cache state
untouched: the metadata block is compared byte for byte."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
from paper_2512_17452_amd.binding import _ids, _ptr, _stream
from harness import MAX_ABS_TOL, MEAN_ABS_TOL, Pair, rand_q, rand_tokens

pytestmark = pytest.mark.gpu

OUT_OF_PAGES, PT_OVERFLOW, DEVICE_FLAG, WORKSPACE, INVALID, ADMIT_BOUND = -2, -3, -5, -6, -1, -8


def _meta_bytes(pool):
    torch.cuda.synchronize()
    return pool.meta_buf.cpu().numpy().copy()


def _refused(fn, code, pool):
    before = _meta_bytes(pool)
    with pytest.raises(wg.WgkvError) as e:
        fn()
    assert e.value.code == code, e.value
    np.testing.assert_array_equal(_meta_bytes(pool), before)


def test_pool_short_of_pages_refuses_prefill_and_decode():
    Hk, d, P, W = 2, 64, 4, 16
    nlp = W // P
    # 36 tokens, all admitted: 20 leave the window = 5 global pages per head; with the 4 ring pages: 18 pages
    pr = Pair(1, 4, Hk, d, wg.BF16, P, W, 2, 32, 18, max_call_seqs=2, max_call_tokens=256)
    dev = pr.dev
    rng = np.random.default_rng(31)
    k, v, g = rand_tokens(rng, 40, Hk, d, torch.bfloat16)
    g[:] = 0.9
    # (1) a prefill that would need 6 global pages per head does not fit
    _refused(lambda: pr.pool.prefill_admit(0, [0], [40], k.to(dev), v.to(dev), g.to(dev), tau=0.5), OUT_OF_PAGES, pr.pool)
    # (2) 36 tokens fit exactly; the state is the oracle's
    pr.prefill(0, [0], [36], k[:36], v[:36], g[:36], 0.5)
    pr.check_state()
    assert pr.orc.free_top == 0 and pr.orc.global_len(0, 0, 0) == 20
    # (3) the next token promotes into a sixth page per head: refused, nothing moves
    _refused(lambda: pr.pool.decode_step(0, [0], k[36:37].to(dev), v[36:37].to(dev), g[36:37].to(dev), tau=0.5),
             OUT_OF_PAGES, pr.pool)
    # (4) so is the first token of another sequence (it needs its ring pages)
    _refused(lambda: pr.pool.decode_step(0, [1], k[36:37].to(dev), v[36:37].to(dev), g[36:37].to(dev), tau=0.5),
             OUT_OF_PAGES, pr.pool)
    pr.check_state()
    pr.check_attend(0, [0], rand_q(rng, 1, 4, d, torch.bfloat16))
    assert nlp == 4


def test_page_table_row_too_narrow():
    Hk, d, P, W = 2, 64, 4, 8
    pr = Pair(1, 4, Hk, d, wg.BF16, P, W, 1, 3, 64, max_call_seqs=1, max_call_tokens=256)   # 3 global pages per head
    dev = pr.dev
    rng = np.random.default_rng(32)
    k, v, g = rand_tokens(rng, 40, Hk, d, torch.bfloat16)
    g[:] = 0.9
    _refused(lambda: pr.pool.prefill_admit(0, [0], [W + 13], k.to(dev), v.to(dev), g.to(dev), tau=0.5), PT_OVERFLOW, pr.pool)
    pr.prefill(0, [0], [W + 12], k[:W + 12], v[:W + 12], g[:W + 12], 0.5)   # exactly three full pages
    pr.check_state()
    _refused(lambda: pr.pool.decode_step(0, [0], k[:1].to(dev), v[:1].to(dev), g[:1].to(dev), tau=0.5), PT_OVERFLOW, pr.pool)
    pr.check_state()


def _smallest_accepted(call, lo, hi):
    """Smallest workspace size in (lo, hi] that `call(size)` accepts (rc 0); rc -6 below it."""
    assert call(hi) == 0
    while hi - lo > 1:
        mid = (lo + hi) // 2
        rc = call(mid)
        assert rc in (0, WORKSPACE), rc
        if rc == 0:
            hi = mid
        else:
            lo = mid
    return hi


def test_workspace_one_byte_short():
    Hq, Hk, d, P, W, T = 8, 2, 128, 16, 32, 200
    pr = Pair(1, Hq, Hk, d, wg.BF16, P, W, 2, 32, 256, max_call_seqs=2, max_call_tokens=512)
    pool, dev, L = pr.pool, pr.dev, pr.pool.L
    rng = np.random.default_rng(33)
    k, v, g = rand_tokens(rng, T, Hk, d, torch.bfloat16)
    kd, vd, gd = k.to(dev), v.to(dev), g.to(dev)
    full = pool.workspace.numel()
    seqs, ntok = _ids([0]), _ids([T])

    def prefill(size, ids=seqs):
        return L.wgkv_prefill_admit(pool.h, 0, 1, ids, ntok, _ptr(kd), _ptr(vd), _ptr(gd), None, None, 0, 0.5,
                                    None, _ptr(pool.workspace), size, _stream())

    # the threshold is found on slot 1 (freed after every accepted call), the checks run on slot 0
    def probe(size):
        rc = prefill(size, _ids([1]))
        if rc == 0:
            pool.free_seq(1)
        return rc
    need = _smallest_accepted(probe, 0, full)
    pool.status()
    before = _meta_bytes(pool)
    assert prefill(need - 1) == WORKSPACE
    np.testing.assert_array_equal(_meta_bytes(pool), before)
    assert prefill(need) == 0
    pr.orc.push_tokens(0, [0], [T], k.float().numpy(), v.float().numpy(), g.numpy(), 0.5)
    pr.touched.add((0, 0))
    pr.check_state()

    # decode form of attend
    q = rand_q(rng, 1, Hq, d, torch.bfloat16).to(dev)
    out = torch.zeros((1, Hq, d), dtype=torch.float32, device=dev)
    one = _ids([1])

    def attend(size):
        return L.wgkv_attend(pool.h, 0, 1, seqs, one, _ptr(q), None, None, None, 0.5, 0.1, _ptr(out),
                             _ptr(pool.workspace), size, _stream())
    need = _smallest_accepted(attend, 0, full)
    out.fill_(7.0)
    assert attend(need - 1) == WORKSPACE
    torch.cuda.synchronize()
    assert (out == 7.0).all()          # nothing was launched
    assert attend(need) == 0

    # prefill-chunk form of attend (needs four query heads per kv head)
    pr2 = Pair(1, 8, 2, 128, wg.BF16, 16, 32, 1, 32, 128, max_call_seqs=1, max_call_tokens=256)
    p2 = pr2.pool
    Tq = 48
    kc, vc, gc = rand_tokens(rng, Tq, 2, 128, torch.bfloat16)
    qc = rand_q(rng, Tq, 8, 128, torch.bfloat16).to(dev)
    kcd, vcd, gcd = kc.to(dev), vc.to(dev), gc.to(dev)
    outc = torch.zeros((Tq, 8, 128), dtype=torch.float32, device=dev)
    nq = _ids([Tq])

    def attend_chunk(size):
        return L.wgkv_attend(p2.h, 0, 1, seqs, nq, _ptr(qc), _ptr(kcd), _ptr(vcd), _ptr(gcd), 0.5, 0.1, _ptr(outc),
                             _ptr(p2.workspace), size, _stream())
    need = _smallest_accepted(attend_chunk, 0, p2.workspace.numel())
    outc.fill_(7.0)
    assert attend_chunk(need - 1) == WORKSPACE
    torch.cuda.synchronize()
    assert (outc == 7.0).all()
    assert attend_chunk(need) == 0
    torch.cuda.synchronize()
    assert torch.isfinite(outc).all()


def test_replayed_graph_past_the_last_free_page_sets_the_sticky_flag():
    Hq, Hk, d, P, W = 8, 2, 128, 4, 8
    # two sequences; 20 tokens each, all admitted: 12 global entries = 3 pages per head, 2 ring pages per head
    n_pages = 2 * Hk * (3 + 2) + Hk        # one more global page per head of one sequence, then nothing
    pr = Pair(1, Hq, Hk, d, wg.BF16, P, W, 2, 16, n_pages, max_call_seqs=2, max_call_tokens=64)
    dev = pr.dev
    rng = np.random.default_rng(34)
    k, v, g = rand_tokens(rng, 40, Hk, d, torch.bfloat16)
    g[:] = 0.9
    pr.prefill(0, [0, 1], [20, 20], k, v, g, 0.5)
    pr.check_state()
    assert pr.orc.free_top == Hk
    kb = torch.zeros((1, Hk, d), dtype=torch.bfloat16, device=dev)
    vb = torch.zeros_like(kb)
    gb = torch.full((1, Hk), 0.9, dtype=torch.float32, device=dev)
    qb = torch.zeros((1, Hq, d), dtype=torch.bfloat16, device=dev)
    ob = torch.zeros((1, Hq, d), dtype=torch.float32, device=dev)
    scale = 1.0 / math.sqrt(d)
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            pr.pool.decode_step(0, [0], kb, vb, gb, tau=0.5)
            pr.pool.attend(0, [0], qb, ob, scale)
    torch.cuda.current_stream().wait_stream(side)
    good = 0
    for step in range(7):            # steps 0..3 fit (the fourth fills the new page), 4..6 find no page
        k1, v1, _ = rand_tokens(rng, 1, Hk, d, torch.bfloat16)
        q1 = rand_q(rng, 1, Hq, d, torch.bfloat16)
        kb.copy_(k1); vb.copy_(v1); qb.copy_(q1)
        ob.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        if step < 4:
            pr.orc.push_tokens(0, [0], [1], k1.float().numpy(), v1.float().numpy(), gb.cpu().numpy(), 0.5)
            good += 1
        # attention still runs on whatever state there is: after a refused step that is the last good state
        ref = pr.orc.attend_cached(0, 0, q1[0].float().numpy(), scale)
        err = np.abs(ob[0].cpu().numpy().astype(np.float64) - ref)
        assert err.max() <= MAX_ABS_TOL and err.mean() <= MEAN_ABS_TOL, (step, err.max())
    assert good == 4 and pr.orc.free_top == 0
    free, flag = pr.pool.status()
    assert flag == OUT_OF_PAGES and free == 0
    rc = pr.pool.L.wgkv_status(pr.pool.h, _stream(), None, None)
    assert rc == DEVICE_FLAG           # sticky
    # the state equals the oracle's at the last good step (check_state asserts a clear flag: compare by hand)
    m = {kk: vv.cpu().numpy() for kk, vv in pr.pool.meta().items()}
    for s in (0, 1):
        assert int(m["seq_len"][s, 0]) == pr.orc.seq_len(s, 0)
        for h in range(Hk):
            lp, gp, rg, _ = pr.orc.head_tables(s, 0, h)
            assert int(m["global_len"][s, 0, h]) == pr.orc.global_len(s, 0, h)
            np.testing.assert_array_equal(m["local_pt"][s, 0, h], lp)
            np.testing.assert_array_equal(m["global_pt"][s, 0, h], gp)
            np.testing.assert_array_equal(m["ring_g"][s, 0, h].view(np.uint32), rg.view(np.uint32))
    # pages come back, the flag is cleared, and direct calls go on from the device's state
    pr.pool.free_seq(1)
    pr.orc.free_seq(1)
    pr.touched.discard((1, 0))
    pr.pool.clear_error()
    free, flag = pr.pool.status()
    assert flag == 0 and free == pr.orc.free_top
    k1, v1, g1 = rand_tokens(rng, 1, Hk, d, torch.bfloat16)
    g1[:] = 0.9
    pr.decode(0, [0], k1, v1, g1, 0.5)
    pr.check_state()
    pr.check_attend(0, [0], rand_q(rng, 1, Hq, d, torch.bfloat16))


@pytest.mark.parametrize("n_first,n_second", [(700, 333), (700, 21)])
def test_recycled_pages_with_non_finite_rows(n_first, n_second):
    """A freed sequence leaves inf / nan rows in its pages; the next owner of those pages, shorter and
    with partly filled last pages, must not see them."""
    Hq, Hk, d, P, W = 8, 2, 128, 16, 32
    max_gp = n_first // P + 2
    pr = Pair(1, Hq, Hk, d, wg.BF16, P, W, 1, max_gp, Hk * (max_gp + W // P) + 1, max_call_seqs=1,
              max_call_tokens=n_first)
    rng = np.random.default_rng(35)
    k, v, g = rand_tokens(rng, n_first, Hk, d, torch.bfloat16)
    g[:] = 0.9
    v[:] = float("inf")
    k[:] = float("nan")
    pr.pool.prefill_admit(0, [0], [n_first], k.to(pr.dev), v.to(pr.dev), g.to(pr.dev), tau=0.5)
    pr.pool.free_seq(0)
    free, flag = pr.pool.status()
    assert flag == 0 and free == pr.cfg.n_pages
    # the oracle never saw the first sequence; its free stack must be brought to the same order
    k0, v0, g0 = rand_tokens(rng, n_first, Hk, d, torch.bfloat16)
    g0[:] = 0.9
    pr.orc.push_tokens(0, [0], [n_first], k0.float().numpy(), v0.float().numpy(), g0.numpy(), 0.5)
    pr.orc.free_seq(0)
    k, v, g = rand_tokens(rng, n_second, Hk, d, torch.bfloat16, rates=[0.7, 0.35])
    pr.prefill(0, [0], [n_second], k, v, g, 0.5)
    pr.check_state()
    assert np.isnan(pr.pool.pool_pages().float().cpu().numpy()).any()       # stale rows are still there
    pr.check_attend(0, [0], rand_q(rng, 1, Hq, d, torch.bfloat16))
    for _ in range(P + 3):
        k1, v1, g1 = rand_tokens(rng, 1, Hk, d, torch.bfloat16)
        pr.decode(0, [0], k1, v1, g1, 0.5)
        pr.check_attend(0, [0], rand_q(rng, 1, Hq, d, torch.bfloat16))
    # the chunk form reads the same pages
    T = 40
    kc, vc, gc = rand_tokens(rng, T, Hk, d, torch.bfloat16)
    qc = rand_q(rng, T, Hq, d, torch.bfloat16)
    out = torch.full((T, Hq, d), float("nan"), dtype=torch.float32, device=pr.dev)
    pr.pool.attend(0, [0], qc.to(pr.dev), out, 1.0 / math.sqrt(d), n_q=[T], k_chunk=kc.to(pr.dev),
                   v_chunk=vc.to(pr.dev), g_chunk=gc.to(pr.dev), tau=0.5)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()


def test_gate_form_of_prefill_admit_checks_its_limits():
    # more than 16 kv heads: the linear gate kernel does not cover them, the call must say so
    Hk, d, dim = 32, 64, 64
    pr = Pair(1, Hk, Hk, d, wg.BF16, 16, 16, 1, 8, 2 * Hk * 4, max_call_seqs=1, max_call_tokens=64)
    dev, L, pool = pr.dev, pr.pool.L, pr.pool
    rng = np.random.default_rng(36)
    k, v, g = rand_tokens(rng, 20, Hk, d, torch.bfloat16)
    hidden = torch.zeros((20, dim), dtype=torch.bfloat16, device=dev)
    w = torch.zeros((Hk, dim), dtype=torch.bfloat16, device=dev)
    _refused(lambda: pool.prefill_admit(0, [0], [20], k.to(dev), v.to(dev), None, hidden=hidden, gate_w=w, tau=0.5),
             INVALID, pool)
    # given scores, the same shape is fine
    pr.prefill(0, [0], [20], k, v, g, 0.5)
    pr.check_state()
    # misaligned hidden rows
    pr8 = Pair(1, 8, 8, d, wg.BF16, 16, 16, 1, 8, 64, max_call_seqs=1, max_call_tokens=64)
    hid = torch.zeros((21 * dim + 8,), dtype=torch.bfloat16, device=dev)
    w8 = torch.zeros((8, dim), dtype=torch.bfloat16, device=dev)
    k8, v8, _ = rand_tokens(rng, 20, 8, d, torch.bfloat16)
    rc = L.wgkv_prefill_admit(pr8.pool.h, 0, 1, _ids([0]), _ids([20]), _ptr(k8.to(dev)), _ptr(v8.to(dev)), None,
                              C.c_void_p(hid.data_ptr() + 2), _ptr(w8), dim, 0.5, None, _ptr(pr8.pool.workspace),
                              pr8.pool.workspace.numel(), _stream())
    assert rc == INVALID
    assert L.wgkv_gate_scores(wg.BF16, 20, dim, 8, C.c_void_p(hid.data_ptr() + 2), _ptr(w8),
                              _ptr(torch.zeros((20, 8), device=dev)), _stream()) == INVALID


def _sparse_scores(rng, n, Hk, per_chunk, chunk, W):
    """Scores with exactly `per_chunk` values >= 0.5 per head in every chunk of `chunk` tokens, none of them among
    the last W of a chunk: a call that feeds one chunk then admits exactly `per_chunk` tokens per head (the ones
    among the chunk's first chunk - W tokens; the W tokens that leave the ring hold none)."""
    g = (0.4 * rng.random((n, Hk))).astype(np.float32)
    for c0 in range(0, n, chunk):
        for h in range(Hk):
            g[c0 + rng.choice(chunk - W, per_chunk, replace=False), h] = 0.9
    return torch.from_numpy(g)


def test_bound_on_admitted_tokens_lets_a_pool_sized_for_the_admitted_cache_run_without_status():
    Hq, Hk, d, P, W, chunk, n_chunks, per_chunk = 4, 2, 64, 4, 16, 64, 6, 6
    n = chunk * n_chunks
    # ring pages + the admitted cache if every head admits `per_chunk` tokens in every chunk, and nothing more
    n_pages = Hk * (W // P + (n_chunks * per_chunk + P - 1) // P)
    rng = np.random.default_rng(35)
    k, v, _ = rand_tokens(rng, n, Hk, d, torch.bfloat16)
    g = _sparse_scores(rng, n, Hk, per_chunk, chunk, W)
    # without the bound the host has to assume that every leaving token is admitted: refused at once or after a
    # few chunks (no wgkv_status in the loop to tighten its count)
    pr0 = Pair(1, Hq, Hk, d, wg.BF16, P, W, 1, 32, n_pages, max_call_seqs=1, max_call_tokens=chunk)
    with pytest.raises(wg.WgkvError) as e:
        for c in range(n_chunks):
            sl = slice(c * chunk, (c + 1) * chunk)
            pr0.pool.prefill_admit(0, [0], [chunk], k[sl].to(pr0.dev), v[sl].to(pr0.dev), g[sl].to(pr0.dev), tau=0.5)
    assert e.value.code == OUT_OF_PAGES
    # with it the same pool takes the whole prompt; the state and the attention are the oracle's
    pr = Pair(1, Hq, Hk, d, wg.BF16, P, W, 1, 32, n_pages, max_call_seqs=1, max_call_tokens=chunk)
    for c in range(n_chunks):
        sl = slice(c * chunk, (c + 1) * chunk)
        pr.prefill(0, [0], [chunk], k[sl], v[sl], g[sl], 0.5, max_admitted_per_head=per_chunk)
    pr.check_state()
    # what left the window was admitted at 6 per chunk; the last W tokens are still in the ring
    adm = int((g[:n - W, 0] >= 0.5).sum())
    assert pr.orc.global_len(0, 0, 0) == adm and pr.orc.free_top >= 0
    pr.check_attend(0, [0], rand_q(rng, 1, Hq, d, torch.bfloat16))
    with pytest.raises(wg.WgkvError) as e:
        pr.pool.prefill_admit(0, [0], [1], k[:1].to(pr.dev), v[:1].to(pr.dev), g[:1].to(pr.dev), tau=0.5,
                              max_admitted_per_head=-1)
    assert e.value.code == INVALID


def test_broken_bound_on_admitted_tokens_is_refused_on_the_device():
    Hq, Hk, d, P, W, chunk = 4, 2, 64, 4, 16, 64
    pr = Pair(1, Hq, Hk, d, wg.BF16, P, W, 2, 32, 200, max_call_seqs=2, max_call_tokens=2 * chunk)
    rng = np.random.default_rng(36)
    k, v, _ = rand_tokens(rng, 3 * chunk, Hk, d, torch.bfloat16)
    g = _sparse_scores(rng, 3 * chunk, Hk, 6, chunk, W)
    pr.prefill(0, [0, 1], [chunk, chunk], k[:2 * chunk], v[:2 * chunk], g[:2 * chunk], 0.5, max_admitted_per_head=6)
    pr.check_state()
    # third chunk for sequence 1: head 1 admits one token more than promised (7 of the tokens that leave)
    g3 = g[2 * chunk:].clone()
    g3[:] = 0.1
    g3[:7, 1] = 0.9     # the W tokens that leave the ring hold no admitted one
    before = _meta_bytes(pr.pool)
    dev = pr.dev
    pr.pool.prefill_admit(0, [1], [chunk], k[2 * chunk:].to(dev), v[2 * chunk:].to(dev), g3.to(dev), tau=0.5,
                          max_admitted_per_head=6)    # accepted by the host, which cannot know
    free, flag = pr.pool.status()
    assert flag == ADMIT_BOUND
    after = _meta_bytes(pr.pool)
    # nothing but the flag has changed
    diff = np.nonzero(before != after)[0]
    assert 0 < diff.size <= 4, diff
    pr.pool.clear_error()
    pr.check_state()                # still the state after two chunks: the oracle never saw the third
    # within the bound (7 admitted, bound 7) the same chunk goes through
    pr.prefill(0, [1], [chunk], k[2 * chunk:], v[2 * chunk:], g3, 0.5, max_admitted_per_head=7)
    pr.check_state()
    pr.check_attend(0, [0, 1], rand_q(rng, 2, Hq, d, torch.bfloat16))
