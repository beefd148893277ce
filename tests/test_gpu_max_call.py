"""Calls at the largest sizes the boundary takes: WGKV_MAX_CALL_SEQS = 128 sequences and WGKV_MAX_CALL_UNITS = 1024
(sequence, kv head) units in one call, through every entry point of the path (chunked prompts of ragged lengths
with empty ones, decode steps with and without the promotion ahead, decode attention, page scoring and selection,
eviction), state and outputs against the oracle; one sequence or one unit more is refused by the host."""
import math

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
from harness import Pair, rand_q, rand_tokens
from oracle import quest_select
from test_gpu_prefill_chunks import _flow

pytestmark = pytest.mark.gpu

INVALID = -1


def test_128_sequences_and_1024_units_in_every_call():
    rng = np.random.default_rng(128)
    L, Hk, G, d, P, W, B = 2, 8, 1, 64, 4, 8, 128
    Hq = Hk * G
    max_chunk, max_gp = 40, 40
    pair = Pair(L, Hq, Hk, d, wg.BF16, P, W, B, max_gp, B * L * Hk * (max_gp + W // P) + 8, max_call_seqs=B,
                max_call_tokens=B * max_chunk)
    seqs = [int(s) for s in rng.permutation(B)]          # all 128 slots, out of order
    for chunk in range(2):
        lens = [int(x) for x in rng.integers(0, max_chunk + 1, B)]
        lens[3] = 0 if chunk == 0 else 2   # an empty piece; every slot has a token before the first decode step
        lens[7] = 1                        # (a first token in a step with the promotion ahead changes page numbers)
        lens = [max(x, 1) for x in lens] if chunk == 1 else lens
        for l in range(L):
            k, v, g = rand_tokens(rng, sum(lens), Hk, d, pair.tdt, rates=list(rng.uniform(0.2, 0.9, Hk)))
            pair.prefill(l, seqs, lens, k, v, g, 0.5)
    pair.check_state()
    for step in range(W + 3):
        if step % 2 == 0:
            pair.pool.decode_promote(seqs, tau=0.5)
        for l in range(L):
            k, v, g = rand_tokens(rng, B, Hk, d, pair.tdt, rates=[0.7] * Hk)
            pair.decode(l, seqs, k, v, g, 0.5)
    pair.check_state()
    for l in range(L):
        pair.check_attend(l, seqs, rand_q(rng, B, Hq, d, pair.tdt), 1.0 / math.sqrt(d))
    # page scoring and selection over all 1024 heads
    lm = pair.pool.quest_landmarks()
    pair.pool.quest_update(1, seqs, lm)
    q = rand_q(rng, B, Hq, d, pair.tdt)
    n_pg = [-(-pair.orc.global_len(s, 1, h) // P) for s in seqs for h in range(Hk)]
    scores, sel, cnt = pair.pool.quest_select(1, seqs, q.to(pair.dev), lm, 3, max(n_pg) + 1)
    scores, sel, cnt = scores.cpu().numpy(), sel.cpu().numpy(), cnt.cpu().numpy()
    for b, s in enumerate(seqs):
        for h in range(Hk):
            u = b * Hk + h
            ref = pair.orc.quest_page_scores(1, s, h, q[b].float().numpy())
            if n_pg[u]:
                assert np.abs(scores[u, :n_pg[u]] - ref).max() <= 2e-5 * max(1.0, float(np.abs(ref).max()))
            want = quest_select(scores[u, :n_pg[u]], 3)
            assert cnt[u] == len(want) and np.array_equal(sel[u, :cnt[u]], want)
    # eviction of half of every head, then the step and the attention again
    n_max = max(pair.orc.global_len(s, 0, h) for s in seqs for h in range(Hk))
    pair.evict(0, seqs, rng.random((B * Hk, n_max + 1)).astype(np.float32), 0.5)
    pair.check_state()
    k, v, g = rand_tokens(rng, B, Hk, d, pair.tdt, rates=[0.7] * Hk)
    pair.decode(0, seqs, k, v, g, 0.5)
    pair.check_attend(0, seqs, rand_q(rng, B, Hq, d, pair.tdt), 1.0 / math.sqrt(d))
    pair.check_state()


@pytest.mark.parametrize("shape", [(32, 8, 128, wg.BF16),   # matrix-core kernel
                                   (8, 8, 64, wg.F32)])     # plain kernel
def test_chunked_prefill_of_128_sequences(shape):
    """Gate-free flow (scores given): prefill-form attention of every chunk row against the definition, admission
    state against the oracle, 128 sequences of ragged lengths = 1024 units per call."""
    rng = np.random.default_rng(1024)
    lens = [int(x) for x in rng.integers(1, 40, 128)]
    _flow(128, lens, 16, 8, 4, 64, 77, use_gate=False, shape=shape)


def test_one_more_sequence_or_unit_than_a_call_takes_is_refused():
    # 129 slots exist, a call may name 128 of them
    cfg = wg.Config(1, 8, 8, 64, wg.BF16, 4, 8, 129, 8, 129 * 8 * 10)
    pool = wg.Pool(cfg, 128, 256)
    dev = pool.device
    k = torch.zeros((129, 8, 64), dtype=torch.bfloat16, device=dev)
    g = torch.zeros((129, 8), dtype=torch.float32, device=dev)
    with pytest.raises(wg.WgkvError) as e:
        pool.decode_step(0, list(range(129)), k, k, g)
    assert e.value.code == INVALID
    pool.decode_step(0, list(range(128)), k[:128], k[:128], g[:128])
    free, flag = pool.status()
    assert flag == 0
    # 16 kv heads: 64 sequences are 1024 units, 65 are one head row too many
    cfg = wg.Config(1, 16, 16, 64, wg.BF16, 4, 8, 65, 8, 65 * 16 * 10)
    with pytest.raises(wg.WgkvError) as e:
        wg.Pool(cfg, 65, 256)                            # a workspace for 65 x 16 units is not handed out either
    assert e.value.code == INVALID
    pool = wg.Pool(cfg, 64, 256)
    k = torch.zeros((65, 16, 64), dtype=torch.bfloat16, device=dev)
    g = torch.zeros((65, 16), dtype=torch.float32, device=dev)
    with pytest.raises(wg.WgkvError) as e:
        pool.decode_step(0, list(range(65)), k, k, g)
    assert e.value.code == INVALID
    pool.decode_step(0, list(range(64)), k[:64], k[:64], g[:64])
    free, flag = pool.status()
    assert flag == 0
