"""A decode step (lazy promotion + decode attention for every layer) captured in a HIP graph and
replayed: every replay must be one more token, equal to the oracle's step, with eager work and
synchronisation between the replays; afterwards wgkv_status brings the host bookkeeping back in
step and direct calls continue."""
import math

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
from harness import Pair, rand_tokens, MAX_ABS_TOL, MEAN_ABS_TOL

pytestmark = pytest.mark.gpu


def test_decode_step_graph_replay():
    rng = np.random.default_rng(17)
    L, Hq, Hk, d, P, W, B, T = 3, 32, 8, 128, 16, 32, 2, 300
    max_gp = (T + 64) // P + 4
    pair = Pair(L, Hq, Hk, d, wg.BF16, P, W, B, max_gp, B * L * Hk * (max_gp + W // P) + 16, max_call_seqs=B,
                max_call_tokens=B * T)
    dev, seqs = pair.dev, [0, 1]
    for l in range(L):
        k, v, g = rand_tokens(rng, 2 * T - 40, Hk, d, pair.tdt, rates=[0.6] * Hk)
        pair.prefill(l, seqs, [T, T - 40], k, v, g, 0.5)
    # one eager step first: everything is warm before the capture
    for l in range(L):
        k, v, g = rand_tokens(rng, B, Hk, d, pair.tdt, rates=[0.7] * Hk)
        pair.decode(l, seqs, k, v, g, 0.5)
    pair.check_state()
    scale = 1.0 / math.sqrt(d)
    # static buffers of the graph
    kb = torch.zeros((L, B, Hk, d), dtype=torch.bfloat16, device=dev)
    vb = torch.zeros_like(kb)
    gb = torch.zeros((L, B, Hk), dtype=torch.float32, device=dev)
    qb = torch.zeros((L, B, Hq, d), dtype=torch.bfloat16, device=dev)
    ob = torch.zeros((L, B, Hq, d), dtype=torch.float32, device=dev)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for l in range(L):
                pair.pool.decode_step(l, seqs, kb[l], vb[l], gb[l], tau=0.5)
                pair.pool.attend(l, seqs, qb[l], ob[l], scale)
    torch.cuda.current_stream().wait_stream(side)
    n_replays = 2 * P + 5          # crosses page boundaries of the global caches and wraps the ring
    for step in range(n_replays):
        ks, vs, gs, qs = [], [], [], []
        for l in range(L):
            k, v, g = rand_tokens(rng, B, Hk, d, pair.tdt, rates=[0.8] * Hk)
            ks.append(k); vs.append(v); gs.append(g)
            qs.append(torch.from_numpy(rng.standard_normal((B, Hq, d)).astype(np.float32)).to(pair.tdt))
        kb.copy_(torch.stack(ks)); vb.copy_(torch.stack(vs)); gb.copy_(torch.stack(gs)); qb.copy_(torch.stack(qs))
        ob.fill_(float("nan"))       # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        out = ob.cpu().numpy().astype(np.float64)
        for l in range(L):
            pair.orc.push_tokens(l, seqs, [1] * B, ks[l].float().numpy(), vs[l].float().numpy(), gs[l].numpy(), 0.5)
            ref = np.stack([pair.orc.attend_cached(s, l, qs[l][i].float().numpy(), scale) for i, s in enumerate(seqs)])
            err = np.abs(out[l] - ref)
            assert np.isfinite(out[l]).all() and err.max() <= MAX_ABS_TOL and err.mean() <= MEAN_ABS_TOL, (step, l)
    # the host has not seen the replays: status re-reads the device, then everything matches and goes on
    pair.check_state()
    for l in range(L):
        k, v, g = rand_tokens(rng, B, Hk, d, pair.tdt, rates=[0.7] * Hk)
        pair.decode(l, seqs, k, v, g, 0.5)
        q = torch.from_numpy(rng.standard_normal((B, Hq, d)).astype(np.float32)).to(pair.tdt)
        pair.check_attend(l, seqs, q)
    pair.check_state()
