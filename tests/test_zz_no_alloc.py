"""wgkv_attend_decode_static (the decode attention entry point that takes no workspace: its
partial results live in an array inside the library's device image) against wgkv_attend on the same
state, on two calls in a row, the second with a smaller input."""
import math

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
from harness import MAX_ABS_TOL, MEAN_ABS_TOL, Pair, rand_q, rand_tokens

pytestmark = pytest.mark.gpu


def _both(pair, layer, seqs, q, scale):
    dev = pair.dev
    c = pair.cfg
    a = torch.full((len(seqs), c.n_q_heads, c.head_dim), float("nan"), dtype=torch.float32, device=dev)
    b = torch.full_like(a, float("nan"))
    qd = q.to(dev)
    pair.pool.attend(layer, seqs, qd, a, scale)
    pair.pool.attend_decode_static(layer, seqs, qd, b, scale)
    torch.cuda.synchronize()
    return a, b


@pytest.mark.parametrize("dtype,d,Hq,Hk,P,W", [(wg.BF16, 128, 32, 8, 16, 64), (wg.F32, 64, 8, 2, 16, 32)])
def test_static_scratch_entry_matches_workspace_entry(dtype, d, Hq, Hk, P, W):
    rng = np.random.default_rng(2512)
    tdt = torch.float32 if dtype == wg.F32 else torch.bfloat16
    B, T = 6, 3000
    max_gp = T // P + 8
    pair = Pair(2, Hq, Hk, d, dtype, P, W, B, max_gp, 2 * B * Hk * (max_gp + W // P) + 32, max_call_seqs=B,
                max_call_tokens=B * T)
    lens = [T, T - 517, 1200, 77, W - 3, 2049]
    for layer in (0, 1):
        k, v, g = rand_tokens(rng, sum(lens), Hk, d, tdt, rates=list(np.linspace(0.05, 0.9, Hk)))
        pair.prefill(layer, list(range(B)), lens, k, v, g, 0.5)
    scale = 1.0 / math.sqrt(d)
    # first call: all six sequences; second call, right after it: two of them, in another order, other layer
    for layer, seqs in ((0, [0, 1, 2, 3, 4, 5]), (1, [4, 1])):
        q = rand_q(rng, len(seqs), Hq, d, tdt)
        a, b = _both(pair, layer, seqs, q, scale)
        assert torch.isfinite(b).all()
        if dtype == wg.BF16:   # one block per compute unit in both entry points: the same split, the same bits
            assert torch.equal(a, b), (layer, (a - b).abs().max().item())
        ref = np.stack([pair.orc.attend_cached(s, layer, q[i].float().numpy(), scale) for i, s in enumerate(seqs)])
        for x in (a, b):
            err = np.abs(x.cpu().numpy().astype(np.float64) - ref)
            if dtype == wg.F32:
                assert err.max() <= 2e-5, err.max()
            else:
                assert err.max() <= MAX_ABS_TOL and err.mean() <= MEAN_ABS_TOL, (err.max(), err.mean())
    # decode steps in between keep working, and the entry point follows the state
    for step in range(3):
        k, v, g = rand_tokens(rng, 2, Hk, d, tdt)
        pair.decode(0, [5, 0], k, v, g, 0.5)
        q = rand_q(rng, 2, Hq, d, tdt)
        a, b = _both(pair, 0, [5, 0], q, scale)
        ref = np.stack([pair.orc.attend_cached(s, 0, q[i].float().numpy(), scale) for i, s in enumerate([5, 0])])
        err = np.abs(b.cpu().numpy().astype(np.float64) - ref)
        assert err.max() <= (2e-5 if dtype == wg.F32 else MAX_ABS_TOL)


def test_static_scratch_entry_rejects_what_does_not_fit():
    # group 8 x head_dim 128: the partials of 512 blocks do not fit the static array
    pair = Pair(1, 8, 1, 128, wg.BF16, 16, 32, 1, 16, 64, max_call_seqs=1, max_call_tokens=64)
    rng = np.random.default_rng(1)
    k, v, g = rand_tokens(rng, 40, 1, 128, torch.bfloat16)
    pair.prefill(0, [0], [40], k, v, g, 0.5)
    q = rand_q(rng, 1, 8, 128, torch.bfloat16).to(pair.dev)
    out = torch.zeros((1, 8, 128), dtype=torch.float32, device=pair.dev)
    with pytest.raises(wg.WgkvError) as e:
        pair.pool.attend_decode_static(0, [0], q, out, 0.1)
    assert e.value.code == -6
    pair.pool.attend(0, [0], q, out, 0.1)   # the entry point with a workspace takes it
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
