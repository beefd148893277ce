"""Pins of the oracle's training-time Write-Gated Attention (Sec. 3.2: mask m_ij, weighted
softmax, log-space bias) and of its gradients against things that are not the oracle:
the library's scaled-dot-product attention with an additive bias built here, the library's
reverse-mode differentiation of it, central differences, the multiplicative form of the
paper's first equation, and identities that hold for any input."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import (attend_definition, attend_soft, soft_attn_backward, soft_attn_backward_sampled, soft_attn_forward,
                    sparsity_loss)


def _inputs(seed, T, Hq, Hk, d, g_kind="uniform"):
    r = np.random.default_rng(seed)
    Q = r.standard_normal((T, Hq, d)).astype(np.float32)
    K = r.standard_normal((T, Hk, d)).astype(np.float32)
    V = r.standard_normal((T, Hk, d)).astype(np.float32)
    if g_kind == "uniform":
        g = r.uniform(0.02, 0.98, (T, Hk)).astype(np.float32)
    elif g_kind == "binary":
        g = (r.uniform(0, 1, (T, Hk)) < 0.4).astype(np.float32)
    else:
        g = np.full((T, Hk), float(g_kind), np.float32)
    dO = r.standard_normal((T, Hq, d)).astype(np.float32)
    return Q, K, V, g, dO


def _library(Q, K, V, g, W, scale, eps, need_grad=False):
    """Library attention in fp64 with the bias matrix log(max(1(i-j<W), g_j) + eps) written out."""
    T, Hq, d = Q.shape
    Hk = K.shape[1]
    G = Hq // Hk
    q = torch.from_numpy(Q).double().permute(1, 0, 2).clone().requires_grad_(need_grad)       # [Hq, T, d]
    k = torch.from_numpy(K).double().permute(1, 0, 2).clone().requires_grad_(need_grad)       # [Hk, T, d]
    v = torch.from_numpy(V).double().permute(1, 0, 2).clone().requires_grad_(need_grad)
    gt = torch.from_numpy(g).double().t().clone().requires_grad_(need_grad)                   # [Hk, T]
    i = torch.arange(T)[:, None]
    j = torch.arange(T)[None, :]
    window = (i - j < W).double()                                                          # [T, T]
    m = torch.maximum(window[None], gt[:, None, :].expand(Hk, T, T))
    bias = torch.log(m + eps).masked_fill((j > i)[None], float("-inf"))                    # causal
    bias = bias.repeat_interleave(G, dim=0)                                                # [Hq, T, T]
    out = F.scaled_dot_product_attention(q[None], k.repeat_interleave(G, dim=0)[None],
                                         v.repeat_interleave(G, dim=0)[None], attn_mask=bias[None], scale=scale)[0]
    return out.permute(1, 0, 2), (q, k, v, gt)


@pytest.mark.parametrize("T,Hq,Hk,d,W,eps", [(40, 4, 2, 8, 6, 1e-6), (97, 8, 2, 16, 16, 1e-3), (33, 2, 2, 4, 64, 1e-6)])
def test_forward_matches_library_attention_with_bias(T, Hq, Hk, d, W, eps):
    Q, K, V, g, _ = _inputs(1, T, Hq, Hk, d)
    scale = 1 / math.sqrt(d)
    out, lse = soft_attn_forward(Q, K, V, g, W, scale, eps)
    ref, _ = _library(Q, K, V, g, W, scale, eps)
    np.testing.assert_allclose(out, ref.detach().numpy(), rtol=1e-11, atol=1e-12)
    # lse against a direct log-sum-exp of the first rows, written out here
    for i in (0, 1, T // 2, T - 1):
        for qh in range(Hq):
            h = qh // (Hq // Hk)
            s = np.array([scale * float(Q[i, qh].astype(np.float64) @ K[j, h].astype(np.float64))
                          + math.log(max(1.0 if i - j < W else 0.0, float(g[j, h])) + eps) for j in range(i + 1)])
            assert abs(lse[i, qh] - (s.max() + math.log(np.exp(s - s.max()).sum()))) < 1e-11


def test_forward_is_the_multiplicative_form():
    """exp(s) * m / sum exp(s) * m (first Write-Gated Attention equation) as eps -> 0."""
    T, Hq, Hk, d, W = 50, 4, 2, 8, 7
    Q, K, V, g, _ = _inputs(2, T, Hq, Hk, d)
    scale = 1 / math.sqrt(d)
    out, _ = soft_attn_forward(Q, K, V, g, W, scale, 1e-300)
    for i in (0, 5, 20, 49):
        for qh in range(Hq):
            h = qh // 2
            s = np.array([scale * float(Q[i, qh].astype(np.float64) @ K[j, h].astype(np.float64)) for j in range(i + 1)])
            m = np.array([max(1.0 if i - j < W else 0.0, float(g[j, h])) for j in range(i + 1)])
            w = np.exp(s - s.max()) * m
            ref = (w[:, None] * V[: i + 1, h].astype(np.float64)).sum(0) / w.sum()
            np.testing.assert_allclose(out[i, qh], ref, rtol=1e-11, atol=1e-13)


def test_binary_gate_gives_the_hard_mask_and_ones_give_plain_attention():
    T, Hq, Hk, d, W = 60, 4, 2, 8, 5
    Q, K, V, gb, _ = _inputs(3, T, Hq, Hk, d, "binary")
    scale = 1 / math.sqrt(d)
    hard = attend_definition(K, V, gb, Q, np.arange(T), W, 0.5, scale)
    soft, _ = soft_attn_forward(Q, K, V, gb, W, scale, 1e-300)   # log(0 + 1e-300): weight 1e-300
    np.testing.assert_allclose(soft, hard, rtol=1e-10, atol=1e-12)
    ones = np.ones_like(gb)
    plain = F.scaled_dot_product_attention(torch.from_numpy(Q).double().permute(1, 0, 2)[None],
                                           torch.from_numpy(K).double().permute(1, 0, 2).repeat_interleave(2, 0)[None],
                                           torch.from_numpy(V).double().permute(1, 0, 2).repeat_interleave(2, 0)[None],
                                           is_causal=True, scale=scale)[0].permute(1, 0, 2).numpy()
    # a bias that is the same for every key cancels in the softmax, whatever eps is
    np.testing.assert_allclose(soft_attn_forward(Q, K, V, ones, W, scale, 0.25)[0], plain, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("T,Hq,Hk,d,W,eps", [(40, 4, 2, 8, 6, 1e-6), (70, 8, 2, 16, 16, 1e-3), (20, 2, 1, 4, 64, 1e-6)])
def test_backward_matches_library_differentiation(T, Hq, Hk, d, W, eps):
    Q, K, V, g, dO = _inputs(4, T, Hq, Hk, d)
    scale = 1 / math.sqrt(d)
    dQ, dK, dV, dg = soft_attn_backward(Q, K, V, g, dO, W, scale, eps)
    out, (q, k, v, gt) = _library(Q, K, V, g, W, scale, eps, need_grad=True)
    out.backward(torch.from_numpy(dO).double())
    np.testing.assert_allclose(dQ, q.grad.permute(1, 0, 2).numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dK, k.grad.permute(1, 0, 2).numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dV, v.grad.permute(1, 0, 2).numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dg, gt.grad.t().numpy(), rtol=1e-9, atol=1e-11)
    assert np.abs(dK).max() > 1e-3 and (np.abs(dg).max() > 1e-3 if T > W else np.all(dg == 0))


def test_backward_matches_central_differences():
    T, Hq, Hk, d, W, eps = 12, 2, 1, 4, 3, 1e-2
    Q, K, V, g, dO = _inputs(5, T, Hq, Hk, d)
    scale = 0.7
    grads = dict(zip("QKVg", soft_attn_backward(Q, K, V, g, dO, W, scale, eps)))

    def loss(Q_, K_, V_, g_):
        return float((soft_attn_forward(Q_, K_, V_, g_, W, scale, eps)[0] * dO.astype(np.float64)).sum())

    r = np.random.default_rng(6)
    args = {"Q": Q, "K": K, "V": V, "g": g}
    # steps that are exact in fp32 around fp32 values rounded to few bits
    for name in "QKVg":
        args[name] = (np.round(args[name] * 64) / 64).astype(np.float32)
    grads = dict(zip("QKVg", soft_attn_backward(args["Q"], args["K"], args["V"], args["g"], dO, W, scale, eps)))
    h = 2.0 ** -10
    for name in "QKVg":
        for _ in range(12):
            idx = tuple(int(r.integers(0, n)) for n in args[name].shape)
            hi = {k_: v_.copy() for k_, v_ in args.items()}
            lo = {k_: v_.copy() for k_, v_ in args.items()}
            hi[name][idx] += h
            lo[name][idx] -= h
            fd = (loss(hi["Q"], hi["K"], hi["V"], hi["g"]) - loss(lo["Q"], lo["K"], lo["V"], lo["g"])) / (2 * h)
            assert abs(fd - grads[name][idx]) <= 2e-5 * max(1.0, abs(fd)), (name, idx, fd, grads[name][idx])


def test_backward_identities():
    T, Hq, Hk, d, W, eps = 64, 8, 2, 16, 9, 1e-6
    Q, K, V, g, dO = _inputs(7, T, Hq, Hk, d)
    scale = 1 / math.sqrt(d)
    dQ, dK, dV, dg = soft_attn_backward(Q, K, V, g, dO, W, scale, eps)
    G = Hq // Hk
    # every row of weights sums to one: the dV of a kv head add up to the dO of its query heads
    np.testing.assert_allclose(dV.sum(0), dO.astype(np.float64).reshape(T, Hk, G, d).sum((0, 2)), rtol=1e-10, atol=1e-10)
    # the output depends on q and k through q . k only: scaling q up and k down changes nothing
    for h in range(Hk):
        lhs = (Q[:, h * G:(h + 1) * G].astype(np.float64) * dQ[:, h * G:(h + 1) * G]).sum()
        rhs = (K[:, h].astype(np.float64) * dK[:, h]).sum()
        assert abs(lhs - rhs) < 1e-9 * max(1.0, abs(lhs))
    # the last W positions are inside the window of every query that sees them, where m_ij = 1
    # does not depend on g_j (g < 1)
    assert np.all(dg[T - W:] == 0.0) and np.abs(dg[: T - W]).max() > 0
    # a score of exactly 1 outside the window ties with nothing (indicator 0): it does follow g
    g1 = g.copy(); g1[3] = 1.0
    assert np.abs(soft_attn_backward(Q, K, V, g1, dO, W, scale, eps)[3][3]).max() > 0
    # a loss that ignores the output has zero gradients
    z = soft_attn_backward(Q, K, V, g, np.zeros_like(dO), W, scale, eps)
    assert all(np.all(x == 0) for x in z)


def test_sampled_gradients_are_the_full_ones():
    """The sampled form used at sizes the full function cannot reach gives the same numbers, and so
    does the per-row forward used there (the library-pinned functions are the reference)."""
    T, Hq, Hk, d, W, eps = 90, 8, 2, 16, 11, 1e-4
    Q, K, V, g, dO = _inputs(9, T, Hq, Hk, d)
    scale = 1 / math.sqrt(d)
    dQ, dK, dV, dg = soft_attn_backward(Q, K, V, g, dO, W, scale, eps)
    rows = [0, 10, 11, 57, 89]
    for h, j_first in ((0, 60), (1, 0), (1, 89), (0, 90)):
        sQ, sK, sV, sg = soft_attn_backward_sampled(Q, K, V, g, dO, W, scale, eps, rows, h, j_first)
        np.testing.assert_allclose(sQ, dQ[rows], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(sK, dK[j_first:, h], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(sV, dV[j_first:, h], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(sg, dg[j_first:, h], rtol=1e-12, atol=1e-14)
    out, _ = soft_attn_forward(Q, K, V, g, W, scale, eps)
    np.testing.assert_allclose(attend_soft(K, V, g, Q[rows], rows, W, scale, use_log=True, eps=eps), out[rows],
                               rtol=1e-12, atol=1e-14)


def test_sparsity_loss_matches_library_differentiation():
    r = np.random.default_rng(8)
    g = r.uniform(0, 1, (5, 37, 3)).astype(np.float32)
    loss, dg = sparsity_loss(g)
    gt = torch.from_numpy(g).double().requires_grad_(True)
    ref = (gt + gt * (1 - gt)).mean()
    ref.backward()
    assert abs(loss - ref.item()) < 1e-14
    np.testing.assert_allclose(dg, gt.grad.numpy(), rtol=1e-13, atol=1e-16)
    # closed forms: g = 0 -> 0, g = 1 -> 1, g = 1/2 -> 3/4
    assert sparsity_loss(np.zeros(4, np.float32))[0] == 0.0 and sparsity_loss(np.ones(4, np.float32))[0] == 1.0
    assert sparsity_loss(np.full(4, 0.5, np.float32))[0] == 0.75
