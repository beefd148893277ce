"""Training-time Write-Gated Attention kernels (Sec. 3.2, log-space form) against the fp64
oracle, through the C ABI: forward output and log-sum-exp, and the gradients for q, k, v and
the gate scores; several tiles with ragged ends, windows longer than the sequence, packed
sequences with an empty one, scores at the ends of [0, 1]."""
import math

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
import wgkv_workloads as wl
from oracle import attend_soft, soft_attn_backward, soft_attn_backward_sampled, soft_attn_forward
from oracle import sparsity_loss as oracle_sparsity_loss

pytestmark = pytest.mark.gpu

# Forward: the bar of the attention kernels (products of bf16 values are exact in fp32, the
# weights are rounded to bf16 before the second product: relative 2^-9 each, averaging out
# over the keys of a row).
FWD_MAX, FWD_MEAN = 1e-2, 1e-3
LSE_TOL = 1e-4   # fp32 sum of fp32 exponentials against fp64
# Backward: p and dS enter their products rounded to bf16 (relative error up to 2^-9 = 2e-3 per
# term, independent between terms), everything else is fp32.  A gradient entry is a sum of such
# terms, so its error is a few 1e-3 of the size of the entries of that tensor; the bar is taken
# relative to the largest entry of the reference: 1e-2 at most, 1e-3 on average.
BWD_MAX, BWD_MEAN = 1e-2, 1e-3


def _cfg(seed, Hk):
    return wl.WorkloadConfig(f"soft_{seed}", 700 + seed, 1, 1, Hk * 4, Hk, 128, "bf16", 8, 4, 0.5, 1, 1, 0,
                             "uniform_10_40")


def _inputs(seed, rows, Hk, g_kind="law"):
    cfg = _cfg(seed, Hk)
    Hq, d = Hk * 4, 128
    q = wl.draw_normal(cfg, "q", (rows, Hq, d))
    k = wl.draw_normal(cfg, "k", (rows, Hk, d))
    v = wl.draw_normal(cfg, "v", (rows, Hk, d))
    dout = wl.draw_normal(cfg, "dout", (rows, Hq, d))
    if g_kind == "law":      # the score law of the decode workloads: most mass near 0, a tail up to 1
        g = torch.from_numpy(wl.draw_scores(cfg, 0, 0, rows, wl.unit_rates(cfg)))
    else:                    # uniform, with exact zeros and ones mixed in
        r = np.random.default_rng(cfg.seed)
        gn = r.uniform(0, 1, (rows, Hk)).astype(np.float32)
        gn[r.uniform(0, 1, gn.shape) < 0.1] = 0.0
        gn[r.uniform(0, 1, gn.shape) < 0.1] = 1.0
        g = torch.from_numpy(gn)
    return q, k, v, g, dout


def _oracle(q, k, v, g, dout, n_tokens, W, scale, eps, backward=True):
    f = lambda x: x.float().numpy()
    outs, lses, grads = [], [], [[], [], [], []]
    r0 = 0
    for T in n_tokens:
        sl = slice(r0, r0 + T)
        o, l = soft_attn_forward(f(q[sl]), f(k[sl]), f(v[sl]), f(g[sl]), W, scale, eps)
        outs.append(o); lses.append(l)
        if backward:
            for acc, x in zip(grads, soft_attn_backward(f(q[sl]), f(k[sl]), f(v[sl]), f(g[sl]), f(dout[sl]), W, scale, eps)):
                acc.append(x)
        r0 += T
    cat = lambda xs: np.concatenate(xs, 0)
    return cat(outs), cat(lses), [cat(x) for x in grads] if backward else None


def _check(name, got, ref, tol_max, tol_mean, relative):
    got = got.double().cpu().numpy()
    assert got.shape == ref.shape and np.isfinite(got).all(), name
    # a reference that vanishes (one key: dS is exactly zero) leaves the rounding of terms of order
    # one that cancel; the floor keeps the bar meaningful there
    unit = max(np.abs(ref).max(), 1e-3) if relative else 1.0
    err = np.abs(got - ref)
    assert err.max() <= tol_max * unit and err.mean() <= tol_mean * unit, (name, err.max() / unit, err.mean() / unit)


CASES = [
    # seed, tokens per sequence, kv heads, W, eps, score kind
    (1, [300], 2, 64, 1e-6, "law"),          # several query blocks and key tiles, ragged ends
    (2, [1], 1, 8, 1e-6, "law"),
    (3, [130], 1, 256, 1e-6, "law"),         # window longer than the sequence: plain causal attention
    (4, [100, 0, 77], 2, 32, 1e-3, "ends"),  # packed sequences, an empty one, scores of exactly 0 and 1
    (5, [513], 1, 100, 1e-6, "ends"),        # window not a multiple of the tile, keys far outside it
    (6, [64, 128], 1, 1, 1e-6, "law"),       # window of one: only the token itself is unweighted
    (9, [200], 1, 16, 0.0, "ends"),          # eps = 0: a score of exactly 0 removes the key outside the window
    # windows one off a tile of 32 keys: where the backward kernels' paths without mask tests begin
    (11, [257], 1, 33, 1e-6, "ends"),
    (12, [420, 130], 1, 63, 1e-6, "law"),
    (13, [257], 1, 96, 1e-6, "law"),
]


@pytest.mark.parametrize("seed,n_tokens,Hk,W,eps,kind", CASES)
def test_forward_and_backward_match_fp64(seed, n_tokens, Hk, W, eps, kind):
    dev = torch.device("cuda:0")
    rows = sum(n_tokens)
    q, k, v, g, dout = _inputs(seed, rows, Hk, kind)
    scale = 1 / math.sqrt(128)
    print("case", seed, n_tokens, Hk, W, eps, kind, flush=True)
    qd, kd, vd, gd, dd = (x.to(dev) for x in (q, k, v, g, dout))
    out, lse = wg.soft_attn_forward(qd, kd, vd, gd, n_tokens, W, scale, eps)
    dq, dk, dv, dg = wg.soft_attn_backward(qd, kd, vd, gd, out, lse, dd, n_tokens, W, scale, eps)
    torch.cuda.synchronize()
    ref_out, ref_lse, (rq, rk, rv, rg) = _oracle(q, k, v, g, dout, n_tokens, W, scale, eps)
    _check("out", out, ref_out, FWD_MAX, FWD_MEAN, False)
    _check("lse", lse, ref_lse, LSE_TOL, LSE_TOL, False)
    _check("dq", dq, rq, BWD_MAX, BWD_MEAN, True)
    _check("dk", dk, rk, BWD_MAX, BWD_MEAN, True)
    _check("dv", dv, rv, BWD_MAX, BWD_MEAN, True)
    if np.abs(rg).max() > 0:
        _check("dg", dg, rg, BWD_MAX, BWD_MEAN, True)
    else:
        assert torch.all(dg == 0)
    # keys that no query sees from outside its window get exactly zero
    r0 = 0
    for T in n_tokens:
        tail = slice(r0 + max(T - W, 0), r0 + T)
        assert torch.all(dg[tail] == 0)
        r0 += T


def test_full_training_length_on_sampled_outputs():
    """The longest training sample (32K tokens, Llama-3.1-8B head shape, window 256), the launch
    the benchmark times: sampled query rows of out and dq, the last 400 keys of one kv head for
    dk, dv, dg (they include keys outside the window of later queries), and two identities that
    hold at any size."""
    dev = torch.device("cuda:0")
    T, Hk, W, eps = 32768, 8, 256, 1e-6
    Hq, scale = 4 * Hk, 1 / math.sqrt(128)
    cfg = wl.get_config("llama8b_32layer_b8_128k")
    q = wl.draw_normal(cfg, "q", (T, Hq, 128), device=dev)
    k = wl.draw_normal(cfg, "k", (T, Hk, 128), device=dev)
    v = wl.draw_normal(cfg, "v", (T, Hk, 128), device=dev)
    dout = wl.draw_normal(cfg, "dout", (T, Hq, 128), device=dev)
    g = wl.draw_scores(cfg, 0, 0, T, wl.unit_rates(cfg), device=dev)
    out, lse = wg.soft_attn_forward(q, k, v, g, [T], W, scale, eps)
    dq, dk, dv, dg = wg.soft_attn_backward(q, k, v, g, out, lse, dout, [T], W, scale, eps)
    torch.cuda.synchronize()
    f = lambda x: x.float().cpu().numpy()
    qn, kn, vn, gn, dn = f(q), f(k), f(v), f(g), f(dout)
    rows = [0, 255, 256, 4097, 20000, T - 1]
    print("oracle: sampled rows", flush=True)
    ref_out = attend_soft(kn, vn, gn, qn[rows], rows, W, scale, use_log=True, eps=eps)
    _check("out rows", out[rows], ref_out, FWD_MAX, FWD_MEAN, False)
    h, j_first = 3, T - 400
    rq, rk, rv, rg = soft_attn_backward_sampled(qn, kn, vn, gn, dn, W, scale, eps, rows, h, j_first)
    print("oracle: done", flush=True)
    _check("dq rows", dq[rows], rq, BWD_MAX, BWD_MEAN, True)
    _check("dk tail", dk[j_first:, h], rk, BWD_MAX, BWD_MEAN, True)
    _check("dv tail", dv[j_first:, h], rv, BWD_MAX, BWD_MEAN, True)
    assert np.abs(rg[: 400 - W]).max() > 0 and np.all(rg[400 - W:] == 0)
    _check("dg tail", dg[j_first:, h], rg, BWD_MAX, BWD_MEAN, True)
    # rows of weights sum to one: the dv of a kv head add up to the dout of its query heads
    lhs = dv.double().sum(0)
    rhs = dout.double().view(T, Hk, 4, 128).sum((0, 2))
    assert (lhs - rhs).abs().max().item() <= 2e-3 * rhs.abs().max().item()
    # the output sees q and k through q . k only
    for hh in range(Hk):
        a = (q[:, 4 * hh:4 * hh + 4].double() * dq[:, 4 * hh:4 * hh + 4].double()).sum().item()
        b = (k[:, hh].double() * dk[:, hh].double()).sum().item()
        unit = (q[:, 4 * hh:4 * hh + 4].double() * dq[:, 4 * hh:4 * hh + 4].double()).abs().sum().item()
        assert abs(a - b) <= 1e-3 * unit, (hh, a, b, unit)
    assert all(bool(torch.isfinite(x).all()) for x in (out, lse, dq, dk, dv, dg))


def test_backward_is_the_same_on_every_run():
    dev = torch.device("cuda:0")
    q, k, v, g, dout = (x.to(dev) for x in _inputs(7, 700, 2))
    scale = 1 / math.sqrt(128)
    out, lse = wg.soft_attn_forward(q, k, v, g, [700], 64, scale, 1e-6)
    first = wg.soft_attn_backward(q, k, v, g, out, lse, dout, [700], 64, scale, 1e-6)
    again = wg.soft_attn_backward(q, k, v, g, out, lse, dout, [700], 64, scale, 1e-6)
    out2, lse2 = wg.soft_attn_forward(q, k, v, g, [700], 64, scale, 1e-6)
    assert torch.equal(out, out2) and torch.equal(lse, lse2)
    assert all(torch.equal(a, b) for a, b in zip(first, again))


def test_argument_errors_are_reported_before_anything_runs():
    dev = torch.device("cuda:0")
    L = wg.load_library()
    q, k, v, g, dout = (x.to(dev) for x in _inputs(8, 16, 1))
    import ctypes as C
    n = (C.c_int32 * 1)(16)
    p = lambda t: C.c_void_p(t.data_ptr())
    out = torch.zeros((16, 4, 128), device=dev)
    lse = torch.zeros((16, 4), device=dev)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    call = lambda dtype, Hq, Hk, d, W, eps: L.wgkv_soft_attn_forward(dtype, 1, n, Hq, Hk, d, W, p(q), p(k), p(v), p(g),
                                                                     0.1, eps, p(out), p(lse), st)
    assert call(wg.BF16, 4, 1, 128, 8, 1e-6) == 0
    assert call(wg.F32, 4, 1, 128, 8, 1e-6) == -1       # fp32 tensors are not supported
    assert call(wg.BF16, 8, 1, 128, 8, 1e-6) == -1      # eight query heads per kv head
    assert call(wg.BF16, 4, 1, 64, 8, 1e-6) == -1
    assert call(wg.BF16, 4, 1, 128, 0, 1e-6) == -1
    assert call(wg.BF16, 4, 1, 128, 8, -1.0) == -1
    # workspace too small for the backward call
    dq = torch.zeros_like(out); dk = torch.zeros((16, 1, 128), device=dev); dv = torch.zeros_like(dk)
    dg = torch.zeros((16, 1), device=dev); ws = torch.zeros(256, dtype=torch.uint8, device=dev)
    need = L.wgkv_soft_attn_workspace_bytes(16, 4)
    assert need >= 16 * 4 * 4
    rc = L.wgkv_soft_attn_backward(wg.BF16, 1, n, 4, 1, 128, 8, p(q), p(k), p(v), p(g), 0.1, 1e-6, p(out), p(lse),
                                   p(dout), p(dq), p(dk), p(dv), p(dg), p(ws), need - 1, st)
    assert rc == -6
    torch.cuda.synchronize()


@pytest.mark.parametrize("n", [1, 255, 4097, 3_000_001])
def test_sparsity_loss_and_its_gradient(n):
    """Sec. 3.3 sparsity term: fp32 sums of n terms in [0, 1] against fp64 (relative 1e-6), the
    gradient element by element (one multiply-add in fp32), a partial call with a larger
    normaliser, and the same bits on a second run."""
    dev = torch.device("cuda:0")
    cfg = _cfg(20, 1)
    g = torch.from_numpy(wl.draw_scores(cfg, 0, 0, n, wl.unit_rates(cfg))[:, 0].copy())
    loss, dg = wg.sparsity_loss(g.to(dev))
    ref, rdg = oracle_sparsity_loss(g.numpy())
    assert abs(loss.item() - ref) <= 1e-6 * max(ref, 1e-30)
    assert np.abs(dg.cpu().numpy().astype(np.float64) - rdg).max() <= 3e-7 / n
    loss2, none = wg.sparsity_loss(g.to(dev), n_total=4 * n, need_grad=False)
    assert none is None and abs(loss2.item() - ref / 4) <= 1e-6 * max(ref / 4, 1e-30)
    assert torch.equal(wg.sparsity_loss(g.to(dev))[0], loss)
