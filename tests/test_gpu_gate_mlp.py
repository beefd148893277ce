"""Write-Gate MLP kernel (Sec. 3.2 feature and gate equations) against the fp64 oracle,
through the C ABI: matrix-core path (bf16, head_dim 64/128, width % 32 == 0), the plain
path (fp32 or other shapes), ragged token counts, the admission decisions that the scores
lead to, and the shape of the chunked-prefill workload."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2512_17452_amd as wg
import wgkv_workloads as wl
from oracle import Oracle, OracleConfig, gate_mlp

pytestmark = pytest.mark.gpu
# bf16 path: both sides round the normalised features to bf16; what is left is fp32 accumulation
# of 2d products (order differs from fp64: ~1e-6 relative), fp32 erf/exp (~1e-7), and the rare
# feature whose fp32 normalisation falls on the other side of a bf16 rounding boundary (each
# moves one pre-activation by ~|w| 2^-8 ~ 2e-4 and the logit by ~1e-5).  Scores are in (0, 1).
TOL_BF16 = 2e-4
TOL_F32 = 2e-5


def _inputs(dtype, T, Hk, d, width, seed):
    cfg = wl.WorkloadConfig(f"gate_mlp_{seed}", 900 + seed, 1, 1, Hk * 4, Hk, d, "bf16" if dtype == torch.bfloat16 else "f32",
                            8, 4, 0.5, T, T, 0, "mlp_gate")
    k = wl.draw_normal(cfg, "k_pre", (T, Hk, d), std=1.5)
    kr = wl.draw_normal(cfg, "k_rope", (T, Hk, d), std=0.7)   # stands in for the rotated keys: any tensor of that shape
    w1, b1, w2, b2 = wl.draw_gate_mlp(cfg, width)
    return k, kr, w1, b1, w2, b2


def _oracle(k, kr, w1, b1, w2, b2, eps, bf16):
    f = lambda x: x.float().numpy()
    return gate_mlp(f(k), f(kr), f(w1), f(b1), f(w2), f(b2), eps=eps, feature_bf16=bf16)


@pytest.mark.parametrize("dtype,T,Hk,d,width,eps", [
    (torch.bfloat16, 1000, 8, 128, 512, 1e-6),    # matrix cores: several blocks and a ragged tail
    (torch.bfloat16, 129, 4, 64, 96, 1e-5),       # matrix cores, head_dim 64
    (torch.bfloat16, 1, 8, 128, 32, 1e-6),
    (torch.bfloat16, 37, 3, 32, 48, 1e-6),        # plain kernel, bf16
    (torch.bfloat16, 20, 2, 128, 40, 1e-6),       # width not a multiple of 32: plain kernel
    (torch.float32, 65, 8, 64, 40, 1e-6),         # plain kernel, fp32
    (torch.float32, 9, 2, 128, 512, 0.0),
])
def test_gate_mlp_scores_match_fp64(dtype, T, Hk, d, width, eps):
    dev = torch.device("cuda:0")
    ins = _inputs(dtype, T, Hk, d, width, T + width)
    g = wg.gate_mlp_scores(*[x.to(dev) for x in ins], eps=eps).cpu().numpy()
    logit, ref = _oracle(*ins, eps, dtype == torch.bfloat16)
    tol = TOL_BF16 if dtype == torch.bfloat16 else TOL_F32
    assert g.shape == (T, Hk) and np.isfinite(g).all()
    assert np.abs(g - ref).max() <= tol, np.abs(g - ref).max()
    assert 0.05 < ref.mean() < 0.95 and ref.std() > 0.1       # the recipe really spreads the scores
    # admission decisions agree with the fp64 ones wherever the score is not within the tolerance of tau
    for tau in (0.1, 0.5):
        far = np.abs(ref - tau) > tol
        assert np.array_equal((g >= tau)[far], (ref >= tau)[far])


def test_gate_mlp_empty_and_bad_arguments():
    dev = torch.device("cuda:0")
    k, kr, w1, b1, w2, b2 = [x.to(dev) for x in _inputs(torch.bfloat16, 8, 2, 128, 64, 5)]
    out = wg.gate_mlp_scores(k[:0], kr[:0], w1, b1, w2, b2)
    assert out.shape == (0, 2)
    with pytest.raises(wg.WgkvError):
        wg.gate_mlp_scores(k, kr, w1, b1, w2, b2, eps=-1.0)
    L = wg.load_library()
    p = lambda t: C.c_void_p(t.data_ptr())
    g = torch.empty((8, 2), dtype=torch.float32, device=dev)
    # a key pointer that is not 16-byte aligned is refused before anything is launched
    rc = L.wgkv_gate_mlp_scores(wg.BF16, 7, 2, 128, 64, C.c_void_p(k.data_ptr() + 2), p(kr), p(w1), p(b1), p(w2), p(b2),
                                1e-6, p(g), None)
    assert rc == -1
    rc = L.wgkv_gate_mlp_scores(wg.BF16, 8, 2, 128, 0, p(k), p(kr), p(w1), p(b1), p(w2), p(b2), 1e-6, p(g), None)
    assert rc == -1


def test_gate_mlp_feeds_admission():
    """Scores of the MLP drive wgkv_prefill_admit; the cache state equals the oracle's, which is
    fed the fp64 scores, provided no score lies within the tolerance of tau (asserted)."""
    dev = torch.device("cuda:0")
    T, Hq, Hk, d, width, W, P = 700, 32, 8, 128, 256, 64, 16
    k, kr, w1, b1, w2, b2 = _inputs(torch.bfloat16, T, Hk, d, width, 77)
    v = wl.draw_normal(wl.WorkloadConfig("gate_mlp_v", 977, 1, 1, Hq, Hk, d, "bf16", W, P, 0.35, T, T, 0, "mlp_gate"),
                       "v", (T, Hk, d))
    _, ref = _oracle(k, kr, w1, b1, w2, b2, 1e-6, True)
    # tau: the middle of the gap between fp64 scores that is wide enough and closest to 0.35
    srt = np.sort(ref.ravel())
    gaps = np.nonzero(np.diff(srt) > 4 * TOL_BF16)[0]
    mids = 0.5 * (srt[gaps] + srt[gaps + 1])
    tau = float(np.float32(mids[np.argmin(np.abs(mids - 0.35))]))
    assert 0.3 < tau < 0.4 and np.abs(ref - tau).min() > TOL_BF16
    max_gp = T // P + 2
    n_pages = Hk * (max_gp + W // P + 1) + 8
    pool = wg.Pool(wg.Config(1, Hq, Hk, d, wg.BF16, P, W, 1, max_gp, n_pages), 1, T)
    g = wg.gate_mlp_scores(*[x.to(dev) for x in (k, kr, w1, b1, w2, b2)])
    pool.prefill_admit(0, [0], [T], kr.to(dev), v.to(dev), g, tau=tau)     # the rotated keys are what is cached
    free, flag = pool.status()
    assert flag == 0
    orc = Oracle(OracleConfig(1, Hq, Hk, d, P, W, 1, max_gp, n_pages, False))
    orc.push_tokens(0, [0], [T], None, None, ref.astype(np.float32), tau)
    meta = pool.meta()
    gl = meta["global_len"].cpu().numpy()[0, 0]
    assert [orc.global_len(0, 0, h) for h in range(Hk)] == gl.tolist()
    assert free == orc.free_top
    assert 0.2 < gl.mean() / (T - W) < 0.95


def test_gate_mlp_chunk_of_the_prefill_workload():
    """Shape of one chunk of the chunked-prefill workload (4 x 4096 tokens, 8 kv heads, d 128, width 512);
    the oracle checks a sample of the tokens, all heads."""
    dev = torch.device("cuda:0")
    cfg = wl.get_config(4)
    T, Hk, d, width = cfg.batch * cfg.chunk, cfg.n_kv_heads, cfg.head_dim, 4 * cfg.head_dim
    k = wl.draw_normal(cfg, "k_pre", (T, Hk, d), device=dev, std=1.5)
    kr = wl.draw_normal(cfg, "k_rope", (T, Hk, d), device=dev, std=0.7)
    w1, b1, w2, b2 = wl.draw_gate_mlp(cfg, width, device=dev)
    g = wg.gate_mlp_scores(k, kr, w1, b1, w2, b2).cpu().numpy()
    assert np.isfinite(g).all()
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 31, 32, 127, 128, T - 129, T - 1], rng.integers(0, T, 1500)]))
    _, ref = _oracle(k[rows].cpu(), kr[rows].cpu(), w1.cpu(), b1.cpu(), w2.cpu(), b2.cpu(), 1e-6, True)
    assert np.abs(g[rows] - ref).max() <= TOL_BF16
