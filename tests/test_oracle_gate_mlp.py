"""Pins of the oracle's Write-Gate MLP (Sec. 3.2, feature and gate equations) against
things that are not the oracle: library RMSNorm / GELU / sigmoid routines in fp64,
tabulated values of the normal distribution, invariances of RMSNorm, and a
hand-computed bfloat16 rounding."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import gate_mlp

# standard normal CDF, tabulated: GELU(z) = z * Phi(z)
PHI = {0.5: 0.6914624612740131, 1.0: 0.8413447460685429, 2.0: 0.9772498680518208}


def _weights(seed, Hk, d, width, scale=0.3):
    r = np.random.default_rng(seed)
    W1 = (r.standard_normal((Hk, width, 2 * d)) * scale).astype(np.float32)
    b1 = (r.standard_normal((Hk, width)) * 0.2).astype(np.float32)
    W2 = (r.standard_normal((Hk, width)) * 0.5).astype(np.float32)
    b2 = r.standard_normal((Hk,)).astype(np.float32)
    return W1, b1, W2, b2


def _library(k, kr, W1, b1, W2, b2, eps):
    """The same composition from torch's own routines, fp64."""
    d = k.shape[-1]
    kt, krt = torch.from_numpy(k).double(), torch.from_numpy(kr).double()
    x = torch.cat([F.rms_norm(kt, (d,), eps=eps), F.rms_norm(krt, (d,), eps=eps)], dim=-1)   # [T, H, 2d]
    h = torch.einsum("hue,the->thu", torch.from_numpy(W1).double(), x) + torch.from_numpy(b1).double()
    logit = (F.gelu(h, approximate="none") * torch.from_numpy(W2).double()).sum(-1) + torch.from_numpy(b2).double()
    return logit.numpy(), torch.sigmoid(logit).numpy()


def test_matches_library_routines():
    for seed, (T, Hk, d, width, eps) in enumerate([(7, 2, 8, 16, 1e-6), (5, 3, 64, 40, 1e-5), (3, 8, 128, 96, 0.0)]):
        r = np.random.default_rng(100 + seed)
        k = r.standard_normal((T, Hk, d)).astype(np.float32) * 2.0
        kr = r.standard_normal((T, Hk, d)).astype(np.float32) * 0.5
        W = _weights(seed, Hk, d, width)
        lo, g = gate_mlp(k, kr, *W, eps=eps)
        lo_ref, g_ref = _library(k, kr, *W, eps)
        assert np.abs(lo - lo_ref).max() < 1e-12
        assert np.abs(g - g_ref).max() < 1e-13


def test_constant_keys_give_tabulated_normal_values():
    # RMSNorm of a constant vector is its sign; unit-selecting rows of W1 then make the
    # hidden pre-activations +1 (from k) and -1 (from k_rope): logit = w_a*Phi(1) - w_b*(1-Phi(1))
    d, width = 4, 2
    k = np.full((1, 1, d), 3.0, np.float32)
    kr = np.full((1, 1, d), -2.0, np.float32)
    W1 = np.zeros((1, width, 2 * d), np.float32)
    W1[0, 0, 0] = 1.0          # first feature of the k half
    W1[0, 1, d] = 1.0          # first feature of the k_rope half
    b1 = np.zeros((1, width), np.float32)
    W2 = np.array([[1.0, 2.0]], np.float32)
    b2 = np.zeros((1,), np.float32)
    lo, g = gate_mlp(k, kr, W1, b1, W2, b2, eps=0.0)
    want = 1.0 * PHI[1.0] - 2.0 * (1.0 - PHI[1.0])
    assert abs(lo[0, 0] - want) < 1e-12
    assert abs(g[0, 0] - 1.0 / (1.0 + math.exp(-want))) < 1e-14
    # symmetric output weights: P(|Z| < 1)
    lo2, _ = gate_mlp(k, kr, W1, b1, np.array([[1.0, 1.0]], np.float32), b2, eps=0.0)
    assert abs(lo2[0, 0] - 0.6826894921370859) < 1e-12


def test_zero_first_layer_leaves_bias_path_and_exact_gelu():
    # W1 = 0: g = sigmoid(sum_u W2_u GELU(b1_u) + b2) whatever the keys are.  The exact
    # GELU(2) is 2 Phi(2) = 1.95449974; the tanh approximation would give 1.95459769.
    Hk, d, width = 2, 16, 3
    r = np.random.default_rng(3)
    k = r.standard_normal((4, Hk, d)).astype(np.float32)
    kr = r.standard_normal((4, Hk, d)).astype(np.float32)
    W1 = np.zeros((Hk, width, 2 * d), np.float32)
    b1 = np.array([[0.5, 1.0, 2.0], [0.0, -1.0, 2.0]], np.float32)
    W2 = np.array([[1.0, -1.0, 0.5], [3.0, 1.0, 1.0]], np.float32)
    b2 = np.array([0.25, -0.5], np.float32)
    lo, g = gate_mlp(k, kr, W1, b1, W2, b2)
    want0 = 0.5 * PHI[0.5] - 1.0 * PHI[1.0] + 0.5 * 2.0 * PHI[2.0] + 0.25
    want1 = 0.0 + (-1.0) * (1.0 - PHI[1.0]) + 2.0 * PHI[2.0] - 0.5
    assert np.abs(lo[:, 0] - want0).max() < 1e-12
    assert np.abs(lo[:, 1] - want1).max() < 1e-12
    assert np.abs(g[:, 1] - 1.0 / (1.0 + math.exp(-want1))).max() < 1e-14


def test_rmsnorm_scale_invariance_and_eps_placement():
    Hk, d, width = 2, 32, 24
    r = np.random.default_rng(11)
    k = r.standard_normal((6, Hk, d)).astype(np.float32)
    kr = r.standard_normal((6, Hk, d)).astype(np.float32)
    W = _weights(5, Hk, d, width)
    lo, _ = gate_mlp(k, kr, *W, eps=0.0)
    # powers of two keep the float inputs exact; each half is normalised on its own
    lo_s, _ = gate_mlp(k * 4.0, kr * 0.125, *W, eps=0.0)
    assert np.abs(lo - lo_s).max() < 1e-12
    # eps is added to the MEAN of squares under the root: a constant vector of 1e-3 with
    # eps = 1e-6 has mean square 1e-6, so it is normalised to 1/sqrt(2)
    kc = np.full((1, 1, 4), 1e-3, np.float32)
    W1 = np.zeros((1, 1, 8), np.float32)
    W1[0, 0, 0] = 32.0         # 32/sqrt(2) = 22.6: far in the region where GELU(z) = z
    b1 = np.zeros((1, 1), np.float32)
    lo_e, _ = gate_mlp(kc, kc, W1, b1, np.ones((1, 1), np.float32), np.zeros((1,), np.float32), eps=1e-6)
    kc64 = float(np.float32(1e-3))
    assert abs(lo_e[0, 0] - 32.0 * kc64 / math.sqrt(kc64 * kc64 + 1e-6)) < 1e-9


def test_heads_and_tokens_are_independent():
    Hk, d, width = 3, 16, 8
    r = np.random.default_rng(21)
    k = r.standard_normal((5, Hk, d)).astype(np.float32)
    kr = r.standard_normal((5, Hk, d)).astype(np.float32)
    W1, b1, W2, b2 = _weights(9, Hk, d, width)
    lo, _ = gate_mlp(k, kr, W1, b1, W2, b2)
    W1b, k2 = W1.copy(), k.copy()
    W1b[1] *= -2.0             # another gate for head 1
    k2[3] += 1.0               # another token 3
    lo_b, _ = gate_mlp(k2, kr, W1b, b1, W2, b2)
    same = np.ones_like(lo, dtype=bool)
    same[:, 1] = False
    same[3, :] = False
    assert np.array_equal(lo[same], lo_b[same])
    assert not np.any(lo[~same] == lo_b[~same])
    # a permutation of the heads permutes the scores
    perm = [2, 0, 1]
    lo_p, _ = gate_mlp(k[:, perm], kr[:, perm], W1[perm], b1[perm], W2[perm], b2[perm])
    assert np.array_equal(lo_p, lo[:, perm])


def test_bf16_feature_rounding_by_hand():
    # k = (1, 3): mean square 5, normalised (0.44721360, 1.34164079); the nearest bfloat16
    # values are 0.447265625 (= 229/512) and 1.34375 (= 172/128).  W1 = 32 e_j puts the
    # pre-activation where GELU(z) = z to double precision, so the logit shows the feature.
    k = np.array([[[1.0, 3.0]]], np.float32)
    W1 = np.zeros((1, 2, 4), np.float32)
    W1[0, 0, 0] = 32.0
    W1[0, 1, 1] = 32.0
    b1 = np.zeros((1, 2), np.float32)
    b2 = np.zeros((1,), np.float32)
    for W2, exact, rounded in [([1 / 32, 0.0], 1.0 / math.sqrt(5.0), 0.447265625),
                               ([0.0, 1 / 32], 3.0 / math.sqrt(5.0), 1.34375)]:
        W2 = np.array([W2], np.float32)
        lo, _ = gate_mlp(k, k, W1, b1, W2, b2, eps=0.0, feature_bf16=False)
        assert abs(lo[0, 0] - exact) < 1e-12
        lo_r, _ = gate_mlp(k, k, W1, b1, W2, b2, eps=0.0, feature_bf16=True)
        assert lo_r[0, 0] == rounded
