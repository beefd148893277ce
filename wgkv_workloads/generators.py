"""Seeded random inputs.  Every stream is keyed by (config seed, purpose,
sequence, layer, step) so that any slice of a workload can be regenerated alone.

Scores: a unit (layer, kv head) with target admission rate r at threshold tau
draws g = 1 - (1 - u)^(1/b), u ~ U(0,1), b = log(r) / log(1 - tau).  That is a
Beta(1, b) variable and P(g >= tau) = (1 - tau)^b = r.  The scores are produced
once, as fp32, and the same bytes are handed to every consumer.
"""
import math

import numpy as np
import torch

from .configs import WorkloadConfig

_PURPOSE = {"rates": 1, "scores": 2, "k": 3, "v": 4, "q": 5, "ctx": 6, "gate_w": 7, "hidden": 8,
            "dec_scores": 9, "dec_k": 10, "dec_v": 11, "k_pre": 12, "k_rope": 13, "mlp_w1": 14, "mlp_b1": 15,
            "mlp_w2": 16, "mlp_b2": 17, "dout": 18}


def _rng(cfg: WorkloadConfig, purpose: str, *key) -> np.random.Generator:
    words = [cfg.seed, _PURPOSE[purpose]] + [int(x) for x in key]
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(words)))


def _torch_seed(cfg: WorkloadConfig, purpose: str, *key) -> int:
    ss = np.random.SeedSequence([cfg.seed, _PURPOSE[purpose]] + [int(x) for x in key])
    return int(ss.generate_state(1, dtype=np.uint64)[0] & np.uint64(0x7FFFFFFFFFFFFFFF))


def context_lengths(cfg: WorkloadConfig) -> np.ndarray:
    """Prompt length of every sequence of the batch, uniform in [ctx_min, ctx_max]."""
    r = _rng(cfg, "ctx")
    return r.integers(cfg.ctx_min, cfg.ctx_max + 1, size=cfg.batch).astype(np.int64)


def unit_rates(cfg: WorkloadConfig) -> np.ndarray:
    """Target admission rate of every (layer, kv head), shared by the batch."""
    r = _rng(cfg, "rates")
    shape = (cfg.n_layers, cfg.n_kv_heads)
    if cfg.rate_law == "uniform_10_40":
        out = r.uniform(0.10, 0.40, size=shape)
    elif cfg.rate_law == "beta_2_8":
        out = r.beta(2.0, 8.0, size=shape)
    elif cfg.rate_law == "beta_1p5_8":
        out = r.beta(1.5, 8.0, size=shape)
    elif cfg.rate_law == "ragged_mix":
        # 5 % of heads near-dense, 20 % near-empty, the rest so that the mean is 0.10
        u = r.uniform(size=shape)
        out = np.full(shape, (0.10 - 0.05 * 0.9 - 0.20 * 0.01) / 0.75)
        out[u < 0.05] = 0.9
        out[(u >= 0.05) & (u < 0.25)] = 0.01
    elif cfg.rate_law == "linear_gate":
        out = np.full(shape, 0.5)
    else:
        raise ValueError(cfg.rate_law)
    return np.clip(out, 1e-4, 1.0 - 1e-4)


def score_shape_b(rate: np.ndarray, tau: float) -> np.ndarray:
    return np.log(rate) / math.log(1.0 - tau)


def draw_scores(cfg: WorkloadConfig, seq: int, layer: int, n_tokens: int, rates: np.ndarray,
                purpose: str = "scores", step: int = 0, device=None):
    """fp32 scores [n_tokens, n_kv_heads] of one (sequence, layer).

    device=None: numpy Philox stream, returns a numpy array.  With a torch device the
    uniforms come from a torch generator seeded with the same key and a torch tensor
    on that device is returned (a different but equally reproducible stream; whoever
    needs the scores on both sides copies these bytes)."""
    b = score_shape_b(rates[layer], cfg.tau)
    if device is None:
        r = _rng(cfg, purpose, seq, layer, step)
        u = r.random(size=(n_tokens, cfg.n_kv_heads), dtype=np.float64)
        g = 1.0 - np.power(1.0 - u, 1.0 / b[None, :])
        return np.ascontiguousarray(np.clip(g, 0.0, 1.0).astype(np.float32))
    gen = torch.Generator(device=device)
    gen.manual_seed(_torch_seed(cfg, purpose, seq, layer, step))
    u = torch.rand((n_tokens, cfg.n_kv_heads), generator=gen, device=device, dtype=torch.float64)
    inv_b = torch.as_tensor(1.0 / b, dtype=torch.float64, device=device)[None, :]
    g = 1.0 - torch.pow(1.0 - u, inv_b)
    return g.clamp_(0.0, 1.0).to(torch.float32).contiguous()


def torch_dtype(cfg: WorkloadConfig):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def draw_normal(cfg: WorkloadConfig, purpose: str, shape, device="cpu", key=(), std: float = 1.0,
                dtype=None) -> torch.Tensor:
    """N(0, std^2) tensor rounded to the workload dtype, drawn on `device`.
    (A tensor drawn on the GPU differs from one drawn on the CPU with the same
    key; whoever needs both sides copies the bytes.)"""
    gen = torch.Generator(device=device)
    gen.manual_seed(_torch_seed(cfg, purpose, *key))
    x = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    if std != 1.0:
        x = x * std
    return x.to(dtype or torch_dtype(cfg))


def draw_linear_gate(cfg: WorkloadConfig, device="cpu") -> torch.Tensor:
    """Random-init per-kv-head linear gate weights ~ N(0, 0.02), [n_kv_heads, hidden_dim]."""
    return draw_normal(cfg, "gate_w", (cfg.n_kv_heads, cfg.hidden_dim), device=device, std=0.02)


def draw_gate_mlp(cfg: WorkloadConfig, width: int, device="cpu"):
    """Random-init Write-Gate MLP parameters for every kv head: W1 [Hkv, width, 2d] ~ N(0, 1/(2d)),
    b1 [Hkv, width] ~ N(0, 0.25), W2 [Hkv, width] ~ N(0, 4/width) in the workload dtype (biases fp32),
    b2 [Hkv] ~ N(0, 1): hidden pre-activations and logits of order one, so the scores spread over (0, 1)."""
    Hk, d = cfg.n_kv_heads, cfg.head_dim
    w1 = draw_normal(cfg, "mlp_w1", (Hk, width, 2 * d), device=device, std=(2 * d) ** -0.5)
    b1 = draw_normal(cfg, "mlp_b1", (Hk, width), device=device, std=0.5, dtype=torch.float32)
    w2 = draw_normal(cfg, "mlp_w2", (Hk, width), device=device, std=2.0 * width ** -0.5)
    b2 = draw_normal(cfg, "mlp_b2", (Hk,), device=device, std=1.0, dtype=torch.float32)
    return w1, b1, w2, b2
