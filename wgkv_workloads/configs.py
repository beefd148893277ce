"""The five workload shapes, plus scaled-down variants for parity tests.

Model shapes: Llama-3.1-8B (32 layers, 32 query / 8 kv heads, head_dim 128) and
Qwen3-4B-2507 (36 layers, 32/8, 128); local window 256 and 16-token pages are the
paper's operating point (Sec. 4.1; App. D last paragraph).  tau = 0.5 goes with
the synthetic scores; it is only an argument of the calls.
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    index: int              # position in the list of five workloads (seed key)
    batch: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str              # "f32" | "bf16"
    w_local: int
    page_size: int
    tau: float
    ctx_min: int            # context (prefill) length range, inclusive
    ctx_max: int
    decode_steps: int
    rate_law: str           # how per-unit admission rates are drawn
    chunk: int = 0          # chunked prefill: tokens per chunk (0 = whole prompt)
    hidden_dim: int = 0     # linear gate input width (0 = scores are given)

    @property
    def seed(self) -> int:
        return 251217000 + self.index

    def scaled(self, **kw) -> "WorkloadConfig":
        return replace(self, **kw)


CONFIGS = [
    WorkloadConfig("tiny", 0, 1, 1, 8, 2, 64, "f32", 64, 16, 0.5, 512, 512, 16, "uniform_10_40"),
    WorkloadConfig("llama8b_1layer_32k", 1, 1, 1, 32, 8, 128, "bf16", 256, 16, 0.5, 32768, 32768,
                   128, "beta_2_8"),
    WorkloadConfig("llama8b_32layer_b8_128k", 2, 8, 32, 32, 8, 128, "bf16", 256, 16, 0.5, 65536,
                   131072, 256, "beta_1p5_8"),
    WorkloadConfig("qwen3_4b_36layer_b32_64k", 3, 32, 36, 32, 8, 128, "bf16", 128, 32, 0.5, 65536,
                   65536, 128, "ragged_mix"),
    WorkloadConfig("llama8b_chunked_prefill_128k", 4, 4, 1, 32, 8, 128, "bf16", 256, 16, 0.5,
                   131072, 131072, 0, "linear_gate", chunk=4096, hidden_dim=4096),
]


def get_config(name_or_index) -> WorkloadConfig:
    if isinstance(name_or_index, int):
        return CONFIGS[name_or_index]
    for c in CONFIGS:
        if c.name == name_or_index:
            return c
    raise KeyError(name_or_index)
