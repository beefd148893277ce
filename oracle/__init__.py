"""CPU oracle for the Write-Gated KV hot path -- TEST INFRASTRUCTURE ONLY.

Nothing in the product package may import this.  See wgkv_oracle.c for what it
computes and which passages of the paper each part follows.
"""
from .wgkv_oracle import Oracle, OracleConfig, attend_definition, attend_soft, gate_mlp, linear_gate, quest_select, soft_attn_backward, soft_attn_backward_sampled, soft_attn_forward, sparsity_loss  # noqa: F401
