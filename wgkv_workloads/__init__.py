"""Seeded synthetic inputs and workload shapes shared by the tests, the smoke
check and the benchmark.  Holds no arithmetic of the method itself: only random
draws with the shapes, dtypes and admission-rate structure of the workloads."""
from .configs import WorkloadConfig, CONFIGS, get_config  # noqa: F401
from .generators import (unit_rates, score_shape_b, draw_scores, draw_normal, context_lengths,  # noqa: F401
                         draw_linear_gate, draw_gate_mlp)
