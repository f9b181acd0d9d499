"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the HIP path and the CPU oracle and holds none of the
method's arithmetic: it only draws Q, K, V. The paper's latency workload is one
long-context sample run through LLaDA-1.5 / Dream-7B-Instruct (Section 4.1,
"Implementation Details"); neither the dataset nor the weights are available, so
these tensors stand in for one attention layer's Q, K, V: the models' head shapes,
the paper's context lengths and step counts, and planted per-head structure that
imitates the head-specific patterns the paper shows (column-wise, sliding-window,
mixed; Section 3.2, Figure 1).
"""
from .configs import CONFIGS, WorkloadConfig, get_config  # noqa: F401
from .generator import StepInputs, make_inputs  # noqa: F401
