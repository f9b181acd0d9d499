"""The five named workload configurations (shapes, blocks, rho, schedule)."""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    config_id: int
    B: int
    Hq: int
    Hkv: int
    L: int
    d: int
    dtype: str            # "bf16" or "f32"
    bq: int               # query-block rows
    bk: int               # key-block columns
    rho: float            # kept fraction of key blocks per query block
    T: int                # denoising steps in the schedule (1 = single calls)
    n_dense: int          # steps run with full attention (selection at the last of them)
    sigma: float          # per-step random-walk std on Q, K, V
    planted: bool         # head-specific planted structure (False: plain N(0,1), no 1/sqrt(d))

    @property
    def nqb(self) -> int:
        return self.L // self.bq

    @property
    def nkb(self) -> int:
        return self.L // self.bk

    def scaled(self, **kw) -> "WorkloadConfig":
        """Same recipe at other sizes (used by tests to shrink a config)."""
        return replace(self, **kw)


CONFIGS = {
    # Tiny fp32 case the oracle finishes instantly: 1 dense step (selection on it), 4 sparse steps.
    "tiny": WorkloadConfig("tiny", 1, 1, 2, 2, 256, 64, "f32", 32, 32, 0.3, 5, 1, 0.05, False),
    # LLaDA-8B-shaped single layer.
    "llada4k": WorkloadConfig("llada4k", 2, 1, 32, 32, 4096, 128, "bf16", 64, 64, 0.2, 1, 1, 0.0, True),
    # Same generator at 16k with a 64-step schedule: 8 dense, select once, 56 sparse.
    "llada16k": WorkloadConfig("llada16k", 3, 1, 32, 32, 16384, 128, "bf16", 64, 64, 0.1, 64, 8, 0.05, True),
    # Dream-7B-shaped GQA layer: 28 query heads over 4 KV heads.
    "dream32k": WorkloadConfig("dream32k", 4, 1, 28, 4, 32768, 128, "bf16", 128, 64, 0.1, 1, 1, 0.0, True),
    # Long-context schedule: 1024 steps, dense for the first 20 %.
    "long64k": WorkloadConfig("long64k", 5, 1, 32, 32, 65536, 128, "bf16", 128, 64, 0.05, 1024, 205, 0.02, True),
    # Not one of the five named workloads: a short-running shape (same head dim, blocks and generator as
    # the long-context one) for hardware-counter runs, whose 32-bit counters saturate on longer kernels.
    "probe8k": WorkloadConfig("probe8k", 6, 1, 8, 8, 8192, 128, "bf16", 128, 64, 0.1, 1, 1, 0.0, True),
    # Not one of the five named workloads: the long-context shape (same length, blocks and rho, so every work-group
    # does exactly what it does there) cut to four heads, one of each planted type, so that one sparse-attention
    # launch is short enough for hardware-counter runs.
    "probe64k": WorkloadConfig("probe64k", 9, 1, 4, 4, 65536, 128, "bf16", 128, 64, 0.05, 1, 1, 0.0, True),
    # The paper's own long-context setting (Section 4.1: square blocks of 128, rho = 30 %, skip = 20 %) on the
    # long-context shape: not one of the five named workloads, used for one parity test and one line of measurements.
    "paper64k": WorkloadConfig("paper64k", 8, 1, 32, 32, 65536, 128, "bf16", 128, 128, 0.3, 1024, 205, 0.02, True),
    # Not one of the five named workloads either: twice the longest context the paper runs, four heads (one of
    # each planted type), used by one parity test to show that nothing in the path stops at 64k.
    "probe128k": WorkloadConfig("probe128k", 7, 1, 4, 4, 131072, 128, "bf16", 128, 64, 0.05, 1, 1, 0.0, True),
}


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name]
