"""Algorithm 1 (SparseD step controller) on top of the fp64 oracle. Test infrastructure.

Reading of the step rule (Section 3.3 "Skipping Sparse", Algorithm 1): steps are
numbered from 0; the first ``n_dense = clamp(ceil(T*skip - 1e-9), 1, T)`` steps run
full attention; at the last of them the pattern is selected from that step's Q, K;
every later step runs sparse attention with that one stored pattern ("Sparse
Reusing").
"""
from __future__ import annotations

import math

import oracle


def n_dense_steps(T: int, skip: float) -> int:
    """Number of full-attention steps out of T for a skip fraction."""
    n = int(math.ceil(T * skip - 1e-9))
    return max(1, min(T, n))


def run(inputs_at_step, T: int, n_dense: int, bq: int, bk: int, rho: float, steps_to_keep=None):
    """Run T steps of Algorithm 1.

    ``inputs_at_step(t) -> (q, k, v)`` supplies the step's tensors. Returns a dict with
    ``outputs`` (step -> float64 output, only for steps in ``steps_to_keep`` or all),
    ``index`` (row_ptr, col_idx), ``calls`` (counts of dense / select / sparse).
    """
    outputs = {}
    index = None
    calls = {"dense": 0, "select": 0, "sparse": 0}
    for t in range(T):
        q, k, v = inputs_at_step(t)
        if t < n_dense:
            out = oracle.attn_dense(q, k, v) if (steps_to_keep is None or t in steps_to_keep) else None
            calls["dense"] += 1
            if t == n_dense - 1:
                row_ptr, col_idx, _, _ = oracle.select_pattern(q, k, bq, bk, rho)
                index = (row_ptr, col_idx)
                calls["select"] += 1
        else:
            out = (oracle.attn_sparse(q, k, v, index[0], index[1], bq, bk)
                   if (steps_to_keep is None or t in steps_to_keep) else None)
            calls["sparse"] += 1
        if out is not None:
            outputs[t] = out
    return {"outputs": outputs, "index": index, "calls": calls}
