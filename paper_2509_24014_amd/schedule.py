"""Step controller of one attention layer (Algorithm 1): dense early, select once, sparse after.

Control flow only; every attention and selection call goes through the C ABI.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding


class SparseDLayer:
    """Holds the one piece of state SparseD carries across denoising steps: the block index.

    ``step(q, k, v, t)`` runs step ``t`` (0-based) of a ``T``-step schedule:
    steps ``0 .. n_dense-1`` use full attention; at step ``n_dense-1`` the pattern is selected
    from that step's Q, K (reusing the dense call's row log-sum-exp); steps ``>= n_dense`` use
    sparse attention with the stored pattern.

    Two switches reproduce the paper's ablation rows (Table 2) on the same kernels:
    ``n_dense=0`` is "without skipping" (the pattern is selected from step 0's Q, K and used from
    step 0 on), ``reselect_every_step=True`` is "without sparse reusing" (every sparse step first
    re-selects its pattern from its own Q, K).
    """

    def __init__(self, T: int, skip: float, block_q: int, block_k: int, rho: float, n_dense: Optional[int] = None,
                 reselect_every_step: bool = False):
        self.T = int(T)
        self.block_q, self.block_k, self.rho = int(block_q), int(block_k), float(rho)
        self.n_dense = int(n_dense) if n_dense is not None else binding.n_dense_steps(T, skip)
        self.reselect_every_step = bool(reselect_every_step)
        self.index: Optional[binding.BlockIndex] = None
        self.calls = {"dense": 0, "select": 0, "sparse": 0}
        self._lse = None
        self._workspace = None

    def _select(self, q, k, lse):
        if self._workspace is None:
            need = binding.select_workspace_bytes(q, self.block_q, self.block_k)
            self._workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        self.index = binding.select_pattern(q, k, self.block_q, self.block_k, self.rho, lse_in=lse,
                                            workspace=self._workspace, index=self.index)
        self.calls["select"] += 1

    def step(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, t: int, out: Optional[torch.Tensor] = None):
        if t >= self.n_dense and (self.reselect_every_step or self.index is None):
            if self.index is None and self.n_dense > 0:
                raise RuntimeError("sparse step before the pattern was selected")
            self._select(q, k, None)  # no dense call at this step: selection runs its own statistics pass
        if t < self.n_dense:
            switch = t == self.n_dense - 1
            if switch and self._lse is None:
                self._lse = torch.empty(q.shape[0], q.shape[1], q.shape[2], dtype=torch.float32, device=q.device)
            out = binding.attn_dense(q, k, v, out=out, lse_out=self._lse if switch else None)
            self.calls["dense"] += 1
            if switch:
                self._select(q, k, self._lse)
            return out
        out = binding.attn_sparse(q, k, v, self.index, out=out)
        self.calls["sparse"] += 1
        return out
