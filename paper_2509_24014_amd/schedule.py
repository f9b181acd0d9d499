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
    """

    def __init__(self, T: int, skip: float, block_q: int, block_k: int, rho: float, n_dense: Optional[int] = None):
        self.T = int(T)
        self.block_q, self.block_k, self.rho = int(block_q), int(block_k), float(rho)
        self.n_dense = int(n_dense) if n_dense is not None else binding.n_dense_steps(T, skip)
        self.index: Optional[binding.BlockIndex] = None
        self.calls = {"dense": 0, "select": 0, "sparse": 0}
        self._lse = None
        self._workspace = None

    def step(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, t: int, out: Optional[torch.Tensor] = None):
        if t < self.n_dense:
            switch = t == self.n_dense - 1
            if switch and self._lse is None:
                self._lse = torch.empty(q.shape[0], q.shape[1], q.shape[2], dtype=torch.float32, device=q.device)
            out = binding.attn_dense(q, k, v, out=out, lse_out=self._lse if switch else None)
            self.calls["dense"] += 1
            if switch:
                if self._workspace is None:
                    need = binding.select_workspace_bytes(q, self.block_q, self.block_k)
                    self._workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
                self.index = binding.select_pattern(q, k, self.block_q, self.block_k, self.rho, lse_in=self._lse,
                                                    workspace=self._workspace, index=self.index)
                self.calls["select"] += 1
            return out
        if self.index is None:
            raise RuntimeError("sparse step before the pattern was selected")
        out = binding.attn_sparse(q, k, v, self.index, out=out)
        self.calls["sparse"] += 1
        return out
