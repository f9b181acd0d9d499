"""Seeded Q, K, V generator with planted head-specific structure and per-step drift.

Recipe (all draws from one ``torch.Generator`` seeded ``seed + 1000*config_id`` on the
chosen device; fp32 masters, rounded to the config's dtype on request):

* base: ``Q, K = randn / sqrt(d)``, ``V = randn``  (un-planted configs: plain ``randn`` for all three);
* head type ``h mod 4`` (query-head index), planted terms in disjoint feature ranges so one
  KV head can carry every type under grouped-query attention:
    0 window   dims 0..15  : ``3*sin / 3*cos`` position features at 8 wavelengths
                             ``1024 * 2**(m/2)`` added to Q and K  (locality of a few hundred tokens)
    1 stripe   dims 16..63 : a direction ``u`` of norm 3; ``K[j] += 4u`` on the first 64 keys and 8
                             random later keys, ``Q[i] += u`` on every query  (column-wise pattern)
    2 segment  dims 64..127: per 512-token segment a direction of norm 3 added to that segment's
                             Q and K  (block-diagonal pattern)
    3 random               : nothing planted
  With as many KV heads as query heads, K of head h gets only h's own term; with fewer KV heads,
  K of a KV head gets all three terms and each query head only its own.
* drift between denoising steps: a random walk on the masters, ``X_t = X_{t-1} + sigma*randn``,
  drawn from a generator seeded ``seed + 1000*config_id + 1 + t``.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

from .configs import WorkloadConfig

_SEGMENT = 512
_WINDOW_DIMS = (0, 16)
_STRIPE_DIMS = (16, 64)
_SEGMENT_DIMS = (64, 128)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _unit_rows(n: int, width: int, norm: float, g: torch.Generator, device) -> torch.Tensor:
    x = torch.randn(n, width, generator=g, device=device, dtype=torch.float32)
    return x * (norm / x.norm(dim=-1, keepdim=True))


@dataclass
class StepInputs:
    """fp32 masters of one layer's Q, K, V plus the recipe to step them forward."""

    cfg: WorkloadConfig
    seed: int
    q: torch.Tensor  # [B, Hq, L, d] fp32
    k: torch.Tensor  # [B, Hkv, L, d] fp32
    v: torch.Tensor  # [B, Hkv, L, d] fp32
    step: int = 0

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.cfg.dtype == "bf16" else torch.float32

    def rounded(self):
        """Q, K, V in the config's dtype: exactly what both the HIP path and the oracle consume."""
        dt = self.torch_dtype
        return self.q.to(dt), self.k.to(dt), self.v.to(dt)

    def advance(self) -> None:
        """One denoising step of drift: X += sigma * randn on each of Q, K, V."""
        self.step += 1
        if self.cfg.sigma == 0.0:
            return
        g = _gen(self.q.device, self.seed + 1000 * self.cfg.config_id + 1 + self.step)
        for x in (self.q, self.k, self.v):
            x.add_(torch.randn(x.shape, generator=g, device=x.device, dtype=torch.float32), alpha=self.cfg.sigma)


def make_inputs(cfg: WorkloadConfig, seed: int = 0, device="cpu") -> StepInputs:
    """Draw the step-0 masters for a config."""
    device = torch.device(device)
    g = _gen(device, seed + 1000 * cfg.config_id)
    B, Hq, Hkv, L, d = cfg.B, cfg.Hq, cfg.Hkv, cfg.L, cfg.d
    q = torch.randn(B, Hq, L, d, generator=g, device=device, dtype=torch.float32)
    k = torch.randn(B, Hkv, L, d, generator=g, device=device, dtype=torch.float32)
    v = torch.randn(B, Hkv, L, d, generator=g, device=device, dtype=torch.float32)
    if not cfg.planted:
        return StepInputs(cfg, seed, q, k, v)
    if d < _SEGMENT_DIMS[1]:
        raise ValueError("planted structure needs d >= 128")
    q.mul_(1.0 / math.sqrt(d))
    k.mul_(1.0 / math.sqrt(d))
    group = Hq // Hkv
    pos = torch.arange(L, device=device, dtype=torch.float32)

    # window features: 8 (sin, cos) pairs
    m = torch.arange(8, device=device, dtype=torch.float32)
    omega = 2.0 * math.pi / (1024.0 * torch.pow(2.0, m / 2.0))
    ang = pos[:, None] * omega[None, :]
    window = torch.empty(L, 16, device=device, dtype=torch.float32)
    window[:, 0::2] = 3.0 * torch.sin(ang)
    window[:, 1::2] = 3.0 * torch.cos(ang)

    # stripe directions / positions and segment directions are drawn per KV head so that the
    # query heads of one group agree with the keys they read
    n_seg = (L + _SEGMENT - 1) // _SEGMENT
    stripe_u = _unit_rows(B * Hkv, _STRIPE_DIMS[1] - _STRIPE_DIMS[0], 3.0, g, device).view(B, Hkv, -1)
    seg_e = _unit_rows(B * Hkv * n_seg, _SEGMENT_DIMS[1] - _SEGMENT_DIMS[0], 3.0, g, device).view(B, Hkv, n_seg, -1)
    seg_of = (torch.arange(L, device=device) // _SEGMENT)
    stripe_pos = []
    for _ in range(B * Hkv):
        extra = 64 + torch.randperm(max(L - 64, 1), generator=g, device=device)[:8] if L > 64 else None
        first = torch.arange(min(64, L), device=device)
        stripe_pos.append(first if extra is None else torch.cat([first, extra]))

    for b in range(B):
        for hk in range(Hkv):
            types_here = {0, 1, 2} if group > 1 else {hk % 4}
            if 0 in types_here:
                k[b, hk, :, _WINDOW_DIMS[0]:_WINDOW_DIMS[1]] += window
            if 1 in types_here:
                sp = stripe_pos[b * Hkv + hk]
                k[b, hk, sp, _STRIPE_DIMS[0]:_STRIPE_DIMS[1]] += 4.0 * stripe_u[b, hk]
            if 2 in types_here:
                k[b, hk, :, _SEGMENT_DIMS[0]:_SEGMENT_DIMS[1]] += seg_e[b, hk][seg_of]
        for h in range(Hq):
            hk = h // group
            t = h % 4
            if t == 0:
                q[b, h, :, _WINDOW_DIMS[0]:_WINDOW_DIMS[1]] += window
            elif t == 1:
                q[b, h, :, _STRIPE_DIMS[0]:_STRIPE_DIMS[1]] += stripe_u[b, hk]
            elif t == 2:
                q[b, h, :, _SEGMENT_DIMS[0]:_SEGMENT_DIMS[1]] += seg_e[b, hk][seg_of]
    return StepInputs(cfg, seed, q, k, v)
