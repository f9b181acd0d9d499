"""Helpers shared by the GPU parity tests (not a test module)."""
from __future__ import annotations

import numpy as np
import torch

# Tolerances of the parity gate: bf16 inputs with fp32 accumulation, and fp32 inputs.
BF16_MAX, BF16_MEAN = 2e-2, 2e-3
F32_MAX = 1e-5
TIE_BAND = 1e-5  # relative width of the band around the k-th pooled score inside which rows may differ


def assert_output_close(got: torch.Tensor, want: np.ndarray, dtype: torch.dtype, what: str = ""):
    g = got.detach().to("cpu").to(torch.float64).numpy().reshape(want.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    diff = np.abs(g - want)
    if dtype == torch.bfloat16:
        assert diff.max() <= BF16_MAX, f"{what}: max|d|={diff.max():.3e} > {BF16_MAX}"
        assert diff.mean() <= BF16_MEAN, f"{what}: mean|d|={diff.mean():.3e} > {BF16_MEAN}"
    else:
        assert diff.max() <= F32_MAX, f"{what}: max|d|={diff.max():.3e} > {F32_MAX}"
    return float(diff.max()), float(diff.mean())


def compare_index(gpu_cols: np.ndarray, ora_cols: np.ndarray, apool: np.ndarray, keep: int):
    """Bit-exact comparison of selected key blocks, row by row, with the tie rule.

    gpu_cols / ora_cols: [rows, keep] ascending block indices; apool: [rows, nkb] fp64 oracle
    scores. A row may differ from the oracle only by exchanging blocks whose oracle score lies
    within TIE_BAND (relative) of the oracle's keep-th largest score. Returns
    (tie_rows, tie_blocks); raises AssertionError on any difference outside the band.
    """
    rows, nkb = apool.shape
    gpu_cols = gpu_cols.reshape(rows, keep)
    ora_cols = ora_cols.reshape(rows, keep)
    assert (gpu_cols >= 0).all() and (gpu_cols < nkb).all(), "block index out of range"
    if keep > 1:
        assert (np.diff(gpu_cols, axis=1) > 0).all(), "row not strictly ascending"
    tie_rows = tie_blocks = 0
    differing = np.nonzero((gpu_cols != ora_cols).any(axis=1))[0]
    for r in differing:
        g, o = set(gpu_cols[r].tolist()), set(ora_cols[r].tolist())
        s_k = np.sort(apool[r])[::-1][keep - 1]
        band = TIE_BAND * abs(s_k)
        for J in (g - o) | (o - g):
            assert abs(apool[r, J] - s_k) <= band, (
                f"row {r}: block {J} score {apool[r, J]:.9e} differs from the cut {s_k:.9e} by more than the tie band")
        tie_rows += 1
        tie_blocks += len(g - o)
    return tie_rows, tie_blocks


def random_csr(B, H, nqb, nkb, max_keep, seed, device, allow_empty=True):
    """A ragged CSR index: every row gets a random number (possibly 0) of distinct ascending blocks."""
    rng = np.random.default_rng(seed)
    cap = nqb * max_keep
    row_ptr = np.zeros((B, H, nqb + 1), dtype=np.int32)
    col_idx = np.full((B, H, cap), -1, dtype=np.int32)
    for b in range(B):
        for h in range(H):
            pos = 0
            for I in range(nqb):
                n = int(rng.integers(0 if allow_empty else 1, max_keep + 1))
                cols = np.sort(rng.choice(nkb, n, replace=False))
                col_idx[b, h, pos:pos + n] = cols
                pos += n
                row_ptr[b, h, I + 1] = pos
    return torch.from_numpy(row_ptr).to(device), torch.from_numpy(col_idx).to(device)
