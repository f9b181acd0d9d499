"""The allocation-free selection entry point against sparsed_select_pattern (GPU, through the C ABI).

sparsed_select_pattern_static keeps its scratch in a fixed array inside the library; every call on a GPU
shares it and finds the previous call's contents there. Two calls in a row, the second on a smaller input,
must each give exactly what sparsed_select_pattern gives with a caller's workspace (same kernels, so the
index and the pooled scores are compared bit for bit), and the index must also pass the oracle's tie rule."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2509_24014_amd as sd
from parity_utils import compare_index

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(B, Hq, Hkv, L, D, dtype, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    scale = 0.45
    q = (torch.randn(B, Hq, L, D, generator=g) * scale).to(dtype)
    k = (torch.randn(B, Hkv, L, D, generator=g) * scale).to(dtype)
    return q, k


def _empty_index(B, H, L, bq, bk, rho):
    nqb, nkb = -(-L // bq), -(-L // bk)
    keep = sd.kept_blocks(rho, nkb)
    return sd.BlockIndex(torch.full((B, H, nqb + 1), -7, dtype=torch.int32, device=DEV),
                         torch.full((B, H, nqb * keep), -7, dtype=torch.int32, device=DEV), bq, bk, nkb), keep


def _one_call(B, Hq, Hkv, L, D, dtype, bq, bk, rho, seed, use_lse):
    print(f"static selection: B={B} Hq={Hq} Hkv={Hkv} L={L} D={D} {dtype} {bq}x{bk} rho={rho} lse_in={use_lse}", flush=True)
    q, k = _inputs(B, Hq, Hkv, L, D, dtype, seed)
    qd, kd = q.to(DEV), k.to(DEV)
    nqb, nkb = -(-L // bq), -(-L // bk)
    lse = None
    if use_lse:
        lse = torch.empty(B, Hq, L, dtype=torch.float32, device=DEV)
        sd.attn_dense(qd, kd, kd, lse_out=lse)
    pooled_ref = torch.empty(B, Hq, nqb, nkb, dtype=torch.float32, device=DEV)
    ref = sd.select_pattern(qd, kd, bq, bk, rho, lse_in=lse, pooled_out=pooled_ref)
    ix, keep = _empty_index(B, Hq, L, bq, bk, rho)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    sd.select_pattern_static(qd, kd, bq, bk, rho, ix, lse_in=lse)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before                     # nothing taken from torch's allocator either
    assert torch.equal(ix.row_ptr, ref.row_ptr) and torch.equal(ix.col_idx, ref.col_idx)
    # once more with the pooled scores exposed: bit-identical to the workspace route
    pooled = torch.empty_like(pooled_ref)
    ix2, _ = _empty_index(B, Hq, L, bq, bk, rho)
    sd.select_pattern_static(qd, kd, bq, bk, rho, ix2, lse_in=lse, pooled_out=pooled)
    torch.cuda.synchronize()
    assert torch.equal(pooled, pooled_ref) and torch.equal(ix2.col_idx, ref.col_idx)
    sd.index_validate(ix)
    # and against the oracle, to the bar of every other selection test
    rp, ci, apool, _ = oracle.select_pattern(q, k, bq, bk, rho)
    np.testing.assert_array_equal(ix.row_ptr.cpu().numpy(), rp)
    rel = np.abs(pooled.cpu().double().numpy() - apool) / apool
    assert rel.max() <= 5e-6
    ties = compare_index(ix.col_idx.cpu().numpy(), ci, apool.reshape(-1, nkb), keep)
    print(f"  identical to sparsed_select_pattern; oracle ties {ties}, pooled rel err {rel.max():.2e}", flush=True)


def test_static_selection_matches_workspace_selection_twice_in_a_row():
    # a larger call first, then a smaller one that finds the larger one's leftovers in the shared scratch
    _one_call(1, 4, 2, 2048, 128, torch.bfloat16, 128, 64, 0.2, seed=1, use_lse=False)
    _one_call(1, 2, 2, 512, 64, torch.bfloat16, 64, 64, 0.3, seed=2, use_lse=True)
    _one_call(2, 2, 1, 200, 64, torch.float32, 32, 32, 0.3, seed=3, use_lse=False)   # fp32, ragged length, batch 2


def test_static_selection_rejects_what_does_not_fit():
    B, H, L, D = 1, 32, 65536, 128                                       # 8 MiB of statistics + 64 MiB of pooled scores
    q = torch.zeros(B, H, L, D, dtype=torch.bfloat16, device=DEV)
    need = sd.select_workspace_bytes(q, 128, 64)
    assert need > sd.STATIC_SCRATCH_BYTES
    nqb, nkb = L // 128, L // 64
    keep = sd.kept_blocks(0.05, nkb)
    ix = sd.BlockIndex(torch.zeros(B, H, nqb + 1, dtype=torch.int32, device=DEV),
                       torch.full((B, H, nqb * keep), -7, dtype=torch.int32, device=DEV), 128, 64, nkb)
    with pytest.raises(sd.SparsedError) as e:
        sd.select_pattern_static(q, q, 128, 64, 0.05, ix)
    assert e.value.status == 7 and "built-in" in str(e.value)
    assert (ix.col_idx == -7).all()                                      # nothing was launched
