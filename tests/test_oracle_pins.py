"""Pins for the fp64 oracle: closed forms, library special cases, invariants, brute force.

The paper prints no numeric worked example, so every pin is something the mathematics
fixes independently of the oracle's own code path: torch's fp64 softmax / SDPA (library
routine), a hand-derived closed form (tests/golden/w1_closed_form.txt), invariants of
Eq. 1 / Eq. 3 / Eq. 6, and exhaustive search on tiny inputs.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import schedule as oracle_schedule

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(B, Hq, Hkv, L, d, seed=0, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    q = (torch.randn(B, Hq, L, d, generator=g) * scale).float()
    k = (torch.randn(B, Hkv, L, d, generator=g) * scale).float()
    v = torch.randn(B, Hkv, L, d, generator=g).float()
    return q, k, v


def _torch_probs(q, k):
    """Eq. 1 through torch's fp64 softmax (a library routine, not the oracle's loop)."""
    B, Hq, L, d = q.shape
    rep = Hq // k.shape[1]
    kk = k.double().repeat_interleave(rep, dim=1)
    return torch.softmax(q.double() @ kk.transpose(-1, -2) / math.sqrt(d), dim=-1)


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = np.array([float(x) for x in vals])
    return out


# ----------------------------------------------------------------------------- O1 dense (Eq. 1)
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (6, 1)])
def test_dense_matches_torch_softmax_and_sdpa(Hq, Hkv):
    q, k, v = _rand(2, Hq, Hkv, 96, 16, seed=1)
    got = oracle.attn_dense(q, k, v)
    rep = Hq // Hkv
    P = _torch_probs(q, k)
    want = (P @ v.double().repeat_interleave(rep, dim=1)).numpy()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    sdpa = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double().repeat_interleave(rep, dim=1), v.double().repeat_interleave(rep, dim=1))
    np.testing.assert_allclose(got, sdpa.numpy(), rtol=0, atol=1e-12)


def test_dense_rows_agree_with_full():
    q, k, v = _rand(1, 3, 3, 80, 8, seed=2)
    full = oracle.attn_dense(q, k, v)
    part = oracle.attn_dense_rows(q, k, v, 0, 2, 17, 53)
    np.testing.assert_array_equal(part, full[0, 2, 17:53])


def test_probs_rows_sum_to_one_and_match_torch():
    q, k, _ = _rand(1, 2, 1, 64, 8, seed=3, scale=2.0)
    P = _torch_probs(q, k).numpy()
    for h, i in [(0, 0), (1, 5), (1, 63)]:
        p = oracle.attn_probs_row(q, k, 0, h, i)
        assert abs(p.sum() - 1.0) < 1e-14
        np.testing.assert_allclose(p, P[0, h, i], rtol=1e-12, atol=1e-16)


def test_dense_zero_queries_give_mean_of_values():
    q, k, v = _rand(1, 2, 2, 50, 8, seed=4)
    q.zero_()
    got = oracle.attn_dense(q, k, v)
    want = v.double().mean(dim=2, keepdim=True).expand(-1, -1, 50, -1).numpy()
    np.testing.assert_allclose(got, want, atol=1e-14)


def test_dense_shift_of_all_keys_changes_nothing():
    # adding one vector c to every key adds q.c to every logit of a row: softmax is unchanged.
    # values are multiples of 1/8 so that the shifted keys are exact in float32.
    g = torch.Generator().manual_seed(5)
    q = torch.randint(-8, 9, (1, 2, 40, 4), generator=g).float() / 8
    k = torch.randint(-8, 9, (1, 2, 40, 4), generator=g).float() / 8
    v = torch.randn(1, 2, 40, 4, generator=g)
    c = torch.tensor([3.0, -2.0, 1.5, 0.25])
    a = oracle.attn_dense(q, k, v)
    b = oracle.attn_dense(q, k + c, v)
    np.testing.assert_allclose(a, b, atol=1e-12)


def test_dense_invariant_under_joint_key_value_permutation():
    q, k, v = _rand(1, 2, 2, 48, 8, seed=6)
    perm = torch.randperm(48, generator=torch.Generator().manual_seed(7))
    a = oracle.attn_dense(q, k, v)
    b = oracle.attn_dense(q, k[:, :, perm], v[:, :, perm])
    np.testing.assert_allclose(a, b, atol=1e-13)


def test_dense_is_not_causal():
    # output of row 0 must depend on the last key (bidirectional attention)
    q, k, v = _rand(1, 1, 1, 16, 4, seed=8)
    a = oracle.attn_dense(q, k, v)
    v2 = v.clone()
    v2[0, 0, -1] += 10.0
    b = oracle.attn_dense(q, k, v2)
    assert np.abs(a[0, 0, 0] - b[0, 0, 0]).max() > 1e-3


# ----------------------------------------------------------------------------- O2 pooling (Section 3.3)
@pytest.mark.parametrize("bq,bk", [(8, 8), (16, 8), (8, 4)])
def test_pool_matches_reshape_mean_of_torch_probs(bq, bk):
    q, k, _ = _rand(1, 4, 2, 64, 8, seed=9, scale=1.5)
    got = oracle.pool_scores(q, k, bq, bk)
    P = _torch_probs(q, k).numpy()
    want = P.reshape(1, 4, 64 // bq, bq, 64 // bk, bk).mean(axis=(3, 5))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-16)
    # each pooled row sums to 1/bk (every softmax row sums to 1)
    np.testing.assert_allclose(got.sum(-1), 1.0 / bk, rtol=1e-12)


def test_pool_uniform_when_queries_are_zero():
    q, k, _ = _rand(1, 1, 1, 32, 4, seed=10)
    q.zero_()
    got = oracle.pool_scores(q, k, 8, 4)
    np.testing.assert_allclose(got, 1.0 / 32, rtol=1e-14)


def test_pool_rows_agree_with_full():
    q, k, _ = _rand(1, 2, 2, 64, 8, seed=11)
    full = oracle.pool_scores(q, k, 16, 8)
    part = oracle.pool_scores_rows(q, k, 16, 8, 0, 1, 1, 3)
    np.testing.assert_array_equal(part, full[0, 1, 1:3])


# ----------------------------------------------------------------------------- the count behind "top rho%"
def test_kept_blocks_rule():
    # the five named configurations
    assert oracle.kept_blocks(0.3, 8) == 3
    assert oracle.kept_blocks(0.2, 64) == 13
    assert oracle.kept_blocks(0.1, 256) == 26
    assert oracle.kept_blocks(0.1, 512) == 52
    assert oracle.kept_blocks(0.05, 1024) == 52
    # products that land a rounding error above an integer must not round up
    assert oracle.kept_blocks(0.3, 10) == 3
    assert oracle.kept_blocks(0.7, 10) == 7
    assert oracle.kept_blocks(0.1, 30) == 3
    # clamps
    assert oracle.kept_blocks(1.0, 17) == 17
    assert oracle.kept_blocks(1e-6, 17) == 1
    assert oracle.kept_blocks(0.5, 1) == 1
    for n in range(1, 40):
        for pct in range(1, 101):
            assert oracle.kept_blocks(pct / 100.0, n) == max(1, -((-pct * n) // 100))


# ----------------------------------------------------------------------------- O3 selection (Eq. 6)
def test_select_maximises_kept_mass_by_exhaustive_search():
    rng = np.random.default_rng(12)
    ap = rng.random((1, 2, 5, 8))
    keep = 3
    row_ptr, col_idx, cut = oracle.select_topk(ap, keep)
    for h in range(2):
        for I in range(5):
            best = max(itertools.combinations(range(8), keep), key=lambda s: ap[0, h, I, list(s)].sum())
            got = col_idx[0, h, I * keep:(I + 1) * keep]
            assert tuple(got) == tuple(sorted(best))
            srt = np.sort(ap[0, h, I])[::-1]
            assert cut[0, h, I, 0] == srt[keep - 1] and cut[0, h, I, 1] == srt[keep]
    np.testing.assert_array_equal(row_ptr[0, 0], np.arange(6) * keep)


def test_select_ties_go_to_the_lower_block_index():
    ap = np.full((1, 1, 2, 6), 0.25)
    _, col_idx, _ = oracle.select_topk(ap, 4)
    np.testing.assert_array_equal(col_idx[0, 0], [0, 1, 2, 3, 0, 1, 2, 3])
    ap = np.array([[[[0.1, 0.5, 0.1, 0.5, 0.1, 0.5]]]])
    _, col_idx, _ = oracle.select_topk(ap, 4)          # three 0.5s, then the lowest-index 0.1
    np.testing.assert_array_equal(col_idx[0, 0], [0, 1, 3, 5])
    _, col_idx, _ = oracle.select_topk(ap, 2)          # two lowest-index 0.5s
    np.testing.assert_array_equal(col_idx[0, 0], [1, 3])


def test_select_rho_one_keeps_everything_and_rows_ascend():
    rng = np.random.default_rng(13)
    ap = rng.random((2, 3, 4, 9))
    row_ptr, col_idx, cut = oracle.select_topk(ap, 9)
    np.testing.assert_array_equal(col_idx.reshape(2, 3, 4, 9), np.broadcast_to(np.arange(9), (2, 3, 4, 9)))
    assert np.isnan(cut[..., 1]).all()
    row_ptr, col_idx, _ = oracle.select_topk(ap, 4)
    rows = col_idx.reshape(2, 3, 4, 4)
    assert (np.diff(rows, axis=-1) > 0).all()
    np.testing.assert_array_equal(row_ptr, np.broadcast_to(np.arange(5) * 4, (2, 3, 5)))


def test_select_follows_a_permutation_of_key_blocks():
    rng = np.random.default_rng(14)
    ap = rng.random((1, 1, 6, 12))
    perm = rng.permutation(12)
    _, a, _ = oracle.select_topk(ap, 5)
    _, b, _ = oracle.select_topk(ap[..., perm], 5)
    a = a.reshape(6, 5)
    b = b.reshape(6, 5)
    for I in range(6):
        assert sorted(perm[b[I]]) == sorted(a[I])


def test_select_pattern_uses_post_softmax_pooled_scores():
    # one key block holds a single huge logit, another many moderate ones: ranking by pooled
    # probabilities (post-softmax) picks the huge one; ranking by mean logit would not.
    L, d, bq, bk = 16, 4, 4, 4
    q = torch.zeros(1, 1, L, d)
    k = torch.zeros(1, 1, L, d)
    q[..., 0] = 2.0
    k[0, 0, 0, 0] = 12.0          # block 0: one key with logit 12, three with 0
    k[0, 0, 4:8, 0] = 4.0         # block 1: four keys with logit 4 (mean logit 4 > 3)
    row_ptr, col_idx, ap, _ = oracle.select_pattern(q, k, bq, bk, rho=0.25)
    assert (col_idx.reshape(-1) == 0).all()
    assert ap[0, 0, 0, 0] > ap[0, 0, 0, 1] > ap[0, 0, 0, 2]


def test_isolated_selection_reduces_to_plain_and_splits_ranges():
    rng = np.random.default_rng(15)
    ap = rng.random((1, 2, 3, 10))
    rp0, ci0, _ = oracle.select_topk(ap, oracle.kept_blocks(0.3, 10))
    rp1, ci1 = oracle.select_isolated(ap, 0.3, 10)      # everything is prefill
    np.testing.assert_array_equal(ci0, ci1)
    np.testing.assert_array_equal(rp0, rp1)
    rp2, ci2 = oracle.select_isolated(ap, 0.5, 4)       # 2 of blocks 0..3 and 3 of blocks 4..9
    rows = ci2.reshape(2, 3, 5)
    for h in range(2):
        for I in range(3):
            pre = sorted(np.argsort(-ap[0, h, I, :4])[:2])
            gen = sorted(4 + np.argsort(-ap[0, h, I, 4:])[:3])
            assert list(rows[h, I]) == pre + gen


# ----------------------------------------------------------------------------- O4 sparse (Eq. 3, Eq. 4)
def _random_index(B, H, nqb, nkb, keep, seed):
    rng = np.random.default_rng(seed)
    row_ptr = np.broadcast_to(np.arange(nqb + 1, dtype=np.int32) * keep, (B, H, nqb + 1)).copy()
    col_idx = np.empty((B, H, nqb * keep), dtype=np.int32)
    for b in range(B):
        for h in range(H):
            for I in range(nqb):
                col_idx[b, h, I * keep:(I + 1) * keep] = np.sort(rng.choice(nkb, keep, replace=False))
    return row_ptr, col_idx


def test_sparse_with_every_block_kept_equals_dense():
    q, k, v = _rand(1, 4, 2, 64, 8, seed=16)
    row_ptr, col_idx = _random_index(1, 4, 8, 8, 8, seed=0)
    a = oracle.attn_sparse(q, k, v, row_ptr, col_idx, 8, 8)
    b = oracle.attn_dense(q, k, v)
    np.testing.assert_allclose(a, b, atol=1e-14)


@pytest.mark.parametrize("bq,bk,keep", [(8, 8, 3), (16, 8, 2), (8, 16, 1)])
def test_sparse_matches_bruteforce_mask_sdpa_and_renormalised_dense(bq, bk, keep):
    B, Hq, Hkv, L, d = 1, 4, 2, 64, 8
    q, k, v = _rand(B, Hq, Hkv, L, d, seed=17, scale=1.3)
    nqb, nkb = L // bq, L // bk
    row_ptr, col_idx = _random_index(B, Hq, nqb, nkb, keep, seed=18)
    got = oracle.attn_sparse(q, k, v, row_ptr, col_idx, bq, bk)
    # (a) Eq. 3 + Eq. 4 literally: explicit L x L matrix of 0 / -inf
    brute = oracle.attn_masked_bruteforce(q, k, v, row_ptr, col_idx, bq, bk)
    np.testing.assert_allclose(got, brute, atol=1e-13)
    # (b) library routine: SDPA with a boolean mask expanded element by element
    mask = np.zeros((B, Hq, L, L), dtype=bool)
    for h in range(Hq):
        for I in range(nqb):
            for J in col_idx[0, h, row_ptr[0, h, I]:row_ptr[0, h, I + 1]]:
                mask[0, h, I * bq:(I + 1) * bq, J * bk:(J + 1) * bk] = True
    rep = Hq // Hkv
    sdpa = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double().repeat_interleave(rep, 1), v.double().repeat_interleave(rep, 1),
        attn_mask=torch.from_numpy(mask))
    np.testing.assert_allclose(got, sdpa.numpy(), atol=1e-12)
    # (c) renormalisation identity with the dense probabilities of Eq. 1
    P = _torch_probs(q, k).numpy() * mask
    want = (P @ v.double().repeat_interleave(rep, 1).numpy()) / P.sum(-1, keepdims=True)
    np.testing.assert_allclose(got, want, atol=1e-12)


def test_sparse_rows_ragged_csr_and_empty_row():
    q, k, v = _rand(1, 1, 1, 32, 4, seed=19)
    # rows of different lengths; row 2 is empty -> zeros
    row_ptr = np.array([[[0, 2, 3, 3, 7]]], dtype=np.int32)
    col_idx = np.array([[[1, 3, 0, 0, 1, 2, 3, 0, 0]]], dtype=np.int32)  # capacity 9 > 7 used
    out = oracle.attn_sparse(q, k, v, row_ptr, col_idx, 8, 8)
    assert (out[0, 0, 16:24] == 0).all()
    np.testing.assert_allclose(out[0, 0, 24:32], oracle.attn_dense(q, k, v)[0, 0, 24:32], atol=1e-14)
    brute = oracle.attn_masked_bruteforce(q, k, v, row_ptr, col_idx, 8, 8)
    np.testing.assert_allclose(out, brute, atol=1e-13)
    part = oracle.attn_sparse_rows(q, k, v, row_ptr, col_idx, 8, 8, 0, 0, 1, 3)
    np.testing.assert_array_equal(part, out[0, 0, 8:24])


# ----------------------------------------------------------------------------- closed form W1
# ----------------------------------------------------------------------------- ragged L (partial last blocks)
def test_ragged_pool_matches_ceil_mode_average_pooling():
    """Library special case: torch's avg_pool2d with ceil_mode=True averages a window that hangs over
    the edge over the entries that exist."""
    L, bq, bk = 45, 16, 8
    q, k, _ = _rand(1, 2, 2, L, 8, seed=31)
    P = torch.softmax(q.double() @ k.double().transpose(-1, -2) / math.sqrt(8), dim=-1)
    want = torch.nn.functional.avg_pool2d(P, kernel_size=(bq, bk), stride=(bq, bk), ceil_mode=True)
    got = oracle.pool_scores(q, k, bq, bk)
    assert got.shape == (1, 2, 3, 6)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-15)
    # the row-range entry point gives the same numbers
    np.testing.assert_allclose(got[0, 1, :2], oracle.pool_scores_rows(q, k, bq, bk, 0, 1, 0, 2), rtol=0, atol=0)
    # each row of a full query block still sums to sum over key blocks of (mass / area): check total mass instead
    area = np.array([bk] * 5 + [L - 5 * bk], dtype=np.float64)
    rows = np.array([bq, bq, L - 2 * bq], dtype=np.float64)
    mass = (got * area[None, None, None, :] * rows[None, None, :, None]).sum(-1)
    np.testing.assert_allclose(mass, np.broadcast_to(rows, mass.shape), rtol=1e-12)


def test_ragged_sparse_matches_bruteforce_and_dense():
    L, bq, bk, d = 45, 16, 8, 8
    q, k, v = _rand(1, 2, 1, L, d, seed=32)
    nqb, nkb = 3, 6
    # every block listed: equals dense attention over the 45 real keys
    rp = np.tile(np.arange(nqb + 1, dtype=np.int32) * nkb, (1, 2, 1))
    ci = np.tile(np.arange(nkb, dtype=np.int32), (1, 2, nqb))
    np.testing.assert_allclose(oracle.attn_sparse(q, k, v, rp, ci, bq, bk), oracle.attn_dense(q, k, v), rtol=1e-12, atol=1e-14)
    # a pattern that keeps the partial last key block plus one other, against the explicit L x L mask and against
    # torch SDPA with the boolean mask built from first principles
    rp = np.tile(np.arange(nqb + 1, dtype=np.int32) * 2, (1, 2, 1))
    ci = np.tile(np.array([1, 5, 0, 5, 3, 5], dtype=np.int32), (1, 2, 1))
    got = oracle.attn_sparse(q, k, v, rp, ci, bq, bk)
    np.testing.assert_allclose(got, oracle.attn_masked_bruteforce(q, k, v, rp, ci, bq, bk), rtol=1e-12, atol=1e-14)
    keep = np.zeros((L, L), dtype=bool)
    for i in range(L):
        for j in range(L):
            keep[i, j] = (j // bk) in ci[0, 0, 2 * (i // bq): 2 * (i // bq) + 2]
    want = torch.nn.functional.scaled_dot_product_attention(q.double(), k.double().repeat_interleave(2, 1), v.double().repeat_interleave(2, 1),
                                                            attn_mask=torch.from_numpy(keep))
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-11, atol=1e-13)
    # rows-variant: the rows past L of the last (partial) query block stay zero
    last = oracle.attn_sparse_rows(q, k, v, rp, ci, bq, bk, 0, 1, 2, 3)
    assert last.shape == (bq, d) and (last[L - 2 * bq:] == 0).all()
    np.testing.assert_allclose(last[:L - 2 * bq], got[0, 1, 2 * bq:], rtol=0, atol=0)


def test_ragged_selection_counts_blocks_with_ceil():
    L, bq, bk = 45, 16, 8
    q, k, _ = _rand(1, 1, 1, L, 8, seed=33)
    rp, ci, ap, _ = oracle.select_pattern(q, k, bq, bk, 0.5)
    assert ap.shape[-2:] == (3, 6) and oracle.kept_blocks(0.5, 6) == 3
    assert rp.tolist() == [[[0, 3, 6, 9]]] and ci.shape[-1] == 9
    for I in range(3):
        assert set(ci[0, 0, 3 * I: 3 * I + 3]) == set(np.argsort(-ap[0, 0, I], kind="stable")[:3])


# ----------------------------------------------------------------------------- isolated selection, boundary at a token
def test_range_pooling_matches_sliced_means_of_torch_probs():
    L, bq, bk, ptok = 90, 16, 16, 40                       # the boundary falls inside key block 2; the last block is partial
    q, k, _ = _rand(1, 2, 1, L, 8, seed=41)
    _, _, ap, n_pre, vblock = oracle.select_isolated_tokens(q, k, bq, bk, 0.4, ptok)
    vstart, vend, vb, n_pre2 = oracle.prefill_ranges(L, bk, ptok)
    assert vstart.tolist() == [0, 16, 32, 40, 48, 64, 80] and vend.tolist() == [16, 32, 40, 48, 64, 80, 90]
    assert vb.tolist() == [0, 1, 2, 2, 3, 4, 5] == vblock.tolist() and n_pre == n_pre2 == 3
    P = _torch_probs(q, k)
    for I in range(6):
        rows = P[:, :, I * bq:min((I + 1) * bq, L)]
        for v in range(7):
            want = rows[..., vstart[v]:vend[v]].mean(dim=(-1, -2)).numpy()
            np.testing.assert_allclose(ap[:, :, I, v], want, rtol=1e-12)
    # every probability is counted exactly once: sum of (mean x area) over the ranges = number of rows
    area = (vend - vstart).astype(np.float64)
    rows = np.array([16] * 5 + [10], dtype=np.float64)
    np.testing.assert_allclose((ap * area).sum(-1) * rows, np.broadcast_to(rows, ap.shape[:-1]), rtol=1e-12)


def test_token_boundary_on_a_block_edge_reduces_to_the_block_version():
    q, k, _ = _rand(1, 2, 2, 96, 8, seed=42)
    rp, ci, ap, n_pre, vblock = oracle.select_isolated_tokens(q, k, 16, 16, 0.34, 32)
    a = oracle.pool_scores(q, k, 16, 16)
    rp2, ci2 = oracle.select_isolated(a, 0.34, 2)
    assert n_pre == 2 and vblock.tolist() == list(range(6))
    np.testing.assert_allclose(ap, a, rtol=1e-13)
    assert np.array_equal(rp, rp2) and np.array_equal(ci, ci2)
    # no prefill at all / everything prefill: plain selection
    for ptok in (0, 96):
        rp3, ci3, _, _, _ = oracle.select_isolated_tokens(q, k, 16, 16, 0.34, ptok)
        rp4, ci4, _ = oracle.select_topk(a, oracle.kept_blocks(0.34, 6))
        assert np.array_equal(rp3, rp4) and np.array_equal(ci3, ci4)


def test_token_boundary_rows_are_unions_of_per_range_optima():
    L, bq, bk, ptok, rho = 96, 16, 16, 40, 0.34
    q, k, _ = _rand(1, 3, 1, L, 8, seed=43)
    rp, ci, ap, n_pre, vblock = oracle.select_isolated_tokens(q, k, bq, bk, rho, ptok)
    nv = ap.shape[-1]
    keep_pre, keep_gen = oracle.kept_blocks(rho, n_pre), oracle.kept_blocks(rho, nv - n_pre)
    lengths = set()
    for h in range(3):
        assert rp[0, h, 0] == 0
        for I in range(L // bq):
            row = ci[0, h, rp[0, h, I]:rp[0, h, I + 1]].tolist()
            assert row == sorted(set(row)), "ascending, no duplicates"
            a = ap[0, h, I]
            best_pre = max(itertools.combinations(range(n_pre), keep_pre), key=lambda c: sum(a[list(c)]))
            best_gen = max(itertools.combinations(range(n_pre, nv), keep_gen), key=lambda c: sum(a[list(c)]))
            want = sorted({int(vblock[v]) for v in best_pre + best_gen})
            assert row == want
            lengths.add(len(row))
    assert lengths <= {keep_pre + keep_gen, keep_pre + keep_gen - 1} and len(lengths) == 2   # both cases occur for this seed


def test_closed_form_w1():
    g = _read_golden("w1_closed_form.txt")
    L = 4
    q = torch.tensor(g["q"], dtype=torch.float32).view(1, 1, L, 1)
    k = torch.tensor(np.log(g["w"]), dtype=torch.float32).view(1, 1, L, 1)
    v = torch.tensor(g["v"], dtype=torch.float32).view(1, 1, L, 1)
    tol = 2e-7  # ln 3 and ln 5 are rounded to float32 on input
    np.testing.assert_allclose(oracle.attn_dense(q, k, v).reshape(-1), g["dense"], atol=tol)
    row_ptr, col_idx, ap, _ = oracle.select_pattern(q, k, 2, 2, rho=0.5)
    np.testing.assert_allclose(ap.reshape(-1), g["apool"], atol=tol)
    np.testing.assert_array_equal(row_ptr.reshape(-1), g["row_ptr"].astype(np.int32))
    np.testing.assert_array_equal(col_idx.reshape(-1), g["col_idx"].astype(np.int32))
    np.testing.assert_allclose(oracle.attn_sparse(q, k, v, row_ptr, col_idx, 2, 2).reshape(-1), g["sparse"], atol=tol)


# ----------------------------------------------------------------------------- O6 schedule (Algorithm 1)
def test_n_dense_steps_rule():
    assert oracle_schedule.n_dense_steps(1024, 0.2) == 205
    assert oracle_schedule.n_dense_steps(64, 0.125) == 8
    assert oracle_schedule.n_dense_steps(5, 0.2) == 1
    assert oracle_schedule.n_dense_steps(10, 0.3) == 3       # 10*0.3 = 3.0000000000000004
    assert oracle_schedule.n_dense_steps(10, 0.0) == 1
    assert oracle_schedule.n_dense_steps(10, 1.0) == 10


def test_schedule_counts_and_reuse():
    q, k, v = _rand(1, 2, 2, 32, 4, seed=20)
    seen = []

    def inputs(t):
        seen.append(t)
        return q + 0.01 * t, k, v

    res = oracle_schedule.run(inputs, T=6, n_dense=2, bq=8, bk=8, rho=0.5)
    assert res["calls"] == {"dense": 2, "select": 1, "sparse": 4}
    assert seen == list(range(6))
    # the pattern comes from the last dense step's Q, K and is the one used by every sparse step
    rp, ci, _, _ = oracle.select_pattern(q + 0.01, k, 8, 8, 0.5)
    np.testing.assert_array_equal(res["index"][1], ci)
    np.testing.assert_allclose(res["outputs"][5], oracle.attn_sparse(q + 0.05, k, v, rp, ci, 8, 8), atol=0)
    np.testing.assert_allclose(res["outputs"][1], oracle.attn_dense(q + 0.01, k, v), atol=0)
