"""GPU parity: every entry point of the C ABI against the fp64 oracle, element by element.

Small cases are compared in full; the named full-size workloads are compared on sampled
(head, query-block) units, which the oracle can compute one by one (every unit depends only on
its own query rows and its head's K, V)."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2509_24014_amd as sd
import workload
from parity_utils import BF16_MAX, assert_output_close, compare_index, random_csr

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def _rand_qkv(B, Hq, Hkv, L, D, dtype, seed, scale=None):
    g = torch.Generator(device="cpu").manual_seed(seed)
    scale = (1.0 / math.sqrt(math.sqrt(D))) if scale is None else scale  # logits ~ N(0, 1)
    q = (torch.randn(B, Hq, L, D, generator=g) * scale).to(dtype)
    k = (torch.randn(B, Hkv, L, D, generator=g) * scale).to(dtype)
    v = torch.randn(B, Hkv, L, D, generator=g).to(dtype)
    return q, k, v


def _dev(*ts):
    return tuple(t.to(DEV) for t in ts)


# ----------------------------------------------------------------------------- dense (Eq. 1)
@pytest.mark.parametrize("B,Hq,Hkv,L,D", [
    (1, 2, 2, 256, 128),    # one 256-row work-group per head
    (2, 4, 2, 320, 128),    # 320 = 5 x 64: the 64-row work-group shape, grouped heads, batch 2
    (1, 3, 1, 384, 64),     # 128-row work-groups, head dim 64, 3 query heads on one KV head
    (1, 2, 1, 1024, 128),   # 16 key tiles
    (1, 1, 1, 64, 128),     # a single tile
])
def test_dense_bf16(B, Hq, Hkv, L, D):
    _say(f"dense bf16 B={B} Hq={Hq} Hkv={Hkv} L={L} D={D}")
    q, k, v = _rand_qkv(B, Hq, Hkv, L, D, torch.bfloat16, seed=L + D)
    want = oracle.attn_dense(q, k, v)
    got = sd.attn_dense(*_dev(q, k, v))
    torch.cuda.synchronize()
    assert_output_close(got, want, torch.bfloat16, "dense bf16")


def test_dense_bf16_peaked_rows_and_large_logits():
    # logits spread over +-30: exercises the running-max rescale across tiles
    q, k, v = _rand_qkv(1, 2, 2, 512, 128, torch.bfloat16, seed=7, scale=0.9)
    want = oracle.attn_dense(q, k, v)
    got = sd.attn_dense(*_dev(q, k, v))
    assert_output_close(got, want, torch.bfloat16, "dense bf16 peaked")


def _climbing_qkv(L, D, H, seed):
    """Rows whose logits run away from their first keys: along the keys the logits of even query rows climb by hundreds
    of octaves (slowly at first, then by more than a tile can absorb), those of odd rows fall by as much."""
    g = torch.Generator().manual_seed(seed)
    q = 0.05 * torch.randn(1, H, L, D, generator=g)
    k = 0.05 * torch.randn(1, H, L, D, generator=g)
    sign = torch.where(torch.arange(L) % 2 == 0, 1.0, -1.0)
    q[..., 0] = sign[None, None, :] * (8.0 + torch.rand(1, H, L, generator=g))
    ramp = torch.linspace(0.0, 1.0, L) ** 2
    k[..., 0] = (ramp * 40.0 * math.sqrt(D))[None, None, :] * (1.0 + 0.25 * torch.rand(1, H, L, generator=g))
    # such rows put all their weight on one or two keys, so an output row is nearly a copy of a row of V, and the
    # absolute bar of the parity gate is meant for values of order one: keep V there
    v = 0.5 * torch.randn(1, H, L, D, generator=g)
    return q.to(torch.bfloat16), k.to(torch.bfloat16), v.to(torch.bfloat16)


@pytest.mark.parametrize("L,D", [(1024, 128), (600, 64), (2048 + 40, 128)])
def test_dense_bf16_rows_whose_logits_leave_the_first_tiles_range(L, D):
    """The attention kernels measure every probability of a row against the maximum of its first 32 keys and only
    re-reference a row when a probability leaves the range fp32 holds comfortably. Here that happens over and over
    (even rows) or never while everything after the first tile underflows (odd rows); output and row
    log-sum-exp must match the oracle all the same."""
    q, k, v = _climbing_qkv(L, D, 2, seed=L + D)
    span = float(q[..., 0].float().abs().max() * k[..., 0].float().max()) / math.sqrt(D)
    assert span * 1.4427 > 400
    lse = torch.empty(1, 2, L, dtype=torch.float32, device=DEV)
    got = sd.attn_dense(*_dev(q, k, v), lse_out=lse)
    assert_output_close(got, oracle.attn_dense(q, k, v), torch.bfloat16, "dense bf16, climbing and falling rows")
    logits = q.double() @ k.double().transpose(-1, -2) / math.sqrt(D)
    want = torch.logsumexp(logits, dim=-1)
    # fp32 carries a value of size x (the logit in octaves, the reference, their sum with log2 of the row sum, the
    # result in nats) to x * 2^-24 at each of those steps: the bar grows with the span
    assert (lse.cpu().double() - want).abs().max() < 2e-5 + 1e-6 * span


@pytest.mark.parametrize("bq,bk,L,D", [(128, 64, 1024, 128), (64, 64, 1024, 128), (32, 64, 512, 128), (64, 32, 600, 64), (128, 128, 1000, 128)])
def test_sparse_bf16_rows_whose_logits_leave_the_first_tiles_range(bq, bk, L, D):
    """The same for the block-sparse kernels: the listed blocks lie far apart, so from one listed block to the next
    the logits jump by more than fp32 can exponentiate, in both directions."""
    q, k, v = _climbing_qkv(L, D, 2, seed=bq + bk + L)
    nqb, nkb = -(-L // bq), -(-L // bk)
    rp, ci = random_csr(1, 2, nqb, nkb, min(6, nkb), seed=L + bq, device=DEV)
    got = sd.attn_sparse(*_dev(q, k, v), sd.BlockIndex(rp, ci, bq, bk, nkb))
    want = oracle.attn_sparse(q, k, v, rp.cpu().numpy(), ci.cpu().numpy(), bq, bk)
    assert_output_close(got, want, torch.bfloat16, f"sparse bf16 {bq}x{bk}, climbing and falling rows")


def _climbing_sweep_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        bq = int(rng.choice([32, 64, 128]))
        bk = int(rng.choice([32, 64, 128]))
        Hkv = int(rng.choice([1, 2]))
        Hq = Hkv * int(rng.choice([1, 2]))
        L = int(rng.integers(40, 1500))
        short = int(rng.integers(1, L + 1))            # a second batch element that stops earlier
        cases.append((i, Hq, Hkv, L, short, D, bq, bk))
    return cases


@pytest.mark.parametrize("case", _climbing_sweep_cases(16, seed=4242),
                         ids=lambda c: f"{c[0]}-H{c[1]}/{c[2]}-L{c[3]}/{c[4]}-D{c[5]}-{c[6]}x{c[7]}")
def test_sweep_rows_that_leave_the_first_tiles_range(case):
    """Climbing and falling rows over random shapes: ragged lengths (partial last blocks and tiles), grouped heads,
    two batch elements of different length, every query-block and key-block size; dense and sparse against the
    oracle, the row log-sum-exp against its definition."""
    _, Hq, Hkv, L, short, D, bq, bk = case
    qs, ks, vs = [], [], []
    for b in range(2):
        q1, _, _ = _climbing_qkv(L, D, Hq, seed=case[0] * 7 + b)
        _, k1, v1 = _climbing_qkv(L, D, Hkv, seed=case[0] * 7 + b + 100)
        qs.append(q1), ks.append(k1), vs.append(v1)
    q, k, v = torch.cat(qs), torch.cat(ks), torch.cat(vs)
    lens = torch.tensor([L, short], dtype=torch.int32)
    qd, kd, vd = _dev(q, k, v)
    lens_d = lens.to(DEV)
    nqb, nkb = -(-L // bq), -(-L // bk)
    lse = torch.zeros(2, Hq, L, dtype=torch.float32, device=DEV)
    out = torch.zeros(2, Hq, L, D, dtype=torch.bfloat16, device=DEV)
    sd.attn_dense(qd, kd, vd, out=out, lse_out=lse, seq_lens=lens_d)
    rp, ci = random_csr(2, Hq, nqb, nkb, min(5, nkb), seed=case[0], device=DEV)
    # the shorter sample's rows may only list blocks it has
    nkb_s, nqb_s = -(-short // bk), -(-short // bq)
    rp_h, ci_h = rp.cpu().numpy().copy(), ci.cpu().numpy().copy()
    for h in range(Hq):
        pos = 0
        new_rp = np.zeros(nqb + 1, dtype=np.int32)
        new_ci = np.full(ci_h.shape[2], -1, dtype=np.int32)
        for I in range(nqb):
            row = ci_h[1, h, rp_h[1, h, I]:rp_h[1, h, I + 1]]
            row = row[row < nkb_s] if I < nqb_s else row[:0]
            new_ci[pos:pos + len(row)] = row
            pos += len(row)
            new_rp[I + 1] = pos
        rp_h[1, h], ci_h[1, h] = new_rp, new_ci
    rp, ci = torch.from_numpy(rp_h).to(DEV), torch.from_numpy(ci_h).to(DEV)
    outs = torch.zeros_like(out)
    sd.attn_sparse(qd, kd, vd, sd.BlockIndex(rp, ci, bq, bk, nkb), out=outs, seq_lens=lens_d)
    for b, n in enumerate((L, short)):
        qb, kb, vb = q[b:b + 1, :, :n], k[b:b + 1, :, :n], v[b:b + 1, :, :n]
        assert_output_close(out[b:b + 1, :, :n], oracle.attn_dense(qb, kb, vb), torch.bfloat16, f"dense, sample {b}")
        logits = qb.double() @ kb.double().repeat_interleave(Hq // Hkv, 1).transpose(-1, -2) / math.sqrt(D)
        span = float(logits.abs().max())
        assert (lse[b:b + 1, :, :n].cpu().double() - torch.logsumexp(logits, dim=-1)).abs().max() < 2e-5 + 1e-6 * span
        nq_b = -(-n // bq)
        want = oracle.attn_sparse(qb, kb, vb, rp_h[b:b + 1, :, :nq_b + 1], ci_h[b:b + 1], bq, bk)
        assert_output_close(outs[b:b + 1, :, :n], want, torch.bfloat16, f"sparse {bq}x{bk}, sample {b}")
        assert (out[b, :, n:] == 0).all() and (outs[b, :, n:] == 0).all()      # rows past the length stay untouched


@pytest.mark.parametrize("B,Hq,Hkv,L,D", [(1, 2, 2, 256, 64), (1, 2, 1, 96, 128), (2, 2, 2, 192, 64)])
def test_dense_f32(B, Hq, Hkv, L, D):
    _say(f"dense f32 B={B} Hq={Hq} Hkv={Hkv} L={L} D={D}")
    q, k, v = _rand_qkv(B, Hq, Hkv, L, D, torch.float32, seed=L + D, scale=1.0 if D == 64 else None)
    want = oracle.attn_dense(q, k, v)
    got = sd.attn_dense(*_dev(q, k, v))
    assert_output_close(got, want, torch.float32, "dense f32")


def test_dense_strided_views_and_preallocated_output():
    # Q, K, V stored as [B, L, H, D] (the layout a fused QKV projection leaves) and viewed as [B, H, L, D]
    B, H, L, D = 1, 4, 256, 128
    g = torch.Generator().manual_seed(3)
    qkv = (torch.randn(3, B, L, H, D, generator=g) * 0.3).to(torch.bfloat16)
    q, k, v = (x.transpose(1, 2) for x in qkv)           # non-contiguous views
    want = oracle.attn_dense(q, k, v)
    qd, kd, vd = (x.transpose(1, 2) for x in qkv.to(DEV))
    out = torch.full((B, L, H, D), float("nan"), dtype=torch.bfloat16, device=DEV).transpose(1, 2)
    ret = sd.attn_dense(qd, kd, vd, out=out)
    assert ret.data_ptr() == out.data_ptr()
    assert_output_close(out, want, torch.bfloat16, "dense strided")


@pytest.mark.parametrize("dtype,L,D", [(torch.bfloat16, 512, 128), (torch.float32, 256, 64)])
def test_dense_log_sum_exp_side_output(dtype, L, D):
    q, k, v = _rand_qkv(1, 2, 1, L, D, dtype, seed=11)
    lse = torch.empty(1, 2, L, dtype=torch.float32, device=DEV)
    sd.attn_dense(*_dev(q, k, v), lse_out=lse)
    logits = q.double() @ k.double().repeat_interleave(2, 1).transpose(-1, -2) / math.sqrt(D)
    want = torch.logsumexp(logits, dim=-1)
    assert (lse.cpu().double() - want).abs().max() < 2e-5


# ----------------------------------------------------------------------------- sparse (Eq. 3, Eq. 4)
@pytest.mark.parametrize("bq,L,Hq,Hkv,D", [(128, 1024, 2, 2, 128), (64, 512, 4, 2, 128), (32, 256, 2, 1, 128), (64, 512, 2, 2, 64)])
def test_sparse_bf16_oracle_index_and_ragged_index(bq, L, Hq, Hkv, D):
    _say(f"sparse bf16 bq={bq} L={L} Hq={Hq} Hkv={Hkv} D={D}")
    bk = 64
    q, k, v = _rand_qkv(1, Hq, Hkv, L, D, torch.bfloat16, seed=bq + L)
    qd, kd, vd = _dev(q, k, v)
    # (a) the oracle's own selected pattern
    row_ptr, col_idx, _, _ = oracle.select_pattern(q, k, bq, bk, 0.3)
    ix = sd.BlockIndex(torch.from_numpy(row_ptr).to(DEV), torch.from_numpy(col_idx).to(DEV), bq, bk, L // bk)
    sd.index_validate(ix)
    got = sd.attn_sparse(qd, kd, vd, ix)
    assert_output_close(got, oracle.attn_sparse(q, k, v, row_ptr, col_idx, bq, bk), torch.bfloat16, "sparse bf16")
    # (b) ragged CSR: rows of different lengths, some empty (their output rows must be exactly zero)
    rp, ci = random_csr(1, Hq, L // bq, L // bk, min(5, L // bk), seed=L, device=DEV)
    ix = sd.BlockIndex(rp, ci, bq, bk, L // bk)
    got = sd.attn_sparse(qd, kd, vd, ix)
    want = oracle.attn_sparse(q, k, v, rp.cpu().numpy(), ci.cpu().numpy(), bq, bk)
    assert_output_close(got, want, torch.bfloat16, "sparse bf16 ragged")
    empty = (rp[..., 1:] == rp[..., :-1]).cpu().numpy()
    assert empty.any()
    rows_empty = np.repeat(empty, bq, axis=-1)
    assert (got.cpu().float().numpy()[rows_empty] == 0).all()


@pytest.mark.parametrize("bq,bk,L,D", [(32, 32, 256, 64), (64, 64, 256, 64), (128, 32, 256, 128)])
def test_sparse_f32(bq, bk, L, D):
    q, k, v = _rand_qkv(1, 2, 2, L, D, torch.float32, seed=bq + bk, scale=1.0 if D == 64 else None)
    qd, kd, vd = _dev(q, k, v)
    row_ptr, col_idx, _, _ = oracle.select_pattern(q, k, bq, bk, 0.3)
    ix = sd.BlockIndex(torch.from_numpy(row_ptr).to(DEV), torch.from_numpy(col_idx).to(DEV), bq, bk, L // bk)
    got = sd.attn_sparse(qd, kd, vd, ix)
    assert_output_close(got, oracle.attn_sparse(q, k, v, row_ptr, col_idx, bq, bk), torch.float32, "sparse f32")
    rp, ci = random_csr(1, 2, L // bq, L // bk, 3, seed=5, device=DEV)
    got = sd.attn_sparse(qd, kd, vd, sd.BlockIndex(rp, ci, bq, bk, L // bk))
    want = oracle.attn_sparse(q, k, v, rp.cpu().numpy(), ci.cpu().numpy(), bq, bk)
    assert_output_close(got, want, torch.float32, "sparse f32 ragged")


def test_sparse_with_every_block_listed_equals_dense_kernel_within_rounding():
    q, k, v = _rand_qkv(1, 2, 2, 512, 128, torch.bfloat16, seed=21)
    qd, kd, vd = _dev(q, k, v)
    ix = sd.select_pattern(qd, kd, 128, 64, 1.0)
    assert ix.col_idx.view(1, 2, 4, 8).cpu().eq(torch.arange(8)).all()
    a = sd.attn_sparse(qd, kd, vd, ix)
    want = oracle.attn_dense(q, k, v)
    assert_output_close(a, want, torch.bfloat16, "sparse rho=1")


def test_index_validate_flags_malformed_rows():
    rp, ci = random_csr(1, 2, 4, 8, 3, seed=1, device=DEV, allow_empty=False)
    ix = sd.BlockIndex(rp, ci, 64, 64, 8)
    sd.index_validate(ix)
    bad = ci.clone()
    bad[0, 1, 0] = 8                      # out of range
    with pytest.raises(sd.SparsedError) as e:
        sd.index_validate(sd.BlockIndex(rp, bad, 64, 64, 8))
    assert e.value.status == 8
    bad = ci.clone()
    n0 = int(rp[0, 0, 1])
    if n0 >= 2:
        bad[0, 0, 1] = bad[0, 0, 0]       # not strictly ascending
        with pytest.raises(sd.SparsedError):
            sd.index_validate(sd.BlockIndex(rp, bad, 64, 64, 8))


# ----------------------------------------------------------------------------- selection (Section 3.3, Eq. 6)
def _check_selection(q, k, bq, bk, rho, use_lse, what):
    B, Hq, L, D = q.shape
    nqb, nkb = -(-L // bq), -(-L // bk)
    qd, kd = _dev(q, k)
    pooled = torch.empty(B, Hq, nqb, nkb, dtype=torch.float32, device=DEV)
    lse = None
    if use_lse:
        lse = torch.empty(B, Hq, L, dtype=torch.float32, device=DEV)
        sd.attn_dense(qd, kd, kd, lse_out=lse)   # V is irrelevant for the log-sum-exp
    ix = sd.select_pattern(qd, kd, bq, bk, rho, lse_in=lse, pooled_out=pooled)
    sd.index_validate(ix)
    row_ptr, col_idx, apool, _ = oracle.select_pattern(q, k, bq, bk, rho)
    keep = oracle.kept_blocks(rho, nkb)
    np.testing.assert_array_equal(ix.row_ptr.cpu().numpy(), row_ptr)
    rel = np.abs(pooled.cpu().double().numpy() - apool) / apool
    assert rel.max() < 5e-6, f"{what}: pooled scores off by {rel.max():.2e} relative"
    tie_rows, tie_blocks = compare_index(ix.col_idx.cpu().numpy()[..., :nqb * keep], col_idx, apool.reshape(-1, nkb), keep)
    _say(f"{what}: rows={B * Hq * nqb} keep={keep} tie_rows={tie_rows} tie_blocks={tie_blocks} pooled_rel_err={rel.max():.2e}")
    if not use_lse and q.dtype == torch.bfloat16:
        # with the full workspace the call above pooled in one pass over the keys; with the least workspace the same
        # call runs row statistics and pooled scores as two passes: both must meet the same bar
        pooled2 = torch.empty_like(pooled)
        ws_min = torch.empty(sd.select_workspace_min_bytes(qd, bq, bk), dtype=torch.uint8, device=DEV)
        ix2 = sd.select_pattern(qd, kd, bq, bk, rho, workspace=ws_min, pooled_out=pooled2)
        rel2 = np.abs(pooled2.cpu().double().numpy() - apool) / apool
        assert rel2.max() < 5e-6, f"{what}: two-pass pooled scores off by {rel2.max():.2e} relative"
        compare_index(ix2.col_idx.cpu().numpy()[..., :nqb * keep], col_idx, apool.reshape(-1, nkb), keep)
        assert not torch.equal(pooled2, pooled) or rel.max() == 0     # two different kernels ran
        _say(f"{what}: two-pass route pooled_rel_err={rel2.max():.2e}")
    return ix


@pytest.mark.parametrize("bq,L,Hq,Hkv,D,rho,use_lse", [
    (128, 1024, 2, 2, 128, 0.25, False), (64, 1024, 4, 2, 128, 0.2, True), (32, 512, 2, 1, 64, 0.3, False),
    (128, 512, 2, 2, 128, 1.0, False), (64, 512, 2, 2, 128, 0.01, True)])
def test_select_bf16(bq, L, Hq, Hkv, D, rho, use_lse):
    q, k, _ = _rand_qkv(1, Hq, Hkv, L, D, torch.bfloat16, seed=bq + L, scale=0.45)
    _check_selection(q, k, bq, 64, rho, use_lse, f"select bf16 bq={bq} L={L} rho={rho}")


@pytest.mark.parametrize("bq,bk,L,D,use_lse", [(32, 32, 256, 64, False), (64, 64, 256, 64, True), (128, 32, 512, 128, False)])
def test_select_f32(bq, bk, L, D, use_lse):
    q, k, _ = _rand_qkv(1, 2, 2, L, D, torch.float32, seed=bq + bk, scale=1.0 if D == 64 else 0.45)
    _check_selection(q, k, bq, bk, 0.3, use_lse, f"select f32 {bq}x{bk} L={L}")


@pytest.mark.parametrize("bq,bk,L,D", [(128, 64, 1024, 128), (64, 32, 600, 64), (32, 128, 1000, 128)])
def test_select_one_pass_re_references_rows_whose_logits_climb(bq, bk, L, D):
    """The one-pass pooled-score kernel takes each row's reference from its first 32 keys. Here the logits climb by
    hundreds of octaves along the keys (every row's mass ends up in its last blocks), so the reference has to be
    raised again and again and everything a row has parked so far rescaled. Row log-sum-exp and pooled scores
    must still match the oracle wherever the oracle's value is representable in fp32."""
    H = 2
    g = torch.Generator().manual_seed(L + D)
    q = torch.zeros(1, H, L, D)
    k = torch.zeros(1, H, L, D)
    q[..., 0] = 8.0 + torch.rand(1, H, L, generator=g)                      # q . k / sqrt(D) = q0 * k0 / sqrt(D)
    ramp = torch.linspace(0.0, 1.0, L) ** 2                                 # slow at first, then steep
    k[..., 0] = (ramp * 40.0 * math.sqrt(D))[None, None, :] * (1.0 + 0.25 * torch.rand(1, H, L, generator=g))
    q[..., 1:] = 0.05 * torch.randn(1, H, L, D - 1, generator=g)
    k[..., 1:] = 0.05 * torch.randn(1, H, L, D - 1, generator=g)
    q, k = q.to(torch.bfloat16), k.to(torch.bfloat16)
    logit_span = float((q[..., 0].float().max() * k[..., 0].float().max()) / math.sqrt(D))
    assert logit_span > 300                                                  # > 430 octaves from first to last key
    qd, kd = _dev(q, k)
    nqb, nkb = -(-L // bq), -(-L // bk)
    pooled = torch.empty(1, H, nqb, nkb, dtype=torch.float32, device=DEV)
    ix = sd.select_pattern(qd, kd, bq, bk, 0.25, pooled_out=pooled)
    sd.index_validate(ix)
    row_ptr, col_idx, apool, _ = oracle.select_pattern(q, k, bq, bk, 0.25)
    got = pooled.cpu().double().numpy()
    big = apool > 1e-30                                                      # what fp32 can hold with full precision
    assert big.any() and (~big).any()
    rel = np.abs(got[big] - apool[big]) / apool[big]
    # fp32 logits of this size carry an error of |logit| * 2^-24 octaves, i.e. a relative error of that times ln 2 in
    # the exponential: the bar here scales with the span (the ordinary bar of 5e-6 holds for ordinary logits)
    tol = 5e-6 + 2e-7 * logit_span * 1.4427
    assert rel.max() < tol, f"pooled scores off by {rel.max():.2e} relative (bar {tol:.1e})"
    assert (got[~big] <= 1e-29).all()
    # the two-pass route on the same input, the same bar
    pooled2 = torch.empty_like(pooled)
    ws_min = torch.empty(sd.select_workspace_min_bytes(qd, bq, bk), dtype=torch.uint8, device=DEV)
    sd.select_pattern(qd, kd, bq, bk, 0.25, workspace=ws_min, pooled_out=pooled2)
    got2 = pooled2.cpu().double().numpy()
    assert (np.abs(got2[big] - apool[big]) / apool[big]).max() < tol
    keep = oracle.kept_blocks(0.25, nkb)
    # the kept sets agree wherever the cut is at a representable score
    cut = np.sort(apool.reshape(-1, nkb), axis=1)[:, ::-1][:, keep - 1]
    rows_ok = cut > 1e-30
    g_rows = ix.col_idx.cpu().numpy().reshape(-1, keep)[rows_ok]
    o_rows = col_idx.reshape(-1, keep)[rows_ok]
    compare_index(g_rows, o_rows, apool.reshape(-1, nkb)[rows_ok], keep)
    _say(f"re-reference {bq}x{bk} L={L}: logit span {logit_span:.0f}, pooled rel err {rel.max():.2e}, rows checked {int(rows_ok.sum())}")


def test_select_one_pass_closing_pass_in_several_segments():
    """625 key blocks per row at head dim 64 with 128-row query blocks: the closing pass of the one-pass kernel
    (row weights applied, rows summed) works through the key blocks in segments of 512 here."""
    bq, bk, L, D, rho = 128, 32, 20000, 64, 0.02
    q, k, _ = _rand_qkv(1, 1, 1, L, D, torch.bfloat16, seed=5, scale=0.5)
    _check_selection(q, k, bq, bk, rho, False, "select one pass, 625 key blocks, D=64")


def test_select_ties_resolve_to_lower_block_index():
    # Q = 0 makes every pooled score exactly 1/L: the kept set must be the first k blocks
    q = torch.zeros(1, 2, 512, 128, dtype=torch.bfloat16)
    k = torch.randn(1, 2, 512, 128).to(torch.bfloat16)
    ix = sd.select_pattern(*_dev(q, k), 64, 64, 0.4)
    keep = oracle.kept_blocks(0.4, 8)
    assert ix.col_idx.cpu().view(1, 2, 8, keep).eq(torch.arange(keep)).all()


def test_select_isolated_matches_oracle():
    q, k, _ = _rand_qkv(1, 2, 2, 1024, 128, torch.bfloat16, seed=31, scale=0.45)
    bq, bk, rho, n_pre = 128, 64, 0.25, 6
    ix = sd.select_pattern_isolated(*_dev(q, k), bq, bk, rho, n_pre)
    apool = oracle.pool_scores(q, k, bq, bk)
    rp, ci = oracle.select_isolated(apool, rho, n_pre)
    np.testing.assert_array_equal(ix.row_ptr.cpu().numpy(), rp)
    got, want = ix.col_idx.cpu().numpy(), ci
    keep_pre, keep_gen = oracle.kept_blocks(rho, n_pre), oracle.kept_blocks(rho, 16 - n_pre)
    g = got.reshape(-1, keep_pre + keep_gen)
    w = want.reshape(-1, keep_pre + keep_gen)
    ap = apool.reshape(-1, 16)
    compare_index(g[:, :keep_pre], w[:, :keep_pre], np.where(np.arange(16) < n_pre, ap, -1.0), keep_pre)
    gen_scores = np.where(np.arange(16) >= n_pre, ap, -1.0)
    compare_index(g[:, keep_pre:], w[:, keep_pre:], gen_scores, keep_gen)


# ----------------------------------------------------------------------------- closed form W1 on the GPU
def test_closed_form_w1_embedded_in_head_dim_64():
    # tests/golden/w1_closed_form.txt, padded to L=64 x d=64: the 4 worked rows/keys are spread so that
    # each falls in its own 32-block, all other keys get a logit of -60 (weight e^-60), scale sqrt(64)=8 undone on q.
    from test_oracle_pins import _read_golden
    g = _read_golden("w1_closed_form.txt")
    L, D = 128, 64
    q = torch.zeros(1, 1, L, D)
    k = torch.zeros(1, 1, L, D)
    v = torch.zeros(1, 1, L, D)
    rows = [0, 1, 32, 33]                       # query rows 0,1 in block 0; 2,3 in block 1 (bq = 32)
    keys = [0, 1, 64, 65]                       # keys 0,1 in key block 0; 2,3 in key block 2 (bk = 32)
    k[0, 0, :, 1] = -60.0
    for n, j in enumerate(keys):
        k[0, 0, j, 0] = math.log(g["w"][n])
        k[0, 0, j, 1] = 0.0
        v[0, 0, j, 0] = g["v"][n]
    q[0, 0, :, 1] = 8.0                         # every query pushes the padding keys to logit -60
    for n, i in enumerate(rows):
        q[0, 0, i, 0] = 8.0 * g["q"][n]
    want = oracle.attn_dense(q, k, v)
    np.testing.assert_allclose(want[0, 0, rows, 0], g["dense"], atol=1e-6)
    got = sd.attn_dense(*_dev(q, k, v))
    np.testing.assert_allclose(got.cpu().double().numpy()[0, 0, rows, 0], g["dense"], atol=1e-5)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_closed_form_w1_replicated_through_the_whole_path(dtype):
    """W1 (tests/golden/w1_closed_form.txt) through dense, pooled scores, index and sparse on the GPU.

    Every worked query row and every worked key (with its value) is repeated 16 times, so the 2 x 2 blocks of the
    worked example become 32 x 32 blocks. Repeating a key r times divides each of its probabilities by r and leaves
    block sums, outputs and the ranking as they were; a block mean is then the worked one divided by r = 16."""
    from test_oracle_pins import _read_golden
    g = _read_golden("w1_closed_form.txt")
    rep, L, D, bq, bk = 16, 64, 64, 32, 32
    q = torch.zeros(1, 1, L, D)
    k = torch.zeros(1, 1, L, D)
    v = torch.zeros(1, 1, L, D)
    for n in range(4):
        q[0, 0, n * rep:(n + 1) * rep, 0] = 8.0 * g["q"][n]          # sqrt(64) = 8 undoes the 1/sqrt(d) scale
        k[0, 0, n * rep:(n + 1) * rep, 0] = math.log(g["w"][n])
        v[0, 0, n * rep:(n + 1) * rep, 0] = g["v"][n]
    q, k, v = q.to(dtype), k.to(dtype), v.to(dtype)
    # bf16 rounds ln 3 and ln 5 (relative 2^-9), which moves the probabilities by a few 1e-3
    tol_out, tol_pool = (1e-5, 2e-6) if dtype == torch.float32 else (2e-2, 1e-2)
    qd, kd, vd = _dev(q, k, v)
    lse = torch.empty(1, 1, L, dtype=torch.float32, device=DEV)
    pooled = torch.empty(1, 1, 2, 2, dtype=torch.float32, device=DEV)
    dense = sd.attn_dense(qd, kd, vd, lse_out=lse)
    ix = sd.select_pattern(qd, kd, bq, bk, 0.5, lse_in=lse, pooled_out=pooled)
    ix_own = sd.select_pattern(qd, kd, bq, bk, 0.5)
    sparse = sd.attn_sparse(qd, kd, vd, ix)
    torch.cuda.synchronize()
    want_dense = np.repeat(np.asarray(g["dense"]), rep)
    want_sparse = np.repeat(np.asarray(g["sparse"]), rep)
    np.testing.assert_allclose(dense.cpu().double().numpy()[0, 0, :, 0], want_dense, atol=tol_out)
    np.testing.assert_allclose(pooled.cpu().double().numpy().reshape(-1), np.asarray(g["apool"]) / rep, rtol=tol_pool)
    np.testing.assert_array_equal(ix.row_ptr.cpu().numpy().reshape(-1), np.asarray(g["row_ptr"], dtype=np.int32))
    np.testing.assert_array_equal(ix.col_idx.cpu().numpy().reshape(-1), np.asarray(g["col_idx"], dtype=np.int32))
    np.testing.assert_array_equal(ix_own.col_idx.cpu().numpy().reshape(-1), np.asarray(g["col_idx"], dtype=np.int32))
    np.testing.assert_allclose(sparse.cpu().double().numpy()[0, 0, :, 0], want_sparse, atol=tol_out)
    assert (dense.cpu().float()[0, 0, :, 1:] == 0).all() and (sparse.cpu().float()[0, 0, :, 1:] == 0).all()

# ----------------------------------------------------------------------------- sequence lengths that are not block multiples
@pytest.mark.parametrize("dtype,L,Hq,Hkv,D", [
    (torch.bfloat16, 200, 2, 1, 128),    # 64-row groups; 3 full key tiles + 8 keys
    (torch.bfloat16, 1000, 2, 2, 128),   # 128-row groups; last key tile has 40 keys
    (torch.bfloat16, 1100, 1, 1, 128),   # 256-row groups; last key tile has 12 keys (second sub-tile empty)
    (torch.bfloat16, 65, 2, 2, 64),      # one key in the last tile
    (torch.bfloat16, 31, 1, 1, 128),     # a single partial tile
    (torch.bfloat16, 97, 1, 1, 64),      # 33 keys in the last tile: one key in its second sub-tile
    (torch.float32, 100, 2, 1, 64),
    (torch.float32, 47, 2, 2, 128),
    (torch.float32, 333, 1, 1, 64),
])
def test_dense_ragged_length(dtype, L, Hq, Hkv, D):
    _say(f"dense ragged {dtype} L={L} Hq={Hq} Hkv={Hkv} D={D}")
    q, k, v = _rand_qkv(1, Hq, Hkv, L, D, dtype, seed=L, scale=1.0 if dtype == torch.float32 and D == 64 else None)
    lse = torch.full((1, Hq, L), float("nan"), dtype=torch.float32, device=DEV)
    guard = torch.full((1, Hq, L + 300, D), 7.0, dtype=dtype, device=DEV)   # room behind the output: must stay untouched
    out = guard[:, :, :L]
    got = sd.attn_dense(*_dev(q, k, v), out=out, lse_out=lse)
    torch.cuda.synchronize()
    assert_output_close(got, oracle.attn_dense(q, k, v), dtype, "dense ragged")
    assert (guard[:, :, L:] == 7.0).all(), "rows past L were written"
    logits = (q.double() @ k.double().repeat_interleave(Hq // Hkv, 1).transpose(-1, -2)) / math.sqrt(D)
    want_lse = torch.logsumexp(logits, dim=-1)
    assert (lse.cpu().double() - want_lse).abs().max() < (2e-5 if dtype == torch.float32 else 1e-4)


@pytest.mark.parametrize("dtype,bq,bk,L,Hq,Hkv,D,rho,use_lse", [
    (torch.bfloat16, 128, 64, 1000, 2, 2, 128, 0.25, False),
    (torch.bfloat16, 64, 64, 1100, 2, 1, 128, 0.2, True),
    (torch.bfloat16, 32, 64, 200, 2, 2, 64, 0.5, False),
    (torch.bfloat16, 128, 128, 1000, 2, 2, 128, 0.3, False),   # the paper's square 128 blocks: last one 64 + 40 keys
    (torch.bfloat16, 128, 128, 960, 2, 1, 128, 0.3, True),     # last block 64 keys: its second tile does not exist
    (torch.bfloat16, 64, 128, 900, 2, 2, 128, 0.25, False),    # last block 4 keys
    (torch.bfloat16, 32, 128, 1024, 2, 2, 64, 0.5, True),      # every block full
    (torch.bfloat16, 128, 128, 100, 1, 1, 128, 1.0, False),    # a single partial block
    (torch.bfloat16, 32, 32, 1000, 2, 2, 128, 0.5, False),     # the paper's square 32 blocks: last one 8 keys
    (torch.bfloat16, 32, 32, 992, 2, 1, 64, 0.5, True),        # 31 full blocks: the last tile has one block only
    (torch.bfloat16, 64, 32, 1024, 2, 2, 128, 0.3, False),
    (torch.bfloat16, 64, 32, 50, 1, 1, 128, 1.0, False),       # one tile: a full block and a partial one
    (torch.bfloat16, 32, 32, 20, 1, 1, 64, 1.0, True),         # a single partial block
    (torch.bfloat16, 128, 32, 1000, 2, 2, 128, 0.3, False),    # 128-row query blocks over 32-key blocks: last block 8 keys
    (torch.bfloat16, 128, 32, 992, 2, 1, 64, 0.5, True),       # odd number of blocks
    (torch.bfloat16, 128, 32, 40, 1, 1, 128, 1.0, False),      # one tile: a full block and a partial one
    (torch.float32, 32, 32, 100, 2, 2, 64, 0.5, False),
    (torch.float32, 64, 64, 333, 1, 1, 64, 0.3, True),      # last 64-key block: 13 keys, its second 32-key tile is empty
    (torch.float32, 128, 32, 300, 2, 1, 128, 0.3, False),
    (torch.float32, 128, 128, 300, 2, 1, 128, 0.4, False),     # fp32, 128-key blocks over 32-key tiles: last block 44 keys
    (torch.float32, 32, 128, 520, 2, 2, 64, 0.3, True),        # last block 8 keys
])
def test_select_and_sparse_ragged_length(dtype, bq, bk, L, Hq, Hkv, D, rho, use_lse):
    _say(f"select+sparse ragged {dtype} {bq}x{bk} L={L}")
    q, k, v = _rand_qkv(1, Hq, Hkv, L, D, dtype, seed=L + bq, scale=1.0 if dtype == torch.float32 and D == 64 else 0.45)
    ix = _check_selection(q, k, bq, bk, rho, use_lse, f"select ragged L={L}")
    nqb, nkb = -(-L // bq), -(-L // bk)
    qd, kd, vd = _dev(q, k, v)
    # the GPU's own pattern
    rp, ci = ix.row_ptr.cpu().numpy(), ix.col_idx.cpu().numpy()
    got = sd.attn_sparse(qd, kd, vd, ix)
    assert_output_close(got, oracle.attn_sparse(q, k, v, rp, ci, bq, bk), dtype, "sparse ragged (selected)")
    # a pattern in which EVERY row keeps the partial last key block, plus random others, some rows only that block
    rng = np.random.default_rng(L)
    rows = []
    for I in range(Hq * nqb):
        others = rng.choice(nkb - 1, size=int(rng.integers(0, min(4, nkb - 1) + 1)), replace=False) if nkb > 1 else []
        rows.append(sorted(set(int(x) for x in others) | {nkb - 1}))
    cap = max(sum(len(r) for r in rows[h * nqb:(h + 1) * nqb]) for h in range(Hq))
    rp = np.zeros((1, Hq, nqb + 1), np.int32)
    ci = np.zeros((1, Hq, cap), np.int32)
    for h in range(Hq):
        pos = 0
        for I in range(nqb):
            r = rows[h * nqb + I]
            ci[0, h, pos:pos + len(r)] = r
            pos += len(r)
            rp[0, h, I + 1] = pos
    ix2 = sd.BlockIndex(torch.from_numpy(rp).to(DEV), torch.from_numpy(ci).to(DEV), bq, bk, nkb)
    sd.index_validate(ix2)
    guard = torch.full((1, Hq, L + 200, D), 7.0, dtype=dtype, device=DEV)
    got = sd.attn_sparse(qd, kd, vd, ix2, out=guard[:, :, :L])
    torch.cuda.synchronize()
    assert_output_close(got, oracle.attn_sparse(q, k, v, rp, ci, bq, bk), dtype, "sparse ragged (last block in every row)")
    assert (guard[:, :, L:] == 7.0).all(), "rows past L were written"


@pytest.mark.parametrize("dtype,bq,bk,L,D,ptok,rho", [
    (torch.bfloat16, 128, 64, 1024, 128, 200, 0.3),    # boundary inside key block 3: 8 prefill keys, 56 generation keys
    (torch.bfloat16, 64, 64, 1000, 128, 990, 0.25),    # inside the partial last block
    (torch.bfloat16, 32, 64, 512, 64, 1, 0.4),         # a single prefill key
    (torch.bfloat16, 128, 64, 1024, 128, 1023, 0.3),   # a single generation key
    (torch.bfloat16, 128, 128, 1024, 128, 200, 0.3),   # 128-key blocks: boundary inside the second tile of block 1
    (torch.bfloat16, 64, 128, 1000, 128, 930, 0.4),    # inside the partial last 128-key block
    (torch.bfloat16, 32, 32, 512, 128, 77, 0.5),       # 32-key blocks
    (torch.bfloat16, 64, 32, 500, 64, 490, 0.4),       # inside the partial last 32-key block
    (torch.bfloat16, 128, 32, 640, 128, 333, 0.3),     # 128-row query blocks over 32-key blocks
    (torch.float32, 32, 32, 256, 64, 50, 0.3),
    (torch.float32, 64, 64, 300, 64, 70, 0.4),         # 64-key blocks over 32-key tiles, partial last block
    (torch.float32, 128, 128, 400, 128, 150, 0.4),     # fp32, 128-key blocks
])
def test_isolated_selection_with_the_boundary_inside_a_block(dtype, bq, bk, L, D, ptok, rho):
    _say(f"isolated selection, token boundary: {dtype} {bq}x{bk} L={L} p={ptok}")
    H = 3
    q, k, v = _rand_qkv(1, H, H, L, D, dtype, seed=L + ptok, scale=1.0 if dtype == torch.float32 and D == 64 else 0.6)
    qd, kd, vd = _dev(q, k, v)
    ix = sd.select_pattern_isolated_tokens(qd, kd, bq, bk, rho, ptok)
    sd.index_validate(ix)
    rp_o, ci_o, ap, n_pre, vblock = oracle.select_isolated_tokens(q, k, bq, bk, rho, ptok)
    nv = ap.shape[-1]
    keep_pre, keep_gen = oracle.kept_blocks(rho, n_pre), oracle.kept_blocks(rho, nv - n_pre)
    rp, ci = ix.row_ptr.cpu().numpy(), ix.col_idx.cpu().numpy()
    nqb = -(-L // bq)
    ties = short_rows = 0
    for h in range(H):
        assert rp[0, h, 0] == 0
        for I in range(nqb):
            got = ci[0, h, rp[0, h, I]:rp[0, h, I + 1]].tolist()
            want = ci_o[0, h, rp_o[0, h, I]:rp_o[0, h, I + 1]].tolist()
            assert got == sorted(set(got))
            short_rows += len(got) == keep_pre + keep_gen - 1
            if got == want:
                continue
            # a difference is legal only between entries whose oracle score ties with the cut of their range
            a = ap[0, h, I]
            cut_pre = np.sort(a[:n_pre])[::-1][keep_pre - 1]
            cut_gen = np.sort(a[n_pre:])[::-1][keep_gen - 1]
            for J in set(got) ^ set(want):
                ok = any((abs(a[e] - (cut_pre if e < n_pre else cut_gen)) <= 1e-5 * (cut_pre if e < n_pre else cut_gen))
                         for e in range(nv) if vblock[e] == J)
                assert ok, f"head {h} row {I}: block {J} differs outside the tie band"
            ties += 1
    _say(f"   rows={H * nqb} keep={keep_pre}+{keep_gen} rows_with_the_boundary_block_kept_twice={short_rows} tie_rows={ties}")
    got = sd.attn_sparse(qd, kd, vd, ix)
    assert_output_close(got, oracle.attn_sparse(q, k, v, rp, ci, bq, bk), dtype, "sparse on the token-boundary pattern")
    # on a block edge the token form is the block form
    edge = sd.select_pattern_isolated_tokens(qd, kd, bq, bk, rho, 2 * bk)
    blk = sd.select_pattern_isolated(qd, kd, bq, bk, rho, 2)
    assert torch.equal(edge.row_ptr, blk.row_ptr) and torch.equal(edge.col_idx, blk.col_idx)


def test_window_index_ragged_length():
    from oracle import patterns
    for L, bq, bk, window, sink in [(1000, 128, 64, 256, 70), (333, 32, 32, 50, 0), (821, 32, 64, 8, 410)]:
        # the token-level definition on the padded grid, cut back to the L real tokens
        nqb, nkb = -(-L // bq), -(-L // bk)
        m = patterns.window_token_mask(L, window, sink)
        blocks = np.zeros((nqb, nkb), bool)
        for I in range(nqb):
            for J in range(nkb):
                blocks[I, J] = m[I * bq:(I + 1) * bq, J * bk:(J + 1) * bk].any()
        ptr, col = patterns.rows_to_csr([np.nonzero(r)[0].astype(np.int32) for r in blocks], 2)
        ix = sd.index_fill_window(1, 2, L, bq, bk, window, sink, DEV)
        sd.index_validate(ix)
        assert np.array_equal(ix.row_ptr.cpu().numpy().reshape(2, -1), ptr)
        assert np.array_equal(ix.row_ptr.cpu().numpy().reshape(2, -1)[:, -1], [col.shape[1]] * 2)
        assert np.array_equal(ix.col_idx.cpu().numpy().reshape(2, -1)[:, :col.shape[1]], col)


# ----------------------------------------------------------------------------- strided views through every entry point
@pytest.mark.parametrize("dtype,L,bq,bk,D", [(torch.bfloat16, 1000, 128, 64, 128), (torch.bfloat16, 333, 64, 64, 64), (torch.float32, 200, 32, 32, 64)])
def test_packed_qkv_views_through_select_and_sparse(dtype, L, bq, bk, D):
    """Q, K, V as views of one packed projection output [B, L, 3, H, D] (row stride 3*H*D, head stride D):
    nothing is copied, every kernel sees strided rows, including the partial last tile."""
    B, H = 2, 3
    g = torch.Generator().manual_seed(L)
    packed = (torch.randn(B, L, 3, H, D, generator=g) * 0.6).to(dtype)
    pd = packed.to(DEV)
    q, k, v = (packed[:, :, i].permute(0, 2, 1, 3) for i in range(3))          # [B, H, L, D] views on the host
    qd, kd, vd = (pd[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    assert not qd.is_contiguous() and qd.stride(2) == 3 * H * D
    dense = sd.attn_dense(qd, kd, vd)
    assert_output_close(dense, oracle.attn_dense(q, k, v), dtype, "dense on packed views")
    ix = _check_selection(q, k, bq, bk, 0.3, False, "select on packed views")   # helper copies q, k to the device contiguously
    ixv = sd.select_pattern(qd, kd, bq, bk, 0.3)                                 # the same call on the strided views
    assert torch.equal(ix.row_ptr, ixv.row_ptr) and torch.equal(ix.col_idx, ixv.col_idx)
    got = sd.attn_sparse(qd, kd, vd, ixv)
    want = oracle.attn_sparse(q, k, v, ixv.row_ptr.cpu().numpy(), ixv.col_idx.cpu().numpy(), bq, bk)
    assert_output_close(got, want, dtype, "sparse on packed views")


# ----------------------------------------------------------------------------- streams
def test_calls_run_on_the_callers_stream():
    """Work is enqueued on the stream passed in (here: torch's current stream inside a stream context), so a chain
    dense -> select -> sparse on a side stream needs no synchronisation in between and two chains on two
    streams, each with its own workspace, do not disturb each other."""
    q, k, v = _rand_qkv(1, 4, 2, 1024, 128, torch.bfloat16, seed=5, scale=0.5)
    qd, kd, vd = _dev(q, k, v)
    q2 = (qd.float() * 0.5).to(torch.bfloat16)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    results = []
    torch.cuda.synchronize()
    for s, qq in zip(streams, (qd, q2)):
        with torch.cuda.stream(s):
            lse = torch.empty(1, 4, 1024, dtype=torch.float32, device=DEV)
            dense = sd.attn_dense(qq, kd, vd, lse_out=lse)
            ix = sd.select_pattern(qq, kd, 128, 64, 0.25, lse_in=lse)
            sparse = sd.attn_sparse(qq, kd, vd, ix)
            results.append((qq, dense, ix, sparse))
    for s in streams:
        s.synchronize()
    for qq, dense, ix, sparse in results:
        qc = qq.cpu()
        assert_output_close(dense, oracle.attn_dense(qc, k, v), torch.bfloat16, "dense on a side stream")
        want = oracle.attn_sparse(qc, k, v, ix.row_ptr.cpu().numpy(), ix.col_idx.cpu().numpy(), 128, 64)
        assert_output_close(sparse, want, torch.bfloat16, "sparse on a side stream")
        ref = sd.select_pattern(qq, kd, 128, 64, 0.25)          # default stream, own statistics
        assert torch.equal(ref.row_ptr, ix.row_ptr)
        _, ci_o, apool, _ = oracle.select_pattern(qc, k, 128, 64, 0.25)
        compare_index(ix.col_idx.cpu().numpy(), ci_o, apool.reshape(-1, 16), oracle.kept_blocks(0.25, 16))


# ----------------------------------------------------------------------------- per-sample lengths inside one batch
@pytest.mark.parametrize("dtype,bq,bk,L,D,lens,rho", [
    (torch.bfloat16, 128, 64, 1024, 128, [1024, 70, 333, 640], 0.25),
    (torch.bfloat16, 64, 64, 512, 64, [1, 512, 65, 129], 0.3),
    (torch.bfloat16, 128, 128, 1024, 128, [1024, 70, 333, 640, 129], 0.3),   # 128-key blocks
    (torch.bfloat16, 32, 32, 512, 64, [512, 33, 100, 1, 480], 0.5),          # 32-key blocks
    (torch.float32, 32, 32, 200, 64, [200, 33, 100], 0.4),
])
def test_per_sample_lengths(dtype, bq, bk, L, D, lens, rho):
    """A padded batch with a length per sample: every sample must equal the oracle run on that sample cut to
    its length, and nothing past a sample's length may be written."""
    _say(f"per-sample lengths {dtype} {bq}x{bk} L={L} lens={lens}")
    B, Hq, Hkv = len(lens), 2, 1
    q, k, v = _rand_qkv(B, Hq, Hkv, L, D, dtype, seed=L + D, scale=1.0 if dtype == torch.float32 and D == 64 else 0.5)
    qd, kd, vd = _dev(q, k, v)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    nqb, nkb = -(-L // bq), -(-L // bk)
    out = torch.full((B, Hq, L, D), 7.0, dtype=dtype, device=DEV)
    lse = torch.full((B, Hq, L), 7.0, dtype=torch.float32, device=DEV)
    sd.attn_dense(qd, kd, vd, out=out, lse_out=lse, seq_lens=sl)
    ix = sd.select_pattern(qd, kd, bq, bk, rho, lse_in=lse, seq_lens=sl)
    ix_own = sd.select_pattern(qd, kd, bq, bk, rho, seq_lens=sl)      # statistics pass of its own
    sd.index_validate(ix)
    assert torch.equal(ix.row_ptr, ix_own.row_ptr)
    out_s = torch.full((B, Hq, L, D), 7.0, dtype=dtype, device=DEV)
    sd.attn_sparse(qd, kd, vd, ix, out=out_s, seq_lens=sl)
    torch.cuda.synchronize()
    rp, ci = ix.row_ptr.cpu().numpy(), ix.col_idx.cpu().numpy()
    for b, n in enumerate(lens):
        qb, kb, vb = q[b:b + 1, :, :n], k[b:b + 1, :, :n], v[b:b + 1, :, :n]
        assert_output_close(out[b:b + 1, :, :n], oracle.attn_dense(qb, kb, vb), dtype, f"dense sample {b}")
        assert (out[b, :, n:] == 7.0).all() and (lse[b, :, n:] == 7.0).all() and (out_s[b, :, n:] == 7.0).all()
        rp_o, ci_o, apool, _ = oracle.select_pattern(qb, kb, bq, bk, rho)
        nqb_b, nkb_b = -(-n // bq), -(-n // bk)
        keep = oracle.kept_blocks(rho, nkb_b)
        for h in range(Hq):
            assert rp[b, h, :nqb_b + 1].tolist() == rp_o[0, h].tolist()
            assert (rp[b, h, nqb_b:] == nqb_b * keep).all()           # query blocks the sample does not have: empty rows
            compare_index(ci[b, h, :nqb_b * keep], ci_o[0, h], apool[0, h], keep)
        # sparse output of this sample against the oracle on the GPU's own rows for it
        rp_b = rp[b:b + 1, :, :nqb_b + 1].copy()
        want = oracle.attn_sparse(qb, kb, vb, rp_b, ci[b:b + 1], bq, bk)
        assert_output_close(out_s[b:b + 1, :, :n], want, dtype, f"sparse sample {b}")


@pytest.mark.parametrize("dtype,bq,bk,L,D,lens,pblocks,rho", [
    (torch.bfloat16, 128, 64, 1024, 128, [1024, 700, 200, 129, 64], 4, 0.3),   # prefill of 4 key blocks; two samples no longer than it
    (torch.bfloat16, 64, 128, 1000, 64, [1000, 500, 257], 2, 0.4),
    (torch.float32, 32, 32, 256, 64, [256, 100, 33, 20], 3, 0.5),
])
def test_isolated_selection_with_per_sample_lengths(dtype, bq, bk, L, D, lens, pblocks, rho):
    """Isolated selection in a padded batch: every sample ranks its prefill blocks [0, p) and its generation blocks
    [p, nkb_b) separately, as if passed alone; a sample no longer than the prefill has one range only."""
    B, H = len(lens), 2
    q, k, v = _rand_qkv(B, H, H, L, D, dtype, seed=L + 3 * D, scale=1.0 if dtype == torch.float32 and D == 64 else 0.5)
    qd, kd, vd = _dev(q, k, v)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    ix = sd.select_pattern_isolated(qd, kd, bq, bk, rho, pblocks, seq_lens=sl)
    sd.index_validate(ix)
    out_s = torch.full((B, H, L, D), 7.0, dtype=dtype, device=DEV)
    sd.attn_sparse(qd, kd, vd, ix, out=out_s, seq_lens=sl)
    torch.cuda.synchronize()
    rp, ci = ix.row_ptr.cpu().numpy(), ix.col_idx.cpu().numpy()
    for b, n in enumerate(lens):
        qb, kb, vb = q[b:b + 1, :, :n], k[b:b + 1, :, :n], v[b:b + 1, :, :n]
        nqb_b, nkb_b = -(-n // bq), -(-n // bk)
        n_pre = min(pblocks, nkb_b)
        apool = oracle.pool_scores(qb, kb, bq, bk)
        rp_o, ci_o = oracle.select_isolated(apool, rho, n_pre)
        k_lo, k_hi = oracle.kept_blocks(rho, n_pre), (oracle.kept_blocks(rho, nkb_b - n_pre) if nkb_b > n_pre else 0)
        keep = k_lo + k_hi
        for h in range(H):
            assert rp[b, h, :nqb_b + 1].tolist() == rp_o[0, h].tolist()
            assert (rp[b, h, nqb_b:] == nqb_b * keep).all()
            got = ci[b, h, :nqb_b * keep].reshape(nqb_b, keep)
            want = ci_o[0, h].reshape(nqb_b, keep)
            compare_index(got[:, :k_lo].reshape(-1), want[:, :k_lo].reshape(-1), apool[0, h][:, :n_pre], k_lo)
            if k_hi:
                compare_index(got[:, k_lo:].reshape(-1) - n_pre, want[:, k_lo:].reshape(-1) - n_pre, apool[0, h][:, n_pre:], k_hi)
        rp_b = rp[b:b + 1, :, :nqb_b + 1].copy()
        want = oracle.attn_sparse(qb, kb, vb, rp_b, ci[b:b + 1], bq, bk)
        assert_output_close(out_s[b:b + 1, :, :n], want, dtype, f"sparse sample {b}")
        assert (out_s[b, :, n:] == 7.0).all()


@pytest.mark.parametrize("dtype,bq,bk,L,D,lens,ptok,rho", [
    # boundary inside key block 3; samples longer than it (two ranges, block 3 split), one ending inside block 3 after
    # the boundary (a generation part of 10 keys), one ending before the boundary and one before block 3 (one range each)
    (torch.bfloat16, 128, 64, 1024, 128, [1024, 700, 210, 199, 150, 64], 200, 0.3),
    (torch.bfloat16, 64, 128, 1000, 64, [1000, 500, 301, 300, 257], 300, 0.4),        # 128-key blocks
    (torch.bfloat16, 32, 32, 512, 128, [512, 100, 78, 77, 40], 77, 0.5),              # 32-key blocks
    (torch.float32, 32, 32, 256, 64, [256, 100, 51, 50, 33, 20], 50, 0.3),
])
def test_isolated_selection_token_boundary_with_per_sample_lengths(dtype, bq, bk, L, D, lens, ptok, rho):
    """A prefill boundary inside a key block in a padded batch (Eq. 5 on samples of different length): every sample
    is ranked as if passed alone at its own length, with the boundary at min(p, its length)."""
    B, H = len(lens), 2
    _say(f"isolated selection, token boundary + per-sample lengths: {dtype} {bq}x{bk} L={L} p={ptok} lens={lens}")
    q, k, v = _rand_qkv(B, H, H, L, D, dtype, seed=L + ptok + D, scale=1.0 if dtype == torch.float32 and D == 64 else 0.6)
    qd, kd, vd = _dev(q, k, v)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    ix = sd.select_pattern_isolated_tokens(qd, kd, bq, bk, rho, ptok, seq_lens=sl)
    sd.index_validate(ix)
    out_s = torch.full((B, H, L, D), 7.0, dtype=dtype, device=DEV)
    sd.attn_sparse(qd, kd, vd, ix, out=out_s, seq_lens=sl)
    torch.cuda.synchronize()
    rp, ci = ix.row_ptr.cpu().numpy(), ix.col_idx.cpu().numpy()
    ties = short_rows = 0
    for b, n in enumerate(lens):
        qb, kb, vb = q[b:b + 1, :, :n], k[b:b + 1, :, :n], v[b:b + 1, :, :n]
        nqb_b = -(-n // bq)
        rp_o, ci_o, ap, n_pre, vblock = oracle.select_isolated_tokens(qb, kb, bq, bk, rho, min(ptok, n))
        nv = ap.shape[-1]
        keep_pre = oracle.kept_blocks(rho, n_pre)
        keep_gen = oracle.kept_blocks(rho, nv - n_pre) if nv > n_pre else 0
        for h in range(H):
            assert rp[b, h, 0] == 0 and (rp[b, h, nqb_b:] == rp[b, h, nqb_b]).all()     # query blocks past the sample: empty rows
            for I in range(nqb_b):
                got = ci[b, h, rp[b, h, I]:rp[b, h, I + 1]].tolist()
                want = ci_o[0, h, rp_o[0, h, I]:rp_o[0, h, I + 1]].tolist()
                assert got == sorted(set(got)) and len(got) == len(want)
                short_rows += (keep_gen > 0 and len(got) == keep_pre + keep_gen - 1)
                if got == want:
                    continue
                a = ap[0, h, I]
                cut_pre = np.sort(a[:n_pre])[::-1][keep_pre - 1]
                cut_gen = np.sort(a[n_pre:])[::-1][keep_gen - 1] if keep_gen else 0.0
                for J in set(got) ^ set(want):
                    ok = any((abs(a[e] - (cut_pre if e < n_pre else cut_gen)) <= 1e-5 * (cut_pre if e < n_pre else cut_gen))
                             for e in range(nv) if vblock[e] == J)
                    assert ok, f"sample {b} head {h} row {I}: block {J} differs outside the tie band"
                ties += 1
        # sparse attention on the GPU-built rows of this sample, as if it had been passed alone
        rp_b = rp[b:b + 1, :, :nqb_b + 1].copy()
        want = oracle.attn_sparse(qb, kb, vb, rp_b, ci[b:b + 1], bq, bk)
        assert_output_close(out_s[b:b + 1, :, :n], want, dtype, f"sparse sample {b}")
        assert (out_s[b, :, n:] == 7.0).all()
    _say(f"   rows_with_the_boundary_block_kept_twice={short_rows} tie_rows={ties}")


# ----------------------------------------------------------------------------- seeded sweep over the parameter space
def _sweep_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
        D = int(rng.choice([64, 128]))
        bq = int(rng.choice([32, 64, 128]))
        bk = 64 if dtype == torch.bfloat16 else int(rng.choice([32, 64]))
        Hkv = int(rng.choice([1, 2]))
        Hq = Hkv * int(rng.choice([1, 2, 3]))
        B = int(rng.choice([1, 2]))
        L = int(rng.integers(1, 700 if dtype == torch.bfloat16 else 300))
        rho = float(rng.choice([0.05, 0.2, 0.5, 1.0]))
        cases.append((i, dtype, B, Hq, Hkv, L, D, bq, bk, rho))
    return cases


def _sweep_cases_wide_key_blocks(n, seed):
    """bf16 with 128-key blocks (the paper's square 128 x 128 among them): lengths chosen so that the last block is
    often short, sometimes no longer than one 64-key tile."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        bq = int(rng.choice([32, 64, 128]))
        Hkv = int(rng.choice([1, 2]))
        Hq = Hkv * int(rng.choice([1, 2]))
        B = int(rng.choice([1, 2]))
        L = int(rng.integers(1, 1200))
        rho = float(rng.choice([0.1, 0.3, 0.5, 1.0]))
        cases.append((1000 + i, torch.bfloat16, B, Hq, Hkv, L, D, bq, 128, rho))
    return cases


_SWEEP_IDS = lambda c: f"{c[0]}-{str(c[1])[6:]}-B{c[2]}H{c[3]}/{c[4]}-L{c[5]}-D{c[6]}-{c[7]}x{c[8]}-rho{c[9]}"  # noqa: E731


@pytest.mark.parametrize("case", _sweep_cases_wide_key_blocks(12, seed=77), ids=_SWEEP_IDS)
def test_sweep_select_sparse_with_128_key_blocks(case):
    _sweep_body(case)


def _sweep_cases_narrow_key_blocks(n, seed):
    """bf16 with 32-key blocks (the paper's square 32 x 32 among them): listed blocks are paired up two to a tile."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        bq = int(rng.choice([32, 64, 128]))
        Hkv = int(rng.choice([1, 2]))
        Hq = Hkv * int(rng.choice([1, 2]))
        B = int(rng.choice([1, 2]))
        L = int(rng.integers(1, 700))
        rho = float(rng.choice([0.1, 0.3, 0.5, 1.0]))
        cases.append((2000 + i, torch.bfloat16, B, Hq, Hkv, L, D, bq, 32, rho))
    return cases


@pytest.mark.parametrize("case", _sweep_cases_narrow_key_blocks(16, seed=78), ids=_SWEEP_IDS)
def test_sweep_select_sparse_with_32_key_blocks(case):
    _sweep_body(case)


@pytest.mark.parametrize("case", _sweep_cases(24, seed=2024), ids=_SWEEP_IDS)
def test_sweep_dense_select_sparse(case):
    """Every entry point on shapes drawn at random (seeded): any length from 1 up, both head dims, all block
    shapes, grouped heads, batch 1-2. Dense, selection (index inside the tie band) and sparse on the GPU's index."""
    _sweep_body(case)


def _sweep_body(case):
    i, dtype, B, Hq, Hkv, L, D, bq, bk, rho = case
    _say(f"sweep {case}")
    q, k, v = _rand_qkv(B, Hq, Hkv, L, D, dtype, seed=100 + i, scale=1.0 if dtype == torch.float32 and D == 64 else 0.5)
    qd, kd, vd = _dev(q, k, v)
    assert_output_close(sd.attn_dense(qd, kd, vd), oracle.attn_dense(q, k, v), dtype, "sweep dense")
    nqb, nkb = -(-L // bq), -(-L // bk)
    pooled = torch.empty(B, Hq, nqb, nkb, dtype=torch.float32, device=DEV)
    ix = sd.select_pattern(qd, kd, bq, bk, rho, pooled_out=pooled)
    sd.index_validate(ix)
    row_ptr, col_idx, apool, _ = oracle.select_pattern(q, k, bq, bk, rho)
    keep = oracle.kept_blocks(rho, nkb)
    assert np.array_equal(ix.row_ptr.cpu().numpy(), row_ptr)
    rel = np.abs(pooled.cpu().double().numpy() - apool) / apool
    assert rel.max() < 5e-6, f"pooled scores off by {rel.max():.2e}"
    compare_index(ix.col_idx.cpu().numpy()[..., :nqb * keep], col_idx, apool.reshape(-1, nkb), keep)
    got = sd.attn_sparse(qd, kd, vd, ix)
    want = oracle.attn_sparse(q, k, v, ix.row_ptr.cpu().numpy(), ix.col_idx.cpu().numpy(), bq, bk)
    assert_output_close(got, want, dtype, "sweep sparse")


def test_sweep_window_index_builder():
    from oracle import patterns
    rng = np.random.default_rng(11)
    for _ in range(16):
        bq, bk = int(rng.choice([32, 64, 128])), int(rng.choice([32, 64]))
        L = int(rng.integers(1, 1500))
        window, sink = int(rng.integers(0, 2 * L)), int(rng.integers(0, L + 1))
        H = int(rng.integers(1, 4))
        nqb, nkb = -(-L // bq), -(-L // bk)
        m = patterns.window_token_mask(L, window, sink)
        rows = [np.array([J for J in range(nkb) if m[I * bq:(I + 1) * bq, J * bk:(J + 1) * bk].any()], dtype=np.int32) for I in range(nqb)]
        ptr, col = patterns.rows_to_csr(rows, H)
        ix = sd.index_fill_window(1, H, L, bq, bk, window, sink, DEV)
        sd.index_validate(ix)
        assert np.array_equal(ix.row_ptr.cpu().numpy().reshape(H, -1), ptr), (L, bq, bk, window, sink)
        assert np.array_equal(ix.col_idx.cpu().numpy().reshape(H, -1)[:, :col.shape[1]], col), (L, bq, bk, window, sink)


def _rows_equal_within_ties(got_rows, want_rows, score_rows, cut_of):
    """got/want: lists of block lists; a difference is legal only for blocks whose score ties with the cut."""
    ties = 0
    for r, (g, w) in enumerate(zip(got_rows, want_rows)):
        assert list(g) == sorted(set(g))
        if list(g) == list(w):
            continue
        for J in set(g) ^ set(w):
            sc, cut = score_rows[r](J), cut_of[r](J)
            assert any(abs(a - c) <= 1e-5 * abs(c) for a, c in zip(sc, cut)), f"row {r}: block {J} differs outside the tie band"
        ties += 1
    return ties


def test_sweep_isolated_selection_blocks_and_tokens():
    rng = np.random.default_rng(12)
    for it in range(10):
        dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
        bq = int(rng.choice([32, 64, 128]))
        bk = 64 if dtype == torch.bfloat16 else int(rng.choice([32, 64]))
        D = int(rng.choice([64, 128]))
        L = int(rng.integers(bk + 1, 700 if dtype == torch.bfloat16 else 300))
        rho = float(rng.choice([0.1, 0.3, 0.6]))
        ptok = int(rng.integers(0, L + 1))
        H = 2
        _say(f"isolated sweep {it}: {dtype} {bq}x{bk} L={L} D={D} rho={rho} p={ptok}")
        q, k, _ = _rand_qkv(1, H, 1, L, D, dtype, seed=300 + it, scale=1.0 if dtype == torch.float32 and D == 64 else 0.6)
        qd, kd = _dev(q, k)
        nqb, nkb = -(-L // bq), -(-L // bk)
        # boundary in tokens
        ix = sd.select_pattern_isolated_tokens(qd, kd, bq, bk, rho, ptok)
        sd.index_validate(ix)
        rp_o, ci_o, ap, n_pre, vblock = oracle.select_isolated_tokens(q, k, bq, bk, rho, ptok)
        nv = ap.shape[-1]
        kp, kg = (oracle.kept_blocks(rho, n_pre) if n_pre else 0), (oracle.kept_blocks(rho, nv - n_pre) if nv > n_pre else 0)
        rp, ci = ix.row_ptr.cpu().numpy(), ix.col_idx.cpu().numpy()
        for h in range(H):
            got = [ci[0, h, rp[0, h, I]:rp[0, h, I + 1]].tolist() for I in range(nqb)]
            want = [ci_o[0, h, rp_o[0, h, I]:rp_o[0, h, I + 1]].tolist() for I in range(nqb)]

            def scores(I):
                return lambda J: [ap[0, h, I, e] for e in range(nv) if vblock[e] == J]

            def cuts(I):
                a = ap[0, h, I]
                cp = np.sort(a[:n_pre])[::-1][kp - 1] if kp else np.nan
                cg = np.sort(a[n_pre:])[::-1][kg - 1] if kg else np.nan
                return lambda J: [cp if e < n_pre else cg for e in range(nv) if vblock[e] == J]
            _rows_equal_within_ties(got, want, [scores(I) for I in range(nqb)], [cuts(I) for I in range(nqb)])
        # boundary in blocks
        pb = int(rng.integers(0, nkb + 1))
        ixb = sd.select_pattern_isolated(qd, kd, bq, bk, rho, pb)
        sd.index_validate(ixb)
        apool = oracle.pool_scores(q, k, bq, bk)
        rpb, cib = oracle.select_isolated(apool, rho, pb)
        keep = (oracle.kept_blocks(rho, pb) if pb else 0) + (oracle.kept_blocks(rho, nkb - pb) if nkb > pb else 0)
        assert np.array_equal(ixb.row_ptr.cpu().numpy(), rpb)
        gotb = ixb.col_idx.cpu().numpy()[..., :nqb * keep].reshape(-1, keep)
        wantb = cib.reshape(-1, keep)
        a2 = apool.reshape(-1, nkb)
        for r in range(gotb.shape[0]):
            if list(gotb[r]) == list(wantb[r]):
                continue
            cp = np.sort(a2[r, :pb])[::-1][oracle.kept_blocks(rho, pb) - 1] if pb else np.nan
            cg = np.sort(a2[r, pb:])[::-1][oracle.kept_blocks(rho, nkb - pb) - 1] if nkb > pb else np.nan
            for J in set(gotb[r]) ^ set(wantb[r]):
                cut = cp if J < pb else cg
                assert abs(a2[r, J] - cut) <= 1e-5 * abs(cut), f"block form, row {r}, block {J}"


# ----------------------------------------------------------------------------- fixed patterns (Section 4.1 baselines)
@pytest.mark.parametrize("L,bq,bk,window,sink", [
    (1024, 128, 64, 256, 0),      # sliding window
    (1024, 128, 64, 256, 64),     # window + one sink block
    (512, 32, 64, 100, 70),       # query blocks smaller than key blocks, sinks straddle a block edge
    (512, 64, 64, 0, 0),          # diagonal only
    (512, 64, 64, 4096, 0),       # window wider than the sequence: every block
    (2048, 64, 32, 300, 33),      # fp32 block shape, many rows
    (1024, 128, 64, 64, 410),     # sinks reach past the window of the first rows: the two runs merge
    (1024, 32, 64, 8, 1024),      # every key is a sink
])
def test_window_index_matches_token_level_definition(L, bq, bk, window, sink):
    from oracle import patterns
    _say(f"window index L={L} {bq}x{bk} window={window} sink={sink}")
    H = 3
    rows = patterns.window_block_rows(L, bq, bk, window, sink)
    ptr, col = patterns.rows_to_csr(rows, H)
    assert sd.index_window_entries(L, bq, bk, window, sink) == col.shape[1]
    ix = sd.index_fill_window(1, H, L, bq, bk, window, sink, DEV)
    sd.index_validate(ix)
    assert np.array_equal(ix.row_ptr.cpu().numpy().reshape(H, -1), ptr)
    assert np.array_equal(ix.col_idx.cpu().numpy().reshape(H, -1)[:, :col.shape[1]], col)


@pytest.mark.parametrize("L,bq,bk", [(1024, 128, 64), (1000, 128, 128), (900, 64, 128), (1000, 32, 32), (700, 64, 32), (1000, 128, 32)])
def test_window_index_feeds_the_sparse_kernel(L, bq, bk):
    from oracle import patterns
    H = 2
    q, k, v = _rand_qkv(1, H, H, L, 128, torch.bfloat16, seed=77)
    ix = sd.index_fill_window(1, H, L, bq, bk, 256, 64, DEV)
    got = sd.attn_sparse(*_dev(q, k, v), ix)
    ptr, col = patterns.rows_to_csr(patterns.window_block_rows(L, bq, bk, 256, 64), H)
    want = oracle.attn_sparse(q, k, v, ptr[None], col[None], bq, bk)
    assert_output_close(got, want, torch.bfloat16, "window + sink sparse")


def test_window_index_rejects_small_capacity():
    ix = sd.BlockIndex(torch.zeros(1, 1, 9, dtype=torch.int32, device=DEV), torch.zeros(1, 1, 8, dtype=torch.int32, device=DEV), 64, 64, 8)
    import ctypes
    from paper_2509_24014_amd import binding
    ci = ix._c()
    st = binding.load_library().sparsed_index_fill_window(ctypes.byref(ci), 512, 256, 0, None)
    assert st == 8 and b"cap_per_head" in binding.load_library().sparsed_last_error()
    assert int(ix.row_ptr.abs().sum()) == 0       # nothing was launched


# ----------------------------------------------------------------------------- the tiny schedule, in full
def test_tiny_config_full_schedule():
    cfg = workload.get_config("tiny")
    _say(f"tiny schedule: T={cfg.T} n_dense={cfg.n_dense}")
    inp = workload.make_inputs(cfg, seed=0, device="cpu")
    layer = sd.SparseDLayer(cfg.T, 0.2, cfg.bq, cfg.bk, cfg.rho)
    assert layer.n_dense == cfg.n_dense == 1
    ora_index = None
    for t in range(cfg.T):
        q, k, v = inp.rounded()
        got = layer.step(*_dev(q, k, v), t)
        if t < cfg.n_dense:
            want = oracle.attn_dense(q, k, v)
            if t == cfg.n_dense - 1:
                rp, ci, apool, _ = oracle.select_pattern(q, k, cfg.bq, cfg.bk, cfg.rho)
                keep = oracle.kept_blocks(cfg.rho, cfg.nkb)
                assert keep == 3
                ties = compare_index(layer.index.col_idx.cpu().numpy(), ci, apool.reshape(-1, cfg.nkb), keep)
                _say(f"tiny: ties {ties}")
                ora_index = (layer.index.row_ptr.cpu().numpy(), layer.index.col_idx.cpu().numpy())
                frozen = layer.index.col_idx.clone()
        else:
            # sparse steps are checked against the oracle run on the SAME (GPU-selected) index
            want = oracle.attn_sparse(q, k, v, ora_index[0], ora_index[1], cfg.bq, cfg.bk)
            assert torch.equal(layer.index.col_idx, frozen)      # the pattern is reused, never recomputed
        assert_output_close(got, want, torch.float32, f"tiny step {t}")
        inp.advance()
    assert layer.calls == {"dense": 1, "select": 1, "sparse": 4}


def test_schedule_ablation_modes_against_oracle():
    """Two of Table 2's ablations as the driver runs them: no dense steps (select at step 0 from that
    step's own q, k), and a fresh selection at every sparse step."""
    cfg = workload.get_config("tiny")
    keep = oracle.kept_blocks(cfg.rho, cfg.nkb)
    for mode in ("no_skip", "reselect"):
        inp = workload.make_inputs(cfg, seed=3, device="cpu")
        layer = (sd.SparseDLayer(cfg.T, 0.2, cfg.bq, cfg.bk, cfg.rho, n_dense=0) if mode == "no_skip"
                 else sd.SparseDLayer(cfg.T, 0.2, cfg.bq, cfg.bk, cfg.rho, reselect_every_step=True))
        first_index = None
        for t in range(cfg.T):
            q, k, v = inp.rounded()
            got = layer.step(*_dev(q, k, v), t)
            if t < layer.n_dense:
                want = oracle.attn_dense(q, k, v)
            else:
                selected_now = (mode == "reselect") or t == 0
                if selected_now:
                    _, ci, apool, _ = oracle.select_pattern(q, k, cfg.bq, cfg.bk, cfg.rho)
                    compare_index(layer.index.col_idx.cpu().numpy(), ci, apool.reshape(-1, cfg.nkb), keep)
                if first_index is None:
                    first_index = layer.index.col_idx.clone()
                elif mode == "no_skip":
                    assert torch.equal(layer.index.col_idx, first_index)
                want = oracle.attn_sparse(q, k, v, layer.index.row_ptr.cpu().numpy(), layer.index.col_idx.cpu().numpy(), cfg.bq, cfg.bk)
            assert_output_close(got, want, torch.float32, f"{mode} step {t}")
            inp.advance()
        _say(f"ablation {mode}: calls {layer.calls}")
        if mode == "no_skip":
            assert layer.calls == {"dense": 0, "select": 1, "sparse": cfg.T}
        else:
            assert layer.calls["select"] >= cfg.T - layer.n_dense


# ----------------------------------------------------------------------------- named workloads at full size
def _sample_units(cfg, n_per_type, seed, heads_per_type=2):
    """(head, query block) units: every head type (up to `heads_per_type` heads of each), n_per_type query blocks per
    type, the first and the last query block always among them."""
    rng = np.random.default_rng(seed)
    units = []
    for t in range(4):
        heads = [h for h in range(cfg.Hq) if h % 4 == t]
        picked = [heads[int(i)] for i in rng.permutation(len(heads))[:heads_per_type]]
        blocks = {0, cfg.nqb - 1}
        while len(blocks) < min(n_per_type, cfg.nqb):
            blocks.add(int(rng.integers(cfg.nqb)))
        for n, I in enumerate(sorted(blocks)):
            units.append((picked[n % len(picked)], I))
    return sorted(units)


def _check_workload_sampled(name, n_per_type, check_dense=True):
    cfg = workload.get_config(name)
    _say(f"{name}: generating L={cfg.L} Hq={cfg.Hq} Hkv={cfg.Hkv} {cfg.bq}x{cfg.bk} rho={cfg.rho}")
    inp = workload.make_inputs(cfg, seed=0, device=DEV)
    q, k, v = inp.rounded()
    del inp
    keep = oracle.kept_blocks(cfg.rho, cfg.nkb)
    lse = torch.empty(cfg.B, cfg.Hq, cfg.L, dtype=torch.float32, device=DEV)
    dense = sd.attn_dense(q, k, v, lse_out=lse)
    pooled = torch.empty(cfg.B, cfg.Hq, cfg.nqb, cfg.nkb, dtype=torch.float32, device=DEV)
    ix = sd.select_pattern(q, k, cfg.bq, cfg.bk, cfg.rho, lse_in=lse, pooled_out=pooled)
    pooled_own = torch.empty_like(pooled)
    ix2 = sd.select_pattern(q, k, cfg.bq, cfg.bk, cfg.rho, pooled_out=pooled_own)   # nothing handed over: one pass over the keys
    cols_own = ix2.col_idx.view(cfg.B, cfg.Hq, cfg.nqb, keep)
    sd.index_validate(ix)
    sparse = sd.attn_sparse(q, k, v, ix)
    torch.cuda.synchronize()
    # properties that hold at any size
    assert torch.isfinite(dense.float()).all() and torch.isfinite(sparse.float()).all()
    assert ix.row_ptr.cpu().eq(torch.arange(cfg.nqb + 1, dtype=torch.int32) * keep).all()
    cols = ix.col_idx.view(cfg.B, cfg.Hq, cfg.nqb, keep)
    assert (cols[..., 1:] > cols[..., :-1]).all() and cols.min() >= 0 and cols.max() < cfg.nkb
    np.testing.assert_allclose(pooled.sum(-1).cpu().numpy(), 1.0 / cfg.bk, rtol=2e-5)   # rows of A' sum to 1/bk
    same = (ix2.col_idx == ix.col_idx).view(cfg.B, cfg.Hq, cfg.nqb, keep).all(-1).float().mean().item()
    _say(f"{name}: rows identical between lse_in and own-statistics selection: {100 * same:.2f}%")
    # sampled units against the oracle
    group = cfg.Hq // cfg.Hkv
    tie_rows = tie_blocks = 0
    pooled_err = pooled_own_err = dense_err = sparse_err = 0.0
    units = _sample_units(cfg, n_per_type, seed=1)
    assert len(units) >= 64
    cache = {}
    for (h, I) in units:
        if h not in cache:
            cache.clear()
            cache[h] = (q[:, h:h + 1].float().cpu(), k[:, h // group:h // group + 1].float().cpu(),
                        v[:, h // group:h // group + 1].float().cpu())
        qh, kh, vh = cache[h]
        r0, r1 = I * cfg.bq, (I + 1) * cfg.bq
        if check_dense:
            want = oracle.attn_dense_rows(qh, kh, vh, 0, 0, r0, r1)
            dense_err = max(dense_err, assert_output_close(dense[0, h, r0:r1], want, torch.bfloat16, f"{name} dense h={h} I={I}")[0])
        ap = oracle.pool_scores_rows(qh, kh, cfg.bq, cfg.bk, 0, 0, I, I + 1)
        _, ci, _ = oracle.select_topk(ap.reshape(1, 1, 1, cfg.nkb), keep)
        tr, tb = compare_index(cols[0, h, I].cpu().numpy(), ci.reshape(-1), ap.reshape(1, cfg.nkb), keep)
        tie_rows += tr
        tie_blocks += tb
        rel = np.abs(pooled[0, h, I].cpu().double().numpy() - ap[0]) / ap[0]
        # the gate sits below the 1e-5 tie band of the ranking (Eq. 6) that these scores feed
        assert rel.max() <= 5e-6, f"{name} pooled h={h} I={I}: {rel.max():.2e}"
        pooled_err = max(pooled_err, float(rel.max()))
        # the same unit from the call that was handed no row statistics
        rel_own = np.abs(pooled_own[0, h, I].cpu().double().numpy() - ap[0]) / ap[0]
        assert rel_own.max() <= 5e-6, f"{name} pooled (one pass) h={h} I={I}: {rel_own.max():.2e}"
        pooled_own_err = max(pooled_own_err, float(rel_own.max()))
        compare_index(cols_own[0, h, I].cpu().numpy(), ci.reshape(-1), ap.reshape(1, cfg.nkb), keep)
        # sparse output against the oracle run on the GPU-selected row
        rp1 = np.zeros((1, 1, cfg.nqb + 1), dtype=np.int32)
        rp1[0, 0, I + 1:] = keep
        ci1 = cols[0, h, I].cpu().numpy().reshape(1, 1, keep)
        want = oracle.attn_sparse_rows(qh, kh, vh, rp1, ci1, cfg.bq, cfg.bk, 0, 0, I, I + 1)
        sparse_err = max(sparse_err, assert_output_close(sparse[0, h, r0:r1], want, torch.bfloat16, f"{name} sparse h={h} I={I}")[0])
    _say(f"{name}: {len(units)} units checked; tie_rows={tie_rows} tie_blocks={tie_blocks} "
         f"max pooled rel err={pooled_err:.2e} (one pass: {pooled_own_err:.2e}) dense max|d|={dense_err:.2e} sparse max|d|={sparse_err:.2e}")


def test_workload_llada4k_full_tensor():
    """The 4k LLaDA-shaped layer, compared in full."""
    cfg = workload.get_config("llada4k")
    inp = workload.make_inputs(cfg, seed=0, device=DEV)
    q, k, v = inp.rounded()
    qc, kc, vc = q.cpu(), k.cpu(), v.cpu()
    _say("llada4k: oracle dense")
    want = oracle.attn_dense(qc, kc, vc)
    lse = torch.empty(cfg.B, cfg.Hq, cfg.L, dtype=torch.float32, device=DEV)
    got = sd.attn_dense(q, k, v, lse_out=lse)
    assert_output_close(got, want, torch.bfloat16, "llada4k dense")
    _say("llada4k: oracle selection")
    rp, ci, apool, _ = oracle.select_pattern(qc, kc, cfg.bq, cfg.bk, cfg.rho)
    ix = sd.select_pattern(q, k, cfg.bq, cfg.bk, cfg.rho, lse_in=lse)
    keep = oracle.kept_blocks(cfg.rho, cfg.nkb)
    assert keep == 13
    tr, tb = compare_index(ix.col_idx.cpu().numpy(), ci, apool.reshape(-1, cfg.nkb), keep)
    _say(f"llada4k: selection rows={cfg.Hq * cfg.nqb} tie_rows={tr} tie_blocks={tb}")
    _say("llada4k: oracle sparse (on the GPU-selected index)")
    want = oracle.attn_sparse(qc, kc, vc, ix.row_ptr.cpu().numpy(), ix.col_idx.cpu().numpy(), cfg.bq, cfg.bk)
    got = sd.attn_sparse(q, k, v, ix)
    assert_output_close(got, want, torch.bfloat16, "llada4k sparse")


def test_workload_llada16k_sampled():
    _check_workload_sampled("llada16k", n_per_type=16)


def test_workload_dream32k_gqa_sampled():
    _check_workload_sampled("dream32k", n_per_type=16)


def test_workload_long64k_sampled():
    _check_workload_sampled("long64k", n_per_type=16)


def test_papers_own_long_context_setting_sampled():
    _check_workload_sampled("paper64k", n_per_type=16)


def test_twice_the_papers_longest_context_sampled():
    _check_workload_sampled("probe128k", n_per_type=16)


def _check_schedule_sampled(name, n_per_type):
    """All T steps of Algorithm 1 on a named workload with its per-step drift, on the GPU; at step 0, the switch step,
    the first sparse step and the last step sampled (head, query-block) units are compared with the oracle, the
    sparse ones on the pattern stored at the switch step (Sparse Reusing), which must never change afterwards."""
    cfg = workload.get_config(name)
    T, n_dense = cfg.T, cfg.n_dense
    keep = oracle.kept_blocks(cfg.rho, cfg.nkb)
    group = cfg.Hq // cfg.Hkv
    check_steps = sorted({0, n_dense - 1, n_dense, T - 1})
    units = _sample_units(cfg, n_per_type, seed=2)
    _say(f"{name} schedule: T={T} n_dense={n_dense} checking steps {check_steps}, {len(units)} units each")
    inp = workload.make_inputs(cfg, seed=0, device=DEV)
    layer = sd.SparseDLayer(T, 0.0, cfg.bq, cfg.bk, cfg.rho, n_dense=n_dense)
    out = None
    frozen = None
    worst = {"dense": 0.0, "sparse": 0.0}
    tie_rows = tie_blocks = 0
    for t in range(T):
        q, k, v = inp.rounded()
        out = layer.step(q, k, v, t, out=out)
        if t == n_dense - 1:
            sd.index_validate(layer.index)
            frozen = (layer.index.row_ptr.clone(), layer.index.col_idx.clone())
            cols = frozen[1].view(cfg.B, cfg.Hq, cfg.nqb, keep).cpu().numpy()
        if t in check_steps:
            torch.cuda.synchronize()
            got = out.cpu()
            cache = {}
            for (h, I) in units:
                if h not in cache:
                    cache.clear()
                    cache[h] = (q[:, h:h + 1].float().cpu(), k[:, h // group:h // group + 1].float().cpu(),
                                v[:, h // group:h // group + 1].float().cpu())
                qh, kh, vh = cache[h]
                r0, r1 = I * cfg.bq, (I + 1) * cfg.bq
                if t < n_dense:
                    want = oracle.attn_dense_rows(qh, kh, vh, 0, 0, r0, r1)
                    kind = "dense"
                else:
                    rp1 = np.zeros((1, 1, cfg.nqb + 1), dtype=np.int32)
                    rp1[0, 0, I + 1:] = keep
                    want = oracle.attn_sparse_rows(qh, kh, vh, rp1, cols[0, h, I].reshape(1, 1, keep), cfg.bq, cfg.bk, 0, 0, I, I + 1)
                    kind = "sparse"
                err = assert_output_close(got[0, h, r0:r1], want, torch.bfloat16, f"{name} step {t} {kind} h={h} I={I}")[0]
                worst[kind] = max(worst[kind], err)
                if t == n_dense - 1:
                    # the pattern stored at the switch step against the oracle's ranking of this step's Q, K
                    ap = oracle.pool_scores_rows(qh, kh, cfg.bq, cfg.bk, 0, 0, I, I + 1)
                    _, ci, _ = oracle.select_topk(ap.reshape(1, 1, 1, cfg.nkb), keep)
                    tr, tb = compare_index(cols[0, h, I], ci.reshape(-1), ap.reshape(1, cfg.nkb), keep)
                    tie_rows += tr
                    tie_blocks += tb
            _say(f"{name} schedule: step {t} ok ({len(units)} units)")
        inp.advance()
    torch.cuda.synchronize()
    assert torch.equal(layer.index.row_ptr, frozen[0]) and torch.equal(layer.index.col_idx, frozen[1])   # reused, never recomputed
    assert layer.calls == {"dense": n_dense, "select": 1, "sparse": T - n_dense}
    _say(f"{name} schedule: calls {layer.calls}; dense max|d|={worst['dense']:.2e} sparse max|d|={worst['sparse']:.2e}; "
         f"switch-step index tie_rows={tie_rows} tie_blocks={tie_blocks}")


def test_schedule_llada16k_all_steps_sampled():
    _check_schedule_sampled("llada16k", n_per_type=4)


def test_schedule_long64k_all_steps_sampled():
    _check_schedule_sampled("long64k", n_per_type=4)


def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline():
    """bench.py on the small 4k workload: one JSON line on stdout carrying every field its readers rely on."""
    import json
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "llada4k", "--steps", "2", "--warmup", "1"],
                       capture_output=True, text=True, timeout=300, cwd=root)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["data"] == "synthetic"
    assert d["config"]["workload"] == "llada4k" and "model" not in d["config"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    roof = d["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 2500.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and "traffic" in roof
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]


def test_hot_path_replays_from_a_hip_graph():
    """dense (with row statistics) -> select -> sparse are kernel launches only when the caller brings the workspace
    and the index, so the three calls can be captured once into a HIP graph. Replays on new contents of the same
    buffers, with eager work and synchronisation between them, equal the eager calls bit for bit every time."""
    B, H, L, D, bq, bk, rho = 1, 4, 1024, 128, 64, 64, 0.25
    nqb, nkb = L // bq, L // bk
    keep = sd.kept_blocks(rho, nkb)
    gen = torch.Generator(device=DEV).manual_seed(5)
    q, k, v = (torch.randn(B, H, L, D, device=DEV, generator=gen).to(torch.bfloat16) for _ in range(3))
    lse = torch.empty(B, H, L, dtype=torch.float32, device=DEV)
    out_d, out_s = torch.empty_like(q), torch.empty_like(q)
    index = sd.BlockIndex(torch.empty(B, H, nqb + 1, dtype=torch.int32, device=DEV),
                          torch.empty(B, H, nqb * keep, dtype=torch.int32, device=DEV), bq, bk, nkb)
    ws = torch.empty(sd.select_workspace_bytes(q, bq, bk), dtype=torch.uint8, device=DEV)

    def hot_path():
        sd.attn_dense(q, k, v, out=out_d, lse_out=lse)
        sd.select_pattern(q, k, bq, bk, rho, lse_in=lse, workspace=ws, index=index)
        sd.attn_sparse(q, k, v, index, out=out_s)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        hot_path()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        hot_path()
    for trial in range(4):
        for t in (q, k, v):
            t.copy_(torch.randn(B, H, L, D, device=DEV, generator=gen).to(torch.bfloat16))
        for t in (out_d, out_s, lse):
            t.fill_(float("nan"))
        index.col_idx.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        lse_e = torch.empty_like(lse)
        dense_e = sd.attn_dense(q, k, v, lse_out=lse_e)
        index_e = sd.select_pattern(q, k, bq, bk, rho, lse_in=lse_e)
        sparse_e = sd.attn_sparse(q, k, v, index_e)
        torch.cuda.synchronize()
        assert torch.equal(out_d, dense_e) and torch.equal(lse, lse_e), f"replay {trial}: dense"
        assert torch.equal(index.row_ptr, index_e.row_ptr) and torch.equal(index.col_idx, index_e.col_idx), f"replay {trial}: index"
        assert torch.equal(out_s, sparse_e), f"replay {trial}: sparse"
