"""Pins for the fixed-pattern oracle (sliding window / window + sinks, Section 4.1): closed forms
and special cases of the token-level definition."""
import numpy as np
import pytest

from oracle import patterns


def test_window_zero_with_square_blocks_is_the_block_diagonal():
    rows = patterns.window_block_rows(256, 32, 32, 0, 0)
    assert [r.tolist() for r in rows] == [[i] for i in range(8)]


def test_window_covering_the_sequence_keeps_every_block():
    rows = patterns.window_block_rows(256, 64, 32, 2 * 256, 0)
    assert all(r.tolist() == list(range(8)) for r in rows)


def test_window_reaches_exactly_half_a_window_each_way():
    # block 4 of 8 (tokens 128..159), half window 32: keys 96..191 = blocks 3, 4, 5; one token more adds 2 and 6
    assert patterns.window_block_rows(256, 32, 32, 64, 0)[4].tolist() == [3, 4, 5]
    assert patterns.window_block_rows(256, 32, 32, 66, 0)[4].tolist() == [2, 3, 4, 5, 6]
    # an odd window length rounds the half down
    assert patterns.window_block_rows(256, 32, 32, 67, 0)[4].tolist() == [2, 3, 4, 5, 6]
    assert patterns.window_block_rows(256, 32, 32, 65, 0)[4].tolist() == [3, 4, 5]


def test_sinks_add_leading_blocks_once():
    rows = patterns.window_block_rows(512, 64, 64, 0, 65)   # 65 sink tokens touch key blocks 0 and 1
    assert rows[0].tolist() == [0, 1]
    assert rows[1].tolist() == [0, 1]
    assert rows[5].tolist() == [0, 1, 5]


def test_token_mask_is_symmetric_without_sinks_and_counts_match():
    m = patterns.window_token_mask(100, 10, 0)
    assert (m == m.T).all()
    # row i sees min(i, 5) + 1 + min(99 - i, 5) keys
    want = [min(i, 5) + 1 + min(99 - i, 5) for i in range(100)]
    assert m.sum(1).tolist() == want


def test_rectangular_blocks():
    # 128-row query blocks over 64-key blocks, no window: each query block sees its own two key blocks
    rows = patterns.window_block_rows(512, 128, 64, 0, 0)
    assert [r.tolist() for r in rows] == [[0, 1], [2, 3], [4, 5], [6, 7]]


def test_csr_layout():
    rows = patterns.window_block_rows(256, 64, 64, 0, 64)
    ptr, col = patterns.rows_to_csr(rows, 3)
    assert ptr.shape == (3, 5) and ptr[1].tolist() == [0, 1, 3, 5, 7]
    assert col[2].tolist() == [0, 0, 1, 0, 2, 0, 3]


def test_host_capacity_formula_matches_the_token_level_count():
    """The host-side entry count of the window builder (block arithmetic) against the number of kept blocks
    of the token-level definition, over a seeded sweep that includes lengths that are not block multiples."""
    from paper_2509_24014_amd import binding
    rng = np.random.default_rng(7)
    for _ in range(60):
        bq, bk = int(rng.choice([32, 64, 128])), int(rng.choice([32, 64]))
        L = int(rng.integers(1, 900))
        window, sink = int(rng.integers(0, 2 * L)), int(rng.integers(0, L + 1))
        nqb, nkb = -(-L // bq), -(-L // bk)
        m = patterns.window_token_mask(L, window, sink)
        total = sum(m[I * bq:(I + 1) * bq, J * bk:(J + 1) * bk].any() for I in range(nqb) for J in range(nkb))
        assert binding.index_window_entries(L, bq, bk, window, sink) == total, (L, bq, bk, window, sink)
