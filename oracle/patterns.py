"""Test oracle (never imported by the product): the fixed sparse patterns the paper compares
against (Section 4.1: sliding window; StreamingLLM = window + attention sinks), written from
their token-level definition for bidirectional attention.

A query token i may see key token j when |i - j| <= window_tokens // 2 or j < sink_tokens.
A (query block, key block) pair is kept when ANY of its token pairs may be seen. The token
mask is formed in full and reduced over blocks, with no shortcut through block arithmetic.
"""
import numpy as np


def window_token_mask(L, window_tokens, sink_tokens):
    i = np.arange(L)[:, None]
    j = np.arange(L)[None, :]
    return (np.abs(i - j) <= window_tokens // 2) | (j < sink_tokens)


def window_block_rows(L, bq, bk, window_tokens, sink_tokens):
    """List of ascending key-block lists, one per query block."""
    m = window_token_mask(L, window_tokens, sink_tokens)
    nqb, nkb = -(-L // bq), -(-L // bk)  # the last block of either axis may be partial
    return [np.array([J for J in range(nkb) if m[I * bq:(I + 1) * bq, J * bk:(J + 1) * bk].any()], dtype=np.int32)
            for I in range(nqb)]


def rows_to_csr(rows, heads):
    """(row_ptr [heads, nqb+1], col_idx [heads, total]) with the same rows for every head."""
    ptr = np.zeros(len(rows) + 1, dtype=np.int32)
    ptr[1:] = np.cumsum([len(r) for r in rows])
    col = np.concatenate(rows) if rows else np.zeros(0, np.int32)
    return np.tile(ptr, (heads, 1)), np.tile(col, (heads, 1))
