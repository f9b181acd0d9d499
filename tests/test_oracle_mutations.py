"""The pins must have teeth: plant one plausible mistake at a time in a COPY of the oracle's C source
(on the CPU, never in the GPU path) and check that the pin tests catch it."""
import ctypes
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "oracle.c")

# (name, text to replace, replacement, pin tests that must notice)
MUTANTS = [
    ("dense: 1/sqrt(d) dropped",
     "    p[j] = dot * inv_sqrt_d;", "    p[j] = dot;",
     [lambda: pins.test_dense_matches_torch_softmax_and_sdpa(2, 2)]),
    ("dense: softmax exponent sign flipped",
     "    p[j] = exp(p[j] - m);", "    p[j] = exp(m - p[j]);",
     [lambda: pins.test_probs_rows_sum_to_one_and_match_torch()]),
    ("dense: grouped heads mapped with modulo instead of division",
     "  const int g = h / (Hq / Hkv);\n  const float* khead = k + IDX4(b, g, 0, Hkv, L, d);\n  const float* vhead = v + IDX4(b, g, 0, Hkv, L, d);\n  int fail = 0;",
     "  const int g = h % Hkv;\n  const float* khead = k + IDX4(b, g, 0, Hkv, L, d);\n  const float* vhead = v + IDX4(b, g, 0, Hkv, L, d);\n  int fail = 0;",
     [lambda: pins.test_dense_matches_torch_softmax_and_sdpa(4, 2)]),
    ("dense: output accumulates keys instead of values",
     "        for (int c = 0; c < d; ++c) o[c] += p[j] * (double)vrow[c];\n      }\n    }\n    free(p);",
     "        for (int c = 0; c < d; ++c) o[c] += p[j] * (double)(khead + (size_t)j * d)[c];\n      }\n    }\n    free(p);",
     [lambda: pins.test_dense_zero_queries_give_mean_of_values()]),
    ("pooling: divided by bq only",
     "arow[J] /= (double)rows * (double)colsJ;", "arow[J] /= (double)rows;",
     [lambda: pins.test_pool_uniform_when_queries_are_zero()]),
    ("pooling: query rows indexed with the key block size",
     "probs_row(q + IDX4(b, h, I * bq + r, Hq, L, d), khead, L, d, p);",
     "probs_row(q + IDX4(b, h, I * bk + r, Hq, L, d), khead, L, d, p);",
     [lambda: pins.test_pool_matches_reshape_mean_of_torch_probs(16, 8)]),
    ("pooling: a partial last block is divided by the full block area",
     "arow[J] /= (double)rows * (double)colsJ;", "arow[J] /= (double)bq * (double)bk;",
     [lambda: pins.test_ragged_pool_matches_ceil_mode_average_pooling()]),
    ("sparse: keys past the end of a partial last block are not masked",
     "        if (j >= L) {\n          s[t * bk + c] = -INFINITY;\n          continue;\n        }",
     "        if (j >= L) {\n          s[t * bk + c] = 0.0;\n          continue;\n        }",
     [lambda: pins.test_ragged_sparse_matches_bruteforce_and_dense()]),
    ("token boundary: the block kept by both ranges is listed twice",
     "        if (n > row_begin && cols[n - 1] == vblock[v]) continue; /* the straddling block, kept by both ranges */\n", "",
     [lambda: pins.test_token_boundary_rows_are_unions_of_per_range_optima()]),
    ("range pooling: divided by the block size instead of the range length",
     "arow[v] /= (double)rows * (double)(vend[v] - vstart[v]);", "arow[v] /= (double)rows * 16.0;",
     [lambda: pins.test_range_pooling_matches_sliced_means_of_torch_probs()]),
    ("count rule: floor instead of guarded ceil",
     "int kk = (int)ceil(rho * (double)n - 1e-9);", "int kk = (int)floor(rho * (double)n);",
     [lambda: pins.test_kept_blocks_rule()]),
    ("selection: ties go to the higher index",
     "      if (best < 0 || arow[J] > arow[best]) best = J; /* strict >: the lower index wins ties */",
     "      if (best < 0 || arow[J] >= arow[best]) best = J;",
     [lambda: pins.test_select_ties_go_to_the_lower_block_index()]),
    ("selection: keeps the smallest scores",
     "      if (best < 0 || arow[J] > arow[best]) best = J; /* strict >: the lower index wins ties */",
     "      if (best < 0 || arow[J] < arow[best]) best = J;",
     [lambda: pins.test_select_maximises_kept_mass_by_exhaustive_search()]),
    ("sparse: key offset uses the query block size",
     "        const int j = cols[t] * bk + c;\n        if (j >= L) {",
     "        const int j = cols[t] * bq + c;\n        if (j >= L) {",
     [lambda: pins.test_sparse_matches_bruteforce_mask_sdpa_and_renormalised_dense(16, 8, 2)]),
    ("sparse: normalised by the number of kept keys instead of the softmax sum",
     "        const double p = s[t * bk + c] / z;\n        const float* vrow = vhead + (size_t)j * d;",
     "        const double p = s[t * bk + c] / (double)nkept;\n        const float* vrow = vhead + (size_t)j * d;",
     [lambda: pins.test_sparse_with_every_block_kept_equals_dense()]),
    ("brute-force mask: listed blocks masked OUT",
     "          M[(size_t)i * L + j] = listed ? 0.0 : -INFINITY;",
     "          M[(size_t)i * L + j] = listed ? -INFINITY : 0.0;",
     [lambda: pins.test_sparse_matches_bruteforce_mask_sdpa_and_renormalised_dense(8, 8, 3)]),
    ("isolated selection: generation range ranked over the whole row",
     "    if (keep_gen > 0) mark_topk(arow, n_pre, nkb, keep_gen, mark, NULL, NULL);",
     "    if (keep_gen > 0) mark_topk(arow, 0, nkb, keep_gen, mark, NULL, NULL);",
     [lambda: pins.test_isolated_selection_reduces_to_plain_and_splits_ranges()]),
]


@pytest.mark.parametrize("name,old,new,checks", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, checks, monkeypatch):
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation site not found for: {name}"
    with tempfile.TemporaryDirectory() as tmp:
        c_path, so_path = os.path.join(tmp, "mutant.c"), os.path.join(tmp, "mutant.so")
        with open(c_path, "w") as f:
            f.write(src.replace(old, new, 1))
        subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-w", "-o", so_path, c_path, "-lm"], check=True)
        good = oracle._load()
        monkeypatch.setattr(oracle, "_lib", ctypes.CDLL(so_path))
        try:
            for check in checks:
                with pytest.raises(AssertionError):
                    check()
        finally:
            monkeypatch.setattr(oracle, "_lib", good)
    # and the unmutated oracle still passes the same checks
    for check in checks:
        check()
