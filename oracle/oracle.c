/*
 * SparseD reference oracle: plain, slow, obviously-correct CPU code in fp64.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it. It shares no code, header,
 * table or helper with the HIP library; the HIP library never calls it.
 *
 * Every function follows the paper (SparseD, arXiv 2509.24014) by its plain
 * definition, one query row (or one query block) at a time, with no blocking,
 * fusion or reordering beyond what the definition states:
 *
 *   oracle_attn_dense*        Section 3.1, Eq. 1   A = Softmax(Q K^T / sqrt(d)),  O = A V
 *   oracle_attn_probs_row     Section 3.1, Eq. 1   one row of A
 *   oracle_pool_scores*       Section 3.3 "Isolated Selection": A' = avgpool(A, block)
 *                             and Algorithm 1 (the per-query-block loop)
 *   oracle_kept_blocks        the count behind "Top rho%" of Eq. 2 / Eq. 6
 *   oracle_select_topk        Eq. 6 without the prefill/generation split
 *   oracle_select_isolated    Eq. 5 + Eq. 6 with the split at a block boundary
 *   oracle_attn_sparse*       Eq. 3 with the mask of Eq. 4 taken as a set restriction
 *   oracle_attn_masked_bruteforce   Eq. 3 + Eq. 4 literally: an explicit L x L matrix
 *                             of 0 / -inf added to the logits (tiny inputs only)
 *
 * Storage: inputs are float32 arrays [B, H, L, d], contiguous. float32 holds every
 * bf16 and fp32 input value exactly, so widening to double loses nothing; all
 * arithmetic below is double. Grouped-query attention: query head h reads
 * key/value head h / (Hq / Hkv).
 *
 * Parallelism: OpenMP over independent (batch, head, row) or (batch, head, block)
 * units only; the arithmetic inside a unit is sequential and in the order written.
 *
 * Return value: 0 on success, a negative number on a bad argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX4(b, h, i, H, L, d) ((((size_t)(b) * (size_t)(H) + (size_t)(h)) * (size_t)(L) + (size_t)(i)) * (size_t)(d))

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- Eq. 1, one row: logits, softmax probabilities over all L keys -------- */
/* p[j] = exp(s_j - max) / sum, s_j = (q_i . k_j) / sqrt(d), j = 0..L-1.        */
static void probs_row(const float* qrow, const float* khead, int L, int d, double* p) {
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  double m = -INFINITY;
  for (int j = 0; j < L; ++j) {
    const float* krow = khead + (size_t)j * d;
    double dot = 0.0;
    for (int c = 0; c < d; ++c) dot += (double)qrow[c] * (double)krow[c];
    p[j] = dot * inv_sqrt_d;
    if (p[j] > m) m = p[j];
  }
  double z = 0.0;
  for (int j = 0; j < L; ++j) {
    p[j] = exp(p[j] - m);
    z += p[j];
  }
  for (int j = 0; j < L; ++j) p[j] /= z;
}

static int check_shape(int B, int Hq, int Hkv, int L, int d) {
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || L <= 0 || d <= 0) return -1;
  if (Hq % Hkv != 0) return -2;
  return 0;
}

/* One row of A (Eq. 1) for inspection by the tests. p has L entries. */
int oracle_attn_probs_row(const float* q, const float* k, int B, int Hq, int Hkv, int L, int d,
                          int b, int h, int i, double* p) {
  int rc = check_shape(B, Hq, Hkv, L, d);
  if (rc) return rc;
  if (b < 0 || b >= B || h < 0 || h >= Hq || i < 0 || i >= L) return -3;
  const int g = h / (Hq / Hkv);
  probs_row(q + IDX4(b, h, i, Hq, L, d), k + IDX4(b, g, 0, Hkv, L, d), L, d, p);
  return 0;
}

/* ---- Eq. 1: dense attention for rows [i0, i1) of one (b, h) ---------------- */
/* out is [(i1 - i0), d] doubles.                                              */
int oracle_attn_dense_rows(const float* q, const float* k, const float* v, int B, int Hq, int Hkv,
                           int L, int d, int b, int h, int i0, int i1, double* out) {
  int rc = check_shape(B, Hq, Hkv, L, d);
  if (rc) return rc;
  if (b < 0 || b >= B || h < 0 || h >= Hq || i0 < 0 || i1 > L || i0 > i1) return -3;
  const int g = h / (Hq / Hkv);
  const float* khead = k + IDX4(b, g, 0, Hkv, L, d);
  const float* vhead = v + IDX4(b, g, 0, Hkv, L, d);
  int fail = 0;
#pragma omp parallel
  {
    double* p = (double*)malloc((size_t)L * sizeof(double));
    if (!p) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(dynamic, 4)
    for (int i = i0; i < i1; ++i) {
      if (!p) continue;
      probs_row(q + IDX4(b, h, i, Hq, L, d), khead, L, d, p);
      double* o = out + (size_t)(i - i0) * d;
      for (int c = 0; c < d; ++c) o[c] = 0.0;
      for (int j = 0; j < L; ++j) {
        const float* vrow = vhead + (size_t)j * d;
        for (int c = 0; c < d; ++c) o[c] += p[j] * (double)vrow[c];
      }
    }
    free(p);
  }
  return fail ? -9 : 0;
}

/* Eq. 1 over the whole tensor; out is [B, Hq, L, d] doubles. */
int oracle_attn_dense(const float* q, const float* k, const float* v, int B, int Hq, int Hkv, int L,
                      int d, double* out) {
  int rc = check_shape(B, Hq, Hkv, L, d);
  if (rc) return rc;
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      rc = oracle_attn_dense_rows(q, k, v, B, Hq, Hkv, L, d, b, h, 0, L, out + IDX4(b, h, 0, Hq, L, d));
      if (rc) return rc;
    }
  return 0;
}

/* ---- Section 3.3: A' = avgpool(A, block) for query blocks [I0, I1) --------- */
/* For each query block I (rows I*bq .. I*bq+bq-1) and key block J, the mean of
 * A over the bq x bk rectangle; A is the full-row softmax of Eq. 1. The loop is
 * Algorithm 1's: one query block at a time, never more than bq rows of A alive.
 * When L is not a multiple of a block size the last block of that axis is
 * partial (nqb = ceil(L/bq), nkb = ceil(L/bk)) and its mean runs over the
 * entries that exist. apool is [(I1 - I0), nkb] doubles.                        */
int oracle_pool_scores_rows(const float* q, const float* k, int B, int Hq, int Hkv, int L, int d,
                            int bq, int bk, int b, int h, int I0, int I1, double* apool) {
  int rc = check_shape(B, Hq, Hkv, L, d);
  if (rc) return rc;
  if (bq <= 0 || bk <= 0) return -4;
  const int nqb = (L + bq - 1) / bq, nkb = (L + bk - 1) / bk;
  if (b < 0 || b >= B || h < 0 || h >= Hq || I0 < 0 || I1 > nqb || I0 > I1) return -3;
  const int g = h / (Hq / Hkv);
  const float* khead = k + IDX4(b, g, 0, Hkv, L, d);
  int fail = 0;
#pragma omp parallel
  {
    double* p = (double*)malloc((size_t)L * sizeof(double));
    if (!p) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (int I = I0; I < I1; ++I) {
      if (!p) continue;
      double* arow = apool + (size_t)(I - I0) * nkb;
      for (int J = 0; J < nkb; ++J) arow[J] = 0.0;
      const int rows = (I * bq + bq <= L) ? bq : L - I * bq; /* rows that exist in this query block */
      for (int r = 0; r < rows; ++r) {
        probs_row(q + IDX4(b, h, I * bq + r, Hq, L, d), khead, L, d, p);
        for (int J = 0; J < nkb; ++J) {
          double s = 0.0;
          for (int c = 0; c < bk && J * bk + c < L; ++c) s += p[J * bk + c];
          arow[J] += s;
        }
      }
      for (int J = 0; J < nkb; ++J) {
        const int colsJ = (J * bk + bk <= L) ? bk : L - J * bk; /* keys that exist in this key block */
        arow[J] /= (double)rows * (double)colsJ;
      }
    }
    free(p);
  }
  return fail ? -9 : 0;
}

/* A' for the whole tensor: apool is [B, Hq, nqb, nkb] doubles. */
int oracle_pool_scores(const float* q, const float* k, int B, int Hq, int Hkv, int L, int d, int bq,
                       int bk, double* apool) {
  int rc = check_shape(B, Hq, Hkv, L, d);
  if (rc) return rc;
  if (bq <= 0 || bk <= 0) return -4;
  const int nqb = (L + bq - 1) / bq, nkb = (L + bk - 1) / bk;
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      rc = oracle_pool_scores_rows(q, k, B, Hq, Hkv, L, d, bq, bk, b, h, 0, nqb,
                                   apool + ((size_t)b * Hq + h) * (size_t)nqb * nkb);
      if (rc) return rc;
    }
  return 0;
}

/* ---- "Top rho%": how many of n key blocks are kept -------------------------- */
/* ceil(rho * n), guarded against rho*n landing a hair above an integer, and
 * clamped to [1, n]. The paper only says "top rho%"; this count is the reading
 * both sides take.                                                             */
int oracle_kept_blocks(double rho, int n) {
  if (n <= 0) return 0;
  int kk = (int)ceil(rho * (double)n - 1e-9);
  if (kk < 1) kk = 1;
  if (kk > n) kk = n;
  return kk;
}

/* Keep the `keep` best of arow[lo..hi) ranked by (score descending, block index
 * ascending), mark them in `mark`, and report the keep-th and (keep+1)-th best
 * scores. Selection sort on purpose: the ranking rule is visible in one line.   */
static void mark_topk(const double* arow, int lo, int hi, int keep, unsigned char* mark,
                      double* kth, double* next) {
  double last = NAN;
  for (int t = 0; t < keep; ++t) {
    int best = -1;
    for (int J = lo; J < hi; ++J) {
      if (mark[J]) continue;
      if (best < 0 || arow[J] > arow[best]) best = J; /* strict >: the lower index wins ties */
    }
    mark[best] = 1;
    last = arow[best];
  }
  double nx = NAN;
  int best = -1;
  for (int J = lo; J < hi; ++J) {
    if (mark[J]) continue;
    if (best < 0 || arow[J] > arow[best]) best = J;
  }
  if (best >= 0) nx = arow[best];
  if (kth) *kth = last;
  if (next) *next = nx;
}

/* ---- Eq. 6 (single key range): per query block keep the top-k key blocks ---- */
/* apool [B, Hq, nqb, nkb]; row_ptr [B, Hq, nqb+1] (offsets local to each (b,h));
 * col_idx [B, Hq, nqb*keep], each row ascending; cut [B, Hq, nqb, 2] = the
 * keep-th best score and the best score left out (NaN when keep == nkb).        */
int oracle_select_topk(const double* apool, int B, int Hq, int nqb, int nkb, int keep,
                       int32_t* row_ptr, int32_t* col_idx, double* cut) {
  if (B <= 0 || Hq <= 0 || nqb <= 0 || nkb <= 0 || keep < 1 || keep > nkb) return -1;
  int fail = 0;
#pragma omp parallel
  {
    unsigned char* mark = (unsigned char*)malloc((size_t)nkb);
    if (!mark) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(static)
    for (long u = 0; u < (long)B * Hq * nqb; ++u) {
      if (!mark) continue;
      const long bh = u / nqb;
      const int I = (int)(u % nqb);
      const double* arow = apool + (size_t)u * nkb;
      memset(mark, 0, (size_t)nkb);
      double kth, next;
      mark_topk(arow, 0, nkb, keep, mark, &kth, &next);
      int32_t* cols = col_idx + (size_t)bh * nqb * keep + (size_t)I * keep;
      int n = 0;
      for (int J = 0; J < nkb; ++J)
        if (mark[J]) cols[n++] = J;
      int32_t* rp = row_ptr + (size_t)bh * (nqb + 1);
      rp[I] = I * keep;
      if (I == nqb - 1) rp[nqb] = nqb * keep;
      if (cut) {
        cut[(size_t)u * 2 + 0] = kth;
        cut[(size_t)u * 2 + 1] = next;
      }
    }
    free(mark);
  }
  return fail ? -9 : 0;
}

/* ---- Eq. 5 + Eq. 6: isolated selection -------------------------------------- */
/* Key blocks [0, n_pre) are the prefill range and [n_pre, nkb) the generation
 * range; each range keeps its own top oracle_kept_blocks(rho, range size); the
 * row is their union, ascending. A range of size 0 keeps nothing. Every row has
 * the same length keep_pre + keep_gen.                                          */
int oracle_select_isolated(const double* apool, int B, int Hq, int nqb, int nkb, double rho,
                           int n_pre, int32_t* row_ptr, int32_t* col_idx) {
  if (B <= 0 || Hq <= 0 || nqb <= 0 || nkb <= 0 || n_pre < 0 || n_pre > nkb) return -1;
  const int keep_pre = oracle_kept_blocks(rho, n_pre);
  const int keep_gen = oracle_kept_blocks(rho, nkb - n_pre);
  const int keep = keep_pre + keep_gen;
  unsigned char* mark = (unsigned char*)malloc((size_t)nkb);
  if (!mark) return -9;
  for (long u = 0; u < (long)B * Hq * nqb; ++u) {
    const long bh = u / nqb;
    const int I = (int)(u % nqb);
    const double* arow = apool + (size_t)u * nkb;
    memset(mark, 0, (size_t)nkb);
    if (keep_pre > 0) mark_topk(arow, 0, n_pre, keep_pre, mark, NULL, NULL);
    if (keep_gen > 0) mark_topk(arow, n_pre, nkb, keep_gen, mark, NULL, NULL);
    int32_t* cols = col_idx + (size_t)bh * nqb * keep + (size_t)I * keep;
    int n = 0;
    for (int J = 0; J < nkb; ++J)
      if (mark[J]) cols[n++] = J;
    int32_t* rp = row_ptr + (size_t)bh * (nqb + 1);
    rp[I] = I * keep;
    if (I == nqb - 1) rp[nqb] = nqb * keep;
  }
  free(mark);
  return 0;
}

/* ---- Eq. 5 + Eq. 6 with the prefill / generation boundary at a key TOKEN ----- */
/* The paper splits the keys into the prefill tokens [0, p) and the generation
 * tokens [p, L) and ranks each range on its own (Eq. 5, Eq. 6); it does not say
 * what happens when p falls inside a key block. Reading taken here: the block
 * that holds p is pooled twice, once over its prefill keys and once over its
 * generation keys (each a mean over the entries that exist), and competes in
 * both ranges; it is kept if either range keeps it.
 *
 * oracle_pool_scores_ranges: mean of A over (query block I) x (keys [vstart[v], vend[v]))
 * for nv arbitrary key ranges; out is [B, Hq, nqb, nv] doubles.                 */
int oracle_pool_scores_ranges(const float* q, const float* k, int B, int Hq, int Hkv, int L, int d,
                              int bq, int nv, const int32_t* vstart, const int32_t* vend, double* out) {
  int rc = check_shape(B, Hq, Hkv, L, d);
  if (rc) return rc;
  if (bq <= 0 || nv <= 0) return -4;
  for (int v = 0; v < nv; ++v)
    if (vstart[v] < 0 || vend[v] > L || vstart[v] >= vend[v]) return -4;
  const int nqb = (L + bq - 1) / bq;
  int fail = 0;
#pragma omp parallel
  {
    double* p = (double*)malloc((size_t)L * sizeof(double));
    if (!p) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(dynamic, 1)
    for (long u = 0; u < (long)B * Hq * nqb; ++u) {
      if (!p) continue;
      const int I = (int)(u % nqb);
      const int h = (int)((u / nqb) % Hq), b = (int)(u / nqb / Hq);
      const float* khead = k + IDX4(b, h / (Hq / Hkv), 0, Hkv, L, d);
      double* arow = out + (size_t)u * nv;
      for (int v = 0; v < nv; ++v) arow[v] = 0.0;
      const int rows = (I * bq + bq <= L) ? bq : L - I * bq;
      for (int r = 0; r < rows; ++r) {
        probs_row(q + IDX4(b, h, I * bq + r, Hq, L, d), khead, L, d, p);
        for (int v = 0; v < nv; ++v)
          for (int j = vstart[v]; j < vend[v]; ++j) arow[v] += p[j];
      }
      for (int v = 0; v < nv; ++v) arow[v] /= (double)rows * (double)(vend[v] - vstart[v]);
    }
    free(p);
  }
  return fail ? -9 : 0;
}

/* Ranks the ranges [0, n_pre) and [n_pre, nv) of every pooled row separately,
 * keeps oracle_kept_blocks(rho, size) of each, maps range v to key block vblock[v]
 * (two neighbouring ranges may map to the same block) and writes the union,
 * ascending and without duplicates, as CSR: rows may differ in length by one.
 * row_ptr [B, Hq, nqb+1], col_idx [B, Hq, cap] with cap >= nqb * (keep_pre + keep_gen). */
int oracle_select_isolated_ranges(const double* apool, int B, int Hq, int nqb, int nv, double rho, int n_pre,
                                  const int32_t* vblock, int cap, int32_t* row_ptr, int32_t* col_idx) {
  if (B <= 0 || Hq <= 0 || nqb <= 0 || nv <= 0 || n_pre < 0 || n_pre > nv) return -1;
  const int keep_pre = oracle_kept_blocks(rho, n_pre);
  const int keep_gen = oracle_kept_blocks(rho, nv - n_pre);
  if (cap < nqb * (keep_pre + keep_gen)) return -1;
  unsigned char* mark = (unsigned char*)malloc((size_t)nv);
  if (!mark) return -9;
  for (long bh = 0; bh < (long)B * Hq; ++bh) {
    int32_t* rp = row_ptr + (size_t)bh * (nqb + 1);
    int32_t* cols = col_idx + (size_t)bh * cap;
    int n = 0;
    rp[0] = 0;
    for (int I = 0; I < nqb; ++I) {
      const double* arow = apool + ((size_t)bh * nqb + I) * nv;
      memset(mark, 0, (size_t)nv);
      if (keep_pre > 0) mark_topk(arow, 0, n_pre, keep_pre, mark, NULL, NULL);
      if (keep_gen > 0) mark_topk(arow, n_pre, nv, keep_gen, mark, NULL, NULL);
      const int row_begin = n;
      for (int v = 0; v < nv; ++v) {
        if (!mark[v]) continue;
        if (n > row_begin && cols[n - 1] == vblock[v]) continue; /* the straddling block, kept by both ranges */
        cols[n++] = vblock[v];
      }
      rp[I + 1] = n;
    }
  }
  free(mark);
  return 0;
}

/* ---- Eq. 3 + Eq. 4 as a set restriction: one query block -------------------- */
/* Rows of query block I attend only to keys in the listed key blocks; max, sum
 * and the weighted V-sum run over those keys only. An empty list gives zeros.
 * cols: n_cols block indices (any order, no duplicates). out: [bq, d] doubles.  */
static int sparse_block(const float* q, const float* k, const float* v, int Hq, int Hkv, int L, int d,
                        int bq, int bk, int b, int h, int I, const int32_t* cols, int n_cols,
                        double* out) {
  const int g = h / (Hq / Hkv);
  const float* khead = k + IDX4(b, g, 0, Hkv, L, d);
  const float* vhead = v + IDX4(b, g, 0, Hkv, L, d);
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  const int nkept = n_cols * bk; /* slots; a key beyond L (partial last block) keeps its slot at -inf */
  double* s = (double*)malloc((size_t)(nkept > 0 ? nkept : 1) * sizeof(double));
  if (!s) return -9;
  for (int r = 0; r < bq && I * bq + r < L; ++r) {
    const float* qrow = q + IDX4(b, h, I * bq + r, Hq, L, d);
    double* o = out + (size_t)r * d;
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    if (nkept == 0) continue;
    double m = -INFINITY;
    for (int t = 0; t < n_cols; ++t)
      for (int c = 0; c < bk; ++c) {
        const int j = cols[t] * bk + c;
        if (j >= L) {
          s[t * bk + c] = -INFINITY;
          continue;
        }
        const float* krow = khead + (size_t)j * d;
        double dot = 0.0;
        for (int e = 0; e < d; ++e) dot += (double)qrow[e] * (double)krow[e];
        s[t * bk + c] = dot * inv_sqrt_d;
        if (s[t * bk + c] > m) m = s[t * bk + c];
      }
    double z = 0.0;
    for (int x = 0; x < nkept; ++x) {
      s[x] = exp(s[x] - m);
      z += s[x];
    }
    for (int t = 0; t < n_cols; ++t)
      for (int c = 0; c < bk; ++c) {
        const int j = cols[t] * bk + c;
        if (j >= L) continue;
        const double p = s[t * bk + c] / z;
        const float* vrow = vhead + (size_t)j * d;
        for (int e = 0; e < d; ++e) o[e] += p * (double)vrow[e];
      }
  }
  free(s);
  return 0;
}

/* Sparse attention for query blocks [I0, I1) of one (b, h). row_ptr/col_idx are
 * the whole index ([B,Hq,nqb+1] / [B,Hq,cap_per_head]); out is [(I1-I0)*bq, d]. */
int oracle_attn_sparse_rows(const float* q, const float* k, const float* v, int B, int Hq, int Hkv,
                            int L, int d, int bq, int bk, const int32_t* row_ptr,
                            const int32_t* col_idx, int cap_per_head, int b, int h, int I0, int I1,
                            double* out) {
  int rc = check_shape(B, Hq, Hkv, L, d);
  if (rc) return rc;
  if (bq <= 0 || bk <= 0) return -4;
  const int nqb = (L + bq - 1) / bq, nkb = (L + bk - 1) / bk;
  if (b < 0 || b >= B || h < 0 || h >= Hq || I0 < 0 || I1 > nqb || I0 > I1) return -3;
  const int32_t* rp = row_ptr + ((size_t)b * Hq + h) * (size_t)(nqb + 1);
  const int32_t* ci = col_idx + ((size_t)b * Hq + h) * (size_t)cap_per_head;
  for (int I = I0; I < I1; ++I) {
    if (rp[I] < 0 || rp[I + 1] < rp[I] || rp[I + 1] > cap_per_head) return -5;
    for (int t = rp[I]; t < rp[I + 1]; ++t)
      if (ci[t] < 0 || ci[t] >= nkb) return -5;
  }
  int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int I = I0; I < I1; ++I) {
    int r = sparse_block(q, k, v, Hq, Hkv, L, d, bq, bk, b, h, I, ci + rp[I], rp[I + 1] - rp[I],
                         out + (size_t)(I - I0) * bq * d);
    if (r) {
#pragma omp atomic write
      fail = 1;
    }
  }
  return fail ? -9 : 0;
}

/* Sparse attention over the whole tensor; out is [B, Hq, L, d] doubles. */
int oracle_attn_sparse(const float* q, const float* k, const float* v, int B, int Hq, int Hkv, int L,
                       int d, int bq, int bk, const int32_t* row_ptr, const int32_t* col_idx,
                       int cap_per_head, double* out) {
  int rc = check_shape(B, Hq, Hkv, L, d);
  if (rc) return rc;
  if (bq <= 0 || bk <= 0) return -4;
  const int nqb = (L + bq - 1) / bq;
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      rc = oracle_attn_sparse_rows(q, k, v, B, Hq, Hkv, L, d, bq, bk, row_ptr, col_idx, cap_per_head,
                                   b, h, 0, nqb, out + IDX4(b, h, 0, Hq, L, d));
      if (rc) return rc;
    }
  return 0;
}

/* ---- Eq. 3 + Eq. 4 literally (tiny inputs) ---------------------------------- */
/* Builds the explicit L x L matrix M_S of 0 / -inf element by element from the
 * block list, forms (Q K^T + M_S) / sqrt(d), takes a row softmax with
 * exp(-inf) = 0, multiplies by V. A row whose mask is all -inf gives zeros.
 * out is [B, Hq, L, d] doubles.                                                */
int oracle_attn_masked_bruteforce(const float* q, const float* k, const float* v, int B, int Hq,
                                  int Hkv, int L, int d, int bq, int bk, const int32_t* row_ptr,
                                  const int32_t* col_idx, int cap_per_head, double* out) {
  int rc = check_shape(B, Hq, Hkv, L, d);
  if (rc) return rc;
  if (bq <= 0 || bk <= 0) return -4;
  if ((size_t)L * (size_t)L > ((size_t)1 << 26)) return -6; /* tiny inputs only */
  const int nqb = (L + bq - 1) / bq, nkb = (L + bk - 1) / bk;
  double* M = (double*)malloc((size_t)L * L * sizeof(double));
  double* S = (double*)malloc((size_t)L * L * sizeof(double));
  if (!M || !S) {
    free(M);
    free(S);
    return -9;
  }
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      const int g = h / (Hq / Hkv);
      const int32_t* rp = row_ptr + ((size_t)b * Hq + h) * (size_t)(nqb + 1);
      const int32_t* ci = col_idx + ((size_t)b * Hq + h) * (size_t)cap_per_head;
      /* Eq. 4: M[i][j] = 0 if (i, j) is in the selected set, -inf otherwise. */
      for (int i = 0; i < L; ++i)
        for (int j = 0; j < L; ++j) {
          int listed = 0;
          for (int t = rp[i / bq]; t < rp[i / bq + 1]; ++t)
            if (ci[t] == j / bk) listed = 1;
          M[(size_t)i * L + j] = listed ? 0.0 : -INFINITY;
        }
      (void)nkb;
      /* Eq. 3: Softmax((Q K^T + M) / sqrt(d)) V. */
      for (int i = 0; i < L; ++i) {
        const float* qrow = q + IDX4(b, h, i, Hq, L, d);
        double m = -INFINITY;
        for (int j = 0; j < L; ++j) {
          const float* krow = k + IDX4(b, g, j, Hkv, L, d);
          double dot = 0.0;
          for (int c = 0; c < d; ++c) dot += (double)qrow[c] * (double)krow[c];
          S[(size_t)i * L + j] = (dot + M[(size_t)i * L + j]) / sqrt((double)d);
          if (S[(size_t)i * L + j] > m) m = S[(size_t)i * L + j];
        }
        double* o = out + IDX4(b, h, i, Hq, L, d);
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        if (m == -INFINITY) continue;
        double z = 0.0;
        for (int j = 0; j < L; ++j) {
          S[(size_t)i * L + j] = exp(S[(size_t)i * L + j] - m); /* exp(-inf) = 0 */
          z += S[(size_t)i * L + j];
        }
        for (int j = 0; j < L; ++j) {
          const double p = S[(size_t)i * L + j] / z;
          const float* vrow = v + IDX4(b, g, j, Hkv, L, d);
          for (int c = 0; c < d; ++c) o[c] += p * (double)vrow[c];
        }
      }
    }
  free(M);
  free(S);
  return 0;
}
