/*
 * sparsed.h - C ABI of the MI355X (gfx950) SparseD attention library.
 *
 * SparseD (arXiv 2509.24014) runs full bidirectional attention for the early
 * denoising steps of a diffusion language model, selects one block-sparse
 * pattern per head at a switch step, and reuses it for every later step
 * (Section 3.3, Algorithm 1). The three calls of that algorithm are the three
 * compute entry points below. Plain C11: no C++ or framework types cross this
 * boundary.
 *
 * Conventions for every entry point
 *  - All tensor, index and workspace pointers are DEVICE pointers owned by the
 *    caller. The library never frees them and keeps no reference after a call
 *    returns. Descriptor structs themselves live in HOST memory.
 *  - Work is enqueued on `ex->stream` (a hipStream_t; NULL or ex == NULL means
 *    the default stream) and the call returns without synchronising, except
 *    where a function says it synchronises. The library allocates no device
 *    memory and keeps no state between calls except the thread-local error
 *    message: scratch memory is the caller's (`ex->workspace`), and a call that
 *    needs one and is given none returns SPARSED_ERR_WORKSPACE.
 *    sparsed_attn_dense, sparsed_attn_sparse and the selection entry points
 *    only launch kernels (no allocation, no memset, no copy), so they may be
 *    recorded into a HIP graph on a capturing stream.
 *  - Errors are returned as a sparsed_status; nothing throws or aborts. Every
 *    argument check happens before the first launch: on a status other than
 *    SPARSED_OK and SPARSED_ERR_HIP no kernel was launched and outputs are
 *    untouched. SPARSED_ERR_HIP reports a failed launch; the selection entry
 *    points launch several kernels in a row, so earlier ones of the same call
 *    may already be enqueued (they write only the workspace, pooled_out and
 *    the index). sparsed_last_error() gives a thread-local message.
 *  - Tensors are [B, H, L, D] views with arbitrary element strides for B, H, L
 *    and unit stride for D. `data` must be 16-byte aligned and every stride a
 *    multiple of 8 elements (bf16) or 4 elements (fp32), so that every row is
 *    16-byte aligned. One (batch, head) slab, (L-1)*stride_l + D elements, must
 *    span less than 2^31 bytes.
 *  - Grouped-query attention: q has Hq heads, k and v have Hkv heads with
 *    Hq % Hkv == 0; query head h reads key/value head h / (Hq / Hkv).
 *  - Supported shapes: D in {64, 128}; any L >= 1; block_q in {32, 64, 128};
 *    block_k in {32, 64, 128}; the paper's square settings 32 x 32 and 128 x 128
 *    are among them. L need not be a
 *    multiple of the block sizes: there are nqb = ceil(L / block_q) query blocks
 *    and nkb = ceil(L / block_k) key blocks, the last of each possibly partial
 *    (the paper pools with L // block_size and is silent on a remainder).
 *  - Arithmetic: bf16 tensors are multiplied on the bf16 matrix cores with
 *    fp32 accumulation, softmax in fp32, probabilities rounded to bf16 before
 *    the product with V. fp32 tensors use fp32 matrix cores throughout.
 *    Pooled scores for selection are fp32 from the logits on, for either dtype.
 */
#ifndef SPARSED_H
#define SPARSED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sparsed_status {
  SPARSED_OK = 0,
  SPARSED_ERR_NULL = 1,        /* a required pointer is NULL */
  SPARSED_ERR_SHAPE = 2,       /* dimensions disagree or are not block multiples */
  SPARSED_ERR_DTYPE = 3,       /* unknown dtype or dtypes differ between tensors */
  SPARSED_ERR_STRIDE = 4,      /* misaligned pointer or stride */
  SPARSED_ERR_RANGE = 5,       /* rho outside (0, 1], negative size, ... */
  SPARSED_ERR_UNSUPPORTED = 6, /* head dim / block size the kernels do not cover */
  SPARSED_ERR_WORKSPACE = 7,   /* workspace missing or too small */
  SPARSED_ERR_INDEX = 8,       /* malformed block index */
  SPARSED_ERR_HIP = 9          /* a HIP runtime call failed; see sparsed_last_error() */
} sparsed_status;

typedef enum sparsed_dtype { SPARSED_BF16 = 0, SPARSED_F32 = 1 } sparsed_dtype;

/* A [B, H, L, D] view of device memory. Strides are in elements. */
typedef struct sparsed_tensor {
  void* data;
  int32_t dtype; /* sparsed_dtype */
  int32_t B, H, L, D;
  int64_t stride_b, stride_h, stride_l;
} sparsed_tensor;

/*
 * The sparse pattern M_S of Eq. 4 stored as a per-head CSR over key blocks:
 * query block I of head (b, h) attends to key blocks
 *   col_idx[(b*H + h)*cap_per_head + t],  t in [row_ptr[(b*H+h)*(nqb+1) + I],
 *                                               row_ptr[(b*H+h)*(nqb+1) + I + 1])
 * i.e. offsets in row_ptr are local to the head's slab and row_ptr[.., 0] == 0.
 * Each row is strictly ascending. H is the number of QUERY heads. Rows may have
 * different lengths; an empty row makes that query block's output all zeros.
 */
typedef struct sparsed_block_index {
  int32_t B, H, nqb, nkb;
  int32_t block_q, block_k;
  int32_t cap_per_head; /* entries of col_idx reserved per (b, h) */
  int32_t* row_ptr;     /* device, [B, H, nqb + 1] */
  int32_t* col_idx;     /* device, [B, H, cap_per_head] */
} sparsed_block_index;

/* Optional execution context. A NULL context means: default stream, no extras. */
typedef struct sparsed_exec {
  void* stream;           /* hipStream_t */
  void* workspace;        /* device scratch for the selection calls and sparsed_index_validate, 256-byte aligned */
  size_t workspace_bytes; /* its size */
  float* lse_out;         /* attn_dense: optional [B, Hq, L] fp32, log-sum-exp of each row's scaled logits */
  const float* lse_in;    /* select_pattern: optional [B, Hq, L] fp32 from attn_dense on the SAME q, k */
  float* pooled_out;      /* select_pattern: optional [B, Hq, nqb, nkb] fp32 copy of the pooled scores A' */
  const int32_t* seq_lens; /* optional DEVICE array [B]: per-sample lengths, see below */
} sparsed_exec;

/*
 * Per-sample lengths (not in the paper, whose runs use one length per call): with ex->seq_lens set,
 * batch element b has min(seq_lens[b], L) tokens; its rows and keys at or past that do not exist.
 *  - attn_dense / attn_sparse: those query rows are neither computed nor stored (out and lse_out keep
 *    what they held); keys past the length are masked.
 *  - select_pattern: sample b pools and ranks its own ceil(len / block_k) key blocks and keeps
 *    sparsed_kept_blocks(rho, that many) per query block: row_ptr[I] = I * k_b for its ceil(len / block_q)
 *    query blocks, and the query blocks it does not have get empty rows. pooled_out entries of blocks a
 *    sample does not have are not written. nqb, nkb and cap_per_head are still those of L.
 *  - select_pattern_isolated: the same with two ranges per sample, [0, min(prefill_blocks, its blocks)) and
 *    the rest of its blocks, each with its own count; a sample no longer than the prefill has one range.
 *  - select_pattern_isolated_tokens: the same with the boundary at a key token p; a sample longer than p
 *    splits the key block that holds p as described at that call (its generation part ends at the sample's
 *    length), a sample no longer than p has one range over its own blocks.
 *  - A length <= 0 makes the whole sample a no-op.
 */

/*
 * Full attention of the early denoising steps (Section 3.1, Eq. 1; Algorithm 1,
 * the "Skipping Sparse" branch):
 *     out[b,h,i,:] = sum_j softmax_j(q[b,h,i,:] . k[b,g,j,:] / sqrt(D)) * v[b,g,j,:]
 * over all j in [0, L), no causal mask. q, out: [B, Hq, L, D]; k, v: [B, Hkv, L, D].
 * If ex->lse_out is set it also receives log(sum_j exp(logit_ij)) per row.
 */
sparsed_status sparsed_attn_dense(const sparsed_tensor* q, const sparsed_tensor* k,
                                  const sparsed_tensor* v, sparsed_tensor* out,
                                  const sparsed_exec* ex);

/*
 * Pattern selection at the switch step (Section 3.3 "Isolated Selection" with a
 * single key range, Eq. 6; Algorithm 1, the per-query-block loop):
 *   1. A' = average of the softmax probabilities A of Eq. 1 over each
 *      block_q x block_k rectangle (each row of A normalised over all L keys;
 *      a partial last block is averaged over the entries that exist);
 *   2. for every query block keep the k = sparsed_kept_blocks(rho, nkb) key
 *      blocks with the largest A' (ties: lower block index), listed ascending.
 * The L x L matrix A is never formed. Fills out_block_index->row_ptr / col_idx
 * (every row has exactly k entries, row_ptr[I] = I*k); its B, H, nqb, nkb,
 * block_q, block_k must already describe q and the blocks and cap_per_head must
 * be >= nqb*k, else SPARSED_ERR_INDEX. Needs ex->workspace of at least
 * sparsed_select_workspace_min_bytes() bytes (SPARSED_ERR_WORKSPACE otherwise;
 * sparsed_select_workspace_bytes() lets it pool in one pass over the keys); the
 * workspace holds the row statistics and the pooled scores while the call's
 * kernels run, so calls that may overlap on the GPU need a workspace each.
 */
sparsed_status sparsed_select_pattern(const sparsed_tensor* q, const sparsed_tensor* k,
                                      int32_t block_q, int32_t block_k, double rho,
                                      sparsed_block_index* out_block_index,
                                      const sparsed_exec* ex);

/*
 * sparsed_select_pattern for callers that cannot allocate device memory or bring a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * selection, same kernels and results, with the scratch (row statistics + pooled scores) in a
 * fixed array of SPARSED_STATIC_SCRATCH_BYTES that is part of the library's code object; each GPU
 * the library runs on holds its own copy until the process ends. ex->workspace is ignored;
 * ex->stream, lse_in, pooled_out and seq_lens work as in sparsed_select_pattern. The call
 * allocates and frees nothing (its first call on a device looks the array's device address up
 * once). Returns SPARSED_ERR_WORKSPACE when sparsed_select_workspace_min_bytes() for these arguments
 * (the _min_ form) exceeds SPARSED_STATIC_SCRATCH_BYTES (e.g. 32 heads of 65536 tokens with 128 x 64 blocks need
 * 75 MB; 32 heads of 16384 tokens with 64 x 64 blocks need 10 MB and fit). All calls on one GPU
 * share that GPU's array, which keeps the previous call's contents (every entry a call reads it
 * has written first): calls that may overlap on one GPU race, so keep them on one stream or
 * order them with events.
 */
#define SPARSED_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
sparsed_status sparsed_select_pattern_static(const sparsed_tensor* q, const sparsed_tensor* k,
                                             int32_t block_q, int32_t block_k, double rho,
                                             sparsed_block_index* out_block_index,
                                             const sparsed_exec* ex);

/*
 * Sparse attention of the later steps ("Sparse Reusing"; Eq. 3 with the mask of
 * Eq. 4): rows of query block I attend only to the keys of the key blocks
 * listed for I (those below L, for a partial last block); the softmax is
 * normalised over those keys only. The index
 * contents are trusted (check them with sparsed_index_validate); its shape
 * fields are checked against q.
 */
sparsed_status sparsed_attn_sparse(const sparsed_tensor* q, const sparsed_tensor* k,
                                   const sparsed_tensor* v, const sparsed_block_index* block_index,
                                   sparsed_tensor* out, const sparsed_exec* ex);

/*
 * Isolated selection proper (Section 3.3, Eq. 5 and Eq. 6): key blocks
 * [0, prefill_blocks) and [prefill_blocks, nkb) are ranked separately, each
 * keeping sparsed_kept_blocks(rho, size of its range) blocks (none for an empty
 * range); a row is the ascending union. prefill_blocks == nkb or 0 gives the
 * same result as sparsed_select_pattern. cap_per_head must be >= nqb * (sum of
 * the two counts).
 */
sparsed_status sparsed_select_pattern_isolated(const sparsed_tensor* q, const sparsed_tensor* k,
                                               int32_t block_q, int32_t block_k, double rho,
                                               int32_t prefill_blocks,
                                               sparsed_block_index* out_block_index,
                                               const sparsed_exec* ex);

/*
 * Isolated selection with the boundary given as a key TOKEN (Eq. 5 splits the keys
 * into prefill tokens [0, prefill_tokens) and generation tokens [prefill_tokens, L)).
 * On a block edge this is sparsed_select_pattern_isolated. Otherwise the paper is
 * silent; reading: the key block that holds the boundary is pooled twice, over its
 * prefill keys and over its generation keys (each a mean over the entries that
 * exist), competes in both ranges with those scores, and is listed once if either
 * range keeps it. With n_pre = ceil(prefill_tokens / block_k) and n_gen = nkb -
 * floor(prefill_tokens / block_k), the ranges keep sparsed_kept_blocks(rho, n_pre)
 * and sparsed_kept_blocks(rho, n_gen) entries; a row has their sum or one fewer, so
 * row_ptr is not I*k here. cap_per_head must be >= nqb * (the sum). Workspace:
 * sparsed_select_tokens_workspace_bytes().
 */
sparsed_status sparsed_select_pattern_isolated_tokens(const sparsed_tensor* q, const sparsed_tensor* k,
                                                      int32_t block_q, int32_t block_k, double rho,
                                                      int32_t prefill_tokens,
                                                      sparsed_block_index* out_block_index,
                                                      const sparsed_exec* ex);

/*
 * Fixed pattern of the paper's sparse baselines (Section 4.1: sliding window, and
 * StreamingLLM = window + leading "sink" keys) written as a block index, so the
 * same sparse kernel runs them: query block I keeps every key block holding a
 * key j with |i - j| <= window_tokens/2 for one of its queries i (the window is
 * taken symmetric because attention here is bidirectional), plus the key blocks
 * that overlap the first sink_tokens keys. The same rows for every head; rows
 * have different lengths. idx->B, H, nqb, nkb, block_q, block_k must describe a
 * sequence of seq_len tokens (block counts rounded up); cap_per_head must be >=
 * sparsed_index_window_entries(...), else SPARSED_ERR_INDEX.
 */
sparsed_status sparsed_index_fill_window(sparsed_block_index* idx, int32_t seq_len, int32_t window_tokens,
                                         int32_t sink_tokens, const sparsed_exec* ex);

/* col_idx entries per head that sparsed_index_fill_window writes (-1 on bad arguments). Host only. */
int64_t sparsed_index_window_entries(int32_t seq_len, int32_t block_q, int32_t block_k, int32_t window_tokens,
                                     int32_t sink_tokens);

/* "Top rho%" of n blocks: ceil(rho*n - 1e-9) clamped to [1, n]; 0 if n <= 0. Host only. */
int32_t sparsed_kept_blocks(double rho, int32_t n);

/*
 * Number of full-attention steps of a T-step schedule with skip fraction `skip`
 * (Section 3.3 "Skipping Sparse"): clamp(ceil(T*skip - 1e-9), 1, T). Steps
 * 0 .. n-1 are dense, the pattern is selected at step n-1, steps n .. T-1 are
 * sparse. Host only.
 */
int32_t sparsed_n_dense_steps(int32_t T, double skip);

/*
 * Bytes of workspace the selection calls want for this q and these blocks (0 on bad arguments): the row statistics,
 * the pooled scores and, for bf16 inputs, the slabs of the one-pass pooled-score kernel that is used when no
 * ex->lse_in is handed over (128 x nkb floats for each of up to 1024 resident work-groups: 537 MB for 32
 * heads of 65536 tokens in 128 x 64 blocks). sparsed_select_workspace_min_bytes() is the part every call needs
 * (statistics + pooled scores, 75 MB in that example); with a workspace between the two, or with ex->lse_in set,
 * selection runs as row statistics (unless handed over) followed by pooled scores, two passes over the keys, with
 * the same results up to fp32 summation order.
 */
size_t sparsed_select_workspace_bytes(const sparsed_tensor* q, int32_t block_q, int32_t block_k);
size_t sparsed_select_workspace_min_bytes(const sparsed_tensor* q, int32_t block_q, int32_t block_k);

/* The same for sparsed_select_pattern_isolated_tokens (a little more: two extra pooled columns and row staging). */
size_t sparsed_select_tokens_workspace_bytes(const sparsed_tensor* q, int32_t block_q, int32_t block_k);

/*
 * Checks on the device that every row of the index is in range, strictly
 * ascending and within cap_per_head. SYNCHRONISES the stream. Returns
 * SPARSED_ERR_INDEX if any row is malformed. Needs ex->workspace of at least
 * 256 bytes (its first word counts the malformed rows).
 */
sparsed_status sparsed_index_validate(const sparsed_block_index* idx, const sparsed_exec* ex);

const char* sparsed_status_string(sparsed_status s);
const char* sparsed_last_error(void); /* thread-local, never NULL */
int32_t sparsed_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPARSED_H */
