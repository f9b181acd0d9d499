// Internal interface between the host-side C ABI (api.hip) and the gfx950 kernels.
// Not installed; include/sparsed.h is the public boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sparsed {

// One [B, H, L, D] operand: base pointer and element strides (stride of D is 1).
struct TensorArg {
  const void* ptr;
  int64_t sb, sh, sl;
};

// Arguments of the attention kernels (dense, sparse, and the statistics-only pass).
struct AttnArgs {
  TensorArg q, k, v;
  void* o;
  int64_t o_sb, o_sh, o_sl;
  float* lse;              // optional [B, Hq, L]: natural-log sum-exp of each row's scaled logits
  const int32_t* row_ptr;  // sparse only: [B, Hq, nqb + 1]
  const int32_t* col_idx;  // sparse only: [B, Hq, cap_per_head]
  int32_t B, Hq, Hkv, L;
  const int32_t* seq_lens; // optional [B]: rows and keys of batch element b at or past seq_lens[b] do not exist
  int32_t nqb, cap_per_head, block_k;
  int32_t n_qtiles;        // query tiles per head = ceil(L / rows per work-group)
  float scale_log2;        // log2(e) / sqrt(D)
};

// Arguments of the pooled-score kernels (Section 3.3: A' = avgpool(A, block)). The keys pooled are
// the tokens [key_begin, key_begin + key_len), cut into blocks of block_k from key_begin on (the whole
// sequence for plain selection; one part of the block that holds the prefill boundary otherwise).
struct PoolArgs {
  TensorArg q, k;
  const float* lse;        // [B, Hq, L] natural-log sum-exp of each row over ALL L keys
  float* apool;            // [B, Hq, nqb, out_stride]; block t of the range lands in column out_col0 + t
  int32_t B, Hq, Hkv, L;
  const int32_t* seq_lens; // optional [B] per-sample lengths (only with the whole-sequence key range)
  int32_t nqb, block_k;
  int32_t key_begin, key_len;
  int32_t out_stride, out_col0;
  float scale_log2;        // log2(e) / sqrt(D)
  // one-pass form only (pool1p_bf16_kernel; whole key range, lse unused):
  float* slab;             // scratch, one slab of block_q x slab_ld floats per work-group of the launch
  int32_t slab_ld;         // floats per slab row: the key-block count rounded up to a multiple of 16
  float* lse_out;          // optional [B, Hq, L]: receives the row log-sum-exp
};

// Arguments of the per-row top-k kernel (Eq. 6): one wavefront per pooled row.
struct TopkArgs {
  const float* apool;      // [rows, nkb]
  int32_t* row_ptr;        // [B*H, nqb + 1]
  int32_t* col_idx;        // [B*H, cap_per_head]
  int32_t rows, nqb, nkb;
  int32_t split;           // key blocks [0, split) and [split, nkb) are ranked separately
  int32_t keep_lo, keep_hi;  // kept in each range (keep_hi = 0 and split = nkb for one range)
  int32_t cap_per_head;
  // Prefill boundary inside key block `straddle` (else straddle < 0): that block enters the first range
  // with score part[2r] (its prefill keys) and the second with part[2r+1] (its generation keys); it is
  // listed once even if both keep it, so rows differ in length: entries go to rows_tmp [rows, keep_lo +
  // keep_hi] and counts [rows], and compact_kernel builds the CSR from them.
  // Per-sample lengths (optional): sample b ranks the key blocks it has, ceil(len/block_k) of them, with its own
  // counts kept_blocks(rho, size of each of its ranges), and its query blocks past ceil(len/block_q) get empty rows.
  const int32_t* seq_lens;
  int32_t heads_per_batch, block_q, block_k, L;
  double rho;
  int32_t straddle;
  int32_t boundary;        // the boundary's key token (only with straddle >= 0)
  const float* part;
  int32_t* rows_tmp;
  int32_t* counts;
};

// Builds row_ptr / col_idx of every head from fixed-stride rows and their lengths.
struct CompactArgs {
  const int32_t* rows_tmp;  // [heads * nqb, stride]
  const int32_t* counts;    // [heads * nqb]
  int32_t* row_ptr;         // [heads, nqb + 1]
  int32_t* col_idx;         // [heads, cap_per_head]
  int32_t heads, nqb, stride, cap_per_head;
};

struct ValidateArgs {
  const int32_t* row_ptr;
  const int32_t* col_idx;
  int32_t rows, nqb, nkb, cap_per_head;
  int32_t* bad;            // device counter of malformed rows
};

// Arguments of the fixed-pattern index builder (sliding window + attention sinks).
struct WindowArgs {
  int32_t* row_ptr;
  int32_t* col_idx;
  int32_t heads, nqb, nkb, block_q, block_k, L, cap_per_head;
  int32_t half_window;  // tokens on either side of a query that stay visible
  int32_t sink_blocks;  // leading key blocks that are always visible
};

enum class Mode : int { kDense = 0, kSparse = 1, kStats = 2 };

// Launchers. Each returns the HIP error of the launch. block_q selects the work-group shape for
// the sparse and pooled kernels; dense and stats pick their own query tile from L.
hipError_t launch_attn_bf16(Mode mode, int D, int block_q, AttnArgs a, hipStream_t s);
hipError_t launch_attn_f32(Mode mode, int D, int block_q, AttnArgs a, hipStream_t s);
// bf16 sparse attention for query blocks of 32 or 64 rows (two waves per 32 rows, keys of a tile split between them)
hipError_t launch_attn_bf16_splitk(int D, int block_q, const AttnArgs& a, hipStream_t s);
hipError_t launch_pool_bf16(int D, int block_q, const PoolArgs& a, hipStream_t s);
hipError_t launch_pool_f32(int D, int block_q, const PoolArgs& a, hipStream_t s);
// Pooled scores of bf16 inputs in one pass over the keys (no row statistics needed): `groups` persistent work-groups,
// each with its own slab in a.slab. pool1p_groups: the number of work-groups that fills the chip for this block_q.
hipError_t launch_pool1p_bf16(int D, int block_q, const PoolArgs& a, int groups, hipStream_t s);
int pool1p_groups(int block_q);
// Units of work of that launch: runs of 128 consecutive rows of one head (one, two or four query blocks).
int64_t pool1p_units(int B, int Hq, int nqb, int block_q);
hipError_t launch_topk(const TopkArgs& a, hipStream_t s);
hipError_t launch_compact(const CompactArgs& a, hipStream_t s);
hipError_t launch_validate(const ValidateArgs& a, hipStream_t s);
hipError_t launch_window_index(const WindowArgs& a, hipStream_t s);
// Row I of the window + sink pattern as two disjoint ascending runs of key blocks: the sink blocks
// [0, *sink_end) and the window blocks [*first, *last] that are not sinks already (empty if *first > *last).
// Shared by the host-side sizing and the kernel.
__host__ __device__ inline void window_row_runs(int I, int block_q, int block_k, int L, int half_window, int sink_blocks,
                                                int* sink_end, int* first, int* last) {
  long lo = (long)I * block_q - half_window, hi = (long)(I + 1) * block_q - 1 + half_window;
  if (lo < 0) lo = 0;
  if (hi > L - 1) hi = L - 1;
  const int nkb = (L + block_k - 1) / block_k;
  *sink_end = sink_blocks < nkb ? sink_blocks : nkb;
  *first = (int)(lo / block_k);
  *last = (int)(hi / block_k);
  if (*first < *sink_end) *first = *sink_end;
}
__host__ __device__ inline int window_row_length(int I, int block_q, int block_k, int L, int half_window, int sink_blocks) {
  int sink_end, first, last;
  window_row_runs(I, block_q, block_k, L, half_window, sink_blocks, &sink_end, &first, &last);
  return sink_end + (last >= first ? last - first + 1 : 0);
}
// Matrix-core rate probe: kProbeGroups work-groups x 8 waves, each wave issues 32 MFMAs per iteration.
constexpr int kProbeGroups = 256;
constexpr int kProbeFloats = kProbeGroups * 512;
hipError_t launch_mfma_rate(float* scratch, int iters, int random_operands, hipStream_t s);
// Vector-unit rate probe, same launch shape: each wave issues 64 fp32 instructions per iteration (op 0: fma, 1: exp2).
hipError_t launch_valu_rate(float* scratch, int iters, int op, hipStream_t s);
// Matrix instructions together with vector_per_mfma (0, 2, 3, 4, 5, 6 or 8) vector instructions each, a quarter of them
// exp2, and optionally one LDS operand read each; same launch shape and matrix work as launch_mfma_rate.
hipError_t launch_mix_rate(float* scratch, int iters, int vector_per_mfma, int lds_operands, hipStream_t s);

// Rows per work-group the dense / stats kernels use for this L (0 if L is unsupported).
int dense_qtile_bf16(int L);
int dense_qtile_f32(int L);

}  // namespace sparsed
