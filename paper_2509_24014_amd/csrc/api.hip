// Host side of the C ABI declared in include/sparsed.h: argument validation, the "top rho%"
// count, workspace carving and kernel dispatch. No arithmetic of the method happens here.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "../../include/sparsed.h"
#include "../../include/sparsed_diag.h"
#include "kernels.hpp"

using namespace sparsed;

namespace {

thread_local char g_err[512] = "";

sparsed_status fail(sparsed_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

sparsed_status hip_fail(hipError_t e, const char* what) {
  return fail(SPARSED_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

hipStream_t stream_of(const sparsed_exec* ex) { return ex ? static_cast<hipStream_t>(ex->stream) : nullptr; }

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

int elem_align(int dtype) { return dtype == SPARSED_BF16 ? 8 : 4; }  // elements per 16 bytes

sparsed_status check_tensor(const sparsed_tensor* t, const char* name) {
  if (!t) return fail(SPARSED_ERR_NULL, "%s is NULL", name);
  if (!t->data) return fail(SPARSED_ERR_NULL, "%s.data is NULL", name);
  if (t->dtype != SPARSED_BF16 && t->dtype != SPARSED_F32) return fail(SPARSED_ERR_DTYPE, "%s: unknown dtype %d", name, t->dtype);
  if (t->B <= 0 || t->H <= 0 || t->L <= 0 || t->D <= 0)
    return fail(SPARSED_ERR_SHAPE, "%s: non-positive dimension [%d,%d,%d,%d]", name, t->B, t->H, t->L, t->D);
  if (t->D != 64 && t->D != 128) return fail(SPARSED_ERR_UNSUPPORTED, "%s: head dim %d not in {64,128}", name, t->D);
  const int al = elem_align(t->dtype);
  if (reinterpret_cast<uintptr_t>(t->data) % 16 != 0) return fail(SPARSED_ERR_STRIDE, "%s.data is not 16-byte aligned", name);
  if (t->stride_l < t->D || t->stride_l % al || t->stride_h % al || t->stride_b % al || t->stride_h < 0 || t->stride_b < 0)
    return fail(SPARSED_ERR_STRIDE, "%s: strides (%lld,%lld,%lld) must be multiples of %d elements and stride_l >= D", name,
                (long long)t->stride_b, (long long)t->stride_h, (long long)t->stride_l, al);
  // one (batch, head) slab is addressed with 32-bit byte offsets inside the kernels
  const int64_t slab_bytes = ((int64_t)(t->L - 1) * t->stride_l + t->D) * (t->dtype == SPARSED_BF16 ? 2 : 4);
  if (slab_bytes >= ((int64_t)1 << 31))
    return fail(SPARSED_ERR_STRIDE, "%s: one (batch, head) slab spans %lld bytes, the limit is 2^31", name, (long long)slab_bytes);
  return SPARSED_OK;
}

// q: [B,Hq,L,D]; k (and v): [B,Hkv,L,D]; same dtype; Hq % Hkv == 0.
sparsed_status check_qk(const sparsed_tensor* q, const sparsed_tensor* k, const char* kname) {
  if (q->dtype != k->dtype) return fail(SPARSED_ERR_DTYPE, "q and %s have different dtypes", kname);
  if (q->B != k->B || q->L != k->L || q->D != k->D)
    return fail(SPARSED_ERR_SHAPE, "q [%d,%d,%d,%d] and %s [%d,%d,%d,%d] disagree", q->B, q->H, q->L, q->D, kname, k->B,
                k->H, k->L, k->D);
  if (q->H % k->H != 0) return fail(SPARSED_ERR_SHAPE, "query heads %d not a multiple of %s heads %d", q->H, kname, k->H);
  return SPARSED_OK;
}

sparsed_status check_out(const sparsed_tensor* q, const sparsed_tensor* out) {
  if (out->dtype != q->dtype) return fail(SPARSED_ERR_DTYPE, "out and q have different dtypes");
  if (out->B != q->B || out->H != q->H || out->L != q->L || out->D != q->D) return fail(SPARSED_ERR_SHAPE, "out shape differs from q");
  return SPARSED_OK;
}

sparsed_status check_blocks(const sparsed_tensor* q, int bq, int bk) {
  if (bq != 32 && bq != 64 && bq != 128) return fail(SPARSED_ERR_UNSUPPORTED, "block_q %d not in {32,64,128}", bq);
  if (bk != 32 && bk != 64 && bk != 128) return fail(SPARSED_ERR_UNSUPPORTED, "block_k %d not in {32,64,128}", bk);
  return SPARSED_OK;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

sparsed_status check_index_shape(const sparsed_block_index* ix, const sparsed_tensor* q) {
  if (!ix) return fail(SPARSED_ERR_NULL, "block index is NULL");
  if (!ix->row_ptr || !ix->col_idx) return fail(SPARSED_ERR_NULL, "block index row_ptr / col_idx is NULL");
  if (ix->block_q <= 0 || ix->block_k <= 0) return fail(SPARSED_ERR_INDEX, "block index has non-positive block sizes");
  if (ix->B != q->B || ix->H != q->H || ix->nqb != ceil_div(q->L, ix->block_q) || ix->nkb != ceil_div(q->L, ix->block_k))
    return fail(SPARSED_ERR_INDEX, "block index [B=%d,H=%d,nqb=%d,nkb=%d,%dx%d] does not describe q [%d,%d,%d,%d]", ix->B, ix->H,
                ix->nqb, ix->nkb, ix->block_q, ix->block_k, q->B, q->H, q->L, q->D);
  if (ix->cap_per_head < 0) return fail(SPARSED_ERR_INDEX, "negative cap_per_head");
  return SPARSED_OK;
}

TensorArg targ(const sparsed_tensor* t) { return TensorArg{t->data, t->stride_b, t->stride_h, t->stride_l}; }

float scale_log2(int D) { return (float)(1.4426950408889634 / std::sqrt((double)D)); }

// The caller's workspace, checked: present, large enough, 256-byte aligned.
sparsed_status caller_workspace(const sparsed_exec* ex, size_t need, const char* what, char** out) {
  if (!ex || !ex->workspace) return fail(SPARSED_ERR_WORKSPACE, "%s needs ex->workspace (%zu bytes)", what, need);
  if (ex->workspace_bytes < need) return fail(SPARSED_ERR_WORKSPACE, "%s: workspace %zu bytes < %zu needed", what, ex->workspace_bytes, need);
  if (reinterpret_cast<uintptr_t>(ex->workspace) % 256) return fail(SPARSED_ERR_WORKSPACE, "%s: workspace is not 256-byte aligned", what);
  *out = static_cast<char*>(ex->workspace);
  return SPARSED_OK;
}

// Scratch of the allocation-free selection entry point: a fixed-size array inside the library's code
// object, one copy per GPU at its own address, held until the process ends. Host code never uses the
// array's name as an address: fixed_scratch() asks the runtime for the device address once per device
// (with that device current) and hands that pointer to the kernels like any caller's workspace.
constexpr size_t kFixedScratchBytes = SPARSED_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kFixedScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
char* g_scratch_ptr[kMaxDevices] = {};

sparsed_status fixed_scratch(char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(SPARSED_ERR_HIP, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p || reinterpret_cast<uintptr_t>(p) % 256) return fail(SPARSED_ERR_HIP, "built-in scratch buffer has no usable device address");
    g_scratch_ptr[dev] = static_cast<char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return SPARSED_OK;
}

size_t select_ws_bytes(int B, int Hq, int L, int nqb, int nkb) {
  return align256((size_t)B * Hq * L * sizeof(float)) + align256((size_t)B * Hq * nqb * nkb * sizeof(float));
}

// Scratch of the one-pass pooled-score kernel (bf16 inputs without a handed-over log-sum-exp): one slab of
// block_q x (key blocks rounded up to 16) floats per persistent work-group.
int onepass_slab_ld(int nkb) { return (nkb + 15) & ~15; }
// (a slab holds the 128 rows of a work-group whatever the query-block size)
size_t onepass_slab_bytes(int nkb) { return align256((size_t)128 * onepass_slab_ld(nkb) * sizeof(float)); }
constexpr int kOnepassMinGroups = 256;  // fewer slabs than compute units (and than pooled rows): the two-pass form is used instead

// Extra scratch when the prefill boundary falls inside a key block: the two partial scores of that
// block per pooled row, fixed-stride rows of kept blocks (at most nkb + 1 each) and their lengths.
size_t select_tokens_extra_bytes(int B, int Hq, int nqb, int nkb) {
  const size_t rows = (size_t)B * Hq * nqb;
  return align256(rows * 2 * sizeof(float)) + align256(rows * (size_t)(nkb + 1) * sizeof(int32_t)) + align256(rows * sizeof(int32_t));
}

sparsed_status attention(Mode mode, const sparsed_tensor* q, const sparsed_tensor* k, const sparsed_tensor* v,
                         const sparsed_block_index* ix, sparsed_tensor* out, const sparsed_exec* ex) {
  sparsed_status st;
  if ((st = check_tensor(q, "q")) || (st = check_tensor(k, "k")) || (st = check_tensor(v, "v")) || (st = check_tensor(out, "out")))
    return st;
  if ((st = check_qk(q, k, "k")) || (st = check_qk(q, v, "v")) || (st = check_out(q, out))) return st;
  if (k->H != v->H) return fail(SPARSED_ERR_SHAPE, "k has %d heads, v has %d", k->H, v->H);
  AttnArgs a{};
  a.q = targ(q);
  a.k = targ(k);
  a.v = targ(v);
  a.o = out->data;
  a.o_sb = out->stride_b;
  a.o_sh = out->stride_h;
  a.o_sl = out->stride_l;
  a.lse = (mode == Mode::kDense && ex) ? ex->lse_out : nullptr;
  a.B = q->B;
  a.Hq = q->H;
  a.Hkv = k->H;
  a.L = q->L;
  a.seq_lens = ex ? ex->seq_lens : nullptr;
  a.scale_log2 = scale_log2(q->D);
  int block_q = 0;
  if (mode == Mode::kSparse) {
    if ((st = check_index_shape(ix, q))) return st;
    if ((st = check_blocks(q, ix->block_q, ix->block_k))) return st;
    a.row_ptr = ix->row_ptr;
    a.col_idx = ix->col_idx;
    a.nqb = ix->nqb;
    a.cap_per_head = ix->cap_per_head;
    a.block_k = ix->block_k;
    block_q = ix->block_q;
  }
  const hipError_t e = (q->dtype == SPARSED_BF16) ? launch_attn_bf16(mode, q->D, block_q, a, stream_of(ex))
                                                 : launch_attn_f32(mode, q->D, block_q, a, stream_of(ex));
  if (e != hipSuccess) return hip_fail(e, mode == Mode::kSparse ? "sparse attention launch" : "dense attention launch");
  return SPARSED_OK;
}

// boundary_token >= 0: isolated selection whose prefill / generation boundary is that key token and lies
// strictly inside a key block (prefill_blocks is then ignored).
sparsed_status select_impl(const sparsed_tensor* q, const sparsed_tensor* k, int32_t bq, int32_t bk, double rho,
                           int32_t prefill_blocks, bool isolated, sparsed_block_index* ix, const sparsed_exec* ex,
                           int32_t boundary_token = -1, char* fixed_scratch = nullptr, size_t fixed_scratch_bytes = 0) {
  sparsed_status st;
  if ((st = check_tensor(q, "q")) || (st = check_tensor(k, "k")) || (st = check_qk(q, k, "k"))) return st;
  if ((st = check_blocks(q, bq, bk))) return st;
  if (!(rho > 0.0) || !(rho <= 1.0)) return fail(SPARSED_ERR_RANGE, "rho %g outside (0, 1]", rho);
  if ((st = check_index_shape(ix, q))) return st;
  if (ix->block_q != bq || ix->block_k != bk) return fail(SPARSED_ERR_INDEX, "block index blocks %dx%d differ from %dx%d", ix->block_q, ix->block_k, bq, bk);
  const int nqb = ix->nqb, nkb = ix->nkb;
  const int32_t* seq_lens = ex ? ex->seq_lens : nullptr;
  if (nkb > 8192) return fail(SPARSED_ERR_UNSUPPORTED, "more than 8192 key blocks per row (%d)", nkb);
  int split = nkb, keep_lo, keep_hi = 0;
  const int straddle = boundary_token >= 0 ? boundary_token / bk : -1;  // the key block that holds the boundary
  if (straddle >= 0) {
    split = straddle + 1;  // ranked entries: blocks 0 .. straddle (its prefill part), then its generation part and the rest
    keep_lo = sparsed_kept_blocks(rho, split);
    keep_hi = sparsed_kept_blocks(rho, nkb - straddle);
  } else if (isolated) {
    if (prefill_blocks < 0 || prefill_blocks > nkb) return fail(SPARSED_ERR_RANGE, "prefill_blocks %d outside [0, %d]", prefill_blocks, nkb);
    split = prefill_blocks;
    keep_lo = sparsed_kept_blocks(rho, split);
    keep_hi = sparsed_kept_blocks(rho, nkb - split);
  } else {
    keep_lo = sparsed_kept_blocks(rho, nkb);
  }
  const int keep = keep_lo + keep_hi;
  // the ranking kernel stages one pooled row (and, with a boundary inside a block, its kept entries) in 64 KB of LDS
  if (straddle >= 0 && (int64_t)nkb + 1 + keep > 16384)
    return fail(SPARSED_ERR_UNSUPPORTED, "row of %d key blocks with %d kept entries does not fit the ranking kernel", nkb, keep);
  if ((int64_t)ix->cap_per_head < (int64_t)nqb * keep)
    return fail(SPARSED_ERR_INDEX, "cap_per_head %d < nqb*k = %lld", ix->cap_per_head, (long long)nqb * keep);

  const size_t lse_bytes = align256((size_t)q->B * q->H * q->L * sizeof(float));
  const size_t base_bytes = select_ws_bytes(q->B, q->H, q->L, nqb, nkb);
  const size_t need = base_bytes + (straddle >= 0 ? select_tokens_extra_bytes(q->B, q->H, nqb, nkb) : 0);
  char* ws = nullptr;
  if (fixed_scratch) {  // the allocation-free entry point: scratch of a fixed size that lives in the library's code object
    if (need > fixed_scratch_bytes)
      return fail(SPARSED_ERR_WORKSPACE, "selection needs %zu bytes of scratch, the built-in buffer holds %zu", need, fixed_scratch_bytes);
    ws = fixed_scratch;
  } else if ((st = caller_workspace(ex, need, "pattern selection", &ws))) {
    return st;
  }
  float* lse_buf = reinterpret_cast<float*>(ws);
  float* apool = (ex && ex->pooled_out) ? ex->pooled_out : reinterpret_cast<float*>(ws + lse_bytes);
  hipStream_t s = stream_of(ex);
  const bool bf16 = q->dtype == SPARSED_BF16;

  const float* lse = ex ? ex->lse_in : nullptr;
  PoolArgs p{};
  p.q = targ(q);
  p.k = targ(k);
  p.apool = apool;
  p.B = q->B;
  p.Hq = q->H;
  p.Hkv = k->H;
  p.L = q->L;
  p.seq_lens = seq_lens;
  p.nqb = nqb;
  p.block_k = bk;
  p.key_begin = 0;
  p.key_len = q->L;
  p.out_stride = nkb;
  p.out_col0 = 0;
  p.scale_log2 = scale_log2(q->D);
  hipError_t e = hipSuccess;
  const size_t rows_total = (size_t)pool1p_units(q->B, q->H, nqb, bq);  // units of the one-pass kernel: 128 rows of a head each
  // How many one-pass slabs the scratch behind `need` has room for.
  const size_t ws_bytes = fixed_scratch ? fixed_scratch_bytes : ex->workspace_bytes;
  const size_t slab_bytes = onepass_slab_bytes(nkb);
  size_t slabs = (ws_bytes - need) / slab_bytes;
  if (slabs > (size_t)pool1p_groups(bq)) slabs = (size_t)pool1p_groups(bq);
  if (slabs > rows_total) slabs = rows_total;
  const size_t slabs_needed = rows_total < (size_t)kOnepassMinGroups ? rows_total : (size_t)kOnepassMinGroups;
  if (!lse && bf16 && slabs >= slabs_needed) {
    // 1 + 2. no log-sum-exp handed over: pooled scores A' (and the row log-sum-exp) in one pass over the keys
    p.slab = reinterpret_cast<float*>(ws + need);
    p.slab_ld = onepass_slab_ld(nkb);
    p.lse_out = lse_buf;
    e = launch_pool1p_bf16(q->D, bq, p, (int)slabs, s);
    if (e != hipSuccess) return hip_fail(e, "one-pass pooled-score launch");
    lse = lse_buf;
    p.slab = nullptr;
    p.lse_out = nullptr;
  } else {
    // 1. row log-sum-exp of Eq. 1's logits, unless the caller passes the one attn_dense produced
    if (!lse) {
      AttnArgs a{};
      a.q = targ(q);
      a.k = targ(k);
      a.lse = lse_buf;
      a.B = q->B;
      a.Hq = q->H;
      a.Hkv = k->H;
      a.L = q->L;
      a.seq_lens = seq_lens;
      a.scale_log2 = scale_log2(q->D);
      e = bf16 ? launch_attn_bf16(Mode::kStats, q->D, 0, a, s) : launch_attn_f32(Mode::kStats, q->D, 0, a, s);
      if (e != hipSuccess) return hip_fail(e, "row statistics launch");
      lse = lse_buf;
    }
    // 2. pooled scores A'
    p.lse = lse;
    e = bf16 ? launch_pool_bf16(q->D, bq, p, s) : launch_pool_f32(q->D, bq, p, s);
    if (e != hipSuccess) return hip_fail(e, "pooled-score launch");
  }
  p.lse = lse;
  const size_t rows = (size_t)q->B * q->H * nqb;
  float* part = nullptr;
  int32_t *rows_tmp = nullptr, *counts = nullptr;
  if (straddle >= 0) {
    // the block that holds the boundary once more, pooled over its prefill keys and over its generation keys
    char* extra = ws + base_bytes;
    part = reinterpret_cast<float*>(extra);
    rows_tmp = reinterpret_cast<int32_t*>(extra + align256(rows * 2 * sizeof(float)));
    counts = reinterpret_cast<int32_t*>(extra + align256(rows * 2 * sizeof(float)) + align256(rows * (size_t)(nkb + 1) * sizeof(int32_t)));
    const int block_end = (straddle + 1) * bk < q->L ? (straddle + 1) * bk : q->L;
    PoolArgs pa = p;
    pa.apool = part;
    pa.out_stride = 2;
    pa.key_begin = straddle * bk;
    pa.key_len = boundary_token - straddle * bk;
    e = bf16 ? launch_pool_bf16(q->D, bq, pa, s) : launch_pool_f32(q->D, bq, pa, s);
    if (e != hipSuccess) return hip_fail(e, "pooled-score launch (prefill part of the boundary block)");
    pa.out_col0 = 1;
    pa.key_begin = boundary_token;
    pa.key_len = block_end - boundary_token;
    e = bf16 ? launch_pool_bf16(q->D, bq, pa, s) : launch_pool_f32(q->D, bq, pa, s);
    if (e != hipSuccess) return hip_fail(e, "pooled-score launch (generation part of the boundary block)");
  }
  // 3. per-row top-k into the CSR index
  TopkArgs t{};
  t.apool = apool;
  t.row_ptr = ix->row_ptr;
  t.col_idx = ix->col_idx;
  t.rows = q->B * q->H * nqb;
  t.nqb = nqb;
  t.nkb = nkb;
  t.split = split;
  t.keep_lo = keep_lo;
  t.keep_hi = keep_hi;
  t.cap_per_head = ix->cap_per_head;
  t.seq_lens = seq_lens;
  t.heads_per_batch = q->H;
  t.block_q = bq;
  t.block_k = bk;
  t.L = q->L;
  t.rho = rho;
  t.straddle = straddle;
  t.boundary = boundary_token;
  t.part = part;
  t.rows_tmp = rows_tmp;
  t.counts = counts;
  e = launch_topk(t, s);
  if (e != hipSuccess) return hip_fail(e, "top-k launch");
  if (straddle >= 0) {
    // rows differ in length (the boundary block may be kept by both ranges): build the CSR from the fixed-stride rows
    CompactArgs c{rows_tmp, counts, ix->row_ptr, ix->col_idx, q->B * q->H, nqb, keep, ix->cap_per_head};
    e = launch_compact(c, s);
    if (e != hipSuccess) return hip_fail(e, "index compaction launch");
  }
  return SPARSED_OK;
}

// The three machine probes share one shape: check the arguments, take 512 KiB of the caller's workspace, run a short
// warm-up launch and a timed launch of `iters` iterations on the stream, return the timed launch's milliseconds.
template <typename Launch>
sparsed_status timed_probe(int32_t iters, const sparsed_exec* ex, const char* what, float* ms_out, Launch launch) {
  if (iters <= 0 || iters > 1000000) return fail(SPARSED_ERR_RANGE, "iters must be in [1, 1000000]");
  char* scratch = nullptr;
  const sparsed_status st = caller_workspace(ex, (size_t)kProbeFloats * sizeof(float), what, &scratch);
  if (st != SPARSED_OK) return st;
  hipStream_t s = stream_of(ex);
  hipEvent_t t0 = nullptr, t1 = nullptr;
  hipError_t e = hipEventCreate(&t0);
  if (e == hipSuccess) e = hipEventCreate(&t1);
  if (e == hipSuccess) e = launch(reinterpret_cast<float*>(scratch), iters / 8 + 1, s);  // warm-up
  if (e == hipSuccess) e = hipEventRecord(t0, s);
  if (e == hipSuccess) e = launch(reinterpret_cast<float*>(scratch), iters, s);
  if (e == hipSuccess) e = hipEventRecord(t1, s);
  if (e == hipSuccess) e = hipEventSynchronize(t1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
  if (t0) (void)hipEventDestroy(t0);
  if (t1) (void)hipEventDestroy(t1);
  if (e != hipSuccess) return hip_fail(e, what);
  *ms_out = ms;
  return SPARSED_OK;
}

// matrix instructions of one probe launch: work-groups x waves x 32 per iteration, 2 * 32 * 32 * 16 FLOP each
double probe_flops(int32_t iters) { return (double)kProbeGroups * 8.0 * 32.0 * (double)iters * 2.0 * 32.0 * 32.0 * 16.0; }

}  // namespace

extern "C" {

sparsed_status sparsed_attn_dense(const sparsed_tensor* q, const sparsed_tensor* k, const sparsed_tensor* v, sparsed_tensor* out,
                                  const sparsed_exec* ex) {
  return attention(Mode::kDense, q, k, v, nullptr, out, ex);
}

sparsed_status sparsed_attn_sparse(const sparsed_tensor* q, const sparsed_tensor* k, const sparsed_tensor* v,
                                   const sparsed_block_index* block_index, sparsed_tensor* out, const sparsed_exec* ex) {
  if (!block_index) return fail(SPARSED_ERR_NULL, "block index is NULL");
  return attention(Mode::kSparse, q, k, v, block_index, out, ex);
}

sparsed_status sparsed_select_pattern(const sparsed_tensor* q, const sparsed_tensor* k, int32_t block_q, int32_t block_k, double rho,
                                      sparsed_block_index* out_block_index, const sparsed_exec* ex) {
  return select_impl(q, k, block_q, block_k, rho, 0, false, out_block_index, ex);
}

sparsed_status sparsed_select_pattern_static(const sparsed_tensor* q, const sparsed_tensor* k, int32_t block_q, int32_t block_k,
                                             double rho, sparsed_block_index* out_block_index, const sparsed_exec* ex) {
  char* ws = nullptr;
  const sparsed_status st = fixed_scratch(&ws);
  if (st != SPARSED_OK) return st;
  return select_impl(q, k, block_q, block_k, rho, 0, false, out_block_index, ex, -1, ws, kFixedScratchBytes);
}

sparsed_status sparsed_select_pattern_isolated(const sparsed_tensor* q, const sparsed_tensor* k, int32_t block_q, int32_t block_k,
                                               double rho, int32_t prefill_blocks, sparsed_block_index* out_block_index,
                                               const sparsed_exec* ex) {
  return select_impl(q, k, block_q, block_k, rho, prefill_blocks, true, out_block_index, ex);
}

sparsed_status sparsed_select_pattern_isolated_tokens(const sparsed_tensor* q, const sparsed_tensor* k, int32_t block_q,
                                                      int32_t block_k, double rho, int32_t prefill_tokens,
                                                      sparsed_block_index* out_block_index, const sparsed_exec* ex) {
  if (!q) return fail(SPARSED_ERR_NULL, "q is NULL");
  if (block_k <= 0) return fail(SPARSED_ERR_UNSUPPORTED, "block_k %d", block_k);
  if (prefill_tokens < 0 || prefill_tokens > q->L) return fail(SPARSED_ERR_RANGE, "prefill_tokens %d outside [0, %d]", prefill_tokens, q->L);
  if (prefill_tokens % block_k == 0 || prefill_tokens == q->L)  // on a block edge: the block form
    return select_impl(q, k, block_q, block_k, rho, ceil_div(prefill_tokens, block_k), true, out_block_index, ex);
  return select_impl(q, k, block_q, block_k, rho, 0, true, out_block_index, ex, prefill_tokens);
}

// slabs of the one-pass kernel, if these inputs can use it
size_t onepass_bytes(const sparsed_tensor* q, int32_t block_q, int32_t nkb) {
  if (q->dtype != SPARSED_BF16 || (block_q != 32 && block_q != 64 && block_q != 128)) return 0;
  return (size_t)pool1p_groups(block_q) * onepass_slab_bytes(nkb);
}

size_t sparsed_select_tokens_workspace_bytes(const sparsed_tensor* q, int32_t block_q, int32_t block_k) {
  if (!q || block_q <= 0 || block_k <= 0 || q->B <= 0 || q->H <= 0 || q->L <= 0) return 0;
  const int nqb = ceil_div(q->L, block_q), nkb = ceil_div(q->L, block_k);
  return select_ws_bytes(q->B, q->H, q->L, nqb, nkb) + select_tokens_extra_bytes(q->B, q->H, nqb, nkb) + onepass_bytes(q, block_q, nkb);
}

size_t sparsed_select_workspace_min_bytes(const sparsed_tensor* q, int32_t block_q, int32_t block_k) {
  if (!q || block_q <= 0 || block_k <= 0 || q->B <= 0 || q->H <= 0 || q->L <= 0) return 0;
  return select_ws_bytes(q->B, q->H, q->L, ceil_div(q->L, block_q), ceil_div(q->L, block_k));
}

int32_t sparsed_kept_blocks(double rho, int32_t n) {
  if (n <= 0) return 0;
  double x = std::ceil(rho * (double)n - 1e-9);
  if (!(x >= 1.0)) x = 1.0;
  if (x > (double)n) x = (double)n;
  return (int32_t)x;
}

int32_t sparsed_n_dense_steps(int32_t T, double skip) {
  if (T <= 0) return 0;
  double x = std::ceil((double)T * skip - 1e-9);
  if (!(x >= 1.0)) x = 1.0;
  if (x > (double)T) x = (double)T;
  return (int32_t)x;
}

size_t sparsed_select_workspace_bytes(const sparsed_tensor* q, int32_t block_q, int32_t block_k) {
  if (!q || block_q <= 0 || block_k <= 0 || q->B <= 0 || q->H <= 0 || q->L <= 0) return 0;
  return select_ws_bytes(q->B, q->H, q->L, ceil_div(q->L, block_q), ceil_div(q->L, block_k)) +
         onepass_bytes(q, block_q, ceil_div(q->L, block_k));
}

sparsed_status sparsed_index_validate(const sparsed_block_index* ix, const sparsed_exec* ex) {
  if (!ix) return fail(SPARSED_ERR_NULL, "block index is NULL");
  if (!ix->row_ptr || !ix->col_idx) return fail(SPARSED_ERR_NULL, "block index row_ptr / col_idx is NULL");
  if (ix->B <= 0 || ix->H <= 0 || ix->nqb <= 0 || ix->nkb <= 0 || ix->cap_per_head < 0)
    return fail(SPARSED_ERR_INDEX, "block index has non-positive dimensions");
  char* ws = nullptr;
  const sparsed_status st = caller_workspace(ex, 256, "index validation", &ws);
  if (st != SPARSED_OK) return st;
  hipStream_t s = stream_of(ex);
  int32_t* bad = reinterpret_cast<int32_t*>(ws);  // device counter of malformed rows
  int32_t host_bad = 0;
  hipError_t e = hipMemsetAsync(bad, 0, sizeof(int32_t), s);
  if (e == hipSuccess) {
    ValidateArgs a{ix->row_ptr, ix->col_idx, ix->B * ix->H * ix->nqb, ix->nqb, ix->nkb, ix->cap_per_head, bad};
    e = launch_validate(a, s);
  }
  if (e == hipSuccess) e = hipMemcpyAsync(&host_bad, bad, sizeof(int32_t), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return hip_fail(e, "index validation");
  if (host_bad != 0) return fail(SPARSED_ERR_INDEX, "%d malformed rows in the block index", host_bad);
  return SPARSED_OK;
}

sparsed_status sparsed_index_fill_window(sparsed_block_index* ix, int32_t seq_len, int32_t window_tokens, int32_t sink_tokens,
                                         const sparsed_exec* ex) {
  if (!ix) return fail(SPARSED_ERR_NULL, "block index is NULL");
  if (!ix->row_ptr || !ix->col_idx) return fail(SPARSED_ERR_NULL, "block index row_ptr / col_idx is NULL");
  if (ix->B <= 0 || ix->H <= 0 || ix->block_q <= 0 || ix->block_k <= 0 || seq_len <= 0 ||
      ix->nqb != ceil_div(seq_len, ix->block_q) || ix->nkb != ceil_div(seq_len, ix->block_k))
    return fail(SPARSED_ERR_INDEX, "block index does not describe a sequence of %d tokens", seq_len);
  if (window_tokens < 0 || sink_tokens < 0) return fail(SPARSED_ERR_RANGE, "negative window or sink length");
  WindowArgs a{};
  a.row_ptr = ix->row_ptr;
  a.col_idx = ix->col_idx;
  a.heads = ix->B * ix->H;
  a.nqb = ix->nqb;
  a.nkb = ix->nkb;
  a.block_q = ix->block_q;
  a.block_k = ix->block_k;
  a.L = seq_len;
  a.cap_per_head = ix->cap_per_head;
  a.half_window = window_tokens / 2;
  a.sink_blocks = (sink_tokens + ix->block_k - 1) / ix->block_k;
  int64_t total = 0;
  for (int I = 0; I < ix->nqb; ++I) total += window_row_length(I, a.block_q, a.block_k, a.L, a.half_window, a.sink_blocks);
  if (total > ix->cap_per_head) return fail(SPARSED_ERR_INDEX, "cap_per_head %d < %lld entries the pattern needs", ix->cap_per_head, (long long)total);
  const hipError_t e = launch_window_index(a, stream_of(ex));
  if (e != hipSuccess) return hip_fail(e, "window index launch");
  return SPARSED_OK;
}

int64_t sparsed_index_window_entries(int32_t seq_len, int32_t block_q, int32_t block_k, int32_t window_tokens, int32_t sink_tokens) {
  if (seq_len <= 0 || block_q <= 0 || block_k <= 0 || window_tokens < 0 || sink_tokens < 0) return -1;
  const int sink_blocks = (sink_tokens + block_k - 1) / block_k;
  int64_t total = 0;
  for (int I = 0; I < ceil_div(seq_len, block_q); ++I) total += window_row_length(I, block_q, block_k, seq_len, window_tokens / 2, sink_blocks);
  return total;
}

sparsed_status sparsed_probe_mfma_bf16(int32_t random_operands, int32_t iters, double* tflops_out, const sparsed_exec* ex) {
  if (!tflops_out) return fail(SPARSED_ERR_NULL, "tflops_out is NULL");
  float ms = 0.f;
  const sparsed_status st = timed_probe(iters, ex, "matrix-core rate probe", &ms, [&](float* scratch, int n, hipStream_t s) {
    return launch_mfma_rate(scratch, n, random_operands, s);
  });
  if (st != SPARSED_OK) return st;
  *tflops_out = ms > 0.f ? probe_flops(iters) / ((double)ms * 1e9) : 0.0;
  return SPARSED_OK;
}

sparsed_status sparsed_probe_valu_f32(int32_t op, int32_t iters, double* gops_out, const sparsed_exec* ex) {
  if (!gops_out) return fail(SPARSED_ERR_NULL, "gops_out is NULL");
  if (op != 0 && op != 1) return fail(SPARSED_ERR_RANGE, "op must be 0 (fma) or 1 (exp2)");
  float ms = 0.f;
  const sparsed_status st = timed_probe(iters, ex, "vector-unit rate probe", &ms, [&](float* scratch, int n, hipStream_t s) {
    return launch_valu_rate(scratch, n, op, s);
  });
  if (st != SPARSED_OK) return st;
  // work-groups x waves x lanes x instructions per iteration
  const double ops = (double)kProbeGroups * 8.0 * 64.0 * 64.0 * (double)iters;
  *gops_out = ms > 0.f ? ops / ((double)ms * 1e6) : 0.0;
  return SPARSED_OK;
}

sparsed_status sparsed_probe_mix_bf16(int32_t vector_per_mfma, int32_t lds_operands, int32_t iters, double* tflops_out,
                                      const sparsed_exec* ex) {
  if (!tflops_out) return fail(SPARSED_ERR_NULL, "tflops_out is NULL");
  const int v = vector_per_mfma;
  if (!(v == 0 || v == 2 || v == 3 || v == 4 || v == 5 || v == 6 || v == 8))
    return fail(SPARSED_ERR_RANGE, "vector_per_mfma must be one of 0, 2, 3, 4, 5, 6, 8");
  float ms = 0.f;
  const sparsed_status st = timed_probe(iters, ex, "instruction-mix rate probe", &ms, [&](float* scratch, int n, hipStream_t s) {
    return launch_mix_rate(scratch, n, v, lds_operands != 0, s);
  });
  if (st != SPARSED_OK) return st;
  *tflops_out = ms > 0.f ? probe_flops(iters) / ((double)ms * 1e9) : 0.0;
  return SPARSED_OK;
}

const char* sparsed_status_string(sparsed_status s) {
  switch (s) {
    case SPARSED_OK: return "ok";
    case SPARSED_ERR_NULL: return "null pointer";
    case SPARSED_ERR_SHAPE: return "shape mismatch";
    case SPARSED_ERR_DTYPE: return "dtype mismatch";
    case SPARSED_ERR_STRIDE: return "bad stride or alignment";
    case SPARSED_ERR_RANGE: return "argument out of range";
    case SPARSED_ERR_UNSUPPORTED: return "unsupported configuration";
    case SPARSED_ERR_WORKSPACE: return "workspace missing or too small";
    case SPARSED_ERR_INDEX: return "malformed block index";
    case SPARSED_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

const char* sparsed_last_error(void) { return g_err; }

int32_t sparsed_version(void) { return 100; }

}  // extern "C"
