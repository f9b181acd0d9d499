// Pattern selection for gfx950 (Section 3.3; Algorithm 1's per-query-block loop; Eq. 6):
//   pool_*_kernel  A'[I, J] = mean over the block_q x block_k rectangle of the softmax
//                  probabilities of Eq. 1 (every row normalised over all L keys, via the row
//                  log-sum-exp computed by the statistics pass). One work-group per query block
//                  walks all key tiles once; the L x L matrix never exists.
//   topk_kernel    per pooled row, the k largest entries (ties: lower block index), written
//                  ascending into the per-head CSR block index. One wavefront per row.
// Pooled scores are fp32 from the logits on: the exponentials, the normaliser and every partial
// sum, with a fixed summation order (lane, then wave tree, then waves in order).
#include "kernels.hpp"
#include "tile_bf16.hpp"
#include "tile_f32.hpp"

namespace sparsed {

// ---------------------------------------------------------------------------- pooled scores, bf16
// Sum of one value per lane over the 64 lanes of a wave with DPP row operations (no LDS traffic);
// the total ends up in lane 63.
__device__ __forceinline__ float wave_sum_to_last_lane(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x111, 0xf, 0xf, true));  // row_shr:1
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x112, 0xf, 0xf, true));  // row_shr:2
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x114, 0xf, 0xf, true));  // row_shr:4
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x118, 0xf, 0xf, true));  // row_shr:8
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x142, 0xa, 0xf, true));  // row_bcast:15
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x143, 0xc, 0xf, true));  // row_bcast:31
  return x;
}

// One work-group of NW waves, 32 query rows each, covers NW / QBW consecutive query blocks of QBW waves (one block
// of 128 rows, two of 64 or four of 32 with NW = 4: small query blocks share the work-group's K tiles and keep four
// waves on every SIMD). Same 32-key software pipeline as
// the attention kernels: sub-step u interleaves the matrix work S(u+1) = K(u+1) Q^T with the vector
// work of sub-tile u (p = 2^(s*c - lse), summed per lane). A key block is two sub-tiles; its
// per-lane sums are reduced over the wave, then over the waves of its query block through LDS in a fixed order.
// HALF: key blocks of 32 (the two 32-key sub-tiles of a tile are pooled separately).
template <int D, int NW, bool HALF, int QBW = NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NW >= 4 ? 4 : NW >= 2 ? 2 : 1, NW >= 4 ? 4 : NW >= 2 ? 2 : 1)))
void pool_bf16_kernel(const PoolArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (the body uses device-only types)
  constexpr int NT = NW * 64;
  constexpr int kKBytes = KLayout<D>::kTileBytes;
  __shared__ __attribute__((aligned(1024))) char kbuf0[kKBytes];
  __shared__ __attribute__((aligned(1024))) char kbuf1[kKBytes];
  __shared__ float wsum[2][NW];
  __shared__ float wsum_even[2][NW];  // HALF only: the even sub-tile's sums (wsum then holds the odd one's)

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 31;
  static_assert(NW % QBW == 0, "whole query blocks per work-group");
  constexpr int kBlocksPerGroup = NW / QBW, kBlockRows = 32 * QBW;
  const int lid = xcd_remap(blockIdx.x, gridDim.x);
  const int groups_per_head = (a.nqb + kBlocksPerGroup - 1) / kBlocksPerGroup;
  const int gq = lid % groups_per_head;  // which run of 32 * NW rows of the head
  const int bh = lid / groups_per_head;
  const int b = bh / a.Hq, h = bh % a.Hq;
  const int hk = h / (a.Hq / a.Hkv);
  const int first_wave = (wave / QBW) * QBW;            // first wave of this wave's query block
  const int I = gq * kBlocksPerGroup + wave / QBW;      // this wave's query block

  // length of this batch element (per-sample lengths shorten the whole-sequence key range with it)
  int L = a.L, key_len = a.key_len;
  if (a.seq_lens != nullptr) {
    const int len = a.seq_lens[b];
    L = len < a.L ? len : a.L;
    key_len = L - a.key_begin < key_len ? L - a.key_begin : key_len;
  }
  if (gq * (32 * NW) >= L || key_len <= 0) return;  // uniform over the work-group
  const __bf16* qbase = static_cast<const __bf16*>(a.q.ptr) + b * a.q.sb + h * a.q.sh;
  const __bf16* kbase = static_cast<const __bf16*>(a.k.ptr) + b * a.k.sb + hk * a.k.sh + (int64_t)a.key_begin * a.k.sl;
  const int row0 = gq * (32 * NW) + wave * 32;
  // a query block of the group that the head (or this sample) does not have: its waves run along with all-zero terms
  const bool block_exists = I < a.nqb && I * kBlockRows < L;

  QFrag<D, 1> qf;
  qf.load(qbase, row0, L, a.q.sl, lane);
  // a query row past L (partial last query block) gets an infinite normaliser: all its terms are 0
  const float lse2 = (row0 + j < L) ? a.lse[(int64_t)bh * a.L + row0 + j] * 1.4426950408889634f : __builtin_inff();
  float* arow = a.apool + ((int64_t)bh * a.nqb + I) * a.out_stride + a.out_col0;
  const int rows_here = (L - I * kBlockRows < kBlockRows) ? L - I * kBlockRows : kBlockRows;  // query rows of the block that exist
  const int last_blk = (key_len - 1) / kTileK;
  const int tail_keys = key_len - last_blk * kTileK;  // keys that exist in the last key block of the range
  auto keys_of = [&](int blk) -> int { return blk == last_blk ? tail_keys : kTileK; };

  TileDma<D, NT, false> kdma;
  kdma.init(a.k.sl, wave, lane);
  KFragAddr<D> kaddr;
  kaddr.init(lane);
  const __amdgpu_buffer_rsrc_t krsrc = make_rsrc(kbase, ((int64_t)(key_len - 1) * a.k.sl + D) * 2);
  const int32_t k_tile_bytes = (int32_t)(kTileK * a.k.sl * 2);
  const int n = last_blk + 1;
  const float c = a.scale_log2;

  auto copy_k_any = [&](int tile, char* dst) {  // any tile: past the end repeats the last one, which may be partial
    const int blk = tile < n ? tile : n - 1;
    if (blk == last_blk && tail_keys < kTileK) kdma.issue_partial(krsrc, blk * k_tile_bytes, dst, wave, lane, a.k.sl, tail_keys);
    else kdma.issue(krsrc, blk * k_tile_bytes, dst, wave);
  };
  auto keys_at = [&](int tile) -> int { return tile < n ? keys_of(tile) : 0; };  // keys that exist in a tile (none in a phantom)
  f32x16 s_even[1], s_odd[1];
  float carry = 0.f;  // per-lane sum of the even sub-tile of the key block in progress
  const int g = lane >> 5;
  // masked: apply `valid`, the number of keys of the sub-tile that exist (>= 32: all, <= 0: none)
  auto expsum_sub = [&](f32x16(&s)[1], const bool masked, int valid) -> float {
    if (masked) {
      const int mine = valid - 8 * g;  // register x of lane (j, g) holds key 16*(x/8) + 8*g + x%8
#pragma unroll
      for (int x = 0; x < 16; ++x)
        if (16 * (x >> 3) + (x & 7) >= mine) s[0][x] = -__builtin_inff();
    }
    float part = 0.f;
#pragma unroll
    for (int x = 0; x < 16; ++x) part += __builtin_amdgcn_exp2f(__builtin_fmaf(s[0][x], c, -lse2));
    asm volatile("" : "+v"(part));  // keep the vector work inside the block that holds the matrix work
    return part;
  };
  const int tile_shift = a.block_k == 2 * kTileK ? 1 : 0;  // a 128-key block is pooled over two consecutive tiles
  float block_acc = 0.f;                                   // first thread of a query block: sum over the tiles of the key block in progress
  auto flush_block = [&](int t, float part) {  // after the tile barrier: key tile t is complete
    (void)part;
    if (tid == first_wave * 64 && block_exists) {
      if (HALF) {  // two 32-key blocks per tile; the second may not exist in the last tile
        float ev = 0.f, od = 0.f;
#pragma unroll
        for (int w = 0; w < QBW; ++w) {
          ev += wsum_even[t & 1][first_wave + w];
          od += wsum[t & 1][first_wave + w];
        }
        const int left = key_len - t * kTileK;  // keys from this tile's first on
        arow[2 * t] = ev * (1.0f / (float)(rows_here * (left < 32 ? left : 32)));
        if (left > 32) arow[2 * t + 1] = od * (1.0f / (float)(rows_here * (left - 32 < 32 ? left - 32 : 32)));
        return;
      }
      float tot = block_acc;
#pragma unroll
      for (int w = 0; w < QBW; ++w) tot += wsum[t & 1][first_wave + w];
      if ((t & tile_shift) == tile_shift || t == n - 1) {  // last tile of its key block
        const int J = t >> tile_shift;
        const int keys_here = key_len - J * a.block_k < a.block_k ? key_len - J * a.block_k : a.block_k;
        arow[J] = tot * (1.0f / (float)(rows_here * keys_here));  // mean over the entries that exist
        tot = 0.f;
      }
      block_acc = tot;
    }
  };

  // Tile step t (LDS parity P = t & 1) = sub-steps 2t+1 and 2t+2. On entry S(2t+1) is in s_odd, the
  // per-lane sum of sub-tile 2t in `carry`, K(t+1) in kbuf[1-P]; kbuf[P] is free and receives K(t+2).
  // Tiles past the end of the range are phantoms (a repeated copy, every key masked), so one branch-free
  // step serves the whole range; MASKED steps (the last few) count the keys that exist in each sub-tile.
#define SPARSED_POOL_STEP(P, MASKED, T)                                                            \
  {                                                                                                \
    char* const kb_free = (P) ? kbuf1 : kbuf0;                                                     \
    char* const kb_next = (P) ? kbuf0 : kbuf1;                                                     \
    if (MASKED) copy_k_any((T) + 2, kb_free);                                                      \
    else kdma.issue(krsrc, ((T) + 2 < n ? (T) + 2 : n - 1) * k_tile_bytes, kb_free, wave);         \
    logits_sub<D, 1, false>(kb_next, 0, kaddr, qf, s_even);                                        \
    float part = (HALF ? 0.f : carry) + expsum_sub(s_odd, (MASKED), keys_at(T) - 32);              \
    sched_substep_interleave<D, 1, false>();                                                       \
    part = wave_sum_to_last_lane(part);                                                            \
    if (lane == 63) wsum[(P)][wave] = part;                                                        \
    if (HALF) {                                                                                    \
      const float ev = wave_sum_to_last_lane(carry);                                               \
      if (lane == 63) wsum_even[(P)][wave] = ev;                                                   \
    }                                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                                             \
    logits_sub<D, 1, false>(kb_next, 1, kaddr, qf, s_odd);                                         \
    carry = expsum_sub(s_even, (MASKED), keys_at((T) + 1));                                        \
    sched_substep_interleave<D, 1, false>();                                                       \
    __syncthreads();                                                                               \
    flush_block((T), part);                                                                        \
  }

  // prologue: K(0), K(1) (a repeat of K(0) for a one-tile range) into LDS; S(0); the sums of sub-tile 0
  copy_k_any(0, kbuf0);
  copy_k_any(1, kbuf1);
  __syncthreads();
  logits_sub<D, 1, true>(kbuf0, 0, kaddr, qf, s_even);
  logits_sub<D, 1, true>(kbuf0, 1, kaddr, qf, s_odd);
  carry = expsum_sub(s_even, true, keys_at(0));
  __syncthreads();  // everyone is done with K(0) before tile step 0 lets K(2) overwrite it

  // an unmasked step at tile t touches tiles t, t+1 (sums) and t+2 (copy, possibly a repeat); a partial last
  // block must stay out of its reach on all three counts, a full one only as far as t+1
  const int steady_reach = (tail_keys < kTileK) ? 4 : 2;
  int t = 0;
  while (t + steady_reach < n) {
    SPARSED_POOL_STEP(0, false, t);
    SPARSED_POOL_STEP(1, false, t + 1);
    t += 2;
  }
  for (; t < n; ++t) {
    if (t & 1) {
      SPARSED_POOL_STEP(1, true, t);
    } else {
      SPARSED_POOL_STEP(0, true, t);
    }
  }
#undef SPARSED_POOL_STEP
#endif
}

// ---------------------------------------------------------------------------- pooled scores, fp32
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void pool_f32_kernel(const PoolArgs a) {
  constexpr int NT = NW * 64;
  using T = TileF32<D>;
  __shared__ __attribute__((aligned(16))) float klds[T::kKFloats];
  __shared__ float wsum[NW];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31;
  const int lid = xcd_remap_f(blockIdx.x, gridDim.x);
  const int I = lid % a.nqb;
  const int bh = lid / a.nqb;
  const int b = bh / a.Hq, h = bh % a.Hq;
  const int hk = h / (a.Hq / a.Hkv);

  int L = a.L, key_len = a.key_len;  // length of this batch element
  if (a.seq_lens != nullptr) {
    const int len = a.seq_lens[b];
    L = len < a.L ? len : a.L;
    key_len = L - a.key_begin < key_len ? L - a.key_begin : key_len;
  }
  if (I * (32 * NW) >= L || key_len <= 0) return;  // uniform over the work-group
  const float* qbase = static_cast<const float*>(a.q.ptr) + b * a.q.sb + h * a.q.sh;
  const float* kbase = static_cast<const float*>(a.k.ptr) + b * a.k.sb + hk * a.k.sh + (int64_t)a.key_begin * a.k.sl;
  const int row0 = I * (32 * NW) + wave * 32;

  QFragF32<D> qf;
  qf.load(qbase, row0, L, a.q.sl, lane);
  // a query row past L (partial last query block) gets an infinite normaliser: all its terms are 0
  const float lse2 = (row0 + j < L) ? a.lse[(int64_t)bh * a.L + row0 + j] * 1.4426950408889634f : __builtin_inff();
  float* arow = a.apool + ((int64_t)bh * a.nqb + I) * a.out_stride + a.out_col0;
  const int rows_here = (L - I * (32 * NW) < 32 * NW) ? L - I * (32 * NW) : 32 * NW;  // query rows that exist
  const int g = lane >> 5;

  const int tiles_per_block = a.block_k / kTileKF;
  const int n_tiles = (key_len + kTileKF - 1) / kTileKF;
  const float c = a.scale_log2;
  float acc = 0.f;  // thread 0: running sum of the current key block
  for (int t = 0; t < n_tiles; ++t) {
    const int valid = key_len - t * kTileKF < kTileKF ? key_len - t * kTileKF : kTileKF;  // keys of this tile that exist (>= 1)
    __syncthreads();
    T::template stage<NT>(kbase + (int64_t)t * kTileKF * a.k.sl, a.k.sl, klds, T::kKStride, tid, valid);
    __syncthreads();
    f32x16 s = logits_tile_f32<D>(klds, qf, lane);
    if (valid < kTileKF) {
#pragma unroll
      for (int x = 0; x < 16; ++x)
        if (8 * (x / 4) + 4 * g + (x % 4) >= valid) s[x] = -__builtin_inff();
    }
    float part = 0.f;
#pragma unroll
    for (int x = 0; x < 16; ++x) part += exp2f(__builtin_fmaf(s[x], c, -lse2));
    part = wave_sum_f(part);
    if (lane == 0) wsum[wave] = part;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
      for (int w = 0; w < NW; ++w) acc += wsum[w];
      if ((t + 1) % tiles_per_block == 0 || t == n_tiles - 1) {  // key block complete (the last one may be partial)
        const int J = t / tiles_per_block;
        const int keys_here = key_len - J * a.block_k < a.block_k ? key_len - J * a.block_k : a.block_k;
        arow[J] = acc * (1.0f / (float)(rows_here * keys_here));  // mean over the entries that exist
        acc = 0.f;
      }
    }
  }
}

// ---------------------------------------------------------------------------- per-row top-k
// Scores are non-negative floats, so their bit patterns order like unsigned integers. For one
// range [lo, hi) of the row held in LDS: a bitwise radix descent finds the keep-th largest value T
// and how many entries equal to T are still needed; then one ascending sweep emits every entry
// above T plus the first `need` entries equal to T (lower block index wins ties).
__device__ __forceinline__ int emit_topk_range(const uint32_t* row, int lo, int hi, int keep,
                                               int32_t* out, int lane) {
  if (keep <= 0 || hi <= lo) return 0;
  uint32_t prefix = 0;
  int need = keep;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = (prefix >> bit) | 1u;
    int cnt = 0;
    for (int base = lo; base < hi; base += 64) {
      const int J = base + lane;
      const bool hit = (J < hi) && ((row[J < hi ? J : lo] >> bit) == cand);
      cnt += __builtin_popcountll(__ballot(hit));
    }
    if (cnt >= need)
      prefix |= (1u << bit);
    else
      need -= cnt;
  }
  const uint32_t T = prefix;
  const unsigned long long lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  int n_out = 0, eq_seen = 0;
  for (int base = lo; base < hi; base += 64) {
    const int J = base + lane;
    const uint32_t x = (J < hi) ? row[J] : 0u;
    const bool gt = (J < hi) && (x > T);
    const bool eq = (J < hi) && (x == T);
    const unsigned long long eq_mask = __ballot(eq);
    const int eq_rank = eq_seen + __builtin_popcountll(eq_mask & lt_mask);
    const bool take = gt || (eq && eq_rank < need);
    const unsigned long long take_mask = __ballot(take);
    if (take) out[n_out + __builtin_popcountll(take_mask & lt_mask)] = J;
    n_out += __builtin_popcountll(take_mask);
    eq_seen += __builtin_popcountll(eq_mask);
  }
  return n_out;
}

__global__ __launch_bounds__(64) void topk_kernel(const TopkArgs a) {
  extern __shared__ uint32_t row[];
  const int lane = threadIdx.x;
  const int r = blockIdx.x;
  if (r >= a.rows) return;
  const int bh = r / a.nqb, I = r % a.nqb;
  const uint32_t* src = reinterpret_cast<const uint32_t*>(a.apool) + (int64_t)r * a.nkb;
  const int keep = a.keep_lo + a.keep_hi;
  auto kept = [&](int nblocks) -> int {  // the host's count rule, in the same double arithmetic
    if (nblocks <= 0) return 0;
    double x = ceil(a.rho * (double)nblocks - 1e-9);
    if (!(x >= 1.0)) x = 1.0;
    if (x > (double)nblocks) x = (double)nblocks;
    return (int)x;
  };
  if (a.straddle >= 0) {
    // Prefill boundary at key token a.boundary, inside key block a.straddle. Rows differ in length, so they are
    // staged at a fixed stride (the host's keep_lo + keep_hi) with their lengths; compact_kernel builds the CSR.
    int L = a.L;  // length of this batch element
    if (a.seq_lens != nullptr) {
      const int len = a.seq_lens[bh / a.heads_per_batch];
      L = len < a.L ? len : a.L;
    }
    const int nkb_b = L > 0 ? (L + a.block_k - 1) / a.block_k : 0, nqb_b = L > 0 ? (L + a.block_q - 1) / a.block_q : 0;
    int32_t* tmp = a.rows_tmp + (int64_t)r * keep;
    if (I >= nqb_b) {  // a query block this sample does not have: an empty row
      if (lane == 0) a.counts[r] = 0;
      return;
    }
    if (L <= a.boundary) {
      // a sample no longer than the prefill: one range over the key blocks it has, none of them split
      for (int J = lane; J < nkb_b; J += 64) row[J] = src[J];
      __syncthreads();
      const int keep_b = kept(nkb_b);
      emit_topk_range(row, 0, nkb_b, keep_b, tmp, lane);
      if (lane == 0) a.counts[r] = keep_b;
      return;
    }
    // The ranked row has nkb_b + 1 entries: blocks before the one that holds the boundary, that block's
    // prefill part, its generation part, the blocks after it. Entries [0, Js] are the prefill range.
    const int Js = a.straddle, nv = nkb_b + 1;
    const int keep_lo = kept(Js + 1), keep_hi = kept(nkb_b - Js), keep_b = keep_lo + keep_hi;
    const uint32_t* part = reinterpret_cast<const uint32_t*>(a.part) + (int64_t)r * 2;
    for (int v = lane; v < nv; v += 64) row[v] = v < Js ? src[v] : v == Js ? part[0] : v == Js + 1 ? part[1] : src[v - 1];
    __syncthreads();
    int32_t* sel = reinterpret_cast<int32_t*>(row + nv);  // the kept entries of both ranges, still in LDS
    emit_topk_range(row, 0, Js + 1, keep_lo, sel, lane);
    emit_topk_range(row, Js + 1, nv, keep_hi, sel + keep_lo, lane);
    __syncthreads();
    // entries -> key blocks; the only possible duplicate is the boundary block, at the junction of the two ranges
    const bool dup = keep_lo > 0 && keep_hi > 0 && sel[keep_lo - 1] == Js && sel[keep_lo] == Js + 1;
    for (int t = lane; t < keep_b; t += 64) {
      if (dup && t == keep_lo) continue;
      const int v = sel[t];
      tmp[t - ((dup && t > keep_lo) ? 1 : 0)] = v > Js ? v - 1 : v;
    }
    if (lane == 0) a.counts[r] = keep_b - (dup ? 1 : 0);
    return;
  }
  if (a.seq_lens != nullptr) {
    // per-sample length: this sample ranks the key blocks it has and keeps its own "top rho%" of them
    const int len = a.seq_lens[bh / a.heads_per_batch];
    const int L = len < a.L ? len : a.L;
    const int nkb_b = L > 0 ? (L + a.block_k - 1) / a.block_k : 0, nqb_b = L > 0 ? (L + a.block_q - 1) / a.block_q : 0;
    // With a prefill / generation split (Eq. 5) the sample's two ranges are [0, split) and [split, nkb_b), the
    // first cut to the blocks the sample has; a sample no longer than the prefill has one range only.
    const int split_b = a.split < nkb_b ? a.split : nkb_b;
    const int keep_lo_b = kept(split_b), keep_hi_b = kept(nkb_b - split_b);
    const int keep_b = keep_lo_b + keep_hi_b;
    int32_t* rp = a.row_ptr + (int64_t)bh * (a.nqb + 1);
    if (I < nqb_b) {
      for (int J = lane; J < nkb_b; J += 64) row[J] = src[J];
      __syncthreads();
      int32_t* out_b = a.col_idx + (int64_t)bh * a.cap_per_head + (int64_t)I * keep_b;
      emit_topk_range(row, 0, split_b, keep_lo_b, out_b, lane);
      emit_topk_range(row, split_b, nkb_b, keep_hi_b, out_b + keep_lo_b, lane);
    }
    if (lane == 0) {
      rp[I] = (I < nqb_b ? I : nqb_b) * keep_b;  // query blocks the sample does not have get empty rows
      if (I == a.nqb - 1) rp[a.nqb] = nqb_b * keep_b;
    }
    return;
  }
  for (int J = lane; J < a.nkb; J += 64) row[J] = src[J];
  __syncthreads();

  int32_t* out = a.col_idx + (int64_t)bh * a.cap_per_head + (int64_t)I * keep;
  emit_topk_range(row, 0, a.split, a.keep_lo, out, lane);
  emit_topk_range(row, a.split, a.nkb, a.keep_hi, out + a.keep_lo, lane);
  if (lane == 0) {
    int32_t* rp = a.row_ptr + (int64_t)bh * (a.nqb + 1);
    rp[I] = I * keep;
    if (I == a.nqb - 1) rp[a.nqb] = a.nqb * keep;
  }
}

// Exclusive scan over the 256 threads of a work-group (each brings the sum of its own consecutive rows): returns
// this thread's offset, leaves the grand total in partial[255].
__device__ __forceinline__ int scan_256(int sum, int32_t (&partial)[256], int tid) {
  partial[tid] = sum;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {
    const int add = tid >= off ? partial[tid - off] : 0;
    __syncthreads();
    partial[tid] += add;
    __syncthreads();
  }
  return partial[tid] - sum;
}

// One work-group per head: exclusive scan of the row lengths into row_ptr, then the waves copy the rows to their
// places, a wave per row and a lane per entry.
__global__ __launch_bounds__(256) void compact_kernel(const CompactArgs a) {
  __shared__ int32_t partial[256];
  const int head = blockIdx.x, tid = threadIdx.x;
  const int per = (a.nqb + 255) / 256;  // consecutive rows per thread
  const int first = tid * per, last = first + per < a.nqb ? first + per : a.nqb;
  const int32_t* counts = a.counts + (int64_t)head * a.nqb;
  int sum = 0;
  for (int I = first; I < last; ++I) sum += counts[I];
  int offset = scan_256(sum, partial, tid);
  int32_t* rp = a.row_ptr + (int64_t)head * (a.nqb + 1);
  int32_t* ci = a.col_idx + (int64_t)head * a.cap_per_head;
  for (int I = first; I < last; ++I) {
    rp[I] = offset;
    offset += counts[I];
  }
  if (tid == 255) rp[a.nqb] = partial[255];
  __syncthreads();  // the row pointer written above is visible to the whole work-group
  const int wave = tid >> 6, lane = tid & 63;
  for (int I = wave; I < a.nqb; I += 4) {
    const int beg = rp[I], n = rp[I + 1] - beg;
    const int32_t* src = a.rows_tmp + ((int64_t)head * a.nqb + I) * a.stride;
    for (int t = lane; t < n; t += 64) ci[beg + t] = src[t];
  }
}

// ---------------------------------------------------------------------------- index validation
__global__ __launch_bounds__(256) void validate_kernel(const ValidateArgs a) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= a.rows) return;
  const int bh = r / a.nqb, I = r % a.nqb;
  const int32_t* rp = a.row_ptr + (int64_t)bh * (a.nqb + 1);
  const int32_t beg = rp[I], end = rp[I + 1];
  bool ok = (beg >= 0) && (end >= beg) && (end <= a.cap_per_head) && (I != 0 || beg == 0);
  if (ok) {
    const int32_t* ci = a.col_idx + (int64_t)bh * a.cap_per_head;
    int32_t prev = -1;
    for (int t = beg; t < end; ++t) {
      const int32_t J = ci[t];
      if (J <= prev || J >= a.nkb) ok = false;
      prev = J;
    }
  }
  if (!ok) atomicAdd(a.bad, 1);
}

// ---------------------------------------------------------------------------- fixed patterns
// Sliding window plus attention sinks as a block index (the fixed patterns the paper compares
// against, Section 4.1): query block I keeps the leading `sink_blocks` key blocks and every key
// block that holds a key within `half_window` tokens of one of its queries. One work-group per head: row lengths
// scanned into the row pointer, then a wave per row.
__global__ __launch_bounds__(256) void window_index_kernel(const WindowArgs a) {
  __shared__ int32_t partial[256];
  const int bh = blockIdx.x, tid = threadIdx.x;
  const int per = (a.nqb + 255) / 256;  // consecutive rows per thread
  const int first_row = tid * per, last_row = first_row + per < a.nqb ? first_row + per : a.nqb;
  int sum = 0;
  for (int I = first_row; I < last_row; ++I) sum += window_row_length(I, a.block_q, a.block_k, a.L, a.half_window, a.sink_blocks);
  int offset = scan_256(sum, partial, tid);
  int32_t* rp = a.row_ptr + (int64_t)bh * (a.nqb + 1);
  int32_t* ci = a.col_idx + (int64_t)bh * a.cap_per_head;
  for (int I = first_row; I < last_row; ++I) {
    rp[I] = offset;
    offset += window_row_length(I, a.block_q, a.block_k, a.L, a.half_window, a.sink_blocks);
  }
  if (tid == 255) rp[a.nqb] = partial[255];
  __syncthreads();  // the row pointer written above is visible to the whole work-group
  const int wave = tid >> 6, lane = tid & 63;
  for (int I = wave; I < a.nqb; I += 4) {  // a wave per row, a lane per entry: the sinks, then the window
    int sink_end, first, last;
    window_row_runs(I, a.block_q, a.block_k, a.L, a.half_window, a.sink_blocks, &sink_end, &first, &last);
    int32_t* dst = ci + rp[I];
    for (int J = lane; J < sink_end; J += 64) dst[J] = J;
    for (int J = first + lane; J <= last; J += 64) dst[sink_end + J - first] = J;
  }
}

// ---------------------------------------------------------------------------- launchers
template <int D>
static hipError_t launch_pool_bf16_d(int block_q, const PoolArgs& a, hipStream_t s) {
  // every work-group is four waves = 128 consecutive rows of a head: one, two or four query blocks
  if (block_q != 128 && block_q != 64 && block_q != 32) return hipErrorInvalidValue;
  const int blocks_per_group = 128 / block_q;
  const int64_t total = (int64_t)a.B * a.Hq * ((a.nqb + blocks_per_group - 1) / blocks_per_group);
  if (total <= 0 || total > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)total), block(256);
  switch (block_q) {
    case 128:
      if (a.block_k == 32) hipLaunchKernelGGL((pool_bf16_kernel<D, 4, true, 4>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((pool_bf16_kernel<D, 4, false, 4>), grid, block, 0, s, a);
      break;
    case 64:
      if (a.block_k == 32) hipLaunchKernelGGL((pool_bf16_kernel<D, 4, true, 2>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((pool_bf16_kernel<D, 4, false, 2>), grid, block, 0, s, a);
      break;
    case 32:
      if (a.block_k == 32) hipLaunchKernelGGL((pool_bf16_kernel<D, 4, true, 1>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((pool_bf16_kernel<D, 4, false, 1>), grid, block, 0, s, a);
      break;
  }
  return hipGetLastError();
}

hipError_t launch_pool_bf16(int D, int block_q, const PoolArgs& a, hipStream_t s) {
  if (D == 128) return launch_pool_bf16_d<128>(block_q, a, s);
  if (D == 64) return launch_pool_bf16_d<64>(block_q, a, s);
  return hipErrorInvalidValue;
}

template <int D>
static hipError_t launch_pool_f32_d(int block_q, const PoolArgs& a, hipStream_t s) {
  const int64_t total = (int64_t)a.B * a.Hq * a.nqb;
  if (total <= 0 || total > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)total);
  switch (block_q) {
    case 128: hipLaunchKernelGGL((pool_f32_kernel<D, 4>), grid, dim3(256), 0, s, a); break;
    case 64: hipLaunchKernelGGL((pool_f32_kernel<D, 2>), grid, dim3(128), 0, s, a); break;
    case 32: hipLaunchKernelGGL((pool_f32_kernel<D, 1>), grid, dim3(64), 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_pool_f32(int D, int block_q, const PoolArgs& a, hipStream_t s) {
  if (D == 128) return launch_pool_f32_d<128>(block_q, a, s);
  if (D == 64) return launch_pool_f32_d<64>(block_q, a, s);
  return hipErrorInvalidValue;
}

hipError_t launch_topk(const TopkArgs& a, hipStream_t s) {
  if (a.rows <= 0) return hipErrorInvalidValue;
  const size_t lds = a.straddle >= 0 ? (size_t)(a.nkb + 1 + a.keep_lo + a.keep_hi) * sizeof(uint32_t) : (size_t)a.nkb * sizeof(uint32_t);
  hipLaunchKernelGGL(topk_kernel, dim3((unsigned)a.rows), dim3(64), lds, s, a);
  return hipGetLastError();
}

hipError_t launch_window_index(const WindowArgs& a, hipStream_t s) {
  if (a.heads <= 0 || a.nqb <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(window_index_kernel, dim3((unsigned)a.heads), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_compact(const CompactArgs& a, hipStream_t s) {
  if (a.heads <= 0 || a.nqb <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(compact_kernel, dim3((unsigned)a.heads), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_validate(const ValidateArgs& a, hipStream_t s) {
  if (a.rows <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(validate_kernel, dim3((unsigned)((a.rows + 255) / 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace sparsed
