// Pooled scores in ONE pass over the keys (Section 3.3; Algorithm 1's per-query-block loop), for callers
// that have no row log-sum-exp to hand over.
//
//   A'[I, J] = 1 / (rows x keys) * sum_{r in I} (1 / Z_r) * sum_{j in J} exp(s_rj - m_r),   Z_r = sum_j exp(s_rj - m_r)
//
// The normaliser Z_r of a query row is known only after its last key, so the per-row block sums
// E[r, J] = sum_{j in J} exp(s_rj - m_r) are parked in a scratch slab that belongs to the work-group
// (128 x nkb floats: O(L) per work-group, never O(L^2) in total), and weighted by 1 / Z_r and summed
// over the rows of the query block once the row is complete. Work-groups are persistent: each walks the
// units (128 consecutive rows of a head: one, two or four query blocks) wg, wg + G, ... and reuses its slab.
//
// Reference m_r: the maximum logit of the row's first 32 keys. It is never above the row's true maximum, so
// nothing underflows that the two-pass form (reference = log-sum-exp) would keep. A later logit more than
// 100 octaves above it (never, on real attention logits) is caught by the overflow test on every 32-key
// sub-tile and handled out of line: the reference is raised, and the row's running sums, its staged block
// sums and the ones already in the slab are rescaled.
//
// Matrix work, K tile copies, fragment layouts and the 32-key software pipeline are those of pool_bf16_kernel
// (select.hip); exponentials, sums and weights are fp32 throughout, summed in a fixed order.
#include "kernels.hpp"
#include "tile_bf16.hpp"

namespace sparsed {

namespace {

[[maybe_unused]] constexpr int kChunk = 8;    // block sums staged per row before they go to the slab (32 contiguous bytes per row)
[[maybe_unused]] constexpr int kChunkLd = 8;  // floats per staged row (no padding: one staging store per key block is too rare for its bank conflicts to count)
[[maybe_unused]] constexpr float kOverflow = 1.2676506e30f;  // 2^100: a 32-key partial sum at or above this triggers the re-reference path

// Work-groups per compute unit the kernel is built for: two K tiles + staging is just under a quarter of the LDS.
constexpr int groups_per_cu(int) { return 4; }

}  // namespace

// QBW: waves per query block. A work-group is always NW = 4 waves = 128 consecutive rows of a head: one query block of
// 128 rows, two of 64 or four of 32, which share its K tiles and its slab.
template <int D, int NW, int BK, int QBW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NW >= 4 ? 4 : NW >= 2 ? 2 : 1, NW >= 4 ? 4 : NW >= 2 ? 2 : 1)))
void pool1p_bf16_kernel(const PoolArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (the body uses device-only types)
  constexpr int NT = NW * 64, QT = 32 * NW;
  constexpr int kKBytes = KLayout<D>::kTileBytes;
  constexpr int kSubPerBlock = BK / 32;  // 32-key sub-tiles per key block: 1, 2 or 4
  __shared__ __attribute__((aligned(1024))) char kbuf0[kKBytes];
  __shared__ __attribute__((aligned(1024))) char kbuf1[kKBytes];
  __shared__ __attribute__((aligned(16))) float chunk[NW][32][kChunkLd];
  __shared__ float inv_z[QT];
  // key blocks per segment of the closing pass: the per-wave partial sums of one segment fit the first K buffer
  constexpr int kSeg = (kKBytes / (NW * 4) >= 1024) ? 1024 : (kKBytes / (NW * 4)) & ~63;
  static_assert(kSeg >= 64 && kSeg * NW * 4 <= kKBytes, "segment of partial sums must fit a K buffer");

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 31, g = lane >> 5;
  const int ld = a.slab_ld;  // floats per slab row: nkb rounded up to a whole chunk
  float* const slab = a.slab + (int64_t)blockIdx.x * QT * ld + (int64_t)wave * 32 * ld;  // this wave's 32 rows
  static_assert(NW % QBW == 0, "whole query blocks per work-group");
  constexpr int kBlocksPerGroup = NW / QBW, kBlockRows = 32 * QBW;
  const int groups_per_head = (a.nqb + kBlocksPerGroup - 1) / kBlocksPerGroup;
  const int units = a.B * a.Hq * groups_per_head;  // a unit: QT consecutive rows of one head
  const float c = a.scale_log2;

  TileDma<D, NT, false> kdma;
  kdma.init(a.k.sl, wave, lane);
  KFragAddr<D> kaddr;
  kaddr.init(lane);

  for (int unit = xcd_remap(blockIdx.x, gridDim.x); unit < units; unit += gridDim.x) {
    const int gq = unit % groups_per_head;
    const int bh = unit / groups_per_head;
    const int b = bh / a.Hq, h = bh % a.Hq;
    const int hk = h / (a.Hq / a.Hkv);
    int L = a.L;  // length of this batch element
    if (a.seq_lens != nullptr) {
      const int len = a.seq_lens[b];
      L = len < a.L ? len : a.L;
    }
    if (gq * QT >= L) continue;  // rows this sample does not have (uniform over the work-group)
    const int key_len = L;
    const __bf16* qbase = static_cast<const __bf16*>(a.q.ptr) + b * a.q.sb + h * a.q.sh;
    const __bf16* kbase = static_cast<const __bf16*>(a.k.ptr) + b * a.k.sb + hk * a.k.sh;
    const int row0 = gq * QT + wave * 32;

    QFrag<D, 1> qf;
    qf.load(qbase, row0, L, a.q.sl, lane);
    const int last_blk = (key_len - 1) / kTileK;                 // last 64-key tile that exists
    const int tail_keys = key_len - last_blk * kTileK;           // keys in it
    const int n = last_blk + 1;
    const int nkb_here = (key_len + BK - 1) / BK;                // key blocks this sample has
    auto keys_of = [&](int blk) -> int { return blk == last_blk ? tail_keys : kTileK; };
    auto keys_at = [&](int tile) -> int { return tile < n ? keys_of(tile) : 0; };
    const __amdgpu_buffer_rsrc_t krsrc = make_rsrc(kbase, ((int64_t)(key_len - 1) * a.k.sl + D) * 2);
    const int32_t k_tile_bytes = (int32_t)(kTileK * a.k.sl * 2);
    auto copy_k_any = [&](int tile, char* dst) {  // any tile: past the end repeats the last one, which may be partial
      const int blk = tile < n ? tile : n - 1;
      if (blk == last_blk && tail_keys < kTileK) kdma.issue_partial(krsrc, blk * k_tile_bytes, dst, wave, lane, a.k.sl, tail_keys);
      else kdma.issue(krsrc, blk * k_tile_bytes, dst, wave);
    };

    f32x16 s_even[1], s_odd[1];
    float M = 0.f;     // reference of this lane's row, in octaves (log2 units)
    float lsum = 0.f;  // this lane's share of Z_r
    float eacc = 0.f;  // this lane's share of the block sum in progress
    int sub = 0;       // 32-key sub-tiles summed so far

    // masked: apply `valid`, the number of keys of the sub-tile that exist (>= 32: all, <= 0: none)
    auto mask_sub = [&](f32x16(&s)[1], int valid) {
      const int mine = valid - 8 * g;  // register x of lane (j, g) holds key 16*(x/8) + 8*g + x%8
#pragma unroll
      for (int x = 0; x < 16; ++x)
        if (16 * (x >> 3) + (x & 7) >= mine) s[0][x] = -__builtin_inff();
    };
    auto row_max = [&](const f32x16(&s)[1]) -> float {
      float mx = fmaxf(s[0][0], s[0][1]);
#pragma unroll
      for (int x = 2; x < 16; x += 2) mx = fmaxf(fmaxf(mx, s[0][x]), s[0][x + 1]);
      return pair_max(mx) * c;
    };
    auto exp_sum = [&](const f32x16(&s)[1]) -> float {
      float part = 0.f;
#pragma unroll
      for (int x = 0; x < 16; ++x) part += __builtin_amdgcn_exp2f(__builtin_fmaf(s[0][x], c, -M));
      return part;
    };
    // A block sum is complete: both halves of the row are added and staged; a full chunk (or the last block) goes to the slab.
    auto finish_block = [&](int J) {
      const float e = pair_sum(eacc);
      eacc = 0.f;
      if (J >= nkb_here) return;  // the empty second half of a partial last tile with 32-key blocks
      const int slot = J & (kChunk - 1);
      if (g == 0) chunk[wave][j][slot] = e;
      if (slot == kChunk - 1 || J == nkb_here - 1) {
        const int r = lane >> 1, half = lane & 1;
        const u32x4 w = *reinterpret_cast<const u32x4*>(&chunk[wave][r][half * 4]);
        *reinterpret_cast<u32x4*>(slab + (int64_t)r * ld + (J & ~(kChunk - 1)) + half * 4) = w;
      }
    };
    // Out of line: some 32-key partial sum overflowed the reference. Raise the reference of the rows concerned to
    // their new maximum and rescale everything they have accumulated so far (J_done block sums are complete).
    auto re_reference = [&](const f32x16(&s)[1], int J_done) {
      const float mx = row_max(s);
      const float Mn = fmaxf(M, mx);
      const float alpha = __builtin_amdgcn_exp2f(M - Mn);  // <= 1; exactly 1 where nothing changes
      M = Mn;
      lsum *= alpha;
      eacc *= alpha;
      if (g == 0 && alpha != 1.0f) {
        const int staged_from = J_done & ~(kChunk - 1);
        for (int J = staged_from; J < J_done; ++J) chunk[wave][j][J - staged_from] *= alpha;
        float* row = slab + (int64_t)j * ld;
        for (int J = 0; J < staged_from; ++J) {
          const float v = __hip_atomic_load(row + J, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          row[J] = v * alpha;
        }
      }
    };
    // One 32-key sub-tile: exponentials against the row reference, summed per lane.
    auto expsum_sub = [&](f32x16(&s)[1], const bool masked, int valid) {
      if (masked) mask_sub(s, valid);
      float part = exp_sum(s);
      if (__builtin_amdgcn_ballot_w64(!(part < kOverflow)) != 0) {  // wave-uniform, practically never taken
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");           // this wave's slab stores are complete
        re_reference(s, sub / kSubPerBlock);
        part = exp_sum(s);
      }
      asm volatile("" : "+v"(part));  // keep the vector work inside the block that holds the matrix work
      lsum += part;
      eacc += part;
      ++sub;
      if (sub % kSubPerBlock == 0) finish_block(sub / kSubPerBlock - 1);
    };

    // Tile step t (LDS parity P = t & 1) = sub-tiles 2t+1 and 2t+2. On entry S(2t+1) is in s_odd, K(t+1) in
    // kbuf[1-P]; kbuf[P] is free and receives K(t+2). Tiles past the end are phantoms (a repeated copy, every key
    // masked); MASKED steps (the last few) count the keys that exist in each sub-tile.
#define SPARSED_POOL1P_STEP(P, MASKED, T)                                                          \
  {                                                                                                \
    char* const kb_free = (P) ? kbuf1 : kbuf0;                                                     \
    char* const kb_next = (P) ? kbuf0 : kbuf1;                                                     \
    if (MASKED) copy_k_any((T) + 2, kb_free);                                                      \
    else kdma.issue(krsrc, ((T) + 2 < n ? (T) + 2 : n - 1) * k_tile_bytes, kb_free, wave);         \
    logits_sub<D, 1, false>(kb_next, 0, kaddr, qf, s_even);                                        \
    expsum_sub(s_odd, (MASKED), keys_at(T) - 32);                                                  \
    sched_substep_interleave<D, 1, false>();                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                             \
    logits_sub<D, 1, false>(kb_next, 1, kaddr, qf, s_odd);                                         \
    if ((T) + 1 < n) expsum_sub(s_even, (MASKED), keys_at((T) + 1));                               \
    sched_substep_interleave<D, 1, false>();                                                       \
    __syncthreads();                                                                               \
  }

    // prologue: K(0), K(1) (a repeat of K(0) for a one-tile range) into LDS; S(0); reference and sums of sub-tile 0
    copy_k_any(0, kbuf0);
    copy_k_any(1, kbuf1);
    __syncthreads();
    logits_sub<D, 1, true>(kbuf0, 0, kaddr, qf, s_even);
    logits_sub<D, 1, true>(kbuf0, 1, kaddr, qf, s_odd);
    mask_sub(s_even, keys_at(0));
    M = row_max(s_even);  // at least one key exists, so this is finite
    expsum_sub(s_even, false, 32);
    __syncthreads();  // everyone is done with K(0) before tile step 0 lets K(2) overwrite it

    const int steady_reach = (tail_keys < kTileK) ? 4 : 2;
    int t = 0;
    while (t + steady_reach < n) {
      SPARSED_POOL1P_STEP(0, false, t);
      SPARSED_POOL1P_STEP(1, false, t + 1);
      t += 2;
    }
    for (; t < n; ++t) {
      if (t & 1) {
        SPARSED_POOL1P_STEP(1, true, t);
      } else {
        SPARSED_POOL1P_STEP(0, true, t);
      }
    }
#undef SPARSED_POOL1P_STEP
    if (sub % kSubPerBlock != 0) finish_block(sub / kSubPerBlock);  // a last key block cut short by the end of the keys

    // The rows are complete: 1 / Z_r (0 for rows past the end), the row log-sum-exp for later users, and then
    // A'[I, J] = sum_r E[r, J] / Z_r over the rows of the block, divided by the entries that exist.
    const float ltot = pair_sum(lsum);
    if (g == 0) {
      const bool exists = row0 + j < L;
      inv_z[wave * 32 + j] = exists ? 1.0f / ltot : 0.f;
      if (a.lse_out != nullptr && exists) a.lse_out[(int64_t)bh * a.L + row0 + j] = (M + __builtin_amdgcn_logf(ltot)) * 0.6931471805599453f;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // this wave's slab stores are complete before it reads them back
    __syncthreads();
    float* const partial = reinterpret_cast<float*>(kbuf0);  // [NW][kSeg] (the K buffers are idle now)
    for (int seg = 0; seg < nkb_here; seg += kSeg) {
      const int seg_n = nkb_here - seg < kSeg ? nkb_here - seg : kSeg;
      for (int x = lane; x < seg_n; x += 64) {
        float acc = 0.f;
        const float* col = slab + seg + x;
#pragma unroll 4
        for (int r = 0; r < 32; ++r)
          acc += __hip_atomic_load(col + (int64_t)r * ld, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * inv_z[wave * 32 + r];
        partial[wave * kSeg + x] = acc;
      }
      __syncthreads();
#pragma unroll
      for (int qb = 0; qb < kBlocksPerGroup; ++qb) {  // the query blocks of the group, each summed over its own waves
        const int I = gq * kBlocksPerGroup + qb;
        if (I >= a.nqb || I * kBlockRows >= L) break;  // a block the head (or this sample) does not have
        float* arow = a.apool + ((int64_t)bh * a.nqb + I) * a.out_stride;
        const int rows_here = (L - I * kBlockRows < kBlockRows) ? L - I * kBlockRows : kBlockRows;  // query rows that exist
        for (int x = tid; x < seg_n; x += NT) {
          float tot = 0.f;
#pragma unroll
          for (int w = 0; w < QBW; ++w) tot += partial[(qb * QBW + w) * kSeg + x];
          const int J = seg + x;
          const int keys_here = key_len - J * BK < BK ? key_len - J * BK : BK;
          arow[J] = tot * (1.0f / (float)(rows_here * keys_here));  // mean over the entries that exist
        }
      }
      __syncthreads();  // the partial sums (and, after the last segment, the K buffers) may be overwritten
    }
  }
#endif
}

int pool1p_groups(int) { return 256 * groups_per_cu(4); }

int64_t pool1p_units(int B, int Hq, int nqb, int block_q) {
  const int per = 128 / block_q;  // query blocks per work-group
  return (int64_t)B * Hq * ((nqb + per - 1) / per);
}

template <int D, int QBW>
static hipError_t launch_pool1p_bk(const PoolArgs& a, int groups, hipStream_t s) {
  const dim3 grid((unsigned)groups), block(256);
  switch (a.block_k) {
    case 32: hipLaunchKernelGGL((pool1p_bf16_kernel<D, 4, 32, QBW>), grid, block, 0, s, a); break;
    case 64: hipLaunchKernelGGL((pool1p_bf16_kernel<D, 4, 64, QBW>), grid, block, 0, s, a); break;
    case 128: hipLaunchKernelGGL((pool1p_bf16_kernel<D, 4, 128, QBW>), grid, block, 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// One-pass pooled scores over the whole key range of every sample. a.slab holds `groups` slabs of
// 128 x a.slab_ld floats; a.lse_out (optional) receives the row log-sum-exp.
hipError_t launch_pool1p_bf16(int D, int block_q, const PoolArgs& a, int groups, hipStream_t s) {
  if (block_q != 128 && block_q != 64 && block_q != 32) return hipErrorInvalidValue;
  const int64_t units = pool1p_units(a.B, a.Hq, a.nqb, block_q);
  if (units <= 0 || units > 0x7fffffff || groups < 1 || a.slab == nullptr || a.slab_ld < a.out_stride) return hipErrorInvalidValue;
  if (groups > units) groups = (int)units;
  if (D == 128) {
    if (block_q == 128) return launch_pool1p_bk<128, 4>(a, groups, s);
    if (block_q == 64) return launch_pool1p_bk<128, 2>(a, groups, s);
    return launch_pool1p_bk<128, 1>(a, groups, s);
  } else if (D == 64) {
    if (block_q == 128) return launch_pool1p_bk<64, 4>(a, groups, s);
    if (block_q == 64) return launch_pool1p_bk<64, 2>(a, groups, s);
    return launch_pool1p_bk<64, 1>(a, groups, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace sparsed
