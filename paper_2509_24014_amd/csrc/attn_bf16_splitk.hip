// Block-sparse bf16 attention (Eq. 3 / Eq. 4) for SMALL query blocks (32 or 64 rows).
//
// The general kernel (attn_bf16.hip) gives every wave 32 query rows and all the keys of a tile, so a
// 64-row query block is a work-group of two waves; its K/V double buffers fill the LDS of a compute
// unit after two such groups, which leaves one wave per SIMD and nothing to overlap a wave's softmax
// with. Here a query block gets twice the waves: wave (rw, kh) owns rows 32*rw .. 32*rw+31 and, of
// every 64-key tile, only the 32 keys of half kh. The two key halves of a row keep their own running
// maximum, sum and output accumulator (flash-decoding style) and are merged once, through LDS, at the
// end. Same LDS footprint per group, twice the waves per compute unit.
//
// Per tile step t a wave computes  S(t+1) = K(t+1)[half] Q^T  interleaved with the softmax of S(t),
// then  O += P(t) V(t)[half].  K(t+2) and V(t+1) are copied global -> LDS meanwhile; one barrier per tile.
// Tiles past the end of the list repeat the last one (their logits are never used); a partial last
// key block is masked in the last step (the last two with 128-key blocks), the only ones that apply key counts.
// Listed blocks of 128 keys are walked as two tiles, listed blocks of 32 keys are paired up two to a tile
// (see the notes at `tile_shift` / `half_blocks` below).
#include "kernels.hpp"
#include "tile_bf16.hpp"

namespace sparsed {

// KB: keys per listed block (32, 64 or 128), a compile-time choice so that the common 64 pays nothing for the others.
template <int D, int RW, int KB>
__global__ __launch_bounds__(RW * 128) __attribute__((amdgpu_waves_per_eu(RW >= 2 ? 2 : 1, RW >= 2 ? 2 : 1))) void attn_bf16_splitk_kernel(const AttnArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (the body uses device-only types)
  constexpr int NW = 2 * RW, NT = NW * 64, QT = 32 * RW;
  constexpr int kKBytes = KLayout<D>::kTileBytes, kVBytes = VLayout<D>::kTileBytes;
  constexpr float kOverflow = 1.152921504606847e18f;  // 2^60: a 16-key partial sum at or above this re-references the row
  __shared__ __attribute__((aligned(1024))) char kbuf0[kKBytes];
  __shared__ __attribute__((aligned(1024))) char kbuf1[kKBytes];
  __shared__ __attribute__((aligned(1024))) char vbuf0[kVBytes];
  __shared__ __attribute__((aligned(1024))) char vbuf1[kVBytes];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rw = wave % RW, kh = wave / RW;  // row group and key half of this wave
  const int j = lane & 31, g = lane >> 5;

  const int lid = xcd_remap(blockIdx.x, gridDim.x);
  const int qt = lid % a.n_qtiles;
  const int bh = lid / a.n_qtiles;
  const int b = bh / a.Hq, h = bh % a.Hq;
  const int hk = h / (a.Hq / a.Hkv);
  int L = a.L;  // length of this batch element
  if (a.seq_lens != nullptr) {
    const int len = a.seq_lens[b];
    L = len < a.L ? len : a.L;
  }
  if (qt * QT >= L) return;  // a query block wholly past the end (uniform over the work-group)

  const __bf16* qbase = static_cast<const __bf16*>(a.q.ptr) + b * a.q.sb + h * a.q.sh;
  const __bf16* kbase = static_cast<const __bf16*>(a.k.ptr) + b * a.k.sb + hk * a.k.sh;
  const __bf16* vbase = static_cast<const __bf16*>(a.v.ptr) + b * a.v.sb + hk * a.v.sh;
  const int row0 = qt * QT + rw * 32;

  const int32_t* rp = a.row_ptr + (int64_t)bh * (a.nqb + 1) + qt;
  const int beg = rp[0], end = rp[1];
  // A listed 128-key block is two consecutive tiles. Listed 32-key blocks are paired up in list order:
  // tile t holds entries 2t and 2t + 1, one in each 32-key half, wherever in the sequence they come from
  // (the key half a wave owns is then exactly one listed block; an odd count leaves the last half empty).
  constexpr int tile_shift = KB == 2 * kTileK ? 1 : 0;
  constexpr bool half_blocks = KB == kTileK / 2;
  const int entries = end - beg;
  const int n = half_blocks ? (entries + 1) >> 1 : entries << tile_shift;
  const int32_t* cols = a.col_idx + (int64_t)bh * a.cap_per_head + beg;
  constexpr int unit = half_blocks ? kTileK / 2 : kTileK;  // keys per copy unit: a 32-key block or a 64-key tile
  const int last_blk = (L - 1) / unit;                 // last unit that exists
  const int tail_keys = L - last_blk * unit;           // keys in it

  float M = 0.f, lsum = 0.f;
  f32x16 o[1][D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int x = 0; x < 16; ++x) o[0][dt][x] = 0.f;
  f32x16 s_a[1], s_b[1];  // logits of the tile being normalised and of the next one
  bf16x8 p[1][2];

  TileDma<D, NT, false> kdma;
  TileDma<D, NT, true> vdma;
  if (half_blocks) {
    kdma.init_half(a.k.sl, wave, lane);
    vdma.init_half(a.v.sl, wave, lane);
  } else {
    kdma.init(a.k.sl, wave, lane);
    vdma.init(a.v.sl, wave, lane);
  }
  KFragAddr<D> kaddr;
  VFragAddr<D> vaddr;
  kaddr.init(lane);
  vaddr.init(lane);

  // block numbers of tiles t .. t+3, read with a vector load (see attn_bf16.hip); past the end: the last one
  int opaque_zero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(opaque_zero));
  auto col_at = [&](int t) -> int {  // key TILE number of tile t of the list; with 32-key blocks: the block of this wave's half
    if (half_blocks) {
      const int e = 2 * t + kh;
      return cols[(e < entries ? e : (entries > 0 ? entries - 1 : 0)) + opaque_zero];  // a missing half repeats the last block, masked
    }
    const int idx = t < n ? t : (n > 0 ? n - 1 : 0);
    return (cols[(idx >> tile_shift) + opaque_zero] << tile_shift) + (idx & tile_shift);
  };
  int blk0 = 0, blk1 = 0, blk2 = 0, blk3 = 0;
  if (n > 0) {
    blk0 = col_at(0);
    blk1 = col_at(1);
    blk2 = col_at(2);
    blk3 = col_at(3);
  }
  QFrag<D, 1> qf;  // loaded after the first K/V copies have been issued (see attn_bf16.hip)

  const int64_t slab_rows = (int64_t)(a.L - 1);
  const __amdgpu_buffer_rsrc_t krsrc = make_rsrc(kbase, (slab_rows * a.k.sl + D) * 2);
  const __amdgpu_buffer_rsrc_t vrsrc = make_rsrc(vbase, (slab_rows * a.v.sl + D) * 2);
  const int32_t k_tile_bytes = (int32_t)(unit * a.k.sl * 2), v_tile_bytes = (int32_t)(unit * a.v.sl * 2);  // bytes per copy unit
  // (the second tile of a partial 128-key block may lie wholly past the end: any real tile is copied, all keys masked)
  auto copy_k = [&](int blk, char* dst) {
    const int rb = __builtin_amdgcn_readfirstlane(blk);
    const int ub = rb < last_blk ? rb : last_blk;
    if (ub == last_blk && tail_keys < unit) {
      if (half_blocks) kdma.issue_partial_half(krsrc, ub * k_tile_bytes, dst, wave, lane, a.k.sl, tail_keys);
      else kdma.issue_partial(krsrc, ub * k_tile_bytes, dst, wave, lane, a.k.sl, tail_keys);
    } else {
      kdma.issue(krsrc, ub * k_tile_bytes, dst, wave);
    }
  };
  auto copy_v = [&](int blk, char* dst) {
    const int rb = __builtin_amdgcn_readfirstlane(blk);
    const int ub = rb < last_blk ? rb : last_blk;
    if (ub == last_blk && tail_keys < unit) {
      if (half_blocks) vdma.issue_partial_half(vrsrc, ub * v_tile_bytes, dst, wave, lane, a.v.sl, tail_keys);
      else vdma.issue_partial(vrsrc, ub * v_tile_bytes, dst, wave, lane, a.v.sl, tail_keys);
    } else {
      vdma.issue(vrsrc, ub * v_tile_bytes, dst, wave);
    }
  };

  const float c = a.scale_log2;

  // Softmax of this wave's 32 keys of one tile against the row's fixed reference M (same arithmetic as the
  // general kernel: the reference is set once, from the first tile, and a sub-tile whose probabilities leave
  // the range that is good for is redone out of line): s -> p and this lane's share of the row sum.
  auto mask_half = [&](f32x16(&s)[1], int valid) {
    const int mine = valid - 8 * g;  // register x of lane (j, g) holds key 16*(x/8) + 8*g + x%8 of the half
#pragma unroll
    for (int x = 0; x < 16; ++x)
      if (16 * (x >> 3) + (x & 7) >= mine) s[0][x] = -__builtin_inff();
  };
  auto exp_half = [&](const f32x16(&s)[1], float& part) {
    part = 0.f;
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      u32x4 pk;
#pragma unroll
      for (int x = 0; x < 8; x += 2) {
        const f32x2 two = {__builtin_amdgcn_exp2f(__builtin_fmaf(s[0][8 * m + x], c, -M)),
                           __builtin_amdgcn_exp2f(__builtin_fmaf(s[0][8 * m + x + 1], c, -M))};
        pk[x >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
        part += two[0];
        part += two[1];
      }
      asm volatile("" : "+v"(pk));  // keep the probabilities inside the block that holds the matrix instructions
      p[0][m] = __builtin_bit_cast(bf16x8, pk);
    }
    asm volatile("" : "+v"(part));
  };
  auto row_max = [&](const f32x16(&s)[1]) -> float {
    float mx = fmaxf(s[0][0], s[0][1]);
#pragma unroll
    for (int x = 2; x < 16; x += 2) mx = fmaxf(fmaxf(mx, s[0][x]), s[0][x + 1]);
    return pair_max(mx) * c;
  };
  auto softmax_half = [&](f32x16(&s)[1], float& part, const bool masked, int valid) {
    if (masked) mask_half(s, valid);
    exp_half(s, part);
  };
  // Out of line, practically never taken: raise the reference to at least this tile's maximum, bring the
  // row's sum and output to it, redo the tile's probabilities.
  auto re_reference = [&](const f32x16(&s)[1], float& part) {
    const float Mn = fmaxf(M, row_max(s));
    const float alpha = __builtin_amdgcn_exp2f(M - Mn);  // <= 1; exactly 1 where nothing changes
    M = Mn;
    lsum *= alpha;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int x = 0; x < 16; ++x) o[0][dt][x] *= alpha;
    exp_half(s, part);
  };
  // keys of this wave's half that exist in tile T of the list, whose first block number is `first`
  auto valid_in = [&](int T, int first) -> int {
    const int tile0 = __builtin_amdgcn_readfirstlane(first);
    return half_blocks ? (2 * T + kh < entries ? (tile0 == last_blk ? tail_keys : 32) : 0)
                       : (tile0 > last_blk ? 0 : tile0 == last_blk ? tail_keys : kTileK) - 32 * kh;
  };

  // Tile step t (LDS parity P = t & 1). On entry: S(t) in S_CUR, K(t+1) in kbuf[1-P], V(t) in vbuf[P];
  // kbuf[P] (held K(t)) and vbuf[1-P] (held V(t-1)) are free and receive K(t+2) and V(t+1).
#define SPARSED_SPLITK_STEP(P, MASKED, T, S_CUR, S_NEXT)                                             \
  {                                                                                                \
    char* const kb_free = (P) ? kbuf1 : kbuf0;                                                     \
    char* const kb_next = (P) ? kbuf0 : kbuf1;                                                     \
    char* const vb_this = (P) ? vbuf1 : vbuf0;                                                     \
    char* const vb_free = (P) ? vbuf0 : vbuf1;                                                     \
    copy_k(blk2, kb_free);                                                                         \
    copy_v(blk1, vb_free);                                                                         \
    const int blk_new = col_at((T) + 4);                                                           \
    const int valid = !(MASKED) ? 32 : valid_in((T), blk0);                                         \
    float part;                                                                                    \
    logits_sub<D, 1, false>(kb_next, kh, kaddr, qf, S_NEXT);                                       \
    softmax_half(S_CUR, part, (MASKED), valid);                                                    \
    sched_substep_interleave<D, 1, false>();                                                       \
    if (__builtin_amdgcn_ballot_w64(!(part < kOverflow)) != 0) re_reference(S_CUR, part);          \
    lsum += part;                                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                                             \
    pv_sub<D, 1, true>(vb_this, kh, vaddr, p, o);                                                  \
    blk0 = blk1;                                                                                   \
    blk1 = blk2;                                                                                   \
    blk2 = blk3;                                                                                   \
    blk3 = blk_new;                                                                                \
    __syncthreads();                                                                               \
  }

  if (n > 0) {
    copy_k(blk0, kbuf0);
    copy_k(blk1, kbuf1);
    copy_v(blk0, vbuf0);
    qf.load(qbase, row0, L, a.q.sl, lane);
    __syncthreads();
    logits_sub<D, 1, true>(kbuf0, kh, kaddr, qf, s_a);
    {
      // The first tile fixes the reference: the maximum over the keys of this wave's half that exist. A half
      // with no such key (a short first block) starts from a floor that the first real key re-references.
      f32x16 first[1] = {s_a[0]};
      mask_half(first, valid_in(0, blk0));
      M = fmaxf(row_max(first), -1e30f);
    }
    __syncthreads();  // everyone is done with K(0) before step 0 lets K(2) overwrite it

    int t = 0;
    while (t + 2 < n) {
      SPARSED_SPLITK_STEP(0, false, t, s_a, s_b);
      SPARSED_SPLITK_STEP(1, false, t + 1, s_b, s_a);
      t += 2;
    }
    if (n - t == 2) {  // with 128-key blocks the last two tiles may both be short (a partial last block)
      SPARSED_SPLITK_STEP(0, (tile_shift != 0), t, s_a, s_b);
      SPARSED_SPLITK_STEP(1, true, t + 1, s_b, s_a);
    } else {
      SPARSED_SPLITK_STEP(0, true, t, s_a, s_b);
    }
  }
#undef SPARSED_SPLITK_STEP

  // Merge the two key halves of every row. The waves of half 1 leave their accumulator, reference
  // maximum and sum in the (now idle) K buffers, laid out [value][lane] so that both sides touch
  // consecutive words; the waves of half 0 fold them in, normalise and store.
  static_assert(RW <= 2, "one K buffer and one V buffer per wave of the second key half");
  static_assert(D / 32 * 16 * 64 * 4 <= kKBytes && 2 * 64 * 4 <= kVBytes, "exchange areas must fit the buffers");
  float* const xchg = reinterpret_cast<float*>(rw == 0 ? kbuf0 : kbuf1);   // the accumulator
  float* const xchg2 = reinterpret_cast<float*>(rw == 0 ? vbuf0 : vbuf1);  // reference maximum and sum
  const float ltot_mine = pair_sum(lsum);
  if (kh == 1) {
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int x = 0; x < 16; ++x) xchg[(dt * 16 + x) * 64 + lane] = o[0][dt][x];
    xchg2[lane] = M;
    xchg2[64 + lane] = ltot_mine;
  }
  __syncthreads();
  if (kh == 1) return;
  const float M_other = xchg2[lane], l_other = xchg2[64 + lane];
  const float Mn = fmaxf(M, M_other);
  const float f_mine = __builtin_amdgcn_exp2f(M - Mn), f_other = __builtin_amdgcn_exp2f(M_other - Mn);
  const float ltot = ltot_mine * f_mine + l_other * f_other;
  const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int x = 0; x < 16; ++x) o[0][dt][x] = (o[0][dt][x] * f_mine + xchg[(dt * 16 + x) * 64 + lane] * f_other) * inv;

  // whole-row stores through an LDS transpose (see the epilogue of attn_bf16.hip); the staging slice is this
  // row group's V buffer, whose two exchanged values this wave has already read
  constexpr int kRowBytes = 2 * D, kSlots = D / 8, kRowsPerStore = 64 / kSlots;
  static_assert(32 * kRowBytes <= kVBytes, "staging slice must fit a V buffer");
  char* const stage = rw == 0 ? vbuf0 : vbuf1;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const f32x2 lo = {o[0][dt][4 * q4], o[0][dt][4 * q4 + 1]};
      const f32x2 hi = {o[0][dt][4 * q4 + 2], o[0][dt][4 * q4 + 3]};
      u32x2 w;
      w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
      w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
      *reinterpret_cast<u32x2*>(stage + j * kRowBytes + (((4 * dt + q4) ^ (j & (kSlots - 1))) << 4) + 8 * g) = w;
    }
  __bf16* const obase = static_cast<__bf16*>(a.o) + b * a.o_sb + h * a.o_sh;
#pragma unroll
  for (int it = 0; it < 32 / kRowsPerStore; ++it) {
    const int r = it * kRowsPerStore + lane / kSlots, slot = lane % kSlots;
    const u32x4 w = *reinterpret_cast<const u32x4*>(stage + r * kRowBytes + ((slot ^ (r & (kSlots - 1))) << 4));
    const int grow = row0 + r;
    if (grow < L) *reinterpret_cast<u32x4*>(obase + (int64_t)grow * a.o_sl + slot * 8) = w;
  }
#endif
}

template <int D, int RW>
static hipError_t launch_splitk(const AttnArgs& a, hipStream_t s) {
  const int64_t total = (int64_t)a.B * a.Hq * a.n_qtiles;
  if (total <= 0 || total > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)total), block(RW * 128);
  switch (a.block_k) {
    case 32: hipLaunchKernelGGL((attn_bf16_splitk_kernel<D, RW, 32>), grid, block, 0, s, a); break;
    case 64: hipLaunchKernelGGL((attn_bf16_splitk_kernel<D, RW, 64>), grid, block, 0, s, a); break;
    case 128: hipLaunchKernelGGL((attn_bf16_splitk_kernel<D, RW, 128>), grid, block, 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Sparse attention for query blocks of 32 or 64 rows. a.n_qtiles must be set by the caller.
hipError_t launch_attn_bf16_splitk(int D, int block_q, const AttnArgs& a, hipStream_t s) {
  if (D == 128 && block_q == 64) return launch_splitk<128, 2>(a, s);
  if (D == 128 && block_q == 32) return launch_splitk<128, 1>(a, s);
  if (D == 64 && block_q == 64) return launch_splitk<64, 2>(a, s);
  if (D == 64 && block_q == 32) return launch_splitk<64, 1>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace sparsed
