// bf16 flash-attention forward for gfx950: dense (Eq. 1), block-sparse (Eq. 3 / Eq. 4) and the
// statistics-only pass (row log-sum-exp of Eq. 1's logits) used by pattern selection.
//
// One work-group owns QT = 32*NQ*NW query rows of one (batch, head) and walks 64-key tiles:
// all of them (dense, stats) or the key blocks listed for its query block (sparse; QT == block_q,
// so all rows of the group share one list). K and V tiles are copied global -> LDS directly,
// double-buffered, one barrier per tile (tile_bf16.hpp).
//
// Software pipeline inside every wave. On this chip a matrix instruction runs in the background
// of the wave that issued it while that same wave keeps issuing vector instructions, whereas two
// waves of a SIMD that each run a matrix block and then a vector block drift into doing the same
// kind of work at the same time. So
// a wave works in sub-steps of 32 keys, and sub-step u interleaves, in one instruction stream,
//      matrix:  O += P(u-1) V(u-1)   and   S(u+1) = K(u+1) Q^T
//      vector:  online softmax of S(u)  ->  P(u), running max / sum
// which are independent of each other; S and P are double-buffered in registers (even / odd
// sub-steps) and the tile loop is unrolled by two so that the LDS buffer roles are static.
// Softmax is online with a FIXED reference per query (the row maximum of the first sub-tile, not a
// running maximum; see softmax_sub) and a running sum, fp32; probabilities are rounded to bf16 for
// the second matrix product; the output accumulator is fp32.
#include "kernels.hpp"
#include "tile_bf16.hpp"


namespace sparsed {

// KB: keys per listed block in sparse mode (64 or 128), a compile-time choice.
template <int D, int NQ, int NW, Mode MODE, int KB = kTileK>
__global__ __launch_bounds__(NW * 64)
    __attribute__((amdgpu_waves_per_eu((NQ == 1 && NW >= 4) ? (MODE == Mode::kStats ? 4 : 2) : 1,
                                       (NQ == 1 && NW >= 4) ? (MODE == Mode::kStats ? 4 : 2) : 1))) void attn_bf16_kernel(const AttnArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (the body uses device-only types)
  constexpr int NT = NW * 64;
  constexpr int QT = 32 * NQ * NW;
  constexpr bool kHasV = MODE != Mode::kStats;
  constexpr int kKBytes = KLayout<D>::kTileBytes;
  constexpr int kVBytes = kHasV ? VLayout<D>::kTileBytes : 16;
  constexpr float kOverflow = 1.152921504606847e18f;  // 2^60: a 16-key partial sum at or above this re-references the row
  // Four separate LDS objects on purpose: the compiler tells accesses to different LDS variables
  // apart, so a copy in flight into one buffer does not hold up fragment reads from the others.
  __shared__ __attribute__((aligned(1024))) char kbuf0[kKBytes];
  __shared__ __attribute__((aligned(1024))) char kbuf1[kKBytes];
  __shared__ __attribute__((aligned(1024))) char vbuf0[kVBytes];
  __shared__ __attribute__((aligned(1024))) char vbuf1[kVBytes];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it in a scalar register
  const int g = lane >> 5;

  const int lid = xcd_remap(blockIdx.x, gridDim.x);
  const int qt = lid % a.n_qtiles;
  const int bh = lid / a.n_qtiles;
  const int b = bh / a.Hq, h = bh % a.Hq;
  const int hk = h / (a.Hq / a.Hkv);
  // length of this batch element: the tensor's L unless the caller passed per-sample lengths
  int L = a.L;
  if (a.seq_lens != nullptr) {
    const int len = a.seq_lens[b];
    L = len < a.L ? len : a.L;
  }
  if (qt * QT >= L) return;  // a query tile wholly past the end (uniform over the work-group)

  const __bf16* qbase = static_cast<const __bf16*>(a.q.ptr) + b * a.q.sb + h * a.q.sh;
  const __bf16* kbase = static_cast<const __bf16*>(a.k.ptr) + b * a.k.sb + hk * a.k.sh;
  const __bf16* vbase = kHasV ? static_cast<const __bf16*>(a.v.ptr) + b * a.v.sb + hk * a.v.sh : nullptr;
  const int row0 = qt * QT + wave * (32 * NQ);  // first query row of this wave

  // key tiles to visit
  // A listed key block of 128 keys is two consecutive 64-key tiles of the list. Listed 32-key blocks are
  // paired up in list order: tile t holds entries 2t and 2t + 1, one in each 32-key half, wherever in
  // the sequence they come from (an odd count leaves the last half empty); the waves that copy the
  // upper half of a tile track entry 2t + 1, the others entry 2t.
  constexpr int tile_shift = (MODE == Mode::kSparse && KB == 2 * kTileK) ? 1 : 0;
  constexpr bool half_blocks = MODE == Mode::kSparse && KB == kTileK / 2;
  constexpr int unit = half_blocks ? kTileK / 2 : kTileK;  // keys per copy unit: a 32-key block or a 64-key tile
  static_assert(!half_blocks || NW >= 2, "32-key blocks need a wave per tile half");
  const int my_half = (half_blocks && 2 * wave >= NW) ? 1 : 0;
  int n, entries = 0;
  const int32_t* cols = nullptr;
  if (MODE == Mode::kSparse) {
    const int32_t* rp = a.row_ptr + (int64_t)bh * (a.nqb + 1) + qt;
    const int beg = rp[0], end = rp[1];
    entries = end - beg;
    n = half_blocks ? (entries + 1) >> 1 : entries << tile_shift;
    cols = a.col_idx + (int64_t)bh * a.cap_per_head + beg;
  } else {
    n = (L + kTileK - 1) / kTileK;
  }
  // A sequence length that is not a multiple of the unit leaves the last one partial: its missing keys
  // are masked to -inf in the softmax and its missing rows never fetched. The second tile of a partial
  // 128-key block may lie wholly past the end: no keys, every logit masked.
  const int last_blk = (L - 1) / unit;        // last key tile (32-key blocks: last block) that exists
  const int tail_keys = L - last_blk * unit;  // keys in it
  auto keys_of = [&](int blk) -> int { return blk > last_blk ? 0 : blk == last_blk ? tail_keys : kTileK; };

  float M[NQ], lsum[NQ];
  f32x16 o[NQ][D / 32];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    M[nq] = 0.f;
    lsum[nq] = 0.f;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int x = 0; x < 16; ++x) o[nq][dt][x] = 0.f;
  }
  f32x16 s_even[NQ], s_odd[NQ];        // logits of the even / odd 32-key sub-tiles in flight
  bf16x8 p_even[NQ][2], p_odd[NQ][2];  // their probabilities

  TileDma<D, NT, false> kdma;
  TileDma<D, NT, true> vdma;
  if constexpr (half_blocks) {
    kdma.init_half(a.k.sl, wave, lane);
    vdma.init_half(a.v.sl, wave, lane);
  } else {
    kdma.init(a.k.sl, wave, lane);
    if (kHasV) vdma.init(a.v.sl, wave, lane);
  }
  KFragAddr<D> kaddr;
  VFragAddr<D> vaddr;
  kaddr.init(lane);
  vaddr.init(lane);

  // Sliding window of key-block numbers: blk_i is the block of tile t+i. For sparse the list is
  // read four tiles ahead of its first use, with a VECTOR load on purpose (an opaque zero keeps the
  // address off the scalar path): scalar loads share a counter with LDS reads and return out of
  // order, which would force every fragment read issued meanwhile to be waited for in full.
  int opaque_zero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(opaque_zero));
  // Tiles past the end of the list repeat the last one: the steady loop prefetches up to two tiles
  // ahead without asking whether they exist, and a repeated copy of a real tile into a free buffer is harmless.
  auto col_at = [&](int t) -> int {  // key TILE number of tile t of the list; 32-key blocks: the block in this wave's copy half
    if (half_blocks) {
      const int e = 2 * t + my_half;
      return cols[(e < entries ? e : (entries > 0 ? entries - 1 : 0)) + opaque_zero];  // a missing half repeats the last block, masked
    }
    const int idx = t < n ? t : (n > 0 ? n - 1 : 0);
    if (MODE != Mode::kSparse) return idx;
    return (cols[(idx >> tile_shift) + opaque_zero] << tile_shift) + (idx & tile_shift);
  };
  int blk0 = 0, blk1 = 0, blk2 = 0, blk3 = 0;
  if (n > 0) {  // a query block that kept nothing has no list entry to read
    blk0 = col_at(0);
    blk1 = col_at(1);
    blk2 = col_at(2);
    blk3 = col_at(3);
  }
  QFrag<D, NQ> qf;  // loaded after the first K/V copies have been issued (below)
  auto uni = [&](int v) -> int { return (MODE == Mode::kSparse) ? __builtin_amdgcn_readfirstlane(v) : v; };
  // keys that exist in tile number `tile` of the list (block `blk`): none past the end of the list
  auto keys_at = [&](int tile, int blk) -> int { return tile < n ? keys_of(uni(blk)) : 0; };
  // 32-key blocks: keys that exist in list entry e (= half e % 2 of tile e / 2). Rows ascend, so only the
  // last entry can be the partial last block of the sequence.
  bool last_is_tail = false;
  if (half_blocks && entries > 0) last_is_tail = __builtin_amdgcn_readfirstlane(cols[entries - 1 + opaque_zero]) == last_blk;
  auto half_keys = [&](int e) -> int { return e < entries ? ((e == entries - 1 && last_is_tail) ? tail_keys : kTileK / 2) : 0; };
  const int64_t slab_rows = (int64_t)(a.L - 1);
  const __amdgpu_buffer_rsrc_t krsrc = make_rsrc(kbase, (slab_rows * a.k.sl + D) * 2);
  const __amdgpu_buffer_rsrc_t vrsrc = make_rsrc(kHasV ? vbase : kbase, kHasV ? (slab_rows * a.v.sl + D) * 2 : 0);
  const int32_t k_tile_bytes = (int32_t)(unit * a.k.sl * 2), v_tile_bytes = (int32_t)(unit * a.v.sl * 2);  // per copy unit
  auto copy_k = [&](int blk, char* dst) { kdma.issue(krsrc, uni(blk) * k_tile_bytes, dst, wave); };
  auto copy_v = [&](int blk, char* dst) { vdma.issue(vrsrc, uni(blk) * v_tile_bytes, dst, wave); };
  // the same for a tile that may be the partial last block (prologue and the last few tiles only)
  // (`ln` is the lane number; the tail loop passes a copy the compiler cannot see through, so that the
  // per-lane addresses of a partial copy are worked out there and not carried across the steady loop.)
  auto copy_k_any = [&](int blk, char* dst, int ln) {
    const int ub = uni(blk) < last_blk ? uni(blk) : last_blk;  // a tile past the end: any real tile will do
    if (ub == last_blk && tail_keys < unit) {
      if constexpr (half_blocks) kdma.issue_partial_half(krsrc, ub * k_tile_bytes, dst, wave, ln, a.k.sl, tail_keys);
      else kdma.issue_partial(krsrc, ub * k_tile_bytes, dst, wave, ln, a.k.sl, tail_keys);
    } else {
      kdma.issue(krsrc, ub * k_tile_bytes, dst, wave);
    }
  };
  auto copy_v_any = [&](int blk, char* dst, int ln) {
    const int ub = uni(blk) < last_blk ? uni(blk) : last_blk;
    if (ub == last_blk && tail_keys < unit) {
      if constexpr (half_blocks) vdma.issue_partial_half(vrsrc, ub * v_tile_bytes, dst, wave, ln, a.v.sl, tail_keys);
      else vdma.issue_partial(vrsrc, ub * v_tile_bytes, dst, wave, ln, a.v.sl, tail_keys);
    } else {
      vdma.issue(vrsrc, ub * v_tile_bytes, dst, wave);
    }
  };
  int lane_tail = lane;

  const float c = a.scale_log2;

  // Softmax of one 32-key sub-tile against the row's reference M: s (fp32 logits) -> p (bf16) and this lane's
  // share `part` of the row sum. The reference is NOT the running maximum: it is fixed by the first sub-tile
  // (its row maximum) and every later probability is 2^(s c - M), whatever its size. fp32 and bf16 carry
  // 2^+-126, the quotient O / l does not depend on the reference, and a logit far below it underflows only
  // where it is negligible beside the first sub-tile's own terms; so no maximum is taken, no accumulator
  // rescaled, as long as the probabilities stay below kOverflow. The caller tests `part` for that after the
  // sub-step's instruction block (a branch inside it would cut the block the scheduling hints apply to) and
  // calls re_reference for the rare sub-tile that fails.
  // masked: apply `valid`, the number of keys of this sub-tile that exist (32 or more = all, 0 or less =
  // none: a phantom tile or the empty half of a partial last block). Unmasked steps skip the 16 selects.
  auto mask_sub = [&](f32x16(&s)[NQ], int valid) {
    const int mine = valid - 8 * g;  // register x of lane (j, g) holds key 16*(x/8) + 8*g + x%8 of the sub-tile
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
      for (int x = 0; x < 16; ++x)
        if (16 * (x >> 3) + (x & 7) >= mine) s[nq][x] = -__builtin_inff();
  };
  auto exp_sub = [&](const f32x16(&s)[NQ], bf16x8(&p)[NQ][2], float(&part)[NQ]) {
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      part[nq] = 0.f;
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        u32x4 pk;
#pragma unroll
        for (int x = 0; x < 8; x += 2) {
          const f32x2 two = {__builtin_amdgcn_exp2f(__builtin_fmaf(s[nq][8 * m + x], c, -M[nq])),
                             __builtin_amdgcn_exp2f(__builtin_fmaf(s[nq][8 * m + x + 1], c, -M[nq]))};
          if (kHasV) pk[x >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
          // The denominator is summed from the unrounded fp32 probabilities with plain adds: the row
          // log-sum-exp that pattern selection reuses needs it to ~1e-7, and the packed bf16 dot
          // instruction, one op cheaper, runs on the matrix pipe and stalls the MFMAs it overlaps.
          part[nq] += two[0];
          part[nq] += two[1];
        }
        if (kHasV) {
          // pin: the probabilities must exist HERE, inside the block that holds the matrix
          // instructions, not be sunk by the compiler past the (rare) branch that follows
          asm volatile("" : "+v"(pk));
          p[nq][m] = __builtin_bit_cast(bf16x8, pk);
        }
      }
      asm volatile("" : "+v"(part[nq]));
    }
  };
  auto softmax_sub = [&](f32x16(&s)[NQ], bf16x8(&p)[NQ][2], float(&part)[NQ], const bool masked, int valid) {
    if (masked) mask_sub(s, valid);
    exp_sub(s, p, part);
  };
  auto row_max = [&](const f32x16(&s)[NQ], int nq) -> float {
    float mx = fmaxf(s[nq][0], s[nq][1]);
#pragma unroll
    for (int x = 2; x < 16; x += 2) mx = fmaxf(fmaxf(mx, s[nq][x]), s[nq][x + 1]);
    return pair_max(mx) * c;
  };
  // true if some lane's 16-key partial sum left the range the fixed reference is good for (wave-uniform)
  auto overflowed = [&](const float(&part)[NQ]) -> bool {
    bool bad = false;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) bad = bad || !(part[nq] < kOverflow);
    return __builtin_amdgcn_ballot_w64(bad) != 0;
  };
  // Out of line, practically never taken: raise the reference of every row to at least this sub-tile's maximum,
  // bring what the row has accumulated (sum and output, including the product issued in this sub-step, whose
  // probabilities had the old reference) to the new one, and redo the sub-tile's probabilities.
  auto re_reference = [&](const f32x16(&s)[NQ], bf16x8(&p)[NQ][2], float(&part)[NQ]) {
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      const float Mn = fmaxf(M[nq], row_max(s, nq));
      const float alpha = __builtin_amdgcn_exp2f(M[nq] - Mn);  // <= 1; exactly 1 where nothing changes
      M[nq] = Mn;
      lsum[nq] *= alpha;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int x = 0; x < 16; ++x) o[nq][dt][x] *= alpha;
    }
    exp_sub(s, p, part);
  };

  // Tile step t (LDS parity P = t & 1) = sub-steps 2t+1 and 2t+2 of the 32-key pipeline.
  // On entry: S(2t+1) in s_odd, P(2t) in p_even, K(t+1) in kbuf[1-P], V(t) in vbuf[P]; the buffers
  // kbuf[P] (held K(t)) and vbuf[1-P] (held V(t-1)) are free and receive K(t+2) and V(t+1).
  //   sub-step 2t+1:  S(2t+2) = K(t+1)[0:32] Q^T,   O += P(2t)   V(t)[0:32],   softmax(2t+1) -> p_odd
  //   sub-step 2t+2:  S(2t+3) = K(t+1)[32:64] Q^T,  O += P(2t+1) V(t)[32:64],  softmax(2t+2) -> p_even
  // Tiles past the end of the list are phantoms: their copy repeats the last real tile and all their
  // keys are masked, so they add nothing, and the same branch-free step serves the whole list. MASKED
  // steps (the last few of a list) count the keys that exist in each sub-tile and use the copy that
  // knows about a partial last block; the others assume full, real tiles.
#define SPARSED_ADD_PART \
  _Pragma("unroll") for (int nq_ = 0; nq_ < NQ; ++nq_) lsum[nq_] += part[nq_];
#define SPARSED_TILE_STEP(P, MASKED, T)                                                            \
  {                                                                                                \
    char* const kb_free = (P) ? kbuf1 : kbuf0;                                                     \
    char* const kb_next = (P) ? kbuf0 : kbuf1;                                                     \
    char* const vb_this = (P) ? vbuf1 : vbuf0;                                                     \
    char* const vb_free = (P) ? vbuf0 : vbuf1;                                                     \
    if (MASKED) {                                                                                  \
      copy_k_any(blk2, kb_free, lane_tail);                                                        \
      if (kHasV) copy_v_any(blk1, vb_free, lane_tail);                                             \
    } else {                                                                                       \
      copy_k(blk2, kb_free);                                                                       \
      if (kHasV) copy_v(blk1, vb_free);                                                            \
    }                                                                                              \
    const int valid_odd = !(MASKED) ? 32 : half_blocks ? half_keys(2 * (T) + 1) : keys_at((T), blk0) - 32;     \
    const int valid_even = !(MASKED) ? 32 : half_blocks ? half_keys(2 * (T) + 2) : keys_at((T) + 1, blk1);     \
    const int blk_new = col_at((T) + 4);                                                           \
    float part[NQ];                                                                                \
    logits_sub<D, NQ, false>(kb_next, 0, kaddr, qf, s_even);                                       \
    if (kHasV) pv_sub<D, NQ, false>(vb_this, 0, vaddr, p_even, o);                                 \
    softmax_sub(s_odd, p_odd, part, (MASKED), valid_odd);                                          \
    sched_substep_interleave<D, NQ, kHasV>();                                                      \
    if (overflowed(part)) re_reference(s_odd, p_odd, part);                                        \
    SPARSED_ADD_PART                                                                               \
    __builtin_amdgcn_sched_barrier(0);                                                             \
    logits_sub<D, NQ, false>(kb_next, 1, kaddr, qf, s_odd);                                        \
    if (kHasV) pv_sub<D, NQ, false>(vb_this, 1, vaddr, p_odd, o);                                  \
    softmax_sub(s_even, p_even, part, (MASKED), valid_even);                                       \
    sched_substep_interleave<D, NQ, kHasV>();                                                      \
    if (overflowed(part)) re_reference(s_even, p_even, part);                                      \
    SPARSED_ADD_PART                                                                               \
    blk0 = blk1;                                                                                   \
    blk1 = blk2;                                                                                   \
    blk2 = blk3;                                                                                   \
    blk3 = blk_new;                                                                                \
    __syncthreads();                                                                               \
  }

  if (n > 0) {
    // prologue: K(0), K(1) (a repeat of K(0) if the list has one tile), V(0) into LDS; S(0); softmax(0)
    copy_k_any(blk0, kbuf0, lane);
    copy_k_any(blk1, kbuf1, lane);
    if (kHasV) copy_v_any(blk0, vbuf0, lane);
    // Q last: loads complete in issue order and the compiler's wait for a block number counts loads issued after it
    // conservatively, so Q rows requested before the copies would have to ARRIVE before the copies could be issued
    // (a second trip to memory in front of the first tiles: 1.2 us of a query block's own timeline, most of which the
    // other work-group of the compute unit hides, so the launch as a whole gains little).
    qf.load(qbase, row0, L, a.q.sl, lane);
    __syncthreads();
    logits_sub<D, NQ, true>(kbuf0, 0, kaddr, qf, s_even);
    logits_sub<D, NQ, true>(kbuf0, 1, kaddr, qf, s_odd);
    {
      // the first sub-tile fixes the reference: its row maximum (it always holds a key that exists)
      mask_sub(s_even, half_blocks ? half_keys(0) : keys_at(0, blk0));
      float part[NQ];
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) M[nq] = fmaxf(row_max(s_even, nq), -1e30f);
      exp_sub(s_even, p_even, part);
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) lsum[nq] = part[nq];
    }
    __syncthreads();  // everyone is done with K(0) before tile step 0 lets K(2) overwrite it

    // An unmasked step at tile t touches tiles t, t+1 (softmax) and t+2 (copy, possibly a repeat). A partial
    // last block must stay out of its reach on all three counts; a full last block only as far as t+1.
    // (with 128-key blocks the last block's second tile may not exist at all: same treatment)
    // (and with 32-key blocks an odd count leaves the last tile's second half empty)
    const int steady_reach = (tail_keys < unit || (tile_shift && !(last_blk & 1)) || (half_blocks && (entries & 1))) ? 4 : 2;
    int t = 0;
    while (t + steady_reach < n) {
      SPARSED_TILE_STEP(0, false, t);
      SPARSED_TILE_STEP(1, false, t + 1);
      t += 2;
    }
    if (t + steady_reach - 1 < n) {  // room for one more unmasked step (t is even here): one masked step fewer
      SPARSED_TILE_STEP(0, false, t);
      t += 1;
    }
    asm volatile("" : "+v"(lane_tail));
    for (; t < n; ++t) {
      if (t & 1) {
        SPARSED_TILE_STEP(1, true, t);
      } else {
        SPARSED_TILE_STEP(0, true, t);
      }
    }
  }
#undef SPARSED_TILE_STEP
#undef SPARSED_ADD_PART

  // Combine the two half-row sums, normalise, store. In the accumulator a lane holds 4 consecutive
  // output columns of ONE row at a time, so direct stores would be 8-byte pieces scattered over 32
  // rows. Each wave instead passes its 32 x D tile through its own slice of the (now idle) K/V
  // buffers and writes whole rows: 16 bytes per lane, D/8 lanes per row. The slice keeps 16-byte
  // slot c of row r at position c ^ (r mod slots) so that neither side has bank conflicts beyond 2-way.
  constexpr int kRowBytes = 2 * D, kSlots = D / 8, kRowsPerStore = 64 / kSlots;
  static_assert(32 * kRowBytes * 2 <= kKBytes && (!kHasV || 32 * kRowBytes * 2 <= kVBytes), "two waves share one buffer");
  // (The lane-derived values of this part are worked out afresh from an opaque copy of the lane number, so that
  // none of them is kept in a register, or spilled, across the tile loop.)
  int lane_e = lane;
  asm volatile("" : "+v"(lane_e));
  const int je = lane_e & 31, ge = lane_e >> 5;
  char* const stage = ((wave >> 1) == 0 ? kbuf0 : (wave >> 1) == 1 ? kbuf1 : (wave >> 1) == 2 ? vbuf0 : vbuf1) + (wave & 1) * (32 * kRowBytes);
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const float ltot = pair_sum(lsum[nq]);
    const int row = row0 + nq * 32 + je;
    if (a.lse != nullptr && ge == 0 && row < L)
      a.lse[(int64_t)bh * a.L + row] = (M[nq] + __builtin_amdgcn_logf(ltot)) * 0.6931471805599453f;
    if (kHasV) {
      const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const f32x2 lo = {o[nq][dt][4 * q4] * inv, o[nq][dt][4 * q4 + 1] * inv};
          const f32x2 hi = {o[nq][dt][4 * q4 + 2] * inv, o[nq][dt][4 * q4 + 3] * inv};
          u32x2 w;
          w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
          w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
          // columns 32*dt + 8*q4 + 4*g .. +3 of row j: slot 4*dt + q4, half g
          *reinterpret_cast<u32x2*>(stage + je * kRowBytes + (((4 * dt + q4) ^ (je & (kSlots - 1))) << 4) + 8 * ge) = w;
        }
      __bf16* const obase = static_cast<__bf16*>(a.o) + b * a.o_sb + h * a.o_sh;
#pragma unroll
      for (int it = 0; it < 32 / kRowsPerStore; ++it) {
        const int r = it * kRowsPerStore + lane_e / kSlots, slot = lane_e % kSlots;
        const u32x4 w = *reinterpret_cast<const u32x4*>(stage + r * kRowBytes + ((slot ^ (r & (kSlots - 1))) << 4));
        const int grow = row0 + nq * 32 + r;
        if (grow < L) *reinterpret_cast<u32x4*>(obase + (int64_t)grow * a.o_sl + slot * 8) = w;  // partial last query tile: rows past L are dropped
      }
    }
  }
#endif
}

int dense_qtile_bf16(int L) {
  if (L <= 0) return 0;
  if (L % 256 == 0) return 256;
  if (L % 128 == 0) return 128;
  if (L % 64 == 0) return 64;
  return L >= 1024 ? 256 : L >= 256 ? 128 : 64;  // partial last tile: waste at most one tile of rows
}

template <int D, int NQ, int NW, Mode MODE, int KB = kTileK>
static hipError_t launch_one(const AttnArgs& a, hipStream_t s) {
  const int64_t total = (int64_t)a.B * a.Hq * a.n_qtiles;
  if (total <= 0 || total > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)total), block(NW * 64);
  hipLaunchKernelGGL((attn_bf16_kernel<D, NQ, NW, MODE, KB>), grid, block, 0, s, a);
  return hipGetLastError();
}

template <int D, Mode MODE>
static hipError_t launch_by_qtile(int qtile, const AttnArgs& a, hipStream_t s) {
  switch (qtile) {
    case 256: return launch_one<D, 1, 8, MODE>(a, s);
    case 128:
      if (MODE == Mode::kSparse && a.block_k == 2 * kTileK) return launch_one<D, 1, 4, MODE, 2 * kTileK>(a, s);
      if (MODE == Mode::kSparse && a.block_k == kTileK / 2) return launch_one<D, 1, 4, MODE, kTileK / 2>(a, s);
      return launch_one<D, 1, 4, MODE>(a, s);
    case 64: return launch_one<D, 1, 2, MODE>(a, s);
    case 32: return launch_one<D, 1, 1, MODE>(a, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_attn_bf16(Mode mode, int D, int block_q, AttnArgs a, hipStream_t s) {
  const int qtile = (mode == Mode::kSparse) ? block_q : dense_qtile_bf16(a.L);
  if (qtile == 0) return hipErrorInvalidValue;
  a.n_qtiles = (a.L + qtile - 1) / qtile;
  if (mode == Mode::kSparse && qtile <= 64) return launch_attn_bf16_splitk(D, qtile, a, s);  // small query blocks
  if (D == 128) {
    if (mode == Mode::kDense) return launch_by_qtile<128, Mode::kDense>(qtile, a, s);
    if (mode == Mode::kSparse) return launch_by_qtile<128, Mode::kSparse>(qtile, a, s);
    return launch_by_qtile<128, Mode::kStats>(qtile, a, s);
  }
  if (D == 64) {
    if (mode == Mode::kDense) return launch_by_qtile<64, Mode::kDense>(qtile, a, s);
    if (mode == Mode::kSparse) return launch_by_qtile<64, Mode::kSparse>(qtile, a, s);
    return launch_by_qtile<64, Mode::kStats>(qtile, a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace sparsed
