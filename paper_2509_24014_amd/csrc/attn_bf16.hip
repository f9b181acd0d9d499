// bf16 flash-attention forward for gfx950: dense (Eq. 1), block-sparse (Eq. 3 / Eq. 4) and the
// statistics-only pass (row log-sum-exp of Eq. 1's logits) used by pattern selection.
//
// One work-group owns QT = 32*NQ*NW query rows of one (batch, head) and walks 64-key tiles:
// all of them (dense, stats) or the key blocks listed for its query block (sparse; QT == block_q,
// so all rows of the group share one list). K and V tiles are staged global -> registers -> LDS,
// double-buffered, one barrier per tile; V is transposed on the way in (tile_bf16.hpp).
// Softmax is online (running max / running sum per query, fp32); probabilities are rounded to
// bf16 for the second matrix product; the output accumulator is fp32.
#include "kernels.hpp"
#include "tile_bf16.hpp"

namespace sparsed {

// EXACT_SUM: accumulate the softmax denominator from the unrounded fp32 probabilities. Used whenever
// the row log-sum-exp is an output (pattern selection needs it to ~1e-7), at one more VALU op per key.
template <int D, int NQ, int NW, Mode MODE, bool EXACT_SUM>
__global__ __launch_bounds__(NW * 64, (NW >= 4 ? 2 : 1)) void attn_bf16_kernel(const AttnArgs a) {
  constexpr int NT = NW * 64;
  constexpr int QT = 32 * NQ * NW;
  constexpr bool kHasV = MODE != Mode::kStats;
  constexpr int kKBytes = kTileK * D * 2;
  constexpr int kVBytes = kHasV ? D * kTileK * 2 : 0;
  __shared__ __attribute__((aligned(16))) char lds[2 * (kKBytes + kVBytes)];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, g = lane >> 5;

  const int lid = xcd_remap(blockIdx.x, gridDim.x);
  const int qt = lid % a.n_qtiles;
  const int bh = lid / a.n_qtiles;
  const int b = bh / a.Hq, h = bh % a.Hq;
  const int hk = h / (a.Hq / a.Hkv);

  const __bf16* qbase = static_cast<const __bf16*>(a.q.ptr) + b * a.q.sb + h * a.q.sh;
  const __bf16* kbase = static_cast<const __bf16*>(a.k.ptr) + b * a.k.sb + hk * a.k.sh;
  const __bf16* vbase = kHasV ? static_cast<const __bf16*>(a.v.ptr) + b * a.v.sb + hk * a.v.sh : nullptr;
  const int row0 = qt * QT + wave * (32 * NQ);  // first query row of this wave

  // key tiles to visit
  int n_tiles;
  const int32_t* cols = nullptr;
  if (MODE == Mode::kSparse) {
    const int32_t* rp = a.row_ptr + (int64_t)bh * (a.nqb + 1) + qt;
    const int beg = rp[0], end = rp[1];
    n_tiles = end - beg;
    cols = a.col_idx + (int64_t)bh * a.cap_per_head + beg;
  } else {
    n_tiles = a.L / kTileK;
  }

  QFrag<D, NQ> qf;
  qf.load(qbase + (int64_t)row0 * a.q.sl, a.q.sl, lane);

  float M[NQ], lsum[NQ];
  f32x16 o[NQ][D / 32];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    M[nq] = -1e30f;
    lsum[nq] = 0.f;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int x = 0; x < 16; ++x) o[nq][dt][x] = 0.f;
  }

  // Staging roles. With 8 waves the upper four stage K and the lower four stage V; otherwise
  // every thread stages its share of both (V units may be fewer than threads).
  constexpr int NTK = (NT == 512) ? 256 : NT;
  constexpr int kVUnits = (kTileK / 4) * (D / 8);
  constexpr int NTV = (NT == 512) ? 256 : (NT < kVUnits ? NT : kVUnits);
  constexpr int NTV2 = NTV < kVUnits ? NTV : kVUnits;
  const int ktid = (NT == 512 && kHasV) ? tid - 256 : tid;
  const bool k_role = (NT == 512 && kHasV) ? (tid >= 256) : (tid < NTK);
  const bool v_role = kHasV && tid < NTV2;
  KStage<D, NTK> kst;
  VStage<D, NTV2> vst;
  auto tile_key0 = [&](int t) -> int {
    const int blk = (MODE == Mode::kSparse) ? __builtin_amdgcn_readfirstlane(cols[t]) : t;
    return blk * kTileK;
  };
  auto issue = [&](int t) {
    const int key0 = tile_key0(t);
    if (k_role) kst.load(kbase + (int64_t)key0 * a.k.sl, a.k.sl, ktid);
    if (v_role) vst.load(vbase + (int64_t)key0 * a.v.sl, a.v.sl, tid);
  };
  auto commit = [&](int buf) {
    char* base = lds + buf * (kKBytes + kVBytes);
    if (k_role) kst.store(base, ktid);
    if (v_role) vst.store(base + kKBytes, tid);
  };

  if (n_tiles > 0) {
    issue(0);
    commit(0);
  }
  __syncthreads();

  const float c = a.scale_log2;
  constexpr float kLazyLog2 = 8.0f;
  for (int t = 0; t < n_tiles; ++t) {
    const char* kl = lds + (t & 1) * (kKBytes + kVBytes);
    const char* vl = kl + kKBytes;
    if (t + 1 < n_tiles) issue(t + 1);

    f32x16 s[NQ][2];
    logits_tile<D, NQ>(kl, qf, lane, s);

    bf16x8 pb[NQ][4];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      // row maximum of this tile (v_max3 chain over the lane's 32 keys, then the partner half)
      float mx = fmaxf(s[nq][0][0], s[nq][0][1]);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int x = (ks == 0 ? 2 : 0); x < 16; x += 2) mx = fmaxf(fmaxf(mx, s[nq][ks][x]), s[nq][ks][x + 1]);
      mx = pair_max(mx);
      // Lazy reference maximum: it is raised only when the tile maximum exceeds it by more than
      // kLazyLog2 (probabilities then stay below 2^kLazyLog2, harmless in fp32 / bf16); the common
      // case skips the rescale of the running sum and of the output accumulator altogether.
      const float cand = mx * c;
      const bool raise = cand > M[nq] + kLazyLog2;
      if (__builtin_amdgcn_ballot_w64(raise) != 0) {
        const float Mn = raise ? cand : M[nq];
        const float alpha = __builtin_amdgcn_exp2f(M[nq] - Mn);
        M[nq] = Mn;
        lsum[nq] *= alpha;
        if (kHasV) {
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int x = 0; x < 16; ++x) o[nq][dt][x] *= alpha;
        }
      }
      const float Mr = M[nq];
      float part = 0.f;
      if (kHasV && !EXACT_SUM) {
        // p = 2^(s*c - M), rounded to bf16 in pairs; the row sum is taken over the ROUNDED values
        // (v_dot2 with ones) so that numerator and denominator see the same probabilities.
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int m = 0; m < 2; ++m) {
            u32x4 pk;
#pragma unroll
            for (int x = 0; x < 8; x += 2) {
              const f32x2 two = {__builtin_amdgcn_exp2f(__builtin_fmaf(s[nq][ks][8 * m + x], c, -Mr)),
                                 __builtin_amdgcn_exp2f(__builtin_fmaf(s[nq][ks][8 * m + x + 1], c, -Mr))};
              const bf16x2 r = __builtin_convertvector(two, bf16x2);
              part = __builtin_amdgcn_fdot2_f32_bf16(r, ones, part, false);
              pk[x >> 1] = __builtin_bit_cast(uint32_t, r);
            }
            pb[nq][2 * ks + m] = __builtin_bit_cast(bf16x8, pk);
          }
      } else {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int m = 0; m < 2; ++m) {
            u32x4 pk;
#pragma unroll
            for (int x = 0; x < 8; x += 2) {
              const f32x2 two = {__builtin_amdgcn_exp2f(__builtin_fmaf(s[nq][ks][8 * m + x], c, -Mr)),
                                 __builtin_amdgcn_exp2f(__builtin_fmaf(s[nq][ks][8 * m + x + 1], c, -Mr))};
              part += two[0];
              part += two[1];
              if (kHasV) pk[x >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
            }
            if (kHasV) pb[nq][2 * ks + m] = __builtin_bit_cast(bf16x8, pk);
          }
      }
      lsum[nq] += part;
    }

    if (kHasV) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int mp = 0; mp < 4; ++mp) {
          const bf16x8 vf = *reinterpret_cast<const bf16x8*>(vl + vt_lds_offset(32 * dt + j, 2 * mp + g));
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq)
            o[nq][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[nq][mp], o[nq][dt], 0, 0, 0);
        }
    }

    if (t + 1 < n_tiles) commit((t + 1) & 1);
    __syncthreads();
  }

  // epilogue: combine the two half-row sums, normalise, store
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const float ltot = pair_sum(lsum[nq]);
    const int row = row0 + nq * 32 + j;
    if (a.lse != nullptr && g == 0)
      a.lse[(int64_t)bh * a.L + row] = (M[nq] + __builtin_amdgcn_logf(ltot)) * 0.6931471805599453f;
    if (kHasV) {
      const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
      __bf16* orow = static_cast<__bf16*>(a.o) + b * a.o_sb + h * a.o_sh + (int64_t)row * a.o_sl;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const f32x2 lo = {o[nq][dt][4 * q4] * inv, o[nq][dt][4 * q4 + 1] * inv};
          const f32x2 hi = {o[nq][dt][4 * q4 + 2] * inv, o[nq][dt][4 * q4 + 3] * inv};
          const bf16x2 l2 = __builtin_convertvector(lo, bf16x2);
          const bf16x2 h2 = __builtin_convertvector(hi, bf16x2);
          u32x2 w;
          w[0] = *reinterpret_cast<const uint32_t*>(&l2);
          w[1] = *reinterpret_cast<const uint32_t*>(&h2);
          *reinterpret_cast<u32x2*>(orow + 32 * dt + 8 * q4 + 4 * g) = w;
        }
    }
  }
}

int dense_qtile_bf16(int L) {
  if (L <= 0 || L % 64 != 0) return 0;
  if (L % 256 == 0) return 256;
  if (L % 128 == 0) return 128;
  return 64;
}

template <int D, int NQ, int NW, Mode MODE>
static hipError_t launch_one(const AttnArgs& a, hipStream_t s) {
  const int64_t total = (int64_t)a.B * a.Hq * a.n_qtiles;
  if (total <= 0 || total > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)total), block(NW * 64);
  if (MODE == Mode::kStats || (MODE == Mode::kDense && a.lse != nullptr))
    hipLaunchKernelGGL((attn_bf16_kernel<D, NQ, NW, MODE, true>), grid, block, 0, s, a);
  else
    hipLaunchKernelGGL((attn_bf16_kernel<D, NQ, NW, MODE, false>), grid, block, 0, s, a);
  return hipGetLastError();
}

template <int D, Mode MODE>
static hipError_t launch_by_qtile(int qtile, const AttnArgs& a, hipStream_t s) {
  switch (qtile) {
    case 256: return launch_one<D, 1, 8, MODE>(a, s);
    case 128: return launch_one<D, 1, 4, MODE>(a, s);
    case 64: return launch_one<D, 1, 2, MODE>(a, s);
    case 32: return launch_one<D, 1, 1, MODE>(a, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_attn_bf16(Mode mode, int D, int block_q, AttnArgs a, hipStream_t s) {
  const int qtile = (mode == Mode::kSparse) ? block_q : dense_qtile_bf16(a.L);
  if (qtile == 0 || a.L % qtile != 0) return hipErrorInvalidValue;
  a.n_qtiles = a.L / qtile;
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
