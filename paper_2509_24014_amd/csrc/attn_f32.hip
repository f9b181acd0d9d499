// fp32 flash-attention forward for gfx950: dense (Eq. 1), block-sparse (Eq. 3 / Eq. 4) and the
// statistics-only pass. fp32 inputs, fp32 matrix cores (32x32x2), fp32 softmax, fp32 output:
// this is the path held to 1e-5 against the fp64 reference, not the throughput path.
//
// One work-group of NW waves owns 32*NW query rows of one (batch, head); each wave owns 32 rows.
// Keys are walked in 32-key tiles staged through LDS (single buffer, two barriers per tile).
#include "kernels.hpp"
#include "tile_f32.hpp"

namespace sparsed {

template <int D, int NW, Mode MODE>
__global__ __launch_bounds__(NW * 64) void attn_f32_kernel(const AttnArgs a) {
  constexpr int NT = NW * 64;
  constexpr int QT = 32 * NW;
  constexpr bool kHasV = MODE != Mode::kStats;
  using T = TileF32<D>;
  __shared__ __attribute__((aligned(16))) float klds[T::kKFloats];
  __shared__ __attribute__((aligned(16))) float vlds[kHasV ? T::kVFloats : 4];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31, g = lane >> 5;

  const int lid = xcd_remap_f(blockIdx.x, gridDim.x);
  const int qt = lid % a.n_qtiles;
  const int bh = lid / a.n_qtiles;
  const int b = bh / a.Hq, h = bh % a.Hq;
  const int hk = h / (a.Hq / a.Hkv);
  int L = a.L;  // length of this batch element
  if (a.seq_lens != nullptr) {
    const int len = a.seq_lens[b];
    L = len < a.L ? len : a.L;
  }
  if (qt * QT >= L) return;  // a query tile wholly past the end (uniform over the work-group)

  const float* qbase = static_cast<const float*>(a.q.ptr) + b * a.q.sb + h * a.q.sh;
  const float* kbase = static_cast<const float*>(a.k.ptr) + b * a.k.sb + hk * a.k.sh;
  const float* vbase = kHasV ? static_cast<const float*>(a.v.ptr) + b * a.v.sb + hk * a.v.sh : nullptr;
  const int row0 = qt * QT + wave * 32;

  const int tiles_per_block = (MODE == Mode::kSparse) ? a.block_k / kTileKF : 1;
  int n_tiles;
  const int32_t* cols = nullptr;
  if (MODE == Mode::kSparse) {
    const int32_t* rp = a.row_ptr + (int64_t)bh * (a.nqb + 1) + qt;
    const int beg = rp[0], end = rp[1];
    n_tiles = (end - beg) * tiles_per_block;
    cols = a.col_idx + (int64_t)bh * a.cap_per_head + beg;
  } else {
    n_tiles = (L + kTileKF - 1) / kTileKF;
  }

  QFragF32<D> qf;
  qf.load(qbase, row0, L, a.q.sl, lane);

  float M = -1e30f, lsum = 0.f;
  f32x16 o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int x = 0; x < 16; ++x) o[dt][x] = 0.f;

  const float c = a.scale_log2;
  for (int t = 0; t < n_tiles; ++t) {
    int key0;
    if (MODE == Mode::kSparse) {
      const int blk = __builtin_amdgcn_readfirstlane(cols[t / tiles_per_block]);
      key0 = blk * a.block_k + (t % tiles_per_block) * kTileKF;
    } else {
      key0 = t * kTileKF;
    }
    // keys of this tile that exist: fewer than 32 only at the end of a sequence whose length is not a
    // multiple of the tile; a tile wholly past the end (the later tiles of a partial key block) is skipped
    const int valid = L - key0 < kTileKF ? L - key0 : kTileKF;
    if (valid <= 0) continue;  // uniform over the work-group
    __syncthreads();  // everyone is done reading the previous tile
    T::template stage<NT>(kbase + (int64_t)key0 * a.k.sl, a.k.sl, klds, T::kKStride, tid, valid);
    if (kHasV) T::template stage<NT>(vbase + (int64_t)key0 * a.v.sl, a.v.sl, vlds, D, tid, valid);
    __syncthreads();

    f32x16 s = logits_tile_f32<D>(klds, qf, lane);
    if (valid < kTileKF) {
#pragma unroll
      for (int x = 0; x < 16; ++x)
        if (8 * (x / 4) + 4 * g + (x % 4) >= valid) s[x] = -__builtin_inff();
    }

    float mx = s[0];
#pragma unroll
    for (int x = 1; x < 16; ++x) mx = fmaxf(mx, s[x]);
    mx = fmaxf(mx, other_half_f(mx));
    const float Mn = fmaxf(M, mx * c);
    const float alpha = exp2f(M - Mn);
    M = Mn;
    float part = 0.f;
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      s[x] = exp2f(__builtin_fmaf(s[x], c, -Mn));
      part += s[x];
    }
    lsum = lsum * alpha + part;

    if (kHasV) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt) {
#pragma unroll
        for (int x = 0; x < 16; ++x) o[dt][x] *= alpha;
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          const int key = 8 * (x / 4) + 4 * g + (x % 4);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x2f32(vlds[key * D + 32 * dt + j], s[x], o[dt], 0, 0, 0);
        }
      }
    }
  }

  const float ltot = lsum + other_half_f(lsum);
  const int row = row0 + j;
  if (row >= L) return;  // partial last query tile
  if (a.lse != nullptr && g == 0) a.lse[(int64_t)bh * a.L + row] = (M + log2f(ltot)) * 0.6931471805599453f;
  if (kHasV) {
    const float inv = ltot > 0.f ? 1.0f / ltot : 0.f;
    float* orow = static_cast<float*>(a.o) + b * a.o_sb + h * a.o_sh + (int64_t)row * a.o_sl;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 w;
#pragma unroll
        for (int x = 0; x < 4; ++x) w[x] = o[dt][4 * q4 + x] * inv;
        *reinterpret_cast<f32x4*>(orow + 32 * dt + 8 * q4 + 4 * g) = w;
      }
  }
}

int dense_qtile_f32(int L) {
  if (L <= 0) return 0;
  if (L % 128 == 0) return 128;
  if (L % 64 == 0) return 64;
  if (L % 32 == 0) return 32;
  return L >= 256 ? 128 : L >= 64 ? 64 : 32;  // partial last tile
}

template <int D, int NW, Mode MODE>
static hipError_t launch_one_f32(const AttnArgs& a, hipStream_t s) {
  const int64_t total = (int64_t)a.B * a.Hq * a.n_qtiles;
  if (total <= 0 || total > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL((attn_f32_kernel<D, NW, MODE>), dim3((unsigned)total), dim3(NW * 64), 0, s, a);
  return hipGetLastError();
}

template <int D, Mode MODE>
static hipError_t launch_by_qtile_f32(int qtile, const AttnArgs& a, hipStream_t s) {
  switch (qtile) {
    case 128: return launch_one_f32<D, 4, MODE>(a, s);
    case 64: return launch_one_f32<D, 2, MODE>(a, s);
    case 32: return launch_one_f32<D, 1, MODE>(a, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_attn_f32(Mode mode, int D, int block_q, AttnArgs a, hipStream_t s) {
  const int qtile = (mode == Mode::kSparse) ? block_q : dense_qtile_f32(a.L);
  if (qtile == 0) return hipErrorInvalidValue;
  a.n_qtiles = (a.L + qtile - 1) / qtile;
  if (D == 128) {
    if (mode == Mode::kDense) return launch_by_qtile_f32<128, Mode::kDense>(qtile, a, s);
    if (mode == Mode::kSparse) return launch_by_qtile_f32<128, Mode::kSparse>(qtile, a, s);
    return launch_by_qtile_f32<128, Mode::kStats>(qtile, a, s);
  }
  if (D == 64) {
    if (mode == Mode::kDense) return launch_by_qtile_f32<64, Mode::kDense>(qtile, a, s);
    if (mode == Mode::kSparse) return launch_by_qtile_f32<64, Mode::kSparse>(qtile, a, s);
    return launch_by_qtile_f32<64, Mode::kStats>(qtile, a, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace sparsed
