// Device-side building blocks of the fp32 kernels for gfx950 (wave64, v_mfma_f32_32x32x2_f32).
//
// Same transposed formulation as the bf16 kernels: S^T[key, query] = K . Q^T puts one query in
// each lane (lane = 32*g + j holds query j; register v holds key row 8*(v/4) + 4*g + (v%4) of the
// 32-key tile). With a contraction depth of 2 per instruction, lane (j, g) supplies element g of
// the pair, so the second product O^T += V^T . P^T can take accumulator register v directly as its
// B operand for the key pair {8*(v/4) + (v%4), 8*(v/4) + 4 + (v%4)} and V is read row-major.
// Everything stays fp32: inputs, both products, softmax.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sparsed {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kTileKF = 32;  // keys per K/V tile of the fp32 kernels

__device__ __forceinline__ float other_half_f(float x) { return __shfl_xor(x, 32, 64); }

__device__ __forceinline__ float wave_sum_f(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

__device__ __forceinline__ int xcd_remap_f(int wg, int total) {
  const int q = total >> 3, r = total & 7;
  const int x = wg & 7, n = wg >> 3;
  return x * q + (x < r ? x : r) + n;
}

// K tile in LDS: [32 keys][D + 1] floats (one float of padding per row: lanes reading the same
// column of 32 different rows hit 32 different banks). V tile: [32 keys][D] floats, unpadded.
template <int D>
struct TileF32 {
  static constexpr int kKStride = D + 1;
  static constexpr int kKFloats = kTileKF * kKStride;
  static constexpr int kVFloats = kTileKF * D;

  // Cooperative copy of a [32, D] tile (row stride stride_l) into LDS with row stride dst_stride.
  // Only the first `rows` rows exist (fewer than 32 in the last tile of a sequence whose length is
  // not a multiple of 32); the others are filled from the last existing row and masked by the caller.
  template <int NT>
  __device__ static __forceinline__ void stage(const float* tile, int64_t stride_l, float* lds,
                                               int dst_stride, int tid, int rows) {
    constexpr int kVec = kTileKF * D / 4;  // float4 pieces
    for (int id = tid; id < kVec; id += NT) {
      const int row = id / (D / 4), c4 = id % (D / 4);
      const int src = row < rows ? row : rows - 1;
      const f32x4 x = *reinterpret_cast<const f32x4*>(tile + (int64_t)src * stride_l + c4 * 4);
      float* dst = lds + row * dst_stride + c4 * 4;
      dst[0] = x[0];
      dst[1] = x[1];
      dst[2] = x[2];
      dst[3] = x[3];
    }
  }
};

// Q fragments: lane (j, g) holds Q[row j][2*kk + g] for kk = 0 .. D/2-1.
template <int D>
struct QFragF32 {
  float f[D / 2];
  // qhead: row 0 of the (batch, head) slab; rows at or past L are read from row L-1 (results dropped by the caller)
  __device__ __forceinline__ void load(const float* qhead, int row0, int L, int64_t stride_l, int lane) {
    const int j = lane & 31, g = lane >> 5;
    const int row = row0 + j < L ? row0 + j : L - 1;
    const float* r = qhead + (int64_t)row * stride_l;
#pragma unroll
    for (int kk = 0; kk < D / 2; ++kk) f[kk] = r[2 * kk + g];
  }
};

// S^T for one 32-key tile.
template <int D>
__device__ __forceinline__ f32x16 logits_tile_f32(const float* klds, const QFragF32<D>& q, int lane) {
  const int i = lane & 31, g = lane >> 5;
  f32x16 s;
#pragma unroll
  for (int x = 0; x < 16; ++x) s[x] = 0.f;
  const float* krow = klds + i * TileF32<D>::kKStride + g;
#pragma unroll
  for (int kk = 0; kk < D / 2; ++kk)
    s = __builtin_amdgcn_mfma_f32_32x32x2f32(krow[2 * kk], q.f[kk], s, 0, 0, 0);
  return s;
}

}  // namespace sparsed
