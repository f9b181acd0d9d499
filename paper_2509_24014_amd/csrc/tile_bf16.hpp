// Device-side building blocks of the bf16 kernels for gfx950 (wave64, v_mfma_f32_32x32x16_bf16).
//
// Formulation. A wave owns 32*NQ query rows. For one tile of 64 keys it computes the TRANSPOSED
// logits  S^T[key, query] = K . Q^T  so that in the 32x32 accumulator layout
//     lane = 32*g + j  holds query j,  register v  holds row 8*(v/4) + 4*g + (v%4)
// every lane owns ONE query and 16 keys of it: the softmax row maximum and row sum need one
// exchange between lanes j and j+32 and nothing else, and the running maximum, running sum and
// rescale factor of a query are per-lane scalars.
//
// The rows of the K operand are fed in a permuted order (bits 2 and 3 of the row swapped) so that
// lane (j, g) ends up holding, in registers 8m .. 8m+7 of the accumulator, the 8 CONSECUTIVE keys
// 16m + 8g .. 16m + 8g + 7 of the 32-key sub-tile. Those 8 probabilities, rounded to bf16, are
// exactly the B operand of the second product  O^T[d, query] += V^T[d, key] . P^T[key, query],
// whose A operand is 8 consecutive keys of one column d of V: one 16-byte read from a K-major
// (transposed) copy of the V tile in LDS. The output accumulator again has one query per lane.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sparsed {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kTileK = 64;  // keys per K/V tile of the bf16 kernels (= block_k)

// Lanes j and j+32 hold the two halves of one query's keys. v_permlane32_swap exchanges the upper
// 32 lanes of its first operand with the lower 32 lanes of its second; fed the same value twice it
// returns {x[lane % 32], x[32 + lane % 32]} in every lane, i.e. both halves of the pair.
__device__ __forceinline__ float pair_max(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// Work-groups are dispatched round-robin over the 8 XCDs, each with its own L2. Map the
// hardware id so that every XCD walks one contiguous range of logical ids: neighbours in the
// logical order (same head, adjacent query tiles) then share an L2.
__device__ __forceinline__ int xcd_remap(int wg, int total) {
  const int q = total >> 3, r = total & 7;
  const int x = wg & 7, n = wg >> 3;
  return x * q + (x < r ? x : r) + n;
}

// ---- K tile in LDS: [64 keys][D] bf16, 16-byte chunks XOR-swizzled per row --------------------
// Row r keeps chunk c at position c ^ kswz(r). kswz is distinct over the 8 rows an aligned group
// of 8 lanes reads (rows {0..3, 8..11} or {4..7, 12..15} after the row permutation).
__device__ __forceinline__ int kswz(int r) { return (r & 3) | ((r >> 1) & 4); }
// Permutation of the K rows fed to the first product: swap bits 2 and 3.
__device__ __forceinline__ int krow_perm(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

template <int D>
__device__ __forceinline__ int k_lds_offset(int row, int chunk) {  // bytes
  return row * (2 * D) + ((chunk ^ kswz(row)) << 4);
}

// ---- V tile in LDS, transposed: [D][64 keys] bf16 (128 bytes per row) -------------------------
// Row d keeps the 16-byte chunk c (keys 8c .. 8c+7) at position c ^ vswz(d).
__device__ __forceinline__ int vswz(int d) { return ((d >> 3) ^ d) & 7; }
__device__ __forceinline__ int vt_lds_offset(int d, int chunk) {  // bytes
  return d * (2 * kTileK) + ((chunk ^ vswz(d)) << 4);
}

// Cooperative global -> register -> LDS staging of one K tile by NT threads.
template <int D, int NT>
struct KStage {
  static constexpr int kChunks = kTileK * D / 8;  // 16-byte chunks in the tile
  static constexpr int kPer = kChunks / NT;
  static_assert(kChunks % NT == 0, "K tile must split evenly");
  u32x4 r[kPer];

  __device__ __forceinline__ void load(const __bf16* tile, int64_t stride_l, int tid) {
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
      const int id = c * NT + tid;
      const int row = id / (D / 8), ch = id % (D / 8);
      r[c] = *reinterpret_cast<const u32x4*>(tile + (int64_t)row * stride_l + ch * 8);
    }
  }
  __device__ __forceinline__ void store(char* lds, int tid) const {
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
      const int id = c * NT + tid;
      const int row = id / (D / 8), ch = id % (D / 8);
      *reinterpret_cast<u32x4*>(lds + k_lds_offset<D>(row, ch)) = r[c];
    }
  }
};

// Cooperative staging of one V tile, transposed on the way into LDS. A unit is 4 consecutive keys
// x 8 consecutive columns: four 16-byte global loads, then for each of the 8 columns the four keys'
// values are packed (v_perm_b32) into one 8-byte LDS write. The unit -> thread map makes every
// aligned group of 8 lanes read one full 128-byte line and every aligned group of 16 lanes write
// 16 distinct 8-byte LDS slots.
template <int D, int NT>
struct VStage {
  static constexpr int kUnits = (kTileK / 4) * (D / 8);
  static constexpr int kPer = kUnits / NT;
  static_assert(kUnits % NT == 0, "V tile must split evenly");
  u32x4 r[kPer][4];

  __device__ static __forceinline__ void decode(int u, int& kq, int& dc) {
    if (D == 128) {
      dc = (u & 7) | ((u >> 1) & 8);
      kq = ((u >> 3) & 1) | ((u >> 4) & 14);
    } else {
      dc = u & 7;
      kq = (u >> 3) & 15;
    }
  }
  __device__ __forceinline__ void load(const __bf16* tile, int64_t stride_l, int tid) {
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
      int kq, dc;
      decode(c * NT + tid, kq, dc);
#pragma unroll
      for (int x = 0; x < 4; ++x)
        r[c][x] = *reinterpret_cast<const u32x4*>(tile + (int64_t)(4 * kq + x) * stride_l + dc * 8);
    }
  }
  __device__ __forceinline__ void store(char* lds, int tid) const {
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
      int kq, dc;
      decode(c * NT + tid, kq, dc);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        u32x2 w;
        w[0] = __builtin_amdgcn_perm(r[c][1][e >> 1], r[c][0][e >> 1], sel);
        w[1] = __builtin_amdgcn_perm(r[c][3][e >> 1], r[c][2][e >> 1], sel);
        const int d = dc * 8 + e;
        *reinterpret_cast<u32x2*>(lds + vt_lds_offset(d, kq >> 1) + ((kq & 1) << 3)) = w;
      }
    }
  }
};

// Q fragments of a wave: B operand of the first product. Lane (j, g) holds, for k-step kk, the 8
// values Q[row j][16*kk + 8*g .. +7].
template <int D, int NQ>
struct QFrag {
  bf16x8 f[NQ][D / 16];
  __device__ __forceinline__ void load(const __bf16* qrow0, int64_t stride_l, int lane) {
    const int j = lane & 31, g = lane >> 5;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk)
        f[nq][kk] = *reinterpret_cast<const bf16x8*>(qrow0 + (int64_t)(nq * 32 + j) * stride_l + kk * 16 + g * 8);
  }
};

// S^T for one 64-key tile: s[nq][ks] (ks = 32-key sub-tile) = K_sub . Q_nq^T, fp32.
template <int D, int NQ>
__device__ __forceinline__ void logits_tile(const char* klds, const QFrag<D, NQ>& q, int lane,
                                            f32x16 (&s)[NQ][2]) {
  const int i = lane & 31, g = lane >> 5;
  const int prow = krow_perm(i);
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
      for (int x = 0; x < 16; ++x) s[nq][ks][x] = 0.f;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(klds + k_lds_offset<D>(32 * ks + prow, 2 * kk + g));
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq)
        s[nq][ks] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, q.f[nq][kk], s[nq][ks], 0, 0, 0);
    }
  }
}

}  // namespace sparsed
