// Diagnostic: the rate the bf16 matrix cores sustain on this chip, measured with nothing but matrix
// instructions on register-resident operands. The chip lowers its clock under load and the amount
// depends on how much the operand bits toggle: all-zero operands reach the published peak, operands
// with random mantissas and signs (what real Q, K, V look like) settle well below it. That second
// figure is the ceiling any attention kernel on real data works under, so the benchmark reports it
// beside the published peak.
#include "kernels.hpp"
#include "tile_bf16.hpp"

namespace sparsed {

__global__ __launch_bounds__(512) void mfma_rate_kernel(float* out, int iters, int random_operands) {
#if defined(__HIP_DEVICE_COMPILE__)
  u32x4 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      // two bf16 per word: random sign and mantissa, exponent of 0.5 .. 2
      uint32_t h = (threadIdx.x * 64u + i * 4u + w + blockIdx.x * 7919u) * 2654435761u;
      h ^= h >> 15;
      h *= 2246822519u;
      h ^= h >> 13;
      const uint32_t r = ((h & 0x807f807fu) | 0x3f003f00u) ^ ((h >> 3) & 0x00800080u);
      a[i][w] = random_operands ? r : 0u;
      b[i][w] = random_operands ? ((r * 31u | 0x3f003f00u) & 0xbfffbfffu) : 0u;
    }
  f32x16 acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[u][x] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int u = 0; u < 4; ++u)
        acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[(i + u) & 7]),
                                                         acc[u], 0, 0, 0);
    // keep the accumulators finite and the loop opaque
#pragma unroll
    for (int u = 0; u < 4; ++u) asm volatile("" : "+v"(acc[u]));
  }
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int x = 0; x < 16; ++x) s += acc[u][x];
  out[blockIdx.x * 512 + threadIdx.x] = s;
#endif
}

// 256 work-groups of 8 waves (two per SIMD on a 256-CU part); scratch must hold kProbeFloats floats.
hipError_t launch_mfma_rate(float* scratch, int iters, int random_operands, hipStream_t s) {
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(kProbeGroups), dim3(512), 0, s, scratch, iters, random_operands);
  return hipGetLastError();
}

}  // namespace sparsed
