// Diagnostics. First: the rate the bf16 matrix cores sustain on this chip, measured with nothing but matrix
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

// The vector unit alone: 64 independent fp32 instructions per wave and iteration on 16 register chains, either
// fused multiply-adds or base-2 exponentials. The ratio of the two rates is what an exponential costs in units
// of an ordinary vector instruction, the figure the softmax side of every kernel here is priced with.
template <int OP>
__global__ __launch_bounds__(512) void valu_rate_kernel(float* out, int iters) {
#if defined(__HIP_DEVICE_COMPILE__)
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = -0.5f - 0.001f * (float)((threadIdx.x + i) & 31);
  const float m = 0.999f, b = -0.0005f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        // exp2 of a value in (-1, 0) is in (0.5, 1); its negative is again in (-1, -0.5): the chain stays in range
        if (OP == 1) x[i] = -__builtin_amdgcn_exp2f(x[i]);  // the negation is a source modifier, not an instruction
        else x[i] = __builtin_fmaf(x[i], m, b);
      }
#pragma unroll
    for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(x[i]));
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += x[i];
  out[blockIdx.x * 512 + threadIdx.x] = s;
#endif
}

hipError_t launch_valu_rate(float* scratch, int iters, int op, hipStream_t s) {
  if (op == 1) hipLaunchKernelGGL(valu_rate_kernel<1>, dim3(kProbeGroups), dim3(512), 0, s, scratch, iters);
  else hipLaunchKernelGGL(valu_rate_kernel<0>, dim3(kProbeGroups), dim3(512), 0, s, scratch, iters);
  return hipGetLastError();
}

// The inner loop of attention with everything but its instruction mix taken away: per matrix instruction, VPM
// independent fp32 vector instructions (every fourth an exp2, the others fma) and, if LDS, one 16-byte-per-lane LDS
// read that supplies the next matrix operand (attention reads 1 KiB of K or V per 32x32x16 instruction and wave).
// No dependencies between the streams, no barriers, no global loads: what this reaches is the ceiling for a kernel
// with that mix on this chip.
template <int VPM, bool LDS>
__global__ __launch_bounds__(512) void mix_rate_kernel(float* out, int iters) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr int kWords = 8192;  // 32 KiB walked by every wave
  __shared__ __attribute__((aligned(16))) uint32_t lds[LDS ? kWords : 4];
  u32x4 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      uint32_t h = (threadIdx.x * 64u + i * 4u + w + blockIdx.x * 7919u) * 2654435761u;
      h ^= h >> 15;
      h *= 2246822519u;
      h ^= h >> 13;
      const uint32_t r = ((h & 0x807f807fu) | 0x3f003f00u) ^ ((h >> 3) & 0x00800080u);
      a[i][w] = r;
      b[i][w] = (r * 31u | 0x3f003f00u) & 0xbfffbfffu;
    }
  if (LDS) {
    for (int i = threadIdx.x; i < kWords; i += 512) lds[i] = 0x3f003f00u | ((i * 2654435761u) & 0x807f807fu);
    __syncthreads();
  }
  const u32x4* lp = reinterpret_cast<const u32x4*>(lds) + (threadIdx.x & 63);
  u32x4 nxt[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) nxt[u] = LDS ? lp[u * 64] : a[u];
  f32x16 acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int x = 0; x < 16; ++x) acc[u][x] = 0.f;
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = -0.5f - 0.001f * (float)((threadIdx.x + i) & 31);
  const float m = 0.999f, c = -0.0005f;
  constexpr int VPG = 4 * VPM;  // vector instructions per group of 4 matrix instructions
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      u32x4 cur[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) cur[u] = LDS ? nxt[u] : a[(g + u) & 7];
      if (LDS) {
#pragma unroll
        for (int u = 0; u < 4; ++u) nxt[u] = lp[((g + 1) & 7) * 256 + u * 64];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, cur[u]), __builtin_bit_cast(bf16x8, b[(g + u) & 7]),
                                                         acc[u], 0, 0, 0);
#pragma unroll
      for (int v = 0; v < VPG; ++v) {
        const int i = (g * VPG + v) & 15;
        if ((v & 3) == 3) x[i] = -__builtin_amdgcn_exp2f(x[i]);  // stays in (-1, -0.5)
        else x[i] = __builtin_fmaf(x[i], m, c);
      }
      // issue order: one matrix instruction, its LDS read, its share of the vector instructions
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (LDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        if (VPM > 0) __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) asm volatile("" : "+v"(acc[u]));
#pragma unroll
    for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(x[i]));
  }
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int xx = 0; xx < 16; ++xx) s += acc[u][xx];
#pragma unroll
  for (int i = 0; i < 16; ++i) s += x[i];
  out[blockIdx.x * 512 + threadIdx.x] = s;
#endif
}

hipError_t launch_mix_rate(float* scratch, int iters, int vector_per_mfma, int lds_operands, hipStream_t s) {
  const dim3 grid(kProbeGroups), block(512);
#define SPARSED_MIX(V)                                                                               \
  case V:                                                                                            \
    if (lds_operands) hipLaunchKernelGGL((mix_rate_kernel<V, true>), grid, block, 0, s, scratch, iters); \
    else hipLaunchKernelGGL((mix_rate_kernel<V, false>), grid, block, 0, s, scratch, iters);         \
    break;
  switch (vector_per_mfma) {
    SPARSED_MIX(0) SPARSED_MIX(2) SPARSED_MIX(3) SPARSED_MIX(4) SPARSED_MIX(5) SPARSED_MIX(6) SPARSED_MIX(8)
    default: return hipErrorInvalidValue;
  }
#undef SPARSED_MIX
  return hipGetLastError();
}

// 256 work-groups of 8 waves (two per SIMD on a 256-CU part); scratch must hold kProbeFloats floats.
hipError_t launch_mfma_rate(float* scratch, int iters, int random_operands, hipStream_t s) {
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(kProbeGroups), dim3(512), 0, s, scratch, iters, random_operands);
  return hipGetLastError();
}

}  // namespace sparsed
