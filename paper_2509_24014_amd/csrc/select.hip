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
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NW >= 2 ? 2 : 1, NW >= 2 ? 2 : 1))) void pool_bf16_kernel(const PoolArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (the body uses device-only types)
  constexpr int NT = NW * 64;
  constexpr int kKBytes = KLayout<D>::kTileBytes;
  __shared__ __attribute__((aligned(16))) char lds[2 * kKBytes];
  __shared__ float wsum[2][NW];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 31;
  const int lid = xcd_remap(blockIdx.x, gridDim.x);
  const int I = lid % a.nqb;
  const int bh = lid / a.nqb;
  const int b = bh / a.Hq, h = bh % a.Hq;
  const int hk = h / (a.Hq / a.Hkv);

  const __bf16* qbase = static_cast<const __bf16*>(a.q.ptr) + b * a.q.sb + h * a.q.sh;
  const __bf16* kbase = static_cast<const __bf16*>(a.k.ptr) + b * a.k.sb + hk * a.k.sh;
  const int row0 = I * (32 * NW) + wave * 32;

  QFrag<D, 1> qf;
  qf.load(qbase + (int64_t)row0 * a.q.sl, a.q.sl, lane);
  const float lse2 = a.lse[(int64_t)bh * a.L + row0 + j] * 1.4426950408889634f;
  float* arow = a.apool + ((int64_t)bh * a.nqb + I) * a.nkb;

  TileDma<D, NT, false> kdma;
  kdma.init(a.k.sl, wave, lane);
  KFragAddr<D> kaddr;
  kaddr.init(lane);
  const int n_tiles = a.nkb;
  const __amdgpu_buffer_rsrc_t krsrc = make_rsrc(kbase, ((int64_t)(a.L - 1) * a.k.sl + D) * 2);
  const int32_t k_tile_bytes = (int32_t)(kTileK * a.k.sl * 2);
  kdma.issue(krsrc, 0, lds, wave);
  __syncthreads();

  const float c = a.scale_log2;
  for (int t = 0; t < n_tiles; ++t) {
    const char* kl = lds + (t & 1) * kKBytes;
    if (t + 1 < n_tiles) kdma.issue(krsrc, (t + 1) * k_tile_bytes, lds + ((t + 1) & 1) * kKBytes, wave);

    f32x16 s0[1], s1[1];
    logits_sub<D, 1, true>(kl, 0, kaddr, qf, s0);
    logits_sub<D, 1, true>(kl, 1, kaddr, qf, s1);
    float part = 0.f;
#pragma unroll
    for (int x = 0; x < 16; ++x) part += __builtin_amdgcn_exp2f(__builtin_fmaf(s0[0][x], c, -lse2));
#pragma unroll
    for (int x = 0; x < 16; ++x) part += __builtin_amdgcn_exp2f(__builtin_fmaf(s1[0][x], c, -lse2));
    part = wave_sum(part);
    if (lane == 0) wsum[t & 1][wave] = part;

    __syncthreads();
    if (tid == 0) {
      float tot = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) tot += wsum[t & 1][w];
      arow[t] = tot * a.inv_area;
    }
  }
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

  const float* qbase = static_cast<const float*>(a.q.ptr) + b * a.q.sb + h * a.q.sh;
  const float* kbase = static_cast<const float*>(a.k.ptr) + b * a.k.sb + hk * a.k.sh;
  const int row0 = I * (32 * NW) + wave * 32;

  QFragF32<D> qf;
  qf.load(qbase + (int64_t)row0 * a.q.sl, a.q.sl, lane);
  const float lse2 = a.lse[(int64_t)bh * a.L + row0 + j] * 1.4426950408889634f;
  float* arow = a.apool + ((int64_t)bh * a.nqb + I) * a.nkb;

  const int tiles_per_block = a.block_k / kTileKF;
  const int n_tiles = a.L / kTileKF;
  const float c = a.scale_log2;
  float acc = 0.f;  // thread 0: running sum of the current key block
  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();
    T::template stage<NT>(kbase + (int64_t)t * kTileKF * a.k.sl, a.k.sl, klds, T::kKStride, tid);
    __syncthreads();
    f32x16 s = logits_tile_f32<D>(klds, qf, lane);
    float part = 0.f;
#pragma unroll
    for (int x = 0; x < 16; ++x) part += exp2f(__builtin_fmaf(s[x], c, -lse2));
    part = wave_sum_f(part);
    if (lane == 0) wsum[wave] = part;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
      for (int w = 0; w < NW; ++w) acc += wsum[w];
      if ((t + 1) % tiles_per_block == 0) {
        arow[t / tiles_per_block] = acc * a.inv_area;
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
  for (int J = lane; J < a.nkb; J += 64) row[J] = src[J];
  __syncthreads();

  const int keep = a.keep_lo + a.keep_hi;
  int32_t* out = a.col_idx + (int64_t)bh * a.cap_per_head + (int64_t)I * keep;
  emit_topk_range(row, 0, a.split, a.keep_lo, out, lane);
  emit_topk_range(row, a.split, a.nkb, a.keep_hi, out + a.keep_lo, lane);
  if (lane == 0) {
    int32_t* rp = a.row_ptr + (int64_t)bh * (a.nqb + 1);
    rp[I] = I * keep;
    if (I == a.nqb - 1) rp[a.nqb] = a.nqb * keep;
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

// ---------------------------------------------------------------------------- launchers
template <int D>
static hipError_t launch_pool_bf16_d(int block_q, const PoolArgs& a, hipStream_t s) {
  const int64_t total = (int64_t)a.B * a.Hq * a.nqb;
  if (total <= 0 || total > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)total);
  switch (block_q) {
    case 128: hipLaunchKernelGGL((pool_bf16_kernel<D, 4>), grid, dim3(256), 0, s, a); break;
    case 64: hipLaunchKernelGGL((pool_bf16_kernel<D, 2>), grid, dim3(128), 0, s, a); break;
    case 32: hipLaunchKernelGGL((pool_bf16_kernel<D, 1>), grid, dim3(64), 0, s, a); break;
    default: return hipErrorInvalidValue;
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
  hipLaunchKernelGGL(topk_kernel, dim3((unsigned)a.rows), dim3(64), (size_t)a.nkb * sizeof(uint32_t), s, a);
  return hipGetLastError();
}

hipError_t launch_validate(const ValidateArgs& a, hipStream_t s) {
  if (a.rows <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(validate_kernel, dim3((unsigned)((a.rows + 255) / 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace sparsed
