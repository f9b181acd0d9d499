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
// whose A operand is 8 consecutive keys of one column d of V. The output accumulator again has
// one query per lane.
//
// Data path. K and V tiles go global -> LDS directly (buffer_load_dwordx4 ... lds: lane i of a wave
// deposits its 16 bytes at LDS base + 16*i); the LDS layouts below are realised on the GLOBAL side
// (each lane fetches the chunk that belongs in its LDS slot). K fragments are 16-byte LDS reads. V fragments use the LDS
// transpose read ds_read_b64_tr_b16: within a block of 16 lanes, result lane L gets element (L%4)
// of the 8 bytes addressed by lanes L/4, 4 + L/4, 8 + L/4, 12 + L/4; addressing lane s to
// V[key0 + s/4][col0 + 4*(s%4) ..] hands lane L the four keys key0 .. key0+3 of column col0 + L.
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
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kTileK = 64;  // keys per K/V tile of the bf16 kernels (a listed key block is half a tile, one tile or two)

#define SPARSED_LDS __attribute__((address_space(3)))
#define SPARSED_GLOBAL __attribute__((address_space(1)))

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

// ---- LDS layouts ---------------------------------------------------------------------------------
// LDS serves 256 bytes (64 banks) per clock: a 16-byte-per-lane read is conflict-free when every
// group of 16 consecutive lanes touches 16 different 16-byte positions modulo 256, an 8-byte
// transpose read when every 32 lanes do. A direct global->LDS load writes one contiguous KB per
// wave, so layouts are built from 1 KB pieces; inside a piece the order of the 64 chunks is free
// (each lane simply fetches the chunk that belongs in its slot).
//
// K tile, D = 128 (one KB = 4 rows): the 16 lanes of a fragment read take the SAME logical chunk
// of 16 consecutive rows. Row r keeps chunk c at position c ^ (r & 3) and every 4-row piece is
// padded by 64 bytes, which shifts piece q by 4*q positions: 16 rows -> 16 distinct positions.
// K tile, D = 64 (one KB = 8 rows of 128 bytes): row r keeps chunk c at c ^ ((r >> 1) & 7).
template <int D>
struct KLayout {
  static constexpr int kPieceBytes = (D == 128) ? 1024 + 64 : 1024;
  static constexpr int kRowsPerPiece = 1024 / (2 * D);
  static constexpr int kTileBytes = (kTileK / kRowsPerPiece) * kPieceBytes;
  __device__ static __forceinline__ int swz(int r) { return (D == 128) ? (r & 3) : ((r >> 1) & 7); }
  __device__ static __forceinline__ int offset(int r, int c) {  // bytes, logical chunk c of row r
    return (r / kRowsPerPiece) * kPieceBytes + (r % kRowsPerPiece) * (2 * D) + ((c ^ swz(r)) << 4);
  }
};
// V tile (one piece = 4 rows = 8*D bytes): a transpose read by 32 lanes takes 4 consecutive rows x
// 4 consecutive chunks (one 32-column slice dt). Piece layout [dt][row & 3][chunk & 3]: those 16
// chunks are 256 contiguous bytes.
template <int D>
struct VLayout {
  static constexpr int kPieceBytes = 8 * D;
  static constexpr int kTileBytes = kTileK * 2 * D;
  __device__ static __forceinline__ int offset(int r, int c) {
    return (r >> 2) * kPieceBytes + ((c >> 2) << 8) + ((r & 3) << 6) + ((c & 3) << 4);
  }
};
// Permutation of the K rows fed to the first product: swap bits 2 and 3.
__device__ __forceinline__ int krow_perm(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

// Direct global -> LDS copy of one [64][D] bf16 tile by NT threads (NT/64 waves). Per-lane byte
// offsets into the global tile are precomputed once (they depend on the row stride and the lane
// only); per tile a wave issues kPerWave 16-byte-per-lane loads, each filling one KB of LDS.
template <int D, int NT, bool IS_V>
struct TileDma {
  static constexpr int kWaveLoads = kTileK * D * 2 / 1024;
  static constexpr int kWaves = NT / 64;
  static constexpr int kPerWave = kWaveLoads / kWaves;
  static_assert(kWaveLoads % kWaves == 0, "tile must split evenly over the waves");
  // At head dim 128 one wave-load is four whole rows of the tile for K and for V alike, and a lane fetches the same
  // chunk of its row in every wave-load: the loads of a wave differ by a uniform 4-row step, which rides in the
  // scalar offset, and one per-lane offset serves them all (registers are what the attention kernels are short of).
  // (Used where a wave issues four loads per tile, the 4-wave work-groups; with two the separate offsets measure faster.)
  static constexpr bool kUniformStep = D == 128 && kPerWave >= 4;
  int32_t goff[kUniformStep ? 1 : kPerWave];  // byte offset of this lane's chunk within the global tile, per wave-load
  int32_t step;                               // kUniformStep: bytes between consecutive wave-loads of a wave

  __device__ static __forceinline__ int lds_piece_offset(int wl) {  // where KB number wl of the tile goes
    if (IS_V) return wl * 1024;
    return wl * KLayout<D>::kPieceBytes;
  }
  __device__ __forceinline__ void init(int64_t stride_l, int wave_in_group, int lane) {
    step = (int32_t)(4 * stride_l * 2);
#pragma unroll
    for (int u = 0; u < (kUniformStep ? 1 : kPerWave); ++u) {
      int row, chunk;
      source_of(wave_in_group * kPerWave + u, lane, &row, &chunk);
      goff[u] = (int32_t)(row * stride_l * 2 + chunk * 16);
    }
  }
  // (row, 16-byte chunk) of the global tile that lane `lane` fetches in wave-load number wl
  __device__ static __forceinline__ void source_of(int wl, int lane, int* row, int* chunk) {
    if (IS_V) {
      const int slot = wl * 64 + lane;  // 16-byte slot within the tile
      const int piece = slot / (D / 2), sp = slot % (D / 2);
      *row = 4 * piece + ((sp >> 2) & 3);
      *chunk = 4 * (sp >> 4) + (sp & 3);
    } else {
      const int rpp = KLayout<D>::kRowsPerPiece, cpr = D / 8;
      *row = wl * rpp + lane / cpr;
      *chunk = (lane % cpr) ^ KLayout<D>::swz(*row);
    }
  }
  // Same copy for a tile of which only the first `rows` rows exist (the last key block of a sequence
  // whose length is not a multiple of the tile): the missing rows are fetched from the last row
  // that exists, so every address stays inside the tensor; their logits are masked by the caller.
  __device__ __forceinline__ void issue_partial(__amdgpu_buffer_rsrc_t rsrc, int32_t tile_byte_offset, char* lds_tile,
                                                int wave_in_group, int lane, int64_t stride_l, int rows) const {
    // Worked out afresh at every call on purpose (the lane number is made opaque): these few integer
    // operations run a handful of times per work-group, whereas per-lane offsets hoisted out of the
    // caller's loop would have to live in registers the main loop has none to spare for.
    asm volatile("" : "+v"(lane));
    const int32_t row_bytes = (int32_t)(stride_l * 2);
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const int wl = wave_in_group * kPerWave + u;
      int row, chunk;
      source_of(wl, lane, &row, &chunk);
      if (row >= rows) row = rows - 1;
      char* dst = lds_tile + lds_piece_offset(wl);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (SPARSED_LDS void*)dst, 16, row * row_bytes + chunk * 16, tile_byte_offset, 0, 0);
    }
  }
  // 32-key blocks: a tile is put together from two independent 32-row halves. With at least two waves
  // every wave's loads lie in ONE half; init_half makes its offsets relative to that half's first row,
  // and issue() is then given the byte offset of the 32-key block that belongs in this wave's half.
  static constexpr bool kWaveInOneHalf = 2 * kPerWave <= kWaveLoads;
  __device__ __forceinline__ void init_half(int64_t stride_l, int wave_in_group, int lane) {
    static_assert(kWaveInOneHalf, "needs at least two waves");
    init(stride_l, wave_in_group, lane);
    if (2 * wave_in_group * kPerWave >= kWaveLoads) {
#pragma unroll
      for (int u = 0; u < (kUniformStep ? 1 : kPerWave); ++u) goff[u] -= (int32_t)(32 * stride_l * 2);
    }
  }
  // the same for a 32-key block of which only the first `rows` rows exist (the last block of a sequence)
  __device__ __forceinline__ void issue_partial_half(__amdgpu_buffer_rsrc_t rsrc, int32_t block_byte_offset, char* lds_tile,
                                                     int wave_in_group, int lane, int64_t stride_l, int rows) const {
    asm volatile("" : "+v"(lane));  // worked out afresh at every call, as in issue_partial
    const int32_t row_bytes = (int32_t)(stride_l * 2);
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const int wl = wave_in_group * kPerWave + u;
      int row, chunk;
      source_of(wl, lane, &row, &chunk);
      row &= 31;  // row within the half
      if (row >= rows) row = rows - 1;
      char* dst = lds_tile + lds_piece_offset(wl);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (SPARSED_LDS void*)dst, 16, row * row_bytes + chunk * 16, block_byte_offset, 0, 0);
    }
  }
  // rsrc: buffer descriptor of the (batch, head) slab; tile_byte_offset: wave-uniform byte offset of
  // the tile's first row in it; lds_tile: LDS address of the tile. The buffer form of the direct
  // load is used because the compiler accounts for it on the vector-memory counter only; the
  // global_load form makes it wait for ALL outstanding LDS reads at every later use of one.
  __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rsrc, int32_t tile_byte_offset, char* lds_tile,
                                        int wave_in_group) const {
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      char* dst = lds_tile + lds_piece_offset(wave_in_group * kPerWave + u);
      if (kUniformStep) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (SPARSED_LDS void*)dst, 16, goff[0], tile_byte_offset + u * step, 0, 0);
      else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (SPARSED_LDS void*)dst, 16, goff[u], tile_byte_offset, 0, 0);
    }
  }
};

// Buffer descriptor over `bytes` bytes starting at base (raw dword access, no stride).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, int64_t bytes) {
  const int32_t n = bytes > 0x7fffffff ? 0x7fffffff : (int32_t)bytes;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, n, 0x00020000);
}

// Q fragments of a wave: B operand of the first product. Lane (j, g) holds, for k-step kk, the 8
// values Q[row j][16*kk + 8*g .. +7].
template <int D, int NQ>
struct QFrag {
  bf16x8 f[NQ][D / 16];
  // qhead: row 0 of the (batch, head) slab; row0: first row of this wave; rows at or past L (a partial
  // last query tile) are read from row L-1 and their results dropped by the caller.
  __device__ __forceinline__ void load(const __bf16* qhead, int row0, int L, int64_t stride_l, int lane) {
    const int j = lane & 31, g = lane >> 5;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      int row = row0 + nq * 32 + j;
      row = row < L ? row : L - 1;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk)
        f[nq][kk] = *reinterpret_cast<const bf16x8*>(qhead + (int64_t)row * stride_l + kk * 16 + g * 8);
    }
  }
};

// Per-lane LDS addressing of the K fragments. Lane (i, g) reads, for sub-tile ks and k-step kk, the
// logical chunk 2*kk + g of row 32*ks + perm(i). The swizzle flips bit 0 (g) and the low bits of kk
// by a lane-dependent mask: a handful of per-lane bases, everything else is an immediate.
template <int D>
struct KFragAddr {
  static constexpr int kBases = (D == 128) ? 2 : 4;
  int32_t base[kBases];
  __device__ __forceinline__ void init(int lane) {
    const int i = lane & 31, g = lane >> 5;
    const int prow = krow_perm(i);
    const int y = KLayout<D>::swz(prow);
    const int row_part = KLayout<D>::offset(prow, 0) - ((0 ^ y) << 4);
#pragma unroll
    for (int bq = 0; bq < kBases; ++bq) base[bq] = row_part + 16 * (g ^ (y & 1)) + 32 * (bq ^ (y >> 1));
  }
  __device__ __forceinline__ bf16x8 read(const char* ktile, int ks, int kk) const {
    const int sub = ks * (32 / KLayout<D>::kRowsPerPiece) * KLayout<D>::kPieceBytes;
    return *reinterpret_cast<const bf16x8*>(ktile + base[kk % kBases] + (kk / kBases) * kBases * 32 + sub);
  }
};

// Per-lane LDS addressing of the V fragments (transpose reads). For column slice dt, 16-key step mp
// and half rr, lane l = 32g + 16*blk + Lb addresses row 16*mp + 8*g + 4*rr + Lb/4, logical chunk
// 4*dt + 2*blk + (Lb&3)/2, byte 8*(Lb&1) within the chunk: one per-lane base plus immediates.
template <int D>
struct VFragAddr {
  int32_t base;
  __device__ __forceinline__ void init(int lane) {
    const int g = lane >> 5, blk = (lane >> 4) & 1, Lb = lane & 15;
    base = VLayout<D>::offset(8 * g + (Lb >> 2), 2 * blk + ((Lb & 3) >> 1)) + 8 * (Lb & 1);
  }
  // 8 consecutive keys 16*mp + 8*g .. +7 of column 32*dt + (lane % 32)
  __device__ __forceinline__ bf16x8 read(const char* vtile, int dt, int mp) const {
    const int32_t b = base + 4 * mp * VLayout<D>::kPieceBytes + 256 * dt;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SPARSED_LDS s16x4*)(vtile + b));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SPARSED_LDS s16x4*)(vtile + b + VLayout<D>::kPieceBytes));
    u32x4 w;
    const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    w[0] = l2[0];
    w[1] = l2[1];
    w[2] = h2[0];
    w[3] = h2[1];
    return __builtin_bit_cast(bf16x8, w);
  }
};

// Scheduling hints: ask the backend to lay the enclosing block out as `AHEAD` fragments' worth of
// LDS reads, then (one fragment's matrix ops, one fragment's reads) repeated, then the remaining
// matrix ops. Without this the compiler issues every fragment read right before the MFMA that
// consumes it and eats the full LDS latency once per fragment.
template <int N_FRAGS, int READS_PER_FRAG, int MFMA_PER_FRAG, int AHEAD>
__device__ __forceinline__ void sched_reads_ahead_of_mfma() {
  __builtin_amdgcn_sched_group_barrier(0x100, AHEAD * READS_PER_FRAG, 0);
#pragma unroll
  for (int i = 0; i < N_FRAGS - AHEAD; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_FRAG, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, READS_PER_FRAG, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, AHEAD * MFMA_PER_FRAG, 0);
}

// S^T for one 32-key sub-tile (ks = 0 / 1 of a 64-key tile): s[nq] = K_sub . Q_nq^T, fp32.
template <int D, int NQ, bool HINT>
__device__ __forceinline__ void logits_sub(const char* klds, int ks, const KFragAddr<D>& ka, const QFrag<D, NQ>& q,
                                           f32x16 (&s)[NQ]) {
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
    for (int x = 0; x < 16; ++x) s[nq][x] = 0.f;
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    const bf16x8 kf = ka.read(klds, ks, kk);
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) s[nq] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, q.f[nq][kk], s[nq], 0, 0, 0);
  }
  if (HINT) sched_reads_ahead_of_mfma<D / 16, 1, NQ, 4>();
}

// O^T += V^T . P^T for one 32-key sub-tile: p[nq][m] holds keys 16*(2*ks + m) + 8*g .. +7.
template <int D, int NQ, bool HINT>
__device__ __forceinline__ void pv_sub(const char* vlds, int ks, const VFragAddr<D>& va, const bf16x8 (&p)[NQ][2],
                                       f32x16 (&o)[NQ][D / 32]) {
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      const bf16x8 vf = va.read(vlds, dt, 2 * ks + m);
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) o[nq][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p[nq][m], o[nq][dt], 0, 0, 0);
    }
  if (HINT) sched_reads_ahead_of_mfma<(D / 32) * 2, 2, NQ, 4>();
}

// Layout hint for one software-pipelined sub-step (P V of the previous sub-tile, K Q^T of the next
// one and the softmax of the current one in a single block): a few fragment reads up front, then
// after every matrix instruction its share of the remaining reads and of the softmax's vector
// work, so the vector instructions issue while the matrix instruction of the same wave executes.
template <int D, int NQ, bool HAS_V>
__device__ __forceinline__ void sched_substep_interleave() {
  constexpr int G = 1;  // matrix instructions per group (coarser groups measured no better)
  constexpr int kMfma = (HAS_V ? (D / 32) * 2 * NQ : 0) + (D / 16) * NQ;
  constexpr int kReads = (HAS_V ? (D / 32) * 2 * 2 : 0) + (D / 16);
  constexpr int kAhead = HAS_V ? 4 : 3;
  // vector instructions handed out between the matrix instructions: three after each of the 16 of an attention
  // sub-step at head dim 128 (of 58; the rest follow the last one: measured better than four after each), otherwise all
  constexpr int kValu = (HAS_V ? (D >= 128 ? 48 : 58) : 50) * NQ;
  constexpr int kGroups = kMfma / G;
  constexpr int kValuPer = (kValu + kGroups - 1) / kGroups;
  constexpr int kReadsPer = (kReads - kAhead + kGroups - 1) / kGroups;
  __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
  for (int i = 0; i < kGroups; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, G, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, kReadsPer, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, kValuPer, 0);
  }
}

}  // namespace sparsed
