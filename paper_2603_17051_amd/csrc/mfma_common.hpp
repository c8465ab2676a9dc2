// Device helpers shared by the bf16 MFMA attention kernels (gfx950 / CDNA4).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace astro {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for -inf (no inf - inf)

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32].
// Lane l (i = l % 32, g = l / 32) holds A[i][8g .. 8g+7], B[8g .. 8g+7][i] and
// D[8*(r/4) + 4g + r%4][i] in accumulator register r.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of a 32x32 accumulator tile that register r of lane group g holds.
__device__ __forceinline__ int acc_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// Value of the partner lane (l ^ 32) combined with the own one: v_permlane32_swap
// exchanges the upper half of its first operand with the lower half of the second.
__device__ __forceinline__ float max_with_partner32(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_partner32(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// LDS tiles are [rows][D] bf16 in 16-byte chunks; chunk c of row r is stored at chunk
// position c ^ swizzle(r) so that both access patterns of the kernels spread over the
// banks: 32 lanes reading one chunk column of 32 consecutive rows (row operand of a
// QK-type product), and the transposing read of 8 consecutive rows x 4 chunks.
template <int CPR>
__device__ __forceinline__ int swizzle(int row) {
  if constexpr (CPR == 16)
    return ((row & 3) << 2) | ((row >> 2) & 3);
  else
    return row & (CPR - 1);
}
template <int D>
__device__ __forceinline__ int lds_chunk_offset(int row, int chunk) {  // in bytes
  constexpr int CPR = D / 8;
  return (row * CPR + (chunk ^ swizzle<CPR>(row))) * 16;
}

// 8 contiguous bf16 of one row: element columns 8*chunk .. 8*chunk+7.
template <int D>
__device__ __forceinline__ bf16x8 lds_read_row8(const char* tile, int row, int chunk) {
  return *reinterpret_cast<const bf16x8*>(tile + lds_chunk_offset<D>(row, chunk));
}

// Transposing read (ds_read_b64_tr_b16): within each block of 16 lanes the lanes
// 4r .. 4r+3 together supply row r (16 values) of a 4x16 matrix, and lane i receives
// column i.  With lane i pointing at tile[row0 + i/4][col0 + 4*(i%4) ..] it returns
// tile[row0 + 0..3][col0 + i]: four consecutive ROWS of one column.
template <int D>
__device__ __forceinline__ bf16x4 lds_read_col4(const char* tile, int row0, int col0, int lane16) {
  const int row = row0 + (lane16 >> 2);
  const int col = col0 + 4 * (lane16 & 3);
  const int off = lds_chunk_offset<D>(row, col >> 3) + (col & 7) * 2;
  typedef i16x4 __attribute__((address_space(3))) * lds_ptr;
  i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + off));
  return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ bf16x8 concat4(bf16x4 a, bf16x4 b) {
  return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- global -> LDS staging of [TILE rows][D] bf16 tiles -------------------------------
// A tile's rows come from up to two row-major sources laid end to end (the resident ring
// rows, then the chunk's rows); rows past both are zero-filled.
struct RowSource {
  const __bf16* base0;
  int64_t stride0;  // elements between rows
  int n0;
  const __bf16* base1;
  int64_t stride1;
  int n1;
};

template <int D, int TILE, int THREADS>
struct TilePairLoader {
  static constexpr int CPR = D / 8;
  static constexpr int kChunks = TILE * CPR / THREADS;  // 16-byte chunks per thread per tile
  static_assert(TILE * CPR % THREADS == 0, "tile must divide over the threads");
  u32x4 a[kChunks], b[kChunks];

  __device__ __forceinline__ static u32x4 fetch(const RowSource& s, int j, int c) {
    u32x4 x = {0, 0, 0, 0};
    if (j < s.n0)
      x = *reinterpret_cast<const u32x4*>(s.base0 + (int64_t)j * s.stride0 + c * 8);
    else if (j < s.n0 + s.n1)
      x = *reinterpret_cast<const u32x4*>(s.base1 + (int64_t)(j - s.n0) * s.stride1 + c * 8);
    return x;
  }
  __device__ __forceinline__ void load(const RowSource& sa, const RowSource& sb, int tile) {
#pragma unroll
    for (int u = 0; u < kChunks; ++u) {
      const int cid = threadIdx.x + u * THREADS;
      const int row = cid / CPR, c = cid % CPR;
      a[u] = fetch(sa, tile * TILE + row, c);
      b[u] = fetch(sb, tile * TILE + row, c);
    }
  }
  __device__ __forceinline__ void store(char* lds_a, char* lds_b) const {
#pragma unroll
    for (int u = 0; u < kChunks; ++u) {
      const int cid = threadIdx.x + u * THREADS;
      const int row = cid / CPR, c = cid % CPR;
      const int off = lds_chunk_offset<D>(row, c);
      *reinterpret_cast<u32x4*>(lds_a + off) = a[u];
      *reinterpret_cast<u32x4*>(lds_b + off) = b[u];
    }
  }
};

}  // namespace astro
