// Device helpers shared by the bf16 MFMA attention kernels (gfx950 / CDNA4).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

namespace astro {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for -inf (no inf - inf)

// Transposing read (ds_read_b64_tr_b16): within each block of 16 lanes the lanes
// 4r .. 4r+3 together supply row r (16 values) of a 4x16 matrix, and lane i receives
// column i.  With lane i pointing at tile[row0 + i/4][col0 + 4*(i%4) ..] it returns
// tile[row0 + 0..3][col0 + i]: four consecutive ROWS of one column.
__device__ __forceinline__ bf16x4 lds_read_tr4(const char* lane_ptr) {
  typedef i16x4 __attribute__((address_space(3))) * lds_ptr;
  i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lane_ptr));
  return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ bf16x8 concat4(bf16x4 a, bf16x4 b) {
  return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// sum of the two bf16 halves of a packed pair, added to acc (v_dot2_f32_bf16 with ones)
__device__ __forceinline__ float add_pair(bf16x2 p, float acc) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  return __builtin_amdgcn_fdot2_f32_bf16(p, ones, acc, false);
}

// ---- tiles read as operands of v_mfma_f32_16x16x32_bf16 ------------------------------------
// D[16x16] += A[16x32] * B[32x16].  Lane l (i = l % 16, g = l / 16) holds A[i][8g .. 8g+7],
// B[8g .. 8g+7][i] and D[4g + r][i] in accumulator register r.  Under the chip's power limit this
// shape sustains about 16 % more flop/s than 32x32x16 on N(0,1) operands (1963 vs 1695 TFLOP/s
// with nothing but MFMAs): half the accumulator traffic per flop.
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Chunk swizzle for the two access patterns of that shape.  Depends on row mod 16 only.
//  * row operand (ds_read_b128): lane (i, g) reads chunk c + g of row i.  The LDS serves such a
//    read in four passes of 16 lanes: {0-3, 12-15, 20-23, 24-27}, {4-7, 8-11, 16-19, 28-31} and
//    the same + 32, so one pass holds rows {0-3, 12-15} at chunk c and rows {4-11} at chunk c ^ 1;
//  * column operand (transposing ds_read_b64): 32 lanes per pass read rows r .. r+7 (r = 0 or 8)
//    at two neighbouring chunks {2k, 2k+1}.
// Both are conflict-free when the swizzled chunk is 2 * pair(row) + (row >= 8) with pair()
// distinct over rows 0-7 and over rows 8-15, and pair(rows 12-15) = pair(rows 0-3): pair(row) =
// row for row < 8, (row + 4) mod 8 above.  With 8 chunks per row two rows share the 64 banks,
// the row's parity picks the half, and the same holds with pair() over the rows of one parity.
template <int CPR>
__device__ __forceinline__ int swizzle16(int row) {
  const int hi = (row >> 3) & 1;
  if constexpr (CPR == 16)
    return (((row + (hi << 2)) & 7) << 1) | hi;
  else
    return ((((row >> 1) & 3) ^ (hi << 1)) << 1) | hi;
}
template <int D>
__device__ __forceinline__ int lds_chunk_offset16(int row, int chunk) {  // in bytes
  constexpr int CPR = D / 8;
  return (row * CPR + (chunk ^ swizzle16<CPR>(row))) * 16;
}

// Per-lane LDS byte offsets for a [rows][D] tile, first 16 rows; further row blocks of 16 are
// constant offsets.
template <int D>
struct OperandAddr16 {
  static constexpr int KS = D / 32;  // k-steps of a contraction over D
  static constexpr int DT = D / 16;  // 16-column tiles
  uint32_t row[KS];  // 8 contiguous columns 32*step + 8g .. of row (lane % 16): A operand, contraction over D
  uint32_t tr[DT];   // transposing read: rows 4g + 0..3 of column 16*dt + lane % 16

  __device__ __forceinline__ void init(int lane) {
    const int i16 = lane & 15, g = lane >> 4;
#pragma unroll
    for (int st = 0; st < KS; ++st) row[st] = lds_chunk_offset16<D>(i16, 4 * st + g);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const int r = 4 * g + (i16 >> 2);
      const int c = 16 * dt + 4 * (i16 & 3);
      tr[dt] = lds_chunk_offset16<D>(r, c >> 3) + (c & 7) * 2;
    }
  }
};

// A operand of a product contracting over D: rows row16 .. row16+15 (row16 a multiple of 16)
template <int D>
__device__ __forceinline__ bf16x8 read_rows16(const char* tile, uint32_t addr, int row16) {
  return *reinterpret_cast<const bf16x8*>(tile + addr + row16 * D * 2);
}
// A operand of a product contracting over 32 tile rows starting at row32 (a multiple of 16):
// k-slots 8g .. 8g+3 <- rows row32 + 4g + 0..3, k-slots 8g+4 .. 8g+7 <- rows row32 + 16 + 4g + 0..3:
// the order in which the two 16x16 accumulators over those rows hand over their registers.
template <int D>
__device__ __forceinline__ bf16x8 read_cols16(const char* tile, uint32_t addr, int row32) {
  return concat4(lds_read_tr4(tile + addr + row32 * D * 2), lds_read_tr4(tile + addr + (row32 + 16) * D * 2));
}

// ---- global -> LDS streaming of [TILE rows][D] bf16 tiles -------------------------------
// Tiles are copied by direct-to-LDS buffer loads (16 bytes per lane, no registers): one
// wave instruction fills 1 KB of consecutive LDS, lane i the 16 bytes at i*16, so the lane
// owning physical chunk p of row r fetches logical chunk p ^ swizzle(r) of that row.
// A row source is a raw buffer descriptor whose size ends with its last valid row: rows
// past the end read as zeros (written to LDS as zeros) without touching memory.
struct RowSegment {
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t stride_bytes;
};

__device__ __forceinline__ RowSegment make_segment(const __bf16* base, int64_t stride_elems, int n_rows, int D) {
  RowSegment s;
  const int64_t bytes = n_rows > 0 ? (int64_t)(n_rows - 1) * stride_elems * 2 + D * 2 : 0;
  s.rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
  s.stride_bytes = (uint32_t)(stride_elems * 2);
  return s;
}

template <int D, int TILE, int WAVES>
struct TileStreamer {
  static constexpr int CPR = D / 8;                    // 16-byte chunks per row
  static constexpr int kRowsPerInst = 64 / CPR;        // rows one wave instruction covers
  static constexpr int kInsts = TILE / (kRowsPerInst * WAVES);
  static_assert(TILE % (kRowsPerInst * WAVES) == 0, "tile must divide over the waves");
  int wave, lane_row, lane_chunk_bytes;

  __device__ __forceinline__ void init() {
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    lane_row = wave * kRowsPerInst + lane / CPR;  // row within the first pass of the tile
    lane_chunk_bytes = ((lane % CPR) ^ swizzle16<CPR>(lane_row)) * 16;
  }
  // per-lane byte offset of its row/chunk inside a tile of a source with this stride
  __device__ __forceinline__ uint32_t lane_offset(const RowSegment s) const {
    return (uint32_t)lane_row * s.stride_bytes + (uint32_t)lane_chunk_bytes;
  }
  // Start copying rows [row0, row0 + TILE) of `s` into the LDS tile (asynchronous; complete
  // after s_waitcnt vmcnt(0) + barrier).  row0 must be wave-uniform.
  __device__ __forceinline__ void issue(const RowSegment s, uint32_t lane_off, int row0, char* lds_tile) const {
    typedef __attribute__((address_space(3))) void* lds_ptr;
#pragma unroll
    for (int u = 0; u < kInsts; ++u) {
      const uint32_t rows = (uint32_t)(row0 + u * WAVES * kRowsPerInst);
      char* dst = lds_tile + (u * WAVES + wave) * kRowsPerInst * D * 2;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(s.rsrc, (lds_ptr)dst, 16, (int)(rows * s.stride_bytes + lane_off), 0, 0, 0);
    }
  }
};

// ---- workgroup -> (tile, stream*head) mapping -------------------------------------------
// 1-D grid.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  With
// `by_xcd`, and when the (stream, head) pairs divide evenly over the XCDs, XCD x gets the
// contiguous range of pairs [x*BH/8, (x+1)*BH/8), tiles of one pair consecutive: a pair's
// K/V is then pulled through ONE L2 instead of all eight (an eighth of the fabric reads;
// measured 1.5-2.5 % faster for the kernels that walk the whole window).  Otherwise (e.g.
// 12 heads of one stream, where that split would leave XCDs idle) the plain pair-major
// order is used, in which every XCD streams every pair in flight.
struct WorkItem {
  int tile, bh;
  bool valid;
};
constexpr int kXcds = 8;
__host__ __device__ inline int work_grid_size(int tiles_per_head, int BH) { return tiles_per_head * BH; }
__device__ __forceinline__ WorkItem work_item(int tiles_per_head, int BH, bool by_xcd, int i) {
  WorkItem w;
  w.valid = i < tiles_per_head * BH;
  int j = i, first = 0;
  if (by_xcd && BH % kXcds == 0) {
    j = i / kXcds;                       // index among this XCD's workgroups
    first = (i % kXcds) * (BH / kXcds);  // first pair of this XCD
  }
  const int rel = j / tiles_per_head;
  w.bh = first + rel;
  w.tile = j - rel * tiles_per_head;
  return w;
}

__device__ __forceinline__ WorkItem work_item(int tiles_per_head, int BH, bool by_xcd) {
  return work_item(tiles_per_head, BH, by_xcd, (int)blockIdx.x);
}

// A work item's pair index -> candidate, head and cache stream.  Pairs are ordered (cache
// stream, head, candidate), so the `group` candidates that share one head's ring rows are
// neighbours (same XCD under the contiguous split, same time otherwise).
struct PairIndex {
  int b;         // candidate = stream of the chunk tensors: cache stream * group + g
  int h;         // head
  int cache_b;   // cache stream
  int cache_bh;  // cache stream * H + head
};
__device__ __forceinline__ PairIndex split_pair(int pair, int H, int group) {
  PairIndex x;
  const int g = pair % group;
  x.cache_bh = pair / group;
  x.cache_b = x.cache_bh / H;
  x.h = x.cache_bh - x.cache_b * H;
  x.b = x.cache_b * group + g;
  return x;
}

// Causal blocks inside the chunk (block_rows token rows each, 0 = the whole chunk is one
// block): chunk rows [0, visible_chunk_rows) are the keys query row q sees, and query rows
// [first_query_row_seeing, Nq) are the queries that see key row j.
__device__ __forceinline__ int visible_chunk_rows(int q, int Nq, int block_rows) {
  if (block_rows == 0) return Nq;
  const int end = (q / block_rows + 1) * block_rows;
  return end < Nq ? end : Nq;
}
__device__ __forceinline__ int first_query_row_seeing(int j, int block_rows) {
  return block_rows == 0 ? 0 : (j / block_rows) * block_rows;
}

// ---- turning a gradient w.r.t. rotated queries / keys back in an epilogue ---------------------
// The rotary tables of one call: (cos, sin) per temporal pair and chunk frame of each candidate
// (written by the rotation pre-pass, so they are the values the operands were rotated with), per
// row and per column.  All counts 0 = no rotary embedding.
struct RotaryTables {
  const float2* tab_t;  // [B][n_frames][n_t]
  const float2* tab_h;  // [gh][n_h]
  const float2* tab_w;  // [gw][n_w]
  int n_t, n_h, n_w, gw, T, n_frames;
};
// Position of chunk token `tok` of candidate b, as the three table rows of its pairs.
struct TokenTables {
  const float2 *t, *h, *w;
};
__device__ __forceinline__ TokenTables token_tables(const RotaryTables& r, int b, int tok) {
  const int fi = tok / r.T, rem = tok - fi * r.T;
  const int row = rem / r.gw, col = rem - row * r.gw;
  return TokenTables{r.tab_t + ((int64_t)b * r.n_frames + fi) * r.n_t, r.tab_h + row * r.n_h, r.tab_w + col * r.n_w};
}
__device__ __forceinline__ float2 pair_cos_sin(const RotaryTables& r, const TokenTables& t, int pair) {
  if (pair < r.n_t) return t.t[pair];
  pair -= r.n_t;
  return pair < r.n_h ? t.h[pair] : t.w[pair - r.n_h];
}
// x = four consecutive components 4*quad .. 4*quad+3 (two adjacent pairs) of a gradient w.r.t. the
// rotated vector; returns them w.r.t. the un-rotated one: R(phi)^T applied to each pair.
__device__ __forceinline__ f32x4 unrotate_quad(const RotaryTables& r, const TokenTables& t, int quad, f32x4 x) {
  const float2 a = pair_cos_sin(r, t, 2 * quad), b = pair_cos_sin(r, t, 2 * quad + 1);
  return f32x4{x[0] * a.x + x[1] * a.y, x[1] * a.x - x[0] * a.y, x[2] * b.x + x[3] * b.y, x[3] * b.x - x[2] * b.y};
}

// wait until this wave's outstanding global loads (including direct-to-LDS ones) are done
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }  // vmcnt(0) only
// ... all but the N most recently issued ones (loads complete in issue order)
template <int N>
__device__ __forceinline__ void wait_vmem_except() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 0xF) | ((N >> 4) << 14));
}

}  // namespace astro
