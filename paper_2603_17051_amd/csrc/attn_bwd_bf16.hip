// Chunk attention backward with the cached context detached (Sec. 3.3), bf16 MFMA with
// fp32 accumulation.  Two kernels, no atomics, deterministic:
//   dq    : one workgroup per query tile, walks ALL visible keys (ring + chunk):
//             Delta[q] = <dO_q, O_q> (taken while the query's dO row is loaded, and
//             written out for the second kernel),
//             S^T = K Q~^T - LSE (Q~ arrives pre-multiplied by log2(e)/sqrt(D) and the accumulators
//             start from -LSE*log2(e): the product is the exponent of 2), P^T = exp2(S^T), dP^T = V dO^T,
//             dS^T = P^T o (dP^T - Delta), dQ~^T += K^T dS^T
//   dkv   : one workgroup per tile of CHUNK keys, walks all query tiles:
//             S = Q~ K~^T, P, dV^T += dO^T P, dP = dO V^T, dS, dK~^T += Q~^T dS
//           Cached keys / values get no gradient, so no workgroup exists for them.
// As in the forward every product is arranged so that the accumulator of one product is
// directly the B operand of the next, and the LDS tile of the other operand is read
// either by rows (contraction over D) or through the transposing read (contraction over
// the tile's rows).
#include "kernels.hpp"
#include "mfma_common.hpp"

namespace astro {
namespace {

// Waves per dQ workgroup.  Eight (one workgroup per CU, half the tile traffic from L2) was
// measured slower, 4.87 vs 4.73 ms: a barrier over eight waves and a wider ragged last query tile.
constexpr int kDqWaves = 4;
constexpr int KT = 64;  // rows per LDS tile

struct BwdParams {
  const __bf16* q_rot;
  const __bf16* kc_rot;
  const __bf16* v_chunk;
  const __bf16* k_cache;
  const __bf16* v_cache;
  const __bf16* out;
  const __bf16* dout;
  const float* lse;
  float* delta;   // [B][H][Nq]  -<dO, O>
  float* lse2;    // [B][H][Nq]  -LSE * log2(e), written next to delta by the dQ kernel
  float* dq;      // [B, Nq, H, D]  w.r.t. the un-rotated queries
  float* dk;      // [B, Nq, H, D]  w.r.t. the un-rotated chunk keys
  float* dv;      // [B, Nq, H, D]
  RotaryTables rot;
  float* dk_hist_rot;  // [B][H][C*T][D]   (only when hist_keys)
  float* dv_hist;      // [B, C*T, H, D]
  int hist_keys;       // dK/dV kernel: 0 = the chunk's keys, 1 = the resident ring rows (group must be 1)
  int H, Nq, BH, tiles;  // BH = candidates * heads; tiles = workgroups per pair of the kernel being launched
  int group;             // candidates per cache stream
  int block_rows;        // causal block inside the chunk in token rows, 0 = none
  int64_t cache_rows;
  float scale;
  StreamInts hist_rows;
};

// ---- dQ -----------------------------------------------------------------------
// 16x16x32 MFMAs: a wave's 32 queries are two sub-blocks of 16 (qs); lane (i = lane % 16,
// g = lane / 16) holds, for queries 16*qs + i, the accumulator rows 4g .. 4g+3 of every 16-row tile.
template <int D>
struct DqWave {
  static constexpr int KS = D / 32;  // k-steps of a contraction over D
  static constexpr int DT = D / 16;  // 16-row tiles of dQ~^T
  bf16x8 qreg[2][KS], doreg[2][KS];  // B operands: Q~ and dO rows of this lane's two queries
  f32x4 neg_lse2[2];   // -LSE*log2(e) of the two queries, four copies: the accumulators of S start from it
  // -Delta of the two queries, four copies each: the accumulators of dP^T start from them, so
  // the product comes out as dP^T - Delta
  f32x4 neg_delta[2];
  f32x4 dq[DT][2];
  OperandAddr16<D> addr;
  int g;

  __device__ __forceinline__ void init(int lane) {
    g = lane >> 4;
    addr.init(lane);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int qs = 0; qs < 2; ++qs) dq[dt][qs] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // ---- the pieces of one 32-key block kb of a tile -------------------------------------
  // S^T - LSE*log2(e) = K Q~^T - LSE*log2(e): 16 MFMAs, each pair behind the read of its K fragment
  __device__ __forceinline__ void s_product(const char* ks, int kb, f32x4 (&s)[2][2]) const {
#pragma unroll
    for (int st = 0; st < KS; ++st)
#pragma unroll
      for (int kh = 0; kh < 2; ++kh) {
        const bf16x8 a = read_rows16<D>(ks, addr.row[st], 32 * kb + 16 * kh);
#pragma unroll
        for (int qs = 0; qs < 2; ++qs) s[kh][qs] = mfma16(a, qreg[qs][st], st == 0 ? neg_lse2[qs] : s[kh][qs]);
      }
  }
  // keys of the block that do not count for a query: score replaced so that P and dS are exactly 0
  __device__ __forceinline__ void mask(int kb, const int (&live)[2], f32x4 (&s)[2][2]) const {
#pragma unroll
    for (int kh = 0; kh < 2; ++kh)
#pragma unroll
      for (int qs = 0; qs < 2; ++qs)
#pragma unroll
        for (int r = 0; r < 4; ++r) s[kh][qs][r] = 32 * kb + 16 * kh + 4 * g + r >= live[qs] ? kNegBig : s[kh][qs][r];
  }
  // P^T = exp2(S^T - LSE*log2(e)), in place: 16 exponentials
  __device__ __forceinline__ void probabilities(f32x4 (&s)[2][2]) const {
#pragma unroll
    for (int qs = 0; qs < 2; ++qs)
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int r = 0; r < 4; ++r) s[kh][qs][r] = fast_exp2(s[kh][qs][r]);
  }
  // dP^T - Delta = V dO^T - Delta: 16 MFMAs
  __device__ __forceinline__ void dp_product(const char* vs, int kb, f32x4 (&dp)[2][2]) const {
#pragma unroll
    for (int st = 0; st < KS; ++st)
#pragma unroll
      for (int kh = 0; kh < 2; ++kh) {
        const bf16x8 a = read_rows16<D>(vs, addr.row[st], 32 * kb + 16 * kh);
#pragma unroll
        for (int qs = 0; qs < 2; ++qs) dp[kh][qs] = mfma16(a, doreg[qs][st], st == 0 ? neg_delta[qs] : dp[kh][qs]);
      }
  }
  // dS^T = P^T o (dP^T - Delta) as the B operand of the next product (k-slots 8g .. 8g+3 <- keys
  // 4g .., k-slots 8g+4 .. <- keys 16 + 4g ..): 24 vector-ALU instructions
  __device__ __forceinline__ void ds_operand(const f32x4 (&pr)[2][2], const f32x4 (&dp)[2][2], bf16x8 (&dsb)[2]) const {
#pragma unroll
    for (int qs = 0; qs < 2; ++qs)
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int r = 0; r < 4; ++r) dsb[qs][4 * kh + r] = (__bf16)(pr[kh][qs][r] * dp[kh][qs][r]);
  }
  // dQ~^T[d][q] += K^T[d][key] dS^T[key][q]: 16 MFMAs
  __device__ __forceinline__ void dq_product(const char* ks, int kb, const bf16x8 (&dsb)[2]) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const bf16x8 a = read_cols16<D>(ks, addr.tr[dt], 32 * kb);
#pragma unroll
      for (int qs = 0; qs < 2; ++qs) dq[dt][qs] = mfma16(a, dsb[qs], dq[dt][qs]);
    }
  }

  // One 64-key tile of which the first live[qs] keys count for this lane's query qs (live_min,
  // wave-uniform: the fewest over the wave).  The others lie past the end of their segment
  // (zero rows in LDS) or in a causal block the query does not see; their score is replaced
  // so that P and dS are exactly 0 (left alone, P = exp(0 - LSE) could overflow for a query
  // whose logits are all very negative, and inf * 0 would poison dQ~ = dS K~).
  // Each product reads its operand fragments just ahead of its MFMAs.  Requesting the next
  // product's fragments one MFMA behind the current one (no product then starts by waiting for
  // LDS) was measured slower with the 32x32x16 kernel, 5.05 vs 4.93 ms: it needs all 256
  // registers and the kernel is not bound by LDS latency.
  // Vector-ALU instructions issue while an MFMA executes, also within one wave: the
  // exponentials (which need S only) sit between the MFMAs of the dP product, 4.56 -> 4.41 ms.
  // Going further lost: the dS operand of one query sub-block under the dQ MFMAs of the other
  // (K^T fragments held for both: all 256 registers, 4.64 ms); the scores of the next key block
  // carried along so that the dS operand sits under their MFMAs (spills in the tile loop, 7.4 ms);
  // the first two operand fragments of the dP and dQ products requested one phase early (4.54 vs 4.48 ms).
  __device__ __forceinline__ void tile(const char* ks, const char* vs, const int (&live)[2], int live_min) {
#pragma unroll
    for (int kb = 0; kb < KT / 32; ++kb) {
      f32x4 s[2][2], dp[2][2];  // [16-key half][query sub-block]
      bf16x8 dsb[2];
      s_product(ks, kb, s);
      if (live_min < 32 * (kb + 1)) mask(kb, live, s);
      // keep the phases apart: hoisting every LDS read of a key block to its top costs
      // more registers than two resident waves per SIMD have
      __builtin_amdgcn_sched_barrier(0);
      probabilities(s);
      dp_product(vs, kb, dp);
#pragma unroll
      for (int i = 0; i < 4 * KS; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);  // one exponential
      }
      __builtin_amdgcn_sched_barrier(0);
      ds_operand(s, dp, dsb);
      __builtin_amdgcn_sched_barrier(0);
      dq_product(ks, kb, dsb);
    }
  }
};

template <int D, int OCC, int kWaves>
__global__ void __launch_bounds__(kWaves * 64, OCC) attn_bwd_dq_kernel(BwdParams p) {
  using Wave = DqWave<D>;
  constexpr int TILE_BYTES = KT * D * 2;
  __shared__ __attribute__((aligned(1024))) char lds[4 * TILE_BYTES];  // K0 V0 K1 V1

  const WorkItem item = work_item(p.tiles, p.BH, true);
  if (!item.valid) return;
  const PairIndex pair = split_pair(item.bh, p.H, p.group);
  const int b = pair.b, h = pair.h;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i16 = lane & 15, g = lane >> 4;
  const int hist = p.hist_rows.v[pair.cache_b];
  const int q0 = (item.tile * kWaves + wave) * 32 + i16;  // this lane's queries: q0 and q0 + 16
  const int64_t bh = (int64_t)b * p.H + h;
  // chunk rows each of this lane's queries sees, the fewest any lane of the wave sees (its
  // first query) and the most any wave of the workgroup sees (its last query)
  const int q_last = p.Nq - 1;
  int vis[2];
#pragma unroll
  for (int qs = 0; qs < 2; ++qs) vis[qs] = visible_chunk_rows(q0 + 16 * qs < q_last ? q0 + 16 * qs : q_last, p.Nq, p.block_rows);
  const int q_wave = (item.tile * kWaves + __builtin_amdgcn_readfirstlane(wave)) * 32;
  const int vis_wave = visible_chunk_rows(q_wave < q_last ? q_wave : q_last, p.Nq, p.block_rows);
  const int q_wg = (item.tile + 1) * kWaves * 32 - 1;
  const int vis_wg = visible_chunk_rows(q_wg < q_last ? q_wg : q_last, p.Nq, p.block_rows);
  const int hist_tiles = (hist + KT - 1) / KT;
  const int ntiles = hist_tiles + (vis_wg + KT - 1) / KT;

  Wave w;
  w.init(lane);
#pragma unroll
  for (int qs = 0; qs < 2; ++qs) {
    const int q = q0 + 16 * qs;
    const bool live = q < p.Nq;
    const __bf16* qrow = p.q_rot + (bh * p.Nq + (live ? q : 0)) * D;
    const int64_t token_row = (((int64_t)b * p.Nq + (live ? q : 0)) * p.H + h) * D;
    const __bf16* drow = p.dout + token_row;
    const __bf16* orow = p.out + token_row;
    // Delta = <dO_q, O_q>: this lane holds the quarter 32*st + 8g .. +7 of the row, the lanes
    // i + 16, i + 32, i + 48 the others
    float dsum = 0.f;
#pragma unroll
    for (int st = 0; st < Wave::KS; ++st) {
      bf16x8 x = {0, 0, 0, 0, 0, 0, 0, 0}, y = x, o = x;
      if (live) {
        x = *reinterpret_cast<const bf16x8*>(qrow + st * 32 + g * 8);
        y = *reinterpret_cast<const bf16x8*>(drow + st * 32 + g * 8);
        o = *reinterpret_cast<const bf16x8*>(orow + st * 32 + g * 8);
      }
      w.qreg[qs][st] = x;
      w.doreg[qs][st] = y;
#pragma unroll
      for (int j = 0; j < 8; ++j) dsum = fmaf((float)y[j], (float)o[j], dsum);
    }
    dsum += __shfl_xor(dsum, 16);
    dsum += __shfl_xor(dsum, 32);
    // a dead query row gets P = exp2(0 - big) = 0 everywhere
    const float nl = live ? -p.lse[bh * p.Nq + q] * kLog2e : -1.0e30f;
    w.neg_lse2[qs] = f32x4{nl, nl, nl, nl};
    w.neg_delta[qs] = f32x4{-dsum, -dsum, -dsum, -dsum};
    // the row terms of the query, for the dK/dV kernel (negative there too)
    if (live && g == 0) {
      p.delta[bh * p.Nq + q] = -dsum;
      p.lse2[bh * p.Nq + q] = nl;
    }
  }

  const RowSegment k_hist = make_segment(p.k_cache + (int64_t)pair.cache_bh * p.cache_rows * D, D, hist, D);
  const RowSegment v_hist = make_segment(p.v_cache + (int64_t)pair.cache_bh * p.cache_rows * D, D, hist, D);
  const RowSegment k_chunk = make_segment(p.kc_rot + bh * p.Nq * D, D, p.Nq, D);
  const RowSegment v_chunk = make_segment(p.v_chunk + ((int64_t)b * p.Nq * p.H + h) * D, (int64_t)p.H * D, p.Nq, D);
  TileStreamer<D, KT, kWaves> ts;
  ts.init();
  const uint32_t off_dense = ts.lane_offset(k_hist);
  const uint32_t off_vchunk = ts.lane_offset(v_chunk);
  auto issue = [&](int t) {
    char* kbuf = lds + (t & 1) * 2 * TILE_BYTES;
    if (t < hist_tiles) {
      ts.issue(k_hist, off_dense, t * KT, kbuf);
      ts.issue(v_hist, off_dense, t * KT, kbuf + TILE_BYTES);
    } else {
      ts.issue(k_chunk, off_dense, (t - hist_tiles) * KT, kbuf);
      ts.issue(v_chunk, off_vchunk, (t - hist_tiles) * KT, kbuf + TILE_BYTES);
    }
  };
  issue(0);
  wait_vmem();
  __syncthreads();

  // two tiles per trip so that each LDS buffer is a compile-time offset of the operand reads
  auto step = [&](int t, auto buf_c) __attribute__((always_inline)) {
    if (t + 1 < ntiles) issue(t + 1);
    const char* kbuf = lds + decltype(buf_c)::value * 2 * TILE_BYTES;
    int live[2];
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) live[qs] = t < hist_tiles ? hist - t * KT : vis[qs] - (t - hist_tiles) * KT;
    w.tile(kbuf, kbuf + TILE_BYTES, live, t < hist_tiles ? hist - t * KT : vis_wave - (t - hist_tiles) * KT);
    wait_vmem();
    __syncthreads();
  };
  for (int t = 0; t < ntiles; t += 2) {
    step(t, std::integral_constant<int, 0>{});
    if (t + 1 < ntiles) step(t + 1, std::integral_constant<int, 1>{});
  }

  // dQ~ -> dQ: the rotation is turned back here (each lane holds both halves of its pairs), so the
  // gradient goes out once, token-major, instead of through a rotated fp32 copy and another pass
  const bool rope = p.rot.n_t + p.rot.n_h + p.rot.n_w != 0;
#pragma unroll
  for (int qs = 0; qs < 2; ++qs) {
    const int q = q0 + 16 * qs;
    if (q < p.Nq) {
      float* row = p.dq + (((int64_t)b * p.Nq + q) * p.H + h) * D;
      const TokenTables tt = token_tables(p.rot, b, q);
#pragma unroll
      for (int dt = 0; dt < Wave::DT; ++dt) {
        f32x4 x = w.dq[dt][qs] * p.scale;
        if (rope) x = unrotate_quad(p.rot, tt, 4 * dt + g, x);
        *reinterpret_cast<f32x4*>(row + 16 * dt + 4 * g) = x;
      }
    }
  }
}

// ---- dK, dV of the chunk's keys ---------------------------------------------------
// One workgroup = 8 waves = 128 keys in 4 blocks of 32 (every lane owns one key), each block
// seen by two waves.  The "value" wave computes S = Q~ K~^T, P and dV^T += dO^T P, and hands P
// (bf16, in the lane-private order of its accumulator registers) to its partner through LDS; the
// "key" wave picks it up one period later and computes dP = dO V^T, dS = P o (dP - Delta) and
// dK~^T += Q~^T dS.  Both gradients in one wave need more registers than two waves per SIMD
// have, and two independent workgroups per key tile each compute S and the exponentials (five
// products instead of four; that is how it was before: 1.22 ms at the 12-head, 21-frame,
// batch-4 shape).  A query tile is used in two consecutive periods, so tiles, row terms and P
// live in rings of three LDS slots, and a period is unrolled three times so that every slot is
// a compile-time offset.
constexpr int kPairWaves = 8;
constexpr int kPairThreads = kPairWaves * 64;
constexpr int QT = 64;  // query rows per LDS tile

template <int D>
struct DkvLds {
  static constexpr int TILE_BYTES = QT * D * 2;
  static constexpr int SLOT_TILES = 2 * TILE_BYTES;              // Q~ tile, dO tile
  static constexpr int SLOT_PROBS = 4 * (QT / 32) * 2 * 1024;    // key block x query block x half: 64 lanes x 16 B
  static constexpr int SLOT_TERMS = 2 * QT * 4;                  // LSE*log2e [QT], Delta [QT]
  static constexpr int kProbs = 3 * SLOT_TILES;
  static constexpr int kTerms = kProbs + 3 * SLOT_PROBS;
  static constexpr int kTotal = kTerms + 3 * SLOT_TERMS;
  static_assert(kTotal <= 160 * 1024, "one workgroup per CU must fit the LDS");
};

// Scheduling pattern for a product of kSteps operand fragments (kReads LDS reads and two MFMAs
// each) placed next to independent vector-ALU work: fragment reads run one step ahead of their
// MFMAs, and each pair of MFMAs is followed by a share of the vector-ALU instructions.
template <int kSteps, int kReads>
__device__ __forceinline__ void interleave() {
  __builtin_amdgcn_sched_group_barrier(0x100, 2 * kReads, 0);  // the first two fragments
#pragma unroll
  for (int i = 0; i < kSteps; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);   // two MFMAs
    __builtin_amdgcn_sched_group_barrier(0x002, 10, 0);  // vector-ALU work of the other block
    if (i + 2 < kSteps) __builtin_amdgcn_sched_group_barrier(0x100, kReads, 0);  // the fragment after next
  }
}

// 16x16x32 MFMAs: a wave's 32 keys are two sub-blocks of 16 (ks); lane (i = lane % 16,
// g = lane / 16) holds, for keys 16*ks + i, the accumulator rows 4g .. 4g+3 of every 16-row tile.
// Tile rows below first[ks] (per lane; first_max, wave-uniform, = the largest over the wave) are
// queries of an earlier causal block than the lane's key ks: they do not see it, P = 0.
template <int D>
struct ValueWave {
  static constexpr int KS = D / 32;  // k-steps of a contraction over D
  static constexpr int DT = D / 16;  // 16-row tiles of dV^T
  bf16x8 kreg[2][KS];  // B operand: K~ rows of this lane's two keys
  f32x4 dv[DT][2];
  OperandAddr16<D> addr;
  int g;

  __device__ __forceinline__ void init(int lane) {
    g = lane >> 4;
    addr.init(lane);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) dv[dt][ks] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // ---- the three phases of one block of 32 queries qb of a tile --------------------------
  // S[q][key] - LSE[q]*log2(e), the exponent of 2 (Q~ is pre-multiplied, the accumulators start from
  // the rows' terms): rows = 32 queries in two halves of 16 (qh), column = the lane's key ks
  __device__ __forceinline__ void s_product(const char* qs, int qb, const f32x4 (&l4)[2], f32x4 (&s)[2][2]) const {
#pragma unroll
    for (int st = 0; st < KS; ++st)
#pragma unroll
      for (int qh = 0; qh < 2; ++qh) {
        const bf16x8 a = read_rows16<D>(qs, addr.row[st], 32 * qb + 16 * qh);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) s[qh][ks] = mfma16(a, kreg[ks][st], st == 0 ? l4[qh] : s[qh][ks]);
      }
  }
  // queries of an earlier causal block than the lane's key do not see it: P = 0
  __device__ __forceinline__ void mask(int qb, const int (&first)[2], f32x4 (&s)[2][2]) const {
#pragma unroll
    for (int qh = 0; qh < 2; ++qh)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int r = 0; r < 4; ++r) s[qh][ks][r] = 32 * qb + 16 * qh + 4 * g + r < first[ks] ? kNegBig : s[qh][ks][r];
  }
  // P as the B operand of the next product (k-slots 8g .. 8g+3 <- queries 4g .., 8g+4 .. <- queries
  // 16 + 4g ..), also handed to the key wave through LDS
  __device__ __forceinline__ void probabilities(const f32x4 (&s)[2][2], int qb, char* probs, bf16x8 (&pb)[2]) const {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int r = 0; r < 4; ++r) pb[ks][4 * qh + r] = (__bf16)fast_exp2(s[qh][ks][r]);
    *reinterpret_cast<bf16x8*>(probs + (2 * qb) * 1024) = pb[0];
    *reinterpret_cast<bf16x8*>(probs + (2 * qb + 1) * 1024) = pb[1];
  }
  // dV^T[d][key] += dO^T[d][q] P[q][key]
  __device__ __forceinline__ void dv_product(const char* dos, int qb, const bf16x8 (&pb)[2]) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const bf16x8 a = read_cols16<D>(dos, addr.tr[dt], 32 * qb);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) dv[dt][ks] = mfma16(a, pb[ks], dv[dt][ks]);
    }
  }

  // One tile of 64 queries = two blocks.  A wave's own MFMAs and vector-ALU work overlap only when
  // independent instructions of both kinds are next to each other, so the blocks are software
  // pipelined: the exponentials of block 0 sit between the MFMAs of S(1), those of block 1 between
  // the MFMAs of dV(0).  (Phase by phase, as it was before, a period took about twice the time of
  // its MFMAs.)
  // qs / dos = Q~ and dO tiles, lse_t = -LSE*log2(e) of the tile's rows, probs = this wave's part of a P slot
  __device__ __forceinline__ void tile(const char* qs, const char* dos, const float* lse_t, char* probs,
                                       const int (&first)[2], int first_max) {
    static_assert(QT == 64, "two blocks per tile");
    f32x4 s0[2][2], s1[2][2], l0[2], l1[2];
    bf16x8 p0[2], p1[2];
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
      l0[qh] = *reinterpret_cast<const f32x4*>(lse_t + 16 * qh + 4 * g);
      l1[qh] = *reinterpret_cast<const f32x4*>(lse_t + 32 + 16 * qh + 4 * g);
    }
    s_product(qs, 0, l0, s0);
    if (first_max > 0) mask(0, first, s0);
    __builtin_amdgcn_sched_barrier(0);
    s_product(qs, 1, l1, s1);
    probabilities(s0, 0, probs, p0);
    interleave<2 * KS, 1>();
    __builtin_amdgcn_sched_barrier(0);
    if (first_max > 32) mask(1, first, s1);
    __builtin_amdgcn_sched_barrier(0);
    dv_product(dos, 0, p0);
    probabilities(s1, 1, probs, p1);
    interleave<DT, 2>();
    __builtin_amdgcn_sched_barrier(0);
    dv_product(dos, 1, p1);
  }
};

template <int D>
struct KeyWave {
  static constexpr int KS = D / 32;
  static constexpr int DT = D / 16;
  bf16x8 vreg[2][KS];  // B operand: V rows of this lane's two keys
  f32x4 dk[DT][2];
  OperandAddr16<D> addr;
  int g;

  __device__ __forceinline__ void init(int lane) {
    g = lane >> 4;
    addr.init(lane);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) dk[dt][ks] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // dP[q][key] - Delta[q] = <dO_q, V_key> - Delta[q]: the accumulators start from the rows' terms
  __device__ __forceinline__ void dp_product(const char* dos, int qb, const f32x4 (&d4)[2], f32x4 (&dp)[2][2]) const {
#pragma unroll
    for (int st = 0; st < KS; ++st)
#pragma unroll
      for (int qh = 0; qh < 2; ++qh) {
        const bf16x8 a = read_rows16<D>(dos, addr.row[st], 32 * qb + 16 * qh);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) dp[qh][ks] = mfma16(a, vreg[ks][st], st == 0 ? d4[qh] : dp[qh][ks]);
      }
  }
  // dS = P o (dP - Delta) as the B operand of the last product
  __device__ __forceinline__ void ds_operand(const bf16x8 (&pb)[2], const f32x4 (&dp)[2][2], bf16x8 (&dsb)[2]) const {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int qh = 0; qh < 2; ++qh)
#pragma unroll
        for (int r = 0; r < 4; ++r) dsb[ks][4 * qh + r] = (__bf16)((float)pb[ks][4 * qh + r] * dp[qh][ks][r]);
  }
  // dK~^T[d][key] += Q~^T[d][q] dS[q][key]
  __device__ __forceinline__ void dk_product(const char* qs, int qb, const bf16x8 (&dsb)[2]) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const bf16x8 a = read_cols16<D>(qs, addr.tr[dt], 32 * qb);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) dk[dt][ks] = mfma16(a, dsb[ks], dk[dt][ks]);
    }
  }

  // One tile of 64 queries, software pipelined like the value wave's: dS of block 0 is formed
  // between the MFMAs of dP(1), dS of block 1 between those of dK(0).
  // qs / dos = Q~ and dO tiles, delta_t = -Delta of the tile's rows, probs = the partner's P of this tile
  __device__ __forceinline__ void tile(const char* qs, const char* dos, const float* delta_t, const char* probs) {
    static_assert(QT == 64, "two blocks per tile");
    f32x4 dp0[2][2], dp1[2][2], d0[2], d1[2];
    bf16x8 p0[2], p1[2], ds0[2], ds1[2];
#pragma unroll
    for (int qh = 0; qh < 2; ++qh) {
      d0[qh] = *reinterpret_cast<const f32x4*>(delta_t + 16 * qh + 4 * g);
      d1[qh] = *reinterpret_cast<const f32x4*>(delta_t + 32 + 16 * qh + 4 * g);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      p0[ks] = *reinterpret_cast<const bf16x8*>(probs + ks * 1024);
      p1[ks] = *reinterpret_cast<const bf16x8*>(probs + (2 + ks) * 1024);
    }
    dp_product(dos, 0, d0, dp0);
    __builtin_amdgcn_sched_barrier(0);
    dp_product(dos, 1, d1, dp1);
    ds_operand(p0, dp0, ds0);
    interleave<2 * KS, 1>();
    __builtin_amdgcn_sched_barrier(0);
    dk_product(qs, 0, ds0);
    ds_operand(p1, dp1, ds1);
    interleave<DT, 2>();
    __builtin_amdgcn_sched_barrier(0);
    dk_product(qs, 1, ds1);
  }
};

// Everything one wave does, in its role (kKey: a key wave, else a value wave).  Both roles
// stream the tiles and meet at the same barriers, one per period.
template <int D, bool kKey>
__device__ __forceinline__ void dkv_wave(const BwdParams& p, const WorkItem& item, int wave, char* lds) {
  using L = DkvLds<D>;
  using Wave = std::conditional_t<kKey, KeyWave<D>, ValueWave<D>>;
  const int b = item.bh / p.H, h = item.bh % p.H;
  const int lane = threadIdx.x & 63;
  const int kw = wave & 3;  // key block of the workgroup's four
  const int i16 = lane & 15, g = lane >> 4;
  const int64_t bh = (int64_t)b * p.H + h;
  // this lane's two keys jc and jc + 16: chunk rows, or (non-detached backward) resident ring rows of the stream
  const int n_keys = p.hist_keys ? p.hist_rows.v[b] : p.Nq;
  const int jc = (item.tile * 4 + kw) * 32 + i16;
  const int ntiles = (p.Nq + QT - 1) / QT;
  // first query row that sees each of this lane's keys (ring rows are seen by every query), the
  // largest over the wave (its last key) and the smallest over the workgroup (its first key)
  const int block_rows = p.hist_keys ? 0 : p.block_rows;
  const int j_last = n_keys - 1;
  int first_q[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) first_q[ks] = first_query_row_seeing(jc + 16 * ks < j_last ? jc + 16 * ks : j_last, block_rows);
  const int j_wave = (item.tile * 4 + kw) * 32 + 31;
  const int first_q_wave = first_query_row_seeing(j_wave < j_last ? j_wave : j_last, block_rows);
  const int t_begin = first_query_row_seeing(item.tile * 128, block_rows) / QT;

  Wave w;
  w.init(lane);
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    // B operand of the role's first product: V row (key wave) or K~ row (value wave) of the lane's key ks
    const bool live = jc + 16 * ks < n_keys;
    const int j0 = live ? jc + 16 * ks : 0;
    const __bf16* row;
    if constexpr (kKey)
      row = p.hist_keys ? p.v_cache + (bh * p.cache_rows + j0) * D : p.v_chunk + (((int64_t)b * p.Nq + j0) * p.H + h) * D;
    else
      row = p.hist_keys ? p.k_cache + (bh * p.cache_rows + j0) * D : p.kc_rot + (bh * p.Nq + j0) * D;
#pragma unroll
    for (int st = 0; st < D / 32; ++st) {
      bf16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
      if (live) x = *reinterpret_cast<const bf16x8*>(row + st * 32 + g * 8);
      if constexpr (kKey)
        w.vreg[ks][st] = x;
      else
        w.kreg[ks][st] = x;
    }
  }

  const RowSegment q_rows = make_segment(p.q_rot + bh * p.Nq * D, D, p.Nq, D);
  const RowSegment do_rows = make_segment(p.dout + ((int64_t)b * p.Nq * p.H + h) * D, (int64_t)p.H * D, p.Nq, D);
  TileStreamer<D, QT, kPairWaves> ts;
  ts.init();
  const uint32_t off_q = ts.lane_offset(q_rows), off_do = ts.lane_offset(do_rows);
  // Row terms of a tile's queries: wave 0 fetches LSE*log2e and wave 1 Delta with a direct-to-LDS
  // load of 4 bytes per lane, so no register, branch or wait of the tile loop depends on them.
  // Rows past Nq read as zeros; they cannot contribute: their Q~ and dO rows are zero in LDS as
  // well, so dP, Delta and with them dS and the dV terms are 0.
  const __amdgpu_buffer_rsrc_t term_rows = __builtin_amdgcn_make_buffer_rsrc(
      (void*)((wave == 0 ? p.lse2 : p.delta) + bh * p.Nq), 0, p.Nq * 4, 0x00020000);
  const int term_lane = lane * 4;
  auto issue = [&](int t, int slot) __attribute__((always_inline)) {
    typedef __attribute__((address_space(3))) void* lds_ptr;
    char* qbuf = lds + slot * L::SLOT_TILES;
    ts.issue(q_rows, off_q, t * QT, qbuf);
    ts.issue(do_rows, off_do, t * QT, qbuf + L::TILE_BYTES);
    if (!kKey && wave < 2)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(term_rows, (lds_ptr)(lds + L::kTerms + slot * L::SLOT_TERMS + wave * QT * 4),
                                               4, t * QT * 4 + term_lane, 0, 0, 0);
  };
  issue(t_begin, 0);
  wait_vmem();
  __syncthreads();

  // Period n: the value waves work on tile n (slot S), the key waves on tile n - 1 (slot S - 1),
  // tile n + 1 streams into slot S + 1; the last period has only the key waves' tile left.
  const int probs_lane = kw * (QT / 32) * 2 * 1024 + lane * 16;
  auto period = [&](int n, auto slot_c) __attribute__((always_inline)) {
    constexpr int S = decltype(slot_c)::value, PREV = (S + 2) % 3, NEXT = (S + 1) % 3;
    if (n + 1 < ntiles) issue(n + 1, NEXT);
    if constexpr (kKey) {
      if (n > t_begin)
        w.tile(lds + PREV * L::SLOT_TILES, lds + PREV * L::SLOT_TILES + L::TILE_BYTES,
               reinterpret_cast<const float*>(lds + L::kTerms + PREV * L::SLOT_TERMS) + QT,
               lds + L::kProbs + PREV * L::SLOT_PROBS + probs_lane);
    } else {
      if (n < ntiles) {
        const int first[2] = {first_q[0] - n * QT, first_q[1] - n * QT};
        w.tile(lds + S * L::SLOT_TILES, lds + S * L::SLOT_TILES + L::TILE_BYTES,
               reinterpret_cast<const float*>(lds + L::kTerms + S * L::SLOT_TERMS),
               lds + L::kProbs + S * L::SLOT_PROBS + probs_lane, first, first_q_wave - n * QT);
      }
    }
    wait_vmem();
    __syncthreads();
  };
  for (int n = t_begin;;) {
    period(n, std::integral_constant<int, 0>{});
    if (++n > ntiles) break;
    period(n, std::integral_constant<int, 1>{});
    if (++n > ntiles) break;
    period(n, std::integral_constant<int, 2>{});
    if (++n > ntiles) break;
  }

  // dV as it is; dK~ of chunk keys is turned back to dK here (ring rows keep the rotated frame:
  // the frame a slot holds is looked up by the pass that follows)
  const bool rope = kKey && !p.hist_keys && p.rot.n_t + p.rot.n_h + p.rot.n_w != 0;
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int j = jc + 16 * ks;
    if (j >= n_keys) continue;
    float* row;
    if constexpr (kKey)
      row = p.hist_keys ? p.dk_hist_rot + (bh * p.cache_rows + j) * D : p.dk + (((int64_t)b * p.Nq + j) * p.H + h) * D;
    else
      row = p.hist_keys ? p.dv_hist + (((int64_t)b * p.cache_rows + j) * p.H + h) * D
                        : p.dv + (((int64_t)b * p.Nq + j) * p.H + h) * D;
    TokenTables tt{};
    if (rope) tt = token_tables(p.rot, b, j);
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      f32x4 x;
      if constexpr (kKey) {
        x = w.dk[dt][ks] * kLn2;  // dK~ = dS^T Q~ / sqrt(D), and the staged Q~ carries log2(e)/sqrt(D)
        if (rope) x = unrotate_quad(p.rot, tt, 4 * dt + g, x);
      } else {
        x = w.dv[dt][ks];
      }
      *reinterpret_cast<f32x4*>(row + 16 * dt + 4 * g) = x;
    }
  }
}

template <int D>
__global__ void __launch_bounds__(kPairThreads, 1) attn_bwd_dkv_kernel(BwdParams p) {
  __shared__ __attribute__((aligned(1024))) char lds[DkvLds<D>::kTotal];
  const WorkItem item = work_item(p.tiles, p.BH, false);
  if (!item.valid) return;
  const int n_keys = p.hist_keys ? p.hist_rows.v[item.bh / p.H] : p.Nq;
  if (item.tile * 128 >= n_keys) return;  // whole workgroup, before any barrier
  // waves 0..3 accumulate dV, waves 4..7 dK; the branch is per wave, and both sides execute
  // the same sequence of barriers
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (wave >= 4)
    dkv_wave<D, true>(p, item, wave, lds);
  else
    dkv_wave<D, false>(p, item, wave, lds);
}

template <int D>
BwdParams make_params(const DevGeom& g, const AttnOperands& op, const void* out, const float* lse, const void* dout,
                      float* dq, float* dk, float* dv, void* scratch) {
  BwdParams p;
  p.q_rot = (const __bf16*)op.q_rot;
  p.kc_rot = (const __bf16*)op.kc_rot;
  p.v_chunk = (const __bf16*)op.v_chunk;
  p.k_cache = (const __bf16*)op.k_cache;
  p.v_cache = (const __bf16*)op.v_cache;
  p.out = (const __bf16*)out;
  p.dout = (const __bf16*)dout;
  p.lse = lse;
  p.delta = (float*)scratch;
  p.lse2 = p.delta + (size_t)g.B * g.H * op.Nq;
  p.dq = dq;
  p.dk = dk;
  p.dv = dv;
  p.rot = RotaryTables{op.tab_t, g.tab_h, g.tab_w, g.n_t, g.n_h, g.n_w, g.gw, g.T, op.Nq / g.T};
  p.H = g.H;
  p.BH = g.B * g.H;
  p.tiles = 0;
  p.Nq = op.Nq;
  p.cache_rows = (int64_t)g.C * g.T;
  p.scale = 1.0f / sqrtf((float)D);
  p.hist_rows = op.hist_rows;
  p.group = op.group;
  p.block_rows = op.block_rows;
  p.dk_hist_rot = nullptr;
  p.dv_hist = nullptr;
  p.hist_keys = 0;
  return p;
}

template <int D>
hipError_t launch(const DevGeom& g, const AttnOperands& op, const void* out, const float* lse, const void* dout,
                  float* dq, float* dk, float* dv, void* scratch, hipStream_t stream) {
  BwdParams p = make_params<D>(g, op, out, lse, dout, dq, dk, dv, scratch);
  {
    ProfileScope prof("attn_bwd_dq_bf16", stream);
    const int qtile = kDqWaves * 32;
    p.tiles = (op.Nq + qtile - 1) / qtile;
    attn_bwd_dq_kernel<D, 8 / kDqWaves, kDqWaves><<<dim3(work_grid_size(p.tiles, p.BH)), kDqWaves * 64, 0, stream>>>(p);
  }
  const int ktile = 128;
  {
    ProfileScope prof("attn_bwd_dkv_bf16", stream);
    p.tiles = (op.Nq + ktile - 1) / ktile;
    attn_bwd_dkv_kernel<D><<<dim3(work_grid_size(p.tiles, p.BH)), kPairThreads, 0, stream>>>(p);
  }
  return hipGetLastError();
}

template <int D>
hipError_t launch_hist(const DevGeom& g, const AttnOperands& op, const float* lse, const void* dout, float* dk_hist_rot,
                       float* dv_hist, const void* scratch, hipStream_t stream) {
  BwdParams p = make_params<D>(g, op, nullptr, lse, dout, nullptr, nullptr, nullptr, const_cast<void*>(scratch));
  p.dk_hist_rot = dk_hist_rot;
  p.dv_hist = dv_hist;
  p.hist_keys = 1;
  int max_hist = 0;
  for (int b = 0; b < g.B; ++b) max_hist = op.hist_rows.v[b] > max_hist ? op.hist_rows.v[b] : max_hist;
  if (max_hist == 0) return hipSuccess;
  const int ktile = 128;
  p.tiles = (max_hist + ktile - 1) / ktile;
  ProfileScope prof("attn_bwd_dkv_hist_bf16", stream);
  attn_bwd_dkv_kernel<D><<<dim3(work_grid_size(p.tiles, p.BH)), kPairThreads, 0, stream>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bwd_hist_bf16(const DevGeom& g, const AttnOperands& op, const float* lse, const void* dout,
                                     float* dk_hist_rot, float* dv_hist, const void* scratch, hipStream_t stream) {
  if (op.group != 1) return hipErrorInvalidValue;
  if (g.D == 128) return launch_hist<128>(g, op, lse, dout, dk_hist_rot, dv_hist, scratch, stream);
  return launch_hist<64>(g, op, lse, dout, dk_hist_rot, dv_hist, scratch, stream);
}

// Delta and LSE*log2e per (stream, head, query)
size_t bf16_bwd_workspace_bytes(const DevGeom& g, int Nq) { return 2 * (size_t)g.B * g.H * Nq * sizeof(float); }

hipError_t launch_attn_bwd_bf16(const DevGeom& g, const AttnOperands& op, const void* out, const float* lse,
                                const void* dout, float* dq, float* dk, float* dv, void* scratch,
                                hipStream_t stream) {
  if (g.D == 128) return launch<128>(g, op, out, lse, dout, dq, dk, dv, scratch, stream);
  return launch<64>(g, op, out, lse, dout, dq, dk, dv, scratch, stream);
}

}  // namespace astro
