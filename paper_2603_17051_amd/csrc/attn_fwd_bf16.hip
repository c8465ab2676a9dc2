// Chunk attention forward over the rolling cache, bf16 MFMA with fp32 accumulation.
//
// One workgroup = 4 wavefronts = 4 * 32 consecutive queries of one (stream, head).
// The visible keys (resident ring rows, then the chunk's own rows) are walked in tiles of
// 32; K and V tiles are streamed into a ring of LDS stages by direct-to-LDS loads issued
// two tiles ahead, one barrier per tile.  Everything is computed transposed so that
// every lane owns ONE query:
//   S^T[key][q] = K * Q~^T      (A = K tile from LDS, B = Q~ held in registers; Q~ arrives
//                                pre-multiplied by log2(e)/sqrt(D), so S^T is the exponent of 2)
//   O^T[d][q]  += V^T * P^T     (A = V tile through the transposing LDS read,
//                                B = P^T taken straight from the S^T accumulators)
// so the row maximum / sum of the softmax are in-lane reductions plus one exchange with
// the partner lane l^32, and the rescale factor is a per-lane scalar.
//
// Order inside a tile: the K operand reads are issued first, then the global->LDS loads
// of the tile two ahead (their issue stalls while the memory pipeline is busy, which now
// overlaps the LDS latency of the K reads), then the QK MFMAs, softmax, V reads and PV
// MFMAs.  Runs of full tiles inside one key segment take a branch-free copy of the tile
// code (no tail handling, no segment or end-of-loop tests); only the few tiles around the
// segment boundaries take the general one.
//
// Softmax reference: probabilities are taken relative to a per-query reference M that is
// only raised when a tile's probabilities relative to it sum to more than kSumLimit; fp32
// accumulators and the bf16 exponent range make any smaller excess exact enough, and
// both the row maximum and the 64 accumulator multiplies of a rescale leave the common path.
// A query's first reference is snapped to 0 when its first tile's maximum is moderate, and a wave
// whose references are all 0 takes exp2 of the score itself: no subtraction per score either.
// The softmax's vector-ALU work of a tile has no independent MFMAs of the same wave to sit between
// (taking the probabilities of the first 16 keys between the MFMAs of the other 16 was measured
// slower as the scheduler ordered it, 3.34 vs 3.22 ms, and equal with the exact order pinned in
// assembly, 3.03-3.08 vs 3.01-3.03 ms); the overlap comes from
// three workgroups (three waves per SIMD) being resident per CU.
#include "kernels.hpp"
#include "mfma_common.hpp"

namespace astro {
namespace {

constexpr int KT = 32;                 // keys per LDS tile
constexpr float kSumLimit = 0x1p44f;  // a lane's 16 probabilities may sum to this before the reference moves

struct FwdParams {
  const __bf16* q_rot;
  const __bf16* kc_rot;
  const __bf16* v_chunk;
  const __bf16* k_cache;
  const __bf16* v_cache;
  __bf16* out;
  float* lse;
  // key-range split: workgroup (pair, split, tile) walks the split's share of the key tiles and
  // writes its own normalised output and log-sum-exp to part `split`; a merge launch combines them
  int splits;
  __bf16* out_part;  // [splits][B, Nq, H, D]
  float* lse_part;   // [splits][B][H][Nq]
  int H, Nq, BH, q_tiles, group;  // BH = candidates * heads; group = candidates per cache stream
  int block_rows;                 // causal block inside the chunk in token rows, 0 = none
  int64_t cache_rows;  // C*T
  StreamInts hist_rows;
};

// 16x16x32 MFMAs: a wave's 32 queries are two sub-blocks of 16 (qs); lane (i = lane % 16,
// g = lane / 16) holds, for queries 16*qs + i, the accumulator rows 4g .. 4g+3 of every 16-row
// tile, so a query's row statistics are spread over the four lanes i, i+16, i+32, i+48; they
// are only combined at the end of the kernel and on the rare path that moves the reference.
template <int D>
struct FwdWave {
  static constexpr int KS = D / 32;   // k-steps of the QK product
  static constexpr int KF = 2 * KS;   // K operand fragments of a 32-key tile: step x 16-key half
  static constexpr int DT = D / 16;   // 16-row tiles of O^T

  bf16x8 qreg[2][KS];
  f32x4 o[DT][2];
  float mc[2], l_run[2];  // softmax reference in log2 units (the units of the scores), per-lane partial row sum
  // every reference of the wave is exactly 0 (wave-uniform): the exponent is the score itself
  bool zero_ref;
  OperandAddr16<D> addr;
  int g;

  __device__ __forceinline__ void init(int lane) {
    g = lane >> 4;
    zero_ref = false;
    addr.init(lane);
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
      mc[qs] = kNegBig;
      l_run[qs] = 0.f;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int qs = 0; qs < 2; ++qs) o[dt][qs] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // p = exp2(s - mc) (kZeroRef: mc is 0 for the whole wave, no subtraction) rounded to bf16, packed as the B operands of the PV
  // product (k-slots 8g .. 8g+3 <- keys 4g .., 8g+4 .. <- keys 16 + 4g ..); sum = this lane's
  // part of the row sums, taken over the rounded values.
  template <bool kZeroRef>
  __device__ __forceinline__ void probabilities(const f32x4 (&s)[2][2], bf16x8 (&pb)[2], float (&sum)[2]) const {
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
      sum[qs] = 0.f;
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
#pragma unroll
        for (int r = 0; r < 4; r += 2) {
          const f32x2 e = kZeroRef ? f32x2{fast_exp2(s[kh][qs][r]), fast_exp2(s[kh][qs][r + 1])}
                                   : f32x2{fast_exp2(s[kh][qs][r] - mc[qs]), fast_exp2(s[kh][qs][r + 1] - mc[qs])};
          const bf16x2 pk = __builtin_convertvector(e, bf16x2);
          sum[qs] = add_pair(pk, sum[qs]);
          pb[qs][4 * kh + r] = pk[0];
          pb[qs][4 * kh + r + 1] = pk[1];
        }
    }
  }

  // A operands of the first half of the QK product's k-steps: 32 keys x D/2.  The other half is
  // read behind the MFMAs of the first (registers for all of them at once are not there).
  static constexpr int KH = KF / 2;
  __device__ __forceinline__ void read_k(const char* ks, bf16x8 (&kf)[KH]) const {
#pragma unroll
    for (int j = 0; j < KH; ++j) kf[j] = read_rows16<D>(ks, addr.row[j >> 1], 16 * (j & 1));
  }

  // S^T tile of 32 keys x this wave's 32 queries from K operands in registers.  With kTail
  // and any_dead (wave-uniform), only the first live[qs] rows of the tile count for this lane's
  // query qs: the others lie past their segment (K and V rows zero in LDS) or in a causal block
  // the query does not see, and get a score that makes their probability exactly 0.
  template <bool kTail>
  __device__ __forceinline__ void scores(const bf16x8 (&kf)[KH], const char* ks, const int (&live)[2], bool any_dead,
                                         f32x4 (&s)[2][2]) const {
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    bf16x8 hi[KH];
#pragma unroll
    for (int j = 0; j < KH; ++j) {  // fragment j: k-step j / 2, key half j % 2
#pragma unroll
      for (int qs = 0; qs < 2; ++qs) s[j & 1][qs] = mfma16(kf[j], qreg[qs][j >> 1], j < 2 ? zero : s[j & 1][qs]);
      hi[j] = read_rows16<D>(ks, addr.row[(KH + j) >> 1], 16 * (j & 1));
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // two MFMAs
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // then one LDS read
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < KH; ++j)
#pragma unroll
      for (int qs = 0; qs < 2; ++qs) s[j & 1][qs] = mfma16(hi[j], qreg[qs][(KH + j) >> 1], s[j & 1][qs]);
    if (kTail && any_dead) mask(live, s);
  }

  __device__ __forceinline__ void mask(const int (&live)[2], f32x4 (&s)[2][2]) const {
#pragma unroll
    for (int kh = 0; kh < 2; ++kh)
#pragma unroll
      for (int qs = 0; qs < 2; ++qs)
#pragma unroll
        for (int r = 0; r < 4; ++r) s[kh][qs][r] = 16 * kh + 4 * g + r >= live[qs] ? kNegBig : s[kh][qs][r];
  }

  // The same scores for the rare path that moves the reference: every operand fragment is read
  // right before its MFMAs, so the path adds no registers to what the common one needs.
  template <bool kTail>
  __device__ __forceinline__ void scores_again(const char* ks, const int (&live)[2], bool any_dead, f32x4 (&s)[2][2]) const {
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < KF; ++j) {
      const bf16x8 a = read_rows16<D>(ks, addr.row[j >> 1], 16 * (j & 1));
#pragma unroll
      for (int qs = 0; qs < 2; ++qs) s[j & 1][qs] = mfma16(a, qreg[qs][j >> 1], j < 2 ? zero : s[j & 1][qs]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (kTail && any_dead) mask(live, s);
  }

  // One 32-key tile: kf = its K operands (read from ks), vs = its V rows in LDS; live (per
  // lane and query) and any_dead (wave-uniform) are only looked at when kTail.
  template <bool kTail>
  __device__ __forceinline__ void tile(const bf16x8 (&kf)[KH], const char* ks, const char* vs, const int (&live)[2],
                                       bool any_dead) {
    // Probabilities relative to the current reference.  No maximum is taken on the common
    // path: a tile whose logits outgrow the reference shows up as a huge (or infinite) row
    // sum; only then the scores are computed again (the first copy is gone: the exponentials
    // are taken in place), the reference is raised and the probabilities are redone.
    bf16x8 pb[2];
    float sum[2];
    {
      f32x4 s[2][2];
      scores<kTail>(kf, ks, live, any_dead, s);
      if (__builtin_expect(zero_ref, 1))
        probabilities<true>(s, pb, sum);
      else
        probabilities<false>(s, pb, sum);
    }
    if (__builtin_expect(__any(!(sum[0] <= kSumLimit) || !(sum[1] <= kSumLimit)), 0)) {
      f32x4 s[2][2];
      scores_again<kTail>(ks, live, any_dead, s);
#pragma unroll
      for (int qs = 0; qs < 2; ++qs) {
        float mx = fmaxf(fmaxf(s[0][qs][0], s[0][qs][1]), fmaxf(s[0][qs][2], s[0][qs][3]));
        mx = fmaxf(mx, fmaxf(fmaxf(s[1][qs][0], s[1][qs][1]), fmaxf(s[1][qs][2], s[1][qs][3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));  // over the four lanes that share the query
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // never below -1e28: a query that has seen nothing but masked keys so far (scores of
        // -1e30) keeps probabilities of exactly 0 instead of exp2(rounding error of 1e29)
        float mc_new = fmaxf(fmaxf(mc[qs], mx), -1.0e28f);
        // A query's FIRST reference (nothing accumulated yet) is snapped to 0 when its tile maximum
        // is moderate, as it is for any ordinary logits: while every reference of the wave is 0 the
        // common path needs no subtraction in front of the exponential.  fp32 sums and the bf16
        // exponent range hold 2^44 above and 2^-90 below such a reference.
        if (mc[qs] < -1.0e27f && mc_new > -32.f && mc_new < 32.f) mc_new = 0.f;
        const float alpha = fast_exp2(mc[qs] - mc_new);
        l_run[qs] *= alpha;
        // whole-tuple products: the compiler then updates the accumulators where they are
        // (element by element it copies all of them, which the tile loop has no registers for)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt][qs] = o[dt][qs] * alpha;
        mc[qs] = mc_new;
      }
      zero_ref = __all(mc[0] == 0.f && mc[1] == 0.f);
      probabilities<false>(s, pb, sum);
    }
    l_run[0] += sum[0];
    l_run[1] += sum[1];
    // O^T += V^T P^T.  Half of the V operand fragments are requested up front; those of the
    // second half are read one by one behind the MFMAs of the first, into the registers
    // these have just released.
    constexpr int HALF = DT / 2;
    bf16x8 v0[HALF], v1[HALF];
#pragma unroll
    for (int dt = 0; dt < HALF; ++dt) v0[dt] = read_cols16<D>(vs, addr.tr[dt], 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int dt = 0; dt < HALF; ++dt) {
      o[dt][0] = mfma16(v0[dt], pb[0], o[dt][0]);
      o[dt][1] = mfma16(v0[dt], pb[1], o[dt][1]);
      v1[dt] = read_cols16<D>(vs, addr.tr[HALF + dt], 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // two MFMAs
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // then two LDS reads
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int dt = 0; dt < HALF; ++dt) {
      o[HALF + dt][0] = mfma16(v1[dt], pb[0], o[HALF + dt][0]);
      o[HALF + dt][1] = mfma16(v1[dt], pb[1], o[HALF + dt][1]);
    }
  }
};

// kCausal: the chunk has causal blocks (block_rows > 0), so the chunk rows a query sees differ
// from lane to lane; without it that count is the uniform Nq and costs no vector register.
template <int D, int kStages, int kWaves, int OCC, bool kCausal>
__global__ void __launch_bounds__(kWaves * 64, OCC) attn_fwd_bf16_kernel(FwdParams p) {
  using Wave = FwdWave<D>;
  constexpr int kAhead = kStages - 1;  // tiles in flight ahead of the one being processed
  constexpr int TILE_BYTES = KT * D * 2;
  constexpr int STAGE_BYTES = 2 * TILE_BYTES;  // K tile, V tile
  __shared__ __attribute__((aligned(1024))) char lds[kStages * STAGE_BYTES];
  // per-lane count of visible chunk rows: kept in LDS, not in a register the tile loop has no room for
  __shared__ int vis_lds[kCausal ? 2 * kWaves * 64 : 1];

  const WorkItem item = work_item(p.q_tiles, p.BH * p.splits, true);
  if (!item.valid) return;
  const int split = item.bh % p.splits;
  const PairIndex pair = split_pair(item.bh / p.splits, p.H, p.group);
  const int b = pair.b, h = pair.h;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i16 = lane & 15, g = lane >> 4;
  const int hist = p.hist_rows.v[pair.cache_b];
  const int q0 = (item.tile * kWaves + wave) * 32 + i16;  // this lane's queries: q0 and q0 + 16
  // chunk rows each of this lane's queries sees, the fewest any lane of the wave sees (its first
  // query) and the most any wave of the workgroup sees (its last query)
  const int q_last = p.Nq - 1;
  const int block_rows = kCausal ? p.block_rows : 0;
  const int q_wave = (item.tile * kWaves + __builtin_amdgcn_readfirstlane(wave)) * 32;
  const int q_wg = (item.tile + 1) * kWaves * 32 - 1;
  const int vis_wave = visible_chunk_rows(q_wave < q_last ? q_wave : q_last, p.Nq, block_rows);
  const int vis_wg = visible_chunk_rows(q_wg < q_last ? q_wg : q_last, p.Nq, block_rows);
  if constexpr (kCausal) {
#pragma unroll
    for (int qs = 0; qs < 2; ++qs)
      vis_lds[qs * kWaves * 64 + threadIdx.x] = visible_chunk_rows(q0 + 16 * qs < q_last ? q0 + 16 * qs : q_last, p.Nq, block_rows);
  }
  // key tiles: first the resident ring rows, then the chunk rows the workgroup sees, each with its own tail
  const int hist_tiles = (hist + KT - 1) / KT;
  const int ntiles = hist_tiles + (vis_wg + KT - 1) / KT;
  // this workgroup's share [t_begin, t_end) of them (all of them without a split)
  const int t_begin = (int)((int64_t)split * ntiles / p.splits);
  const int t_end = (int)((int64_t)(split + 1) * ntiles / p.splits);
  const int64_t bh = (int64_t)b * p.H + h;

  Wave w;
  w.init(lane);
  // Q~ as the B operand: lane (i, g) holds Q~[q][32*st + 8g .. +7] of its two queries
#pragma unroll
  for (int qs = 0; qs < 2; ++qs) {
    const int q = q0 + 16 * qs;
    const __bf16* qrow = p.q_rot + (bh * p.Nq + (q < p.Nq ? q : 0)) * D;
#pragma unroll
    for (int st = 0; st < Wave::KS; ++st) {
      bf16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
      if (q < p.Nq) x = *reinterpret_cast<const bf16x8*>(qrow + st * 32 + g * 8);
      w.qreg[qs][st] = x;
    }
  }

  const RowSegment k_hist = make_segment(p.k_cache + (int64_t)pair.cache_bh * p.cache_rows * D, D, hist, D);
  const RowSegment v_hist = make_segment(p.v_cache + (int64_t)pair.cache_bh * p.cache_rows * D, D, hist, D);
  const RowSegment k_chunk = make_segment(p.kc_rot + bh * p.Nq * D, D, p.Nq, D);
  const RowSegment v_chunk = make_segment(p.v_chunk + ((int64_t)b * p.Nq * p.H + h) * D, (int64_t)p.H * D, p.Nq, D);
  using Streamer = TileStreamer<D, KT, kWaves>;
  Streamer ts;
  ts.init();
  const uint32_t off_dense = ts.lane_offset(k_hist);    // stride D: ring K, ring V, rotated chunk K
  const uint32_t off_vchunk = ts.lane_offset(v_chunk);  // stride H*D
  auto issue_hist = [&](int t, char* stage) __attribute__((always_inline)) {
    ts.issue(k_hist, off_dense, t * KT, stage);
    ts.issue(v_hist, off_dense, t * KT, stage + TILE_BYTES);
  };
  auto issue = [&](int t, char* stage) __attribute__((always_inline)) {
    const bool in_hist = t < hist_tiles;
    const int row0 = (in_hist ? t : t - hist_tiles) * KT;
    const RowSegment ks = in_hist ? k_hist : k_chunk;
    const RowSegment vs = in_hist ? v_hist : v_chunk;
    ts.issue(ks, off_dense, row0, stage);
    ts.issue(vs, in_hist ? off_dense : off_vchunk, row0, stage + TILE_BYTES);
  };
  // rows of tile t that count for this lane's query qs, and whether any lane of the wave has fewer than all
  auto live_in = [&](int t, int qs) __attribute__((always_inline)) {
    if (t < hist_tiles) return hist - t * KT;
    if constexpr (kCausal)
      return vis_lds[qs * kWaves * 64 + threadIdx.x] - (t - hist_tiles) * KT;  // own entry: no barrier needed
    else
      return vis_wave - (t - hist_tiles) * KT;
  };
  auto any_dead_in = [&](int t) __attribute__((always_inline)) {
    return (t < hist_tiles ? hist - t * KT : vis_wave - (t - hist_tiles) * KT) < KT;
  };
  // Invariant at the top of tile t: tiles t .. t+kAhead-1 have landed and are visible to
  // every wave except the last of them, whose loads may still be in flight; the stage of
  // tile t+kAhead (= that of tile t-1) is free.
  constexpr int kLoadsPerTile = 2 * Streamer::kInsts;  // per wave
#pragma unroll
  for (int t = 0; t < kAhead; ++t)
    if (t_begin + t < t_end) issue(t_begin + t, lds + t * STAGE_BYTES);
  if (t_end - t_begin >= kAhead && kAhead > 1)
    wait_vmem_except<kLoadsPerTile>();
  else
    wait_vmem();
  __syncthreads();

  // kGeneric: any tile.  kHist: tile t is a full tile of ring rows and tile t+kAhead is one
  // too (possibly ragged), so nothing has to be tested: the bulk of a long window.
  constexpr int kGeneric = 0, kHist = 1;
  auto step = [&](int t, auto stage_c, auto mode_c) __attribute__((always_inline)) {
    constexpr int ST = decltype(stage_c)::value;
    constexpr int MODE = decltype(mode_c)::value;
    char* stage = lds + ST * STAGE_BYTES;
    char* refill = lds + ((ST + kAhead) % kStages) * STAGE_BYTES;
    bf16x8 kf[Wave::KH];
    w.read_k(stage, kf);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (MODE == kHist)
      issue_hist(t + kAhead, refill);
    else if (t + kAhead < t_end)
      issue(t + kAhead, refill);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (MODE == kGeneric) {
      const int live[2] = {live_in(t, 0), live_in(t, 1)};
      w.template tile<true>(kf, stage, stage + TILE_BYTES, live, any_dead_in(t));
    } else {
      const int live[2] = {KT, KT};
      w.template tile<false>(kf, stage, stage + TILE_BYTES, live, false);
    }
    // keep the next tile's K reads behind this tile's last MFMA: started earlier they
    // would need registers that are not there
    __builtin_amdgcn_sched_barrier(0);
    // tile t+1 .. t+kAhead-1 must have landed before the next tile starts; the newest may stay in flight
    if (kAhead > 1 && (MODE != kGeneric || t + kAhead < t_end))
      wait_vmem_except<kLoadsPerTile>();
    else
      wait_vmem();
    __syncthreads();
  };
  // kStages tiles per trip so that every LDS stage is a compile-time offset
  auto group = [&](int t, auto mode_c) __attribute__((always_inline)) {
    constexpr bool kAll = decltype(mode_c)::value != kGeneric;  // all kStages tiles exist
    step(t, std::integral_constant<int, 0>{}, mode_c);
    if (kStages > 1 && (kAll || t + 1 < t_end)) step(t + 1, std::integral_constant<int, 1 % kStages>{}, mode_c);
    if (kStages > 2 && (kAll || t + 2 < t_end)) step(t + 2, std::integral_constant<int, 2 % kStages>{}, mode_c);
    if (kStages > 3 && (kAll || t + 3 < t_end)) step(t + 3, std::integral_constant<int, 3 % kStages>{}, mode_c);
    static_assert(kStages <= 4, "unroll more steps");
  };
  int t = t_begin;
  const int fast_end = hist_tiles < t_end ? hist_tiles : t_end;
  for (; t + kStages - 1 + kAhead < fast_end; t += kStages) group(t, std::integral_constant<int, kHist>{});
  for (; t < t_end; t += kStages) group(t, std::integral_constant<int, kGeneric>{});

  // ---- epilogue: normalise, write O [B, Nq, H, D] bf16 and LSE [B, H, Nq] (of this split's keys)
  __bf16* out = p.out;
  float* lse = p.lse;
  if (p.splits > 1) {
    out = p.out_part + (int64_t)split * ((int64_t)p.BH * p.Nq * D);
    lse = p.lse_part + (int64_t)split * ((int64_t)p.BH * p.Nq);
  }
  // A key range in which a query sees nothing (no tiles at all: a split of a workgroup that sees
  // few keys under the causal mask; or only keys of later causal blocks: row sum 0) reports zero
  // output and a log-sum-exp of -1e30, which is weight 0 in the merge.  Every query sees its own
  // block, so some range of it is real.
#pragma unroll
  for (int qs = 0; qs < 2; ++qs) {
    // the query's row sum: over the four lanes that share it
    float l_tot = w.l_run[qs];
    l_tot += __shfl_xor(l_tot, 16);
    l_tot += __shfl_xor(l_tot, 32);
    const bool nothing = !(l_tot > 0.f);
    const float inv = nothing ? 0.f : 1.f / l_tot;
    const int q = q0 + 16 * qs;
    if (q < p.Nq) {
      __bf16* orow = out + (((int64_t)b * p.Nq + q) * p.H + h) * D;
#pragma unroll
      for (int dt = 0; dt < Wave::DT; ++dt) {
        bf16x4 x;
#pragma unroll
        for (int c = 0; c < 4; ++c) x[c] = (__bf16)(w.o[dt][qs][c] * inv);
        *reinterpret_cast<bf16x4*>(orow + 16 * dt + 4 * g) = x;
      }
      if (g == 0) lse[bh * p.Nq + q] = nothing ? kNegBig : w.mc[qs] * kLn2 + __logf(l_tot);
    }
  }
}

// Combine the per-split results: softmax over the union of the splits' keys is the average of the
// splits' outputs weighted by exp(lse_s - lse).  One wave per (stream, query, head) row.
template <int D>
__global__ void __launch_bounds__(256) fwd_merge_kernel(FwdParams p, int64_t n_rows) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (b*Nq + q)*H + h
  if (row >= n_rows) return;
  const int lane = threadIdx.x & 63;
  const int h = (int)(row % p.H);
  const int64_t bq = row / p.H;
  const int q = (int)(bq % p.Nq);
  const int64_t b = bq / p.Nq;
  const int64_t lse_at = (b * p.H + h) * p.Nq + q;
  const int64_t out_stride = (int64_t)p.BH * p.Nq * D, lse_stride = (int64_t)p.BH * p.Nq;
  float m = kNegBig;
  for (int s = 0; s < p.splits; ++s) m = fmaxf(m, p.lse_part[s * lse_stride + lse_at]);
  float tot = 0.f, a0 = 0.f, a1 = 0.f;
  for (int s = 0; s < p.splits; ++s) {
    const float w = __expf(p.lse_part[s * lse_stride + lse_at] - m);
    tot += w;
    if (lane < D / 2) {
      const bf16x2 o = *reinterpret_cast<const bf16x2*>(p.out_part + s * out_stride + row * D + lane * 2);
      a0 = fmaf(w, (float)o[0], a0);
      a1 = fmaf(w, (float)o[1], a1);
    }
  }
  const float inv = 1.f / tot;
  if (lane < D / 2) {
    const bf16x2 o = {(__bf16)(a0 * inv), (__bf16)(a1 * inv)};
    *reinterpret_cast<bf16x2*>(p.out + row * D + lane * 2) = o;
  }
  if (lane == 0) p.lse[lse_at] = m + __logf(tot);
}

template <int D, int kStages, int kWaves, int OCC, bool kCausal>
hipError_t launch(const DevGeom& g, const AttnOperands& op, void* out, float* lse, void* parts, hipStream_t stream) {
  FwdParams p;
  p.q_rot = (const __bf16*)op.q_rot;
  p.kc_rot = (const __bf16*)op.kc_rot;
  p.v_chunk = (const __bf16*)op.v_chunk;
  p.k_cache = (const __bf16*)op.k_cache;
  p.v_cache = (const __bf16*)op.v_cache;
  p.out = (__bf16*)out;
  p.lse = lse;
  p.H = g.H;
  p.Nq = op.Nq;
  p.cache_rows = (int64_t)g.C * g.T;
  p.hist_rows = op.hist_rows;
  p.group = op.group;
  p.block_rows = op.block_rows;
  const int qtile = kWaves * 32;
  p.BH = g.B * g.H;
  p.q_tiles = (op.Nq + qtile - 1) / qtile;
  // a launch that would leave the chip under two rounds of workgroups is split over the keys
  p.splits = bf16_fwd_splits(g, op, parts != nullptr);
  p.out_part = (__bf16*)parts;
  p.lse_part = (float*)((char*)parts + (size_t)p.splits * p.BH * op.Nq * D * 2);
  dim3 grid(work_grid_size(p.q_tiles, p.BH * p.splits));
  {
    ProfileScope prof("attn_fwd_bf16", stream);
    attn_fwd_bf16_kernel<D, kStages, kWaves, OCC, kCausal><<<grid, dim3(kWaves * 64), 0, stream>>>(p);
  }
  if (p.splits > 1) {
    const int64_t n_rows = (int64_t)p.BH * op.Nq;
    ProfileScope prof("attn_fwd_merge", stream);
    fwd_merge_kernel<D><<<dim3((unsigned)((n_rows + 3) / 4)), 256, 0, stream>>>(p, n_rows);
  }
  return hipGetLastError();
}

}  // namespace

// ---- key-range split of launches that cannot fill the chip -----------------------------------
// The forward holds three workgroups per CU.  With fewer than two rounds of workgroups (one
// stream of 12 heads and 37 query tiles is 444 workgroups on 768 places) each (pair, query
// tile) is cut into `splits` key ranges, enough for two rounds, at most kMaxFwdSplits and
// never less than kMinTilesPerSplit key tiles each.
constexpr int kMaxFwdSplits = 8, kMinTilesPerSplit = 4, kFwdWorkgroupsPerCu = 3;

static int fwd_work_items(const DevGeom& g, int Nq) { return ((Nq + 127) / 128) * g.B * g.H; }

size_t bf16_fwd_split_bytes(const DevGeom& g, int Nq) {
  if (fwd_work_items(g, Nq) >= 2 * kFwdWorkgroupsPerCu * g.n_cus) return 0;
  return (size_t)kMaxFwdSplits * g.B * g.H * Nq * ((size_t)g.D * 2 + sizeof(float));
}

int bf16_fwd_splits(const DevGeom& g, const AttnOperands& op, bool have_parts) {
  if (!have_parts) return 1;
  const int items = fwd_work_items(g, op.Nq), places = kFwdWorkgroupsPerCu * g.n_cus;
  if (items >= 2 * places) return 1;
  int min_hist = INT32_MAX;
  for (int b = 0; b < g.B / op.group; ++b) min_hist = op.hist_rows.v[b] < min_hist ? op.hist_rows.v[b] : min_hist;
  // key tiles of the workgroup that sees the fewest: under causal blocks that is the first query
  // tile, which sees one block of the chunk (a range may still come out empty or unseen for some
  // queries: both report weight 0 to the merge)
  const int chunk_rows = op.block_rows > 0 && op.block_rows < op.Nq ? op.block_rows : op.Nq;
  const int tiles = (min_hist + KT - 1) / KT + (chunk_rows + KT - 1) / KT;
  int s = (2 * places + items - 1) / items;
  if (s > kMaxFwdSplits) s = kMaxFwdSplits;
  if (s > tiles / kMinTilesPerSplit) s = tiles / kMinTilesPerSplit;
  return s < 1 ? 1 : s;
}

hipError_t launch_attn_fwd_bf16(const DevGeom& g, const AttnOperands& op, void* out, float* lse, void* parts,
                                hipStream_t stream) {
  const bool causal = op.block_rows > 0;
  if (g.D == 128)
    return causal ? launch<128, 3, 4, 3, true>(g, op, out, lse, parts, stream) : launch<128, 3, 4, 3, false>(g, op, out, lse, parts, stream);
  return causal ? launch<64, 3, 4, 3, true>(g, op, out, lse, parts, stream) : launch<64, 3, 4, 3, false>(g, op, out, lse, parts, stream);
}

}  // namespace astro
