// Chunk attention forward over the rolling cache, bf16 MFMA with fp32 accumulation.
//
// One workgroup = 4 wavefronts = 4 * 32 consecutive queries of one (stream, head).
// The visible keys (resident ring rows, then the chunk's own rows) are walked in tiles of
// 32; K and V tiles are streamed into a ring of 4 LDS stages by direct-to-LDS loads issued
// three tiles ahead, one barrier per tile.  Everything is computed transposed so that
// every lane owns ONE query:
//   S^T[key][q] = K * Q~^T      (A = K tile from LDS, B = Q~ held in registers)
//   O^T[d][q]  += V^T * P^T     (A = V tile through the transposing LDS read,
//                                B = P^T taken straight from the S^T accumulators)
// so the row maximum / sum of the softmax are in-lane reductions plus one exchange with
// the partner lane l^32, and the rescale factor is a per-lane scalar.
//
// Because tile t+1 is already visible while tile t is processed, its K operands are read
// into registers before the barrier and the MFMAs of the next tile start without an LDS
// round trip.
//
// Softmax reference: probabilities are taken relative to a per-query reference M that is
// only raised when a tile's maximum exceeds it by more than kRescaleSlack (in log2
// units); fp32 accumulators and the bf16 exponent range make any smaller excess exact
// enough, and the 64 accumulator multiplies of a rescale leave the common path.
// MFMA and vector-ALU work of one wave do not overlap on this hardware; the overlap
// comes from two workgroups (two waves per SIMD) being resident per CU.
#include <cstdlib>

#include "kernels.hpp"
#include "mfma_common.hpp"

namespace astro {
namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int KT = 32;                 // keys per LDS tile
constexpr float kRescaleSlack = 40.f;  // log2 units: p <= 2^40 before the reference moves

struct FwdParams {
  const __bf16* q_rot;
  const __bf16* kc_rot;
  const __bf16* v_chunk;
  const __bf16* k_cache;
  const __bf16* v_cache;
  __bf16* out;
  float* lse;
  int H, Nq, BH, q_tiles;
  int64_t cache_rows;  // C*T
  float scale_log2e, scale;
  StreamInts hist_rows;
};

// x *= a in place: keeps the accumulator in its registers on the rare rescale path
__device__ __forceinline__ float scale_in_place(float x, float a) {
  asm volatile("v_mul_f32 %0, %1, %0" : "+v"(x) : "v"(a));
  return x;
}

template <int D, bool KPREF>
struct FwdWave {
  static constexpr int QSTEPS = D / 16;  // MFMA k-steps of the QK product
  static constexpr int DB = D / 32;      // 32-row blocks of O^T

  bf16x8 qreg[QSTEPS];
  bf16x8 kfrag[KPREF ? QSTEPS : 1];  // K operands of the tile about to be processed
  f32x16 o[DB];
  float m_ref, l_run;  // reference (raw dot units), per-lane partial row sum
  OperandAddr<D> addr;
  int g;
  float scale_log2e, slack_raw;

  __device__ __forceinline__ void init(int lane, float sl2e) {
    g = lane >> 5;
    scale_log2e = sl2e;
    slack_raw = kRescaleSlack / sl2e;
    addr.init(lane);
    m_ref = kNegBig;
    l_run = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  }

  __device__ __forceinline__ void load_kfrag(const char* ks) {
#pragma unroll
    for (int st = 0; st < QSTEPS; ++st) kfrag[st] = read_rows8<D>(ks, addr.row[st], 0);
  }

  // One 32-key tile whose K operands are in kfrag; vs = its V tile, ks_next = K tile of the
  // following one (already visible), read into kfrag for the next call.
  // Rows of a tile past the end of its segment are zero in LDS: they add nothing to O
  // (V = 0) but do add exp(0 - M) each to the row sum, which `dead_keys` (their number in
  // this tile, wave-uniform) takes out again.
  __device__ __forceinline__ void tile(const char* ks, const char* vs, const char* ks_next, bool has_next, int dead_keys) {
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 s;
    if constexpr (KPREF) {
#pragma unroll
      for (int st = 0; st < QSTEPS; ++st) s = mfma32(kfrag[st], qreg[st], st == 0 ? zero : s);
      // next tile's K operands: their LDS latency hides under this tile's softmax and PV
      if (has_next) load_kfrag(ks_next);
    } else {
#pragma unroll
      for (int st = 0; st < QSTEPS; ++st) s = mfma32(read_rows8<D>(ks, addr.row[st], 0), qreg[st], st == 0 ? zero : s);
    }

    float mx = fmaxf(s[0], s[1]);
#pragma unroll
    for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, s[r]), s[r + 1]);
    mx = max_with_partner32(mx);
    if (__builtin_expect(__any(mx > m_ref + slack_raw), 0)) {
      const float m_new = fmaxf(m_ref, mx);
      const float alpha = fast_exp2((m_ref - m_new) * scale_log2e);
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = scale_in_place(o[db][r], alpha);
      m_ref = m_new;
    }
    const float mc = m_ref * scale_log2e;
    bf16x8 pb[2];
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      const f32x2 e = {fast_exp2(fmaf(s[r], scale_log2e, -mc)), fast_exp2(fmaf(s[r + 1], scale_log2e, -mc))};
      const bf16x2 pk = __builtin_convertvector(e, bf16x2);
      sum = add_pair(pk, sum);  // the row sum runs over the rounded values the PV product uses
      pb[r >> 3][r & 7] = pk[0];
      pb[r >> 3][(r & 7) + 1] = pk[1];
    }
    if (dead_keys > 0) {
      // keys KT - dead_keys .. KT-1 of the tile are dead; this lane saw those among
      // acc_row(r, g), each as exp2(0 - M) rounded to bf16
      const float e0 = fast_exp2(-mc);
      const f32x2 e = {e0, e0};
      const bf16x2 pk = __builtin_convertvector(e, bf16x2);
      int mine = 0;
#pragma unroll
      for (int r = 0; r < 16; ++r) mine += (acc_row(r, g) >= KT - dead_keys) ? 1 : 0;
      sum -= (float)mine * (float)pk[0];
    }
    l_run += sum;
    // O^T += V^T P^T (16 keys per MFMA k-step)
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int db = 0; db < DB; ++db) o[db] = mfma32(read_cols8<D>(vs, addr.tr[db], 16 * s2), pb[s2], o[db]);
  }
};

template <int D, int kStages, bool KPREF, int OCC>
__global__ void __launch_bounds__(kThreads, OCC) attn_fwd_bf16_kernel(FwdParams p) {
  using Wave = FwdWave<D, KPREF>;
  constexpr int kAhead = kStages - 1;  // tiles in flight ahead of the one being processed
  constexpr int TILE_BYTES = KT * D * 2;
  constexpr int STAGE_BYTES = 2 * TILE_BYTES;  // K tile, V tile
  __shared__ __attribute__((aligned(1024))) char lds[kStages * STAGE_BYTES];

  const WorkItem item = work_item(p.q_tiles, p.BH);
  if (!item.valid) return;
  const int b = item.bh / p.H, h = item.bh % p.H;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i32 = lane & 31, g = lane >> 5;
  const int hist = p.hist_rows.v[b];
  // key tiles: first the resident ring rows, then the chunk's rows, each with its own tail
  const int hist_tiles = (hist + KT - 1) / KT;
  const int ntiles = hist_tiles + (p.Nq + KT - 1) / KT;
  const int q = (item.tile * kWaves + wave) * 32 + i32;
  const int64_t bh = (int64_t)b * p.H + h;

  Wave w;
  w.init(lane, p.scale_log2e);
  // Q~ as the B operand: lane (i32, g) holds Q~[q][16*st + 8g .. +7]
  {
    const __bf16* qrow = p.q_rot + (bh * p.Nq + (q < p.Nq ? q : 0)) * D;
#pragma unroll
    for (int st = 0; st < Wave::QSTEPS; ++st) {
      bf16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
      if (q < p.Nq) x = *reinterpret_cast<const bf16x8*>(qrow + st * 16 + g * 8);
      w.qreg[st] = x;
    }
  }

  const RowSegment k_hist = make_segment(p.k_cache + bh * p.cache_rows * D, D, hist, D);
  const RowSegment v_hist = make_segment(p.v_cache + bh * p.cache_rows * D, D, hist, D);
  const RowSegment k_chunk = make_segment(p.kc_rot + bh * p.Nq * D, D, p.Nq, D);
  const RowSegment v_chunk = make_segment(p.v_chunk + ((int64_t)b * p.Nq * p.H + h) * D, (int64_t)p.H * D, p.Nq, D);
  using Streamer = TileStreamer<D, KT, kWaves>;
  Streamer ts;
  ts.init();
  const uint32_t off_dense = ts.lane_offset(k_hist);    // stride D: ring K, ring V, rotated chunk K
  const uint32_t off_vchunk = ts.lane_offset(v_chunk);  // stride H*D
  auto issue = [&](int t, char* stage) {
    if (t < hist_tiles) {
      ts.issue(k_hist, off_dense, t * KT, stage);
      ts.issue(v_hist, off_dense, t * KT, stage + TILE_BYTES);
    } else {
      ts.issue(k_chunk, off_dense, (t - hist_tiles) * KT, stage);
      ts.issue(v_chunk, off_vchunk, (t - hist_tiles) * KT, stage + TILE_BYTES);
    }
  };
  auto dead_in = [&](int t) {
    const int live = t < hist_tiles ? hist - t * KT : p.Nq - (t - hist_tiles) * KT;
    return live >= KT ? 0 : KT - live;
  };
  // Invariant at the top of tile t: tiles t .. t+kAhead-1 have landed and are visible to
  // every wave except the last of them, whose loads may still be in flight; the stage of
  // tile t+kAhead (= that of tile t-1) is free.
  constexpr int kLoadsPerTile = 2 * Streamer::kInsts;  // per wave
#pragma unroll
  for (int t = 0; t < kAhead; ++t)
    if (t < ntiles) issue(t, lds + t * STAGE_BYTES);
  if (ntiles >= kAhead && kAhead > 1)
    wait_vmem_except<kLoadsPerTile>();
  else
    wait_vmem();
  __syncthreads();
  if constexpr (KPREF) w.load_kfrag(lds);

  auto step = [&](int t, auto stage_c) {
    constexpr int ST = decltype(stage_c)::value;
    if (t + kAhead < ntiles) issue(t + kAhead, lds + ((ST + kAhead) % kStages) * STAGE_BYTES);
    w.tile(lds + ST * STAGE_BYTES, lds + ST * STAGE_BYTES + TILE_BYTES, lds + ((ST + 1) % kStages) * STAGE_BYTES,
           t + 1 < ntiles, dead_in(t));
    // tile t+1 .. t+kAhead-1 must have landed before the next tile starts; the newest may stay in flight
    if (t + kAhead < ntiles && kAhead > 1)
      wait_vmem_except<kLoadsPerTile>();
    else
      wait_vmem();
    __syncthreads();
  };
  // kStages tiles per trip so that every LDS stage is a compile-time offset
  for (int t = 0; t < ntiles; t += kStages) {
    step(t, std::integral_constant<int, 0>{});
    if (kStages > 1 && t + 1 < ntiles) step(t + 1, std::integral_constant<int, 1 % kStages>{});
    if (kStages > 2 && t + 2 < ntiles) step(t + 2, std::integral_constant<int, 2 % kStages>{});
    if (kStages > 3 && t + 3 < ntiles) step(t + 3, std::integral_constant<int, 3 % kStages>{});
  }

  // ---- epilogue: normalise, write O [B, Nq, H, D] bf16 and LSE [B, H, Nq]
  const float l_tot = sum_with_partner32(w.l_run);
  const float inv = 1.f / l_tot;
  if (q < p.Nq) {
    __bf16* orow = p.out + (((int64_t)b * p.Nq + q) * p.H + h) * D;
#pragma unroll
    for (int db = 0; db < Wave::DB; ++db)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        bf16x4 x;
#pragma unroll
        for (int c = 0; c < 4; ++c) x[c] = (__bf16)(w.o[db][4 * rr + c] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * rr + 4 * g) = x;
      }
    if (g == 0) p.lse[bh * p.Nq + q] = w.m_ref * p.scale + __logf(l_tot);
  }
}

template <int D, int kStages, bool KPREF, int OCC>
hipError_t launch(const DevGeom& g, const AttnOperands& op, void* out, float* lse, hipStream_t stream) {
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
  p.scale = 1.0f / sqrtf((float)D);
  p.scale_log2e = p.scale * kLog2e;
  p.hist_rows = op.hist_rows;
  const int qtile = kWaves * 32;
  p.BH = g.B * g.H;
  p.q_tiles = (op.Nq + qtile - 1) / qtile;
  dim3 grid(work_grid_size(p.q_tiles, p.BH));
  ProfileScope prof("attn_fwd_bf16", stream);
  attn_fwd_bf16_kernel<D, kStages, KPREF, OCC><<<grid, dim3(kThreads), 0, stream>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_fwd_bf16(const DevGeom& g, const AttnOperands& op, void* out, float* lse, hipStream_t stream) {
  static const int variant = [] {
    const char* e = getenv("ASTRO_FWD_VARIANT");
    return e ? atoi(e) : 0;
  }();
  if (g.D == 128) {
    if (variant == 1) return launch<128, 4, true, 2>(g, op, out, lse, stream);
    if (variant == 2) return launch<128, 3, false, 2>(g, op, out, lse, stream);
    if (variant == 3) return launch<128, 4, false, 2>(g, op, out, lse, stream);
    return launch<128, 3, false, 3>(g, op, out, lse, stream);
  }
  return launch<64, 3, false, 3>(g, op, out, lse, stream);
}

}  // namespace astro
