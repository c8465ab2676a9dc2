// Chunk attention forward over the rolling cache, bf16 MFMA with fp32 accumulation.
//
// One workgroup = 4 wavefronts = 4 * 32 * NQB consecutive queries of one (stream, head).
// The visible keys (resident ring rows, then the chunk's own rows) are walked in tiles of
// 64; K and V tiles are streamed into LDS by direct-to-LDS loads (two LDS buffers, one
// barrier per tile).  Everything is computed transposed so that every lane owns ONE query:
//   S^T[key][q] = K * Q~^T      (A = K tile from LDS, B = Q~ held in registers)
//   O^T[d][q]  += V^T * P^T     (A = V tile through the transposing LDS read,
//                                B = P^T taken straight from the S^T accumulators)
// so the row maximum / sum of the online softmax are in-lane reductions plus one
// exchange with the partner lane l^32, and the rescale factor is a per-lane scalar.
// MFMA and vector-ALU work of one wave do not overlap on this hardware; the overlap
// comes from two workgroups (two waves per SIMD) being resident per CU.
#include <cstdlib>

#include "kernels.hpp"
#include "mfma_common.hpp"

namespace astro {
namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int KT = 64;  // keys per LDS tile

struct FwdParams {
  const __bf16* q_rot;
  const __bf16* kc_rot;
  const __bf16* v_chunk;
  const __bf16* k_cache;
  const __bf16* v_cache;
  __bf16* out;
  float* lse;
  int H, Nq;
  int64_t cache_rows;  // C*T
  float scale_log2e, scale;
  StreamInts hist_rows;
};

template <int D, int NQB>
struct FwdWave {
  static constexpr int QSTEPS = D / 16;  // MFMA k-steps of the QK product
  static constexpr int DB = D / 32;      // 32-row blocks of O^T

  bf16x8 qreg[NQB][QSTEPS];
  f32x16 o[NQB][DB];
  float m_run[NQB], l_run[NQB];  // running max (raw dot units), per-lane partial row sum
  OperandAddr<D> addr;
  int g;
  float scale_log2e;

  __device__ __forceinline__ void init(int lane, float sl2e) {
    g = lane >> 5;
    scale_log2e = sl2e;
    addr.init(lane);
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      m_run[qb] = kNegBig;
      l_run[qb] = 0.f;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
    }
  }

  // One 64-key tile.  `valid` = number of live keys in the tile (only read when TAIL).
  template <bool TAIL>
  __device__ __forceinline__ void tile(const char* ks, const char* vs, int valid) {
#pragma unroll
    for (int kb = 0; kb < KT / 32; ++kb) {
      // ---- S^T block: keys 32kb .. 32kb+31 of the tile x the wave's queries
      f32x16 s[NQB];
#pragma unroll
      for (int st = 0; st < QSTEPS; ++st) {
        const bf16x8 a = read_rows8<D>(ks, addr.row[st], kb);
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
          if (st == 0) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            s[qb] = mfma32(a, qreg[qb][st], zero);
          } else {
            s[qb] = mfma32(a, qreg[qb][st], s[qb]);
          }
        }
      }
      if (TAIL) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const bool dead = 32 * kb + acc_row(r, g) >= valid;
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb) s[qb][r] = dead ? kNegBig : s[qb][r];
        }
      }
      // ---- online softmax; P^T (bf16) becomes the B operand of the PV product
      bf16x8 pb[NQB][2];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        float mx = fmaxf(s[qb][0], s[qb][1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, s[qb][r]), s[qb][r + 1]);
        mx = max_with_partner32(mx);
        if (__any(mx > m_run[qb])) {
          const float m_new = fmaxf(m_run[qb], mx);
          const float alpha = fast_exp2((m_run[qb] - m_new) * scale_log2e);
          l_run[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
          m_run[qb] = m_new;
        }
        const float mc = m_run[qb] * scale_log2e;
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const f32x2 e = {fast_exp2(fmaf(s[qb][r], scale_log2e, -mc)), fast_exp2(fmaf(s[qb][r + 1], scale_log2e, -mc))};
          const bf16x2 pk = __builtin_convertvector(e, bf16x2);
          // the row sum is taken over the rounded values the PV product uses
          sum = add_pair(pk, sum);
          pb[qb][r >> 3][r & 7] = pk[0];
          pb[qb][r >> 3][(r & 7) + 1] = pk[1];
        }
        l_run[qb] += sum;
      }
      // ---- O^T += V^T P^T for these 32 keys (16 keys per MFMA k-step)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 a = read_cols8<D>(vs, addr.tr[db], 32 * kb + 16 * s2);
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb) o[qb][db] = mfma32(a, pb[qb][s2], o[qb][db]);
        }
      }
    }
  }
};

template <int D, int NQB, int OCC>
__global__ void __launch_bounds__(kThreads, OCC) attn_fwd_bf16_kernel(FwdParams p) {
  using Wave = FwdWave<D, NQB>;
  constexpr int TILE_BYTES = KT * D * 2;
  __shared__ __attribute__((aligned(1024))) char lds[4 * TILE_BYTES];  // K0 V0 K1 V1

  const int b = blockIdx.z, h = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i32 = lane & 31, g = lane >> 5;
  const int hist = p.hist_rows.v[b];
  // key tiles: first the resident ring rows, then the chunk's rows, each with its own tail
  const int hist_tiles = (hist + KT - 1) / KT;
  const int ntiles = hist_tiles + (p.Nq + KT - 1) / KT;
  const int q0 = (blockIdx.x * kWaves + wave) * 32 * NQB;
  const int64_t bh = (int64_t)b * p.H + h;

  Wave w;
  w.init(lane, p.scale_log2e);
  // Q~ as the B operand: lane (i32, g) holds Q~[q0 + 32*qb + i32][16*st + 8g .. +7]
  {
    const __bf16* qh = p.q_rot + bh * (int64_t)p.Nq * D;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int q = q0 + 32 * qb + i32;
#pragma unroll
      for (int st = 0; st < Wave::QSTEPS; ++st) {
        bf16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
        if (q < p.Nq) x = *reinterpret_cast<const bf16x8*>(qh + (int64_t)q * D + st * 16 + g * 8);
        w.qreg[qb][st] = x;
      }
    }
  }

  const RowSegment k_hist = make_segment(p.k_cache + bh * p.cache_rows * D, D, hist, D);
  const RowSegment v_hist = make_segment(p.v_cache + bh * p.cache_rows * D, D, hist, D);
  const RowSegment k_chunk = make_segment(p.kc_rot + bh * p.Nq * D, D, p.Nq, D);
  const RowSegment v_chunk = make_segment(p.v_chunk + ((int64_t)b * p.Nq * p.H + h) * D, (int64_t)p.H * D, p.Nq, D);
  TileStreamer<D, KT, kWaves> ts;
  ts.init();
  const uint32_t off_dense = ts.lane_offset(k_hist);    // stride D: ring K, ring V, rotated chunk K
  const uint32_t off_vchunk = ts.lane_offset(v_chunk);  // stride H*D
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

  for (int t = 0; t < ntiles; ++t) {
    if (t + 1 < ntiles) issue(t + 1);
    const char* kbuf = lds + (t & 1) * 2 * TILE_BYTES;
    const int valid = t < hist_tiles ? hist - t * KT : p.Nq - (t - hist_tiles) * KT;
    if (valid >= KT)
      w.template tile<false>(kbuf, kbuf + TILE_BYTES, KT);
    else
      w.template tile<true>(kbuf, kbuf + TILE_BYTES, valid);
    wait_vmem();
    __syncthreads();
  }

  // ---- epilogue: normalise, write O [B, Nq, H, D] bf16 and LSE [B, H, Nq]
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int q = q0 + 32 * qb + i32;
    const float l_tot = sum_with_partner32(w.l_run[qb]);
    const float inv = 1.f / l_tot;
    if (q < p.Nq) {
      __bf16* orow = p.out + (((int64_t)b * p.Nq + q) * p.H + h) * D;
#pragma unroll
      for (int db = 0; db < Wave::DB; ++db)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          bf16x4 x;
#pragma unroll
          for (int c = 0; c < 4; ++c) x[c] = (__bf16)(w.o[qb][db][4 * rr + c] * inv);
          *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * rr + 4 * g) = x;
        }
      if (g == 0) p.lse[bh * p.Nq + q] = w.m_run[qb] * p.scale + __logf(l_tot);
    }
  }
}

template <int D, int NQB, int OCC>
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
  const int qtile = kWaves * 32 * NQB;
  dim3 grid((op.Nq + qtile - 1) / qtile, g.H, g.B);
  ProfileScope prof("attn_fwd_bf16", stream);
  attn_fwd_bf16_kernel<D, NQB, OCC><<<grid, dim3(kThreads), 0, stream>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_fwd_bf16(const DevGeom& g, const AttnOperands& op, void* out, float* lse, hipStream_t stream) {
  if (g.D == 128) return launch<128, 1, 2>(g, op, out, lse, stream);
  return launch<64, 1, 2>(g, op, out, lse, stream);
}

}  // namespace astro
