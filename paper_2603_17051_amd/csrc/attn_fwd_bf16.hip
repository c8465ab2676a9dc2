// Chunk attention forward over the rolling cache, bf16 MFMA with fp32 accumulation.
//
// One workgroup = 4 wavefronts = 4 * 32 * NQB consecutive queries of one (stream, head).
// The visible keys (resident ring rows, then the chunk's own rows) are walked in tiles of
// 64; K and V tiles are staged through LDS (register prefetch, two LDS buffers, one
// barrier per tile).  Everything is computed transposed so that every lane owns ONE query:
//   S^T[key][q] = K * Q~^T      (A = K tile from LDS, B = Q~ held in registers)
//   O^T[d][q]  += V^T * P^T     (A = V tile through the transposing LDS read,
//                                B = P^T taken straight from the S^T accumulators)
// so the row maximum / sum of the online softmax are in-lane reductions plus one
// exchange with the partner lane l^32, and the rescale factor is a per-lane scalar.
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

template <int D, int NQB, int OCC>
__global__ void __launch_bounds__(kThreads, OCC) attn_fwd_bf16_kernel(FwdParams p) {
  constexpr int QSTEPS = D / 16;  // MFMA k-steps of the QK product
  constexpr int DB = D / 32;      // 32-row blocks of O^T
  constexpr int TILE_BYTES = KT * D * 2;
  __shared__ __attribute__((aligned(16))) char lds[4 * TILE_BYTES];  // K0 V0 K1 V1

  const int b = blockIdx.z, h = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i32 = lane & 31, g = lane >> 5, i16 = lane & 15, blk = (lane >> 4) & 1;
  const int hist = p.hist_rows.v[b];
  const int nk = hist + p.Nq;
  const int ntiles = (nk + KT - 1) / KT;
  const int q0 = (blockIdx.x * kWaves + wave) * 32 * NQB;

  // Q~ as the B operand: lane (i32, g) holds Q~[q0 + 32*qb + i32][16*st + 8g .. +7]
  bf16x8 qreg[NQB][QSTEPS];
  {
    const __bf16* qh = p.q_rot + ((int64_t)b * p.H + h) * (int64_t)p.Nq * D;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int q = q0 + 32 * qb + i32;
#pragma unroll
      for (int st = 0; st < QSTEPS; ++st) {
        bf16x8 x = {0, 0, 0, 0, 0, 0, 0, 0};
        if (q < p.Nq) x = *reinterpret_cast<const bf16x8*>(qh + (int64_t)q * D + st * 16 + g * 8);
        qreg[qb][st] = x;
      }
    }
  }

  f32x16 o[NQB][DB];
  float m_run[NQB], l_run[NQB];  // running max (raw dot units) and per-lane partial sum
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m_run[qb] = kNegBig;
    l_run[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
  }

  const int64_t bh = (int64_t)b * p.H + h;
  const RowSource ksrc{p.k_cache + bh * p.cache_rows * D, D, hist, p.kc_rot + bh * p.Nq * D, D, p.Nq};
  const RowSource vsrc{p.v_cache + bh * p.cache_rows * D, D, hist, p.v_chunk + ((int64_t)b * p.Nq * p.H + h) * D,
                       (int64_t)p.H * D, p.Nq};
  TilePairLoader<D, KT, kThreads> ld;
  ld.load(ksrc, vsrc, 0);
  ld.store(lds, lds + TILE_BYTES);
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    const char* ks = lds + (t & 1) * 2 * TILE_BYTES;
    const char* vs = ks + TILE_BYTES;
    if (t + 1 < ntiles) ld.load(ksrc, vsrc, t + 1);
    const bool tail = (t + 1) * KT > nk;

#pragma unroll
    for (int kb = 0; kb < KT / 32; ++kb) {
      // ---- S^T block: keys 32kb .. 32kb+31 of the tile x the wave's queries
      f32x16 s[NQB];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[qb][r] = 0.f;
#pragma unroll
      for (int st = 0; st < QSTEPS; ++st) {
        const bf16x8 a = lds_read_row8<D>(ks, 32 * kb + i32, 2 * st + g);
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) s[qb] = mfma32(a, qreg[qb][st], s[qb]);
      }
      if (tail) {
        const int key0 = t * KT + 32 * kb;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const bool dead = key0 + acc_row(r, g) >= nk;
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb) s[qb][r] = dead ? kNegBig : s[qb][r];
        }
      }
      // ---- online softmax; P^T (bf16) becomes the B operand of the PV product
      bf16x8 pb[NQB][2];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        float mx = s[qb][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[qb][r]);
        mx = max_with_partner32(mx);
        const float m_new = fmaxf(m_run[qb], mx);
        if (__any(m_new > m_run[qb])) {
          const float alpha = fast_exp2((m_run[qb] - m_new) * p.scale_log2e);
          l_run[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
          m_run[qb] = m_new;
        }
        const float mc = m_run[qb] * p.scale_log2e;
        float pr[16];
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          pr[r] = fast_exp2(fmaf(s[qb][r], p.scale_log2e, -mc));
          sum += pr[r];
        }
        l_run[qb] += sum;
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int j = 0; j < 8; ++j) pb[qb][s2][j] = (__bf16)pr[8 * s2 + j];
      }
      // ---- O^T += V^T P^T for these 32 keys
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const int key0 = 32 * kb + 16 * s2 + 4 * g;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const int col0 = 32 * db + 16 * blk;
          const bf16x8 a = concat4(lds_read_col4<D>(vs, key0, col0, i16), lds_read_col4<D>(vs, key0 + 8, col0, i16));
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb) o[qb][db] = mfma32(a, pb[qb][s2], o[qb][db]);
        }
      }
    }

    if (t + 1 < ntiles) {
      char* kn = lds + ((t + 1) & 1) * 2 * TILE_BYTES;
      ld.store(kn, kn + TILE_BYTES);
    }
    __syncthreads();
  }

  // ---- epilogue: normalise, write O [B, Nq, H, D] bf16 and LSE [B, H, Nq]
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int q = q0 + 32 * qb + i32;
    const float l_tot = sum_with_partner32(l_run[qb]);
    const float inv = 1.f / l_tot;
    if (q < p.Nq) {
      __bf16* orow = p.out + (((int64_t)b * p.Nq + q) * p.H + h) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          bf16x4 w;
#pragma unroll
          for (int c = 0; c < 4; ++c) w[c] = (__bf16)(o[qb][db][4 * rr + c] * inv);
          *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * rr + 4 * g) = w;
        }
      if (g == 0) p.lse[((int64_t)b * p.H + h) * p.Nq + q] = m_run[qb] * p.scale + __logf(l_tot);
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

int g_fwd_variant = 0;  // tuning knob: 0 = 64 queries per wave, 1 = 32 queries per wave

hipError_t launch_attn_fwd_bf16(const DevGeom& g, const AttnOperands& op, void* out, float* lse, hipStream_t stream) {
  if (g.D == 128) {
    if (g_fwd_variant == 1) return launch<128, 1, 2>(g, op, out, lse, stream);
    return launch<128, 2, 1>(g, op, out, lse, stream);
  }
  if (g_fwd_variant == 1) return launch<64, 1, 2>(g, op, out, lse, stream);
  return launch<64, 2, 1>(g, op, out, lse, stream);
}

}  // namespace astro
