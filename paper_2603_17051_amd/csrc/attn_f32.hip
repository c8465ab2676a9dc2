// fp32 debug path of chunk attention over the rolling cache: the definition written as
// plain kernels (score matrix in a scratch buffer, row softmax, products), no MFMA, no
// tiling.  Slow by design; it exists to separate indexing / rotary / ring mistakes from
// MFMA-layout mistakes and to meet a 1e-5 tolerance against the fp64 definition.
#include "kernels.hpp"

namespace astro {
namespace {

struct F32Operands {
  const float* q_rot;
  const float* kc_rot;
  const float* v_chunk;
  const float* k_cache;
  const float* v_cache;
  int H, D, Nq, nk_stride, group;
  int block_rows;  // causal block inside the chunk in token rows, 0 = none
  int64_t cache_rows;
  float scale;
  StreamInts hist_rows;
};

__device__ __forceinline__ const float* key_row(const F32Operands& p, int b, int h, int j) {
  const int cb = b / p.group;  // cache stream of candidate b
  const int hist = p.hist_rows.v[cb];
  if (j < hist) return p.k_cache + (((int64_t)cb * p.H + h) * p.cache_rows + j) * p.D;
  return p.kc_rot + (((int64_t)b * p.H + h) * p.Nq + (j - hist)) * p.D;
}
__device__ __forceinline__ const float* value_row(const F32Operands& p, int b, int h, int j) {
  const int cb = b / p.group;
  const int hist = p.hist_rows.v[cb];
  if (j < hist) return p.v_cache + (((int64_t)cb * p.H + h) * p.cache_rows + j) * p.D;
  return p.v_chunk + (((int64_t)b * p.Nq + (j - hist)) * p.H + h) * p.D;
}
__device__ __forceinline__ float* score_row(float* s, const F32Operands& p, int bh, int q) {
  return s + ((int64_t)bh * p.Nq + q) * p.nk_stride;
}

__device__ float block_reduce(float x, bool is_max, float* red) {
  const int t = threadIdx.x;
  red[t] = x;
  __syncthreads();
  for (int s = blockDim.x / 2; s > 0; s >>= 1) {
    if (t < s) red[t] = is_max ? fmaxf(red[t], red[t + s]) : red[t] + red[t + s];
    __syncthreads();
  }
  const float r = red[0];
  __syncthreads();
  return r;
}

// S[q][j] = scale * <q~_q, k~_j>; grid (ceil(nk_stride/256), Nq, B*H).  A chunk key in a later
// causal block than the query gets a score so low that every later step sees probability 0.
__global__ void scores_kernel(F32Operands p, float* s) {
  const int bh = blockIdx.z, b = bh / p.H, h = bh % p.H, q = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int hist = p.hist_rows.v[b / p.group];
  const int nk = hist + p.Nq;
  if (j >= nk) return;
  if (p.block_rows > 0 && j >= hist && (j - hist) / p.block_rows > q / p.block_rows) {
    score_row(s, p, bh, q)[j] = -3.0e38f;
    return;
  }
  const float* qr = p.q_rot + ((int64_t)bh * p.Nq + q) * p.D;
  const float* kr = key_row(p, b, h, j);
  float acc = 0.f;
  for (int d = 0; d < p.D; ++d) acc = fmaf(qr[d], kr[d], acc);
  score_row(s, p, bh, q)[j] = acc * p.scale;
}

// in place S -> P = softmax row; lse; grid (Nq, B*H), 256 threads
__global__ void softmax_kernel(F32Operands p, float* s, float* lse) {
  __shared__ float red[256];
  const int bh = blockIdx.y, b = bh / p.H, q = blockIdx.x;
  const int nk = p.hist_rows.v[b / p.group] + p.Nq;
  float* row = score_row(s, p, bh, q);
  float m = -3.0e38f;
  for (int j = threadIdx.x; j < nk; j += blockDim.x) m = fmaxf(m, row[j]);
  m = block_reduce(m, true, red);
  float z = 0.f;
  for (int j = threadIdx.x; j < nk; j += blockDim.x) z += expf(row[j] - m);
  z = block_reduce(z, false, red);
  const float l = m + logf(z);
  for (int j = threadIdx.x; j < nk; j += blockDim.x) row[j] = expf(row[j] - l);
  if (threadIdx.x == 0) lse[(int64_t)bh * p.Nq + q] = l;
}

// O[q][d] = sum_j P[q][j] V[j][d]; grid (Nq, B*H), D threads
__global__ void pv_kernel(F32Operands p, const float* s, float* out) {
  const int bh = blockIdx.y, b = bh / p.H, h = bh % p.H, q = blockIdx.x, d = threadIdx.x;
  const int nk = p.hist_rows.v[b / p.group] + p.Nq;
  const float* row = s + ((int64_t)bh * p.Nq + q) * p.nk_stride;
  float acc = 0.f;
  for (int j = 0; j < nk; ++j) acc = fmaf(row[j], value_row(p, b, h, j)[d], acc);
  out[(((int64_t)b * p.Nq + q) * p.H + h) * p.D + d] = acc;
}

// ---- backward -----------------------------------------------------------------
// in place S -> P = exp(S - lse); delta[q] = <dO_q, O_q>; grid (Nq, B*H), 256 threads
__global__ void probs_delta_kernel(F32Operands p, float* s, const float* lse, const float* out, const float* dout,
                                   float* delta) {
  __shared__ float red[256];
  const int bh = blockIdx.y, b = bh / p.H, h = bh % p.H, q = blockIdx.x;
  const int nk = p.hist_rows.v[b / p.group] + p.Nq;
  float* row = score_row(s, p, bh, q);
  const float l = lse[(int64_t)bh * p.Nq + q];
  for (int j = threadIdx.x; j < nk; j += blockDim.x) row[j] = expf(row[j] - l);
  const int64_t off = (((int64_t)b * p.Nq + q) * p.H + h) * p.D;
  float x = 0.f;
  for (int d = threadIdx.x; d < p.D; d += blockDim.x) x += out[off + d] * dout[off + d];
  x = block_reduce(x, false, red);
  if (threadIdx.x == 0) delta[(int64_t)bh * p.Nq + q] = x;
}

// dS[q][j] = P[q][j] * (<dO_q, V_j> - delta_q); grid (ceil(nk_stride/256), Nq, B*H)
__global__ void dscores_kernel(F32Operands p, const float* prob, const float* dout, const float* delta, float* ds) {
  const int bh = blockIdx.z, b = bh / p.H, h = bh % p.H, q = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int nk = p.hist_rows.v[b / p.group] + p.Nq;
  if (j >= nk) return;
  const float* dor = dout + (((int64_t)b * p.Nq + q) * p.H + h) * p.D;
  const float* vr = value_row(p, b, h, j);
  float acc = 0.f;
  for (int d = 0; d < p.D; ++d) acc = fmaf(dor[d], vr[d], acc);
  const int64_t o = ((int64_t)bh * p.Nq + q) * p.nk_stride + j;
  ds[o] = prob[o] * (acc - delta[(int64_t)bh * p.Nq + q]);
}

// dQ~[q][d] = scale * sum_j dS[q][j] K~[j][d]; grid (Nq, B*H), D threads; head-major out
__global__ void dq_kernel(F32Operands p, const float* ds, float* dq_rot) {
  const int bh = blockIdx.y, b = bh / p.H, h = bh % p.H, q = blockIdx.x, d = threadIdx.x;
  const int nk = p.hist_rows.v[b / p.group] + p.Nq;
  const float* row = ds + ((int64_t)bh * p.Nq + q) * p.nk_stride;
  float acc = 0.f;
  for (int j = 0; j < nk; ++j) acc = fmaf(row[j], key_row(p, b, h, j)[d], acc);
  dq_rot[((int64_t)bh * p.Nq + q) * p.D + d] = acc * p.scale;
}

// chunk keys only (the cached context is a constant):
// dK~[jc][d] = scale * sum_q dS[q][hist+jc] Q~[q][d];  dV[jc][d] = sum_q P[q][hist+jc] dO[q][d]
__global__ void dkv_kernel(F32Operands p, const float* prob, const float* ds, const float* dout, float* dk_rot,
                           float* dv) {
  const int bh = blockIdx.y, b = bh / p.H, h = bh % p.H, jc = blockIdx.x, d = threadIdx.x;
  const int j = p.hist_rows.v[b / p.group] + jc;
  float ak = 0.f, av = 0.f;
  for (int q = 0; q < p.Nq; ++q) {
    const int64_t o = ((int64_t)bh * p.Nq + q) * p.nk_stride + j;
    ak = fmaf(ds[o], p.q_rot[((int64_t)bh * p.Nq + q) * p.D + d], ak);
    av = fmaf(prob[o], dout[(((int64_t)b * p.Nq + q) * p.H + h) * p.D + d], av);
  }
  dk_rot[((int64_t)bh * p.Nq + jc) * p.D + d] = ak * p.scale;
  dv[(((int64_t)b * p.Nq + jc) * p.H + h) * p.D + d] = av;
}

F32Operands make_operands(const DevGeom& g, const AttnOperands& op) {
  F32Operands p;
  p.q_rot = (const float*)op.q_rot;
  p.kc_rot = (const float*)op.kc_rot;
  p.v_chunk = (const float*)op.v_chunk;
  p.k_cache = (const float*)op.k_cache;
  p.v_cache = (const float*)op.v_cache;
  p.H = g.H;
  p.D = g.D;
  p.Nq = op.Nq;
  p.nk_stride = g.C * g.T + op.Nq;
  p.cache_rows = (int64_t)g.C * g.T;
  p.scale = (float)(1.0 / sqrt((double)g.D));
  p.group = op.group;
  p.block_rows = op.block_rows;
  p.hist_rows = op.hist_rows;
  return p;
}

}  // namespace

size_t f32_fwd_workspace_floats(const DevGeom& g, int Nq) {
  return (size_t)g.B * g.H * Nq * ((size_t)g.C * g.T + Nq);
}
size_t f32_bwd_workspace_floats(const DevGeom& g, int Nq) {
  return 2 * f32_fwd_workspace_floats(g, Nq) + (size_t)g.B * g.H * Nq;
}

hipError_t launch_attn_fwd_f32(const DevGeom& g, const AttnOperands& op, float* out, float* lse, float* scratch,
                               hipStream_t stream) {
  const F32Operands p = make_operands(g, op);
  const int BH = g.B * g.H;
  scores_kernel<<<dim3((p.nk_stride + 255) / 256, p.Nq, BH), 256, 0, stream>>>(p, scratch);
  softmax_kernel<<<dim3(p.Nq, BH), 256, 0, stream>>>(p, scratch, lse);
  pv_kernel<<<dim3(p.Nq, BH), g.D, 0, stream>>>(p, scratch, out);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_f32(const DevGeom& g, const AttnOperands& op, const float* out, const float* lse,
                               const float* dout, float* dq_rot, float* dk_rot, float* dv, float* scratch,
                               hipStream_t stream) {
  const F32Operands p = make_operands(g, op);
  const int BH = g.B * g.H;
  const size_t mat = f32_fwd_workspace_floats(g, op.Nq);
  float* prob = scratch;
  float* ds = scratch + mat;
  float* delta = scratch + 2 * mat;
  scores_kernel<<<dim3((p.nk_stride + 255) / 256, p.Nq, BH), 256, 0, stream>>>(p, prob);
  probs_delta_kernel<<<dim3(p.Nq, BH), 256, 0, stream>>>(p, prob, lse, out, dout, delta);
  dscores_kernel<<<dim3((p.nk_stride + 255) / 256, p.Nq, BH), 256, 0, stream>>>(p, prob, dout, delta, ds);
  dq_kernel<<<dim3(p.Nq, BH), g.D, 0, stream>>>(p, ds, dq_rot);
  dkv_kernel<<<dim3(p.Nq, BH), g.D, 0, stream>>>(p, prob, ds, dout, dk_rot, dv);
  return hipGetLastError();
}

}  // namespace astro
