// Clip-level forward-process RL loss and its gradient w.r.t. the current velocity prediction
// (Sec. 3.1 eq. (1)-(2), Sec. 3.3 reward normalisation, Sec. 3.4 selective KL; Alg. 1 Phase 2),
// fused into one pass over the four velocity-shaped tensors: HBM-bound, every element is read
// once (4 tensors) and its gradient written once (cache-bypassing loads and stores).  Deterministic: per-block partial sums in a
// workspace, summed in a fixed order by one block.  Two launches (main, final sum) up to 1024
// samples, three (prepare, main, final sum) above.
#include <mutex>

#include "kernels.hpp"

namespace astro {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kElemsPerBlock = 16384;  // elements of one sample a workgroup walks

struct NftParams {
  const void *v_theta, *v_old, *v_ref, *target;
  const float* advantage;
  const int32_t* kl_mask;
  float* grad;
  float* loss;      // [3] total, policy, kl
  float* r_tilde;   // workspace [n]
  float* n_masked;  // workspace [1]
  float* partials;  // workspace [n][blocks_per_sample][3]
  int n, blocks_per_sample;
  int64_t E;
  float inv_a_max, beta, lambda_kl;
};

// r~_i = clip(A_i / A_max, -1, 1) / 2 + 0.5 and the number of masked samples
__global__ void __launch_bounds__(kThreads) nft_prepare_kernel(NftParams p) {
  __shared__ int cnt[kThreads];
  int c = 0;
  for (int i = threadIdx.x; i < p.n; i += kThreads) {
    const float a = p.advantage[i] * p.inv_a_max;
    p.r_tilde[i] = fminf(fmaxf(a, -1.f), 1.f) * 0.5f + 0.5f;
    c += p.kl_mask[i] != 0 ? 1 : 0;
  }
  cnt[threadIdx.x] = c;
  __syncthreads();
  for (int s = kThreads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) cnt[threadIdx.x] += cnt[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) *p.n_masked = (float)cnt[0];
}

template <typename Elem>
struct Chunk;
template <>
struct Chunk<__bf16> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const void* base, int64_t i, float (&x)[N]) {
    const bf16x8 v = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(base) + i));
#pragma unroll
    for (int j = 0; j < N; ++j) x[j] = (float)v[j];
  }
};
template <>
struct Chunk<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const void* base, int64_t i, float (&x)[N]) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + i));
#pragma unroll
    for (int j = 0; j < N; ++j) x[j] = v[j];
  }
};

// Up to this many samples every workgroup derives r~ of its sample and the number of masked
// samples itself (a few KB from L2) and the prepare launch is skipped: at one group of 24 clips the
// three dependent launches took 28 us for 17 us of memory traffic.
constexpr int kMaxSamplesInline = 1024;

// grid (blocks_per_sample, n)
template <typename Elem, bool kInline>
__global__ void __launch_bounds__(kThreads) nft_loss_kernel(NftParams p) {
  constexpr int N = Chunk<Elem>::N;
  const int i = blockIdx.y;
  float r, nm;
  if constexpr (kInline) {
    __shared__ int cnt[kThreads / 64];
    int c = 0;
    for (int j = threadIdx.x; j < p.n; j += kThreads) c += p.kl_mask[j] != 0 ? 1 : 0;
#pragma unroll
    for (int sh = 32; sh > 0; sh >>= 1) c += __shfl_xor(c, sh);
    if ((threadIdx.x & 63) == 0) cnt[threadIdx.x >> 6] = c;
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int wv = 0; wv < kThreads / 64; ++wv) total += cnt[wv];
    nm = (float)total;
    r = fminf(fmaxf(p.advantage[i] * p.inv_a_max, -1.f), 1.f) * 0.5f + 0.5f;
    // the first workgroup leaves both where the final sum reads them
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      p.r_tilde[i] = r;
      if (i == 0) *p.n_masked = nm;
    }
  } else {
    r = p.r_tilde[i];
    nm = *p.n_masked;
  }
  const float c_pol = 2.f * p.beta / (float)p.n;
  const float c_kl = (p.kl_mask[i] != 0 && nm > 0.f) ? 2.f * p.lambda_kl / nm : 0.f;
  const int64_t lo = (int64_t)blockIdx.x * kElemsPerBlock;
  const int64_t hi = lo + kElemsPerBlock < p.E ? lo + kElemsPerBlock : p.E;
  const int64_t base = (int64_t)i * p.E;
  float s_pos = 0.f, s_neg = 0.f, s_ref = 0.f;
  for (int64_t e = lo + (int64_t)threadIdx.x * N; e < hi; e += (int64_t)kThreads * N) {
    float vt[N], vo[N], vr[N], tg[N];
    Chunk<Elem>::load(p.v_theta, base + e, vt);
    Chunk<Elem>::load(p.v_old, base + e, vo);
    Chunk<Elem>::load(p.v_ref, base + e, vr);
    Chunk<Elem>::load(p.target, base + e, tg);
    float g[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const float bd = p.beta * (vt[j] - vo[j]);  // v+ = v_old + beta (v_theta - v_old), v- = v_old - beta (...)
      const float e_pos = (vo[j] - tg[j]) + bd;
      const float e_neg = (vo[j] - tg[j]) - bd;
      const float d_ref = vt[j] - vr[j];
      s_pos = fmaf(e_pos, e_pos, s_pos);
      s_neg = fmaf(e_neg, e_neg, s_neg);
      s_ref = fmaf(d_ref, d_ref, s_ref);
      g[j] = c_pol * (r * e_pos - (1.f - r) * e_neg) + c_kl * d_ref;
    }
    float* go = p.grad + base + e;
#pragma unroll
    for (int j = 0; j < N; j += 4)
      __builtin_nontemporal_store(f32x4{g[j], g[j + 1], g[j + 2], g[j + 3]}, reinterpret_cast<f32x4*>(go + j));
  }
  // block reduction of the three sums
  __shared__ float red[3][kThreads / 64];
  float v[3] = {s_pos, s_neg, s_ref};
#pragma unroll
  for (int k = 0; k < 3; ++k) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v[k] += __shfl_xor(v[k], s);
    if ((threadIdx.x & 63) == 0) red[k][threadIdx.x >> 6] = v[k];
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    float t = 0.f;
#pragma unroll
    for (int wv = 0; wv < kThreads / 64; ++wv) t += red[threadIdx.x][wv];
    p.partials[((int64_t)i * p.blocks_per_sample + blockIdx.x) * 3 + threadIdx.x] = t;
  }
}

// one workgroup: L_policy = (1/n) sum_i [r~_i S+_i + (1 - r~_i) S-_i], L_KL = (1/|M|) sum_{i in M} Sref_i
__global__ void __launch_bounds__(kThreads) nft_finalize_kernel(NftParams p) {
  __shared__ double pol[kThreads], kl[kThreads];
  double a = 0.0, b = 0.0;
  for (int i = threadIdx.x; i < p.n; i += kThreads) {
    double s[3] = {0.0, 0.0, 0.0};
    const float* part = p.partials + (int64_t)i * p.blocks_per_sample * 3;
    for (int blk = 0; blk < p.blocks_per_sample; ++blk)
      for (int k = 0; k < 3; ++k) s[k] += (double)part[blk * 3 + k];
    const double r = (double)p.r_tilde[i];
    a += r * s[0] + (1.0 - r) * s[1];
    if (p.kl_mask[i] != 0) b += s[2];
  }
  pol[threadIdx.x] = a;
  kl[threadIdx.x] = b;
  __syncthreads();
  for (int s = kThreads / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      pol[threadIdx.x] += pol[threadIdx.x + s];
      kl[threadIdx.x] += kl[threadIdx.x + s];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double nm = (double)*p.n_masked;
    const double l_pol = pol[0] / (double)p.n;
    const double l_kl = nm > 0.0 ? kl[0] / nm : 0.0;
    p.loss[0] = (float)(l_pol + (double)p.lambda_kl * l_kl);
    p.loss[1] = (float)l_pol;
    p.loss[2] = (float)l_kl;
  }
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
int blocks_per_sample(int64_t E) { return (int)((E + kElemsPerBlock - 1) / kElemsPerBlock); }

int workspace_bytes_of(int32_t n_samples, int64_t elems_per_sample, size_t* bytes) {
  if (!bytes || n_samples < 1 || n_samples > 65535 || elems_per_sample < 1 || elems_per_sample > ((int64_t)1 << 40))
    return ASTRO_ERR_INVALID_ARG;
  *bytes = align256((size_t)n_samples * sizeof(float)) + 256 +
           align256((size_t)n_samples * blocks_per_sample(elems_per_sample) * 3 * sizeof(float));
  return ASTRO_OK;
}

// Validation and launches shared by the two entry points; `workspace` is device memory of at
// least the bytes workspace_bytes_of() reports (the caller's, or the static array below).
int run_nft_loss(const void* v_theta, const void* v_old, const void* v_ref, const void* target, const float* advantage,
                 const int32_t* kl_mask, int32_t n_samples, int64_t elems_per_sample, int32_t dtype, float a_max,
                 float beta, float lambda_kl, float* loss, float* grad_v_theta, void* workspace, size_t workspace_bytes,
                 hipStream_t stream, bool timed) {
  size_t need = 0;
  if (workspace_bytes_of(n_samples, elems_per_sample, &need) != ASTRO_OK) return ASTRO_ERR_INVALID_ARG;
  if (!v_theta || !v_old || !v_ref || !target || !advantage || !kl_mask || !loss || !grad_v_theta) return ASTRO_ERR_INVALID_ARG;
  if (dtype != ASTRO_BF16 && dtype != ASTRO_F32) return ASTRO_ERR_INVALID_ARG;
  if (!(a_max > 0.f) || !(beta == beta) || !(lambda_kl == lambda_kl)) return ASTRO_ERR_INVALID_ARG;
  // 16-byte vector accesses: every sample must start on a 16-byte boundary in all tensors
  if (elems_per_sample % (dtype == ASTRO_BF16 ? 8 : 4) != 0) return ASTRO_ERR_UNSUPPORTED;
  for (const void* ptr : {v_theta, v_old, v_ref, target, (const void*)grad_v_theta})
    if ((uintptr_t)ptr & 15) return ASTRO_ERR_INVALID_ARG;
  if (blocks_per_sample(elems_per_sample) > 2147483647 / 3) return ASTRO_ERR_UNSUPPORTED;
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return ASTRO_ERR_WORKSPACE;

  NftParams p;
  p.v_theta = v_theta; p.v_old = v_old; p.v_ref = v_ref; p.target = target;
  p.advantage = advantage; p.kl_mask = kl_mask;
  p.grad = grad_v_theta; p.loss = loss;
  char* ws = static_cast<char*>(workspace);
  p.r_tilde = reinterpret_cast<float*>(ws);
  p.n_masked = reinterpret_cast<float*>(ws + align256((size_t)n_samples * sizeof(float)));
  p.partials = reinterpret_cast<float*>(ws + align256((size_t)n_samples * sizeof(float)) + 256);
  p.n = n_samples;
  p.blocks_per_sample = blocks_per_sample(elems_per_sample);
  p.E = elems_per_sample;
  p.inv_a_max = 1.f / a_max; p.beta = beta; p.lambda_kl = lambda_kl;
  {
    // the entry point that must not allocate never creates timing events, even while profiling is on
    ProfileScope prof("nft_loss", stream, timed);
    const dim3 grid(p.blocks_per_sample, n_samples);
    if (n_samples <= kMaxSamplesInline) {
      if (dtype == ASTRO_BF16)
        nft_loss_kernel<__bf16, true><<<grid, kThreads, 0, stream>>>(p);
      else
        nft_loss_kernel<float, true><<<grid, kThreads, 0, stream>>>(p);
    } else {
      nft_prepare_kernel<<<1, kThreads, 0, stream>>>(p);
      if (dtype == ASTRO_BF16)
        nft_loss_kernel<__bf16, false><<<grid, kThreads, 0, stream>>>(p);
      else
        nft_loss_kernel<float, false><<<grid, kThreads, 0, stream>>>(p);
    }
    nft_finalize_kernel<<<1, kThreads, 0, stream>>>(p);
  }
  return hipGetLastError() == hipSuccess ? ASTRO_OK : ASTRO_ERR_HIP;
}

// ---- the entry point that allocates nothing -------------------------------------------------
// r~, the masked count and the per-block partial sums live in a file-scope device array instead
// of a caller's workspace.  Every GPU the library runs on holds its own copy of the array at its
// own address for the life of the process; the host-side name of the array is not that address,
// so the address is asked for once per device (with that device current) and kept.
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return ASTRO_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return ASTRO_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return ASTRO_ERR_HIP;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return ASTRO_OK;
}

}  // namespace
}  // namespace astro

using namespace astro;

extern "C" {

int astro_nft_loss_workspace_bytes(int32_t n_samples, int64_t elems_per_sample, size_t* bytes) {
  return workspace_bytes_of(n_samples, elems_per_sample, bytes);
}

int astro_nft_loss(const void* v_theta, const void* v_old, const void* v_ref, const void* target, const float* advantage,
                   const int32_t* kl_mask, int32_t n_samples, int64_t elems_per_sample, int32_t dtype, float a_max,
                   float beta, float lambda_kl, float* loss, float* grad_v_theta, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
  return run_nft_loss(v_theta, v_old, v_ref, target, advantage, kl_mask, n_samples, elems_per_sample, dtype, a_max, beta,
                      lambda_kl, loss, grad_v_theta, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream), true);
}

int astro_nft_loss_static_bytes(size_t* bytes) {
  if (!bytes) return ASTRO_ERR_INVALID_ARG;
  *bytes = kStaticScratchBytes;
  return ASTRO_OK;
}

int astro_nft_loss_static(const void* v_theta, const void* v_old, const void* v_ref, const void* target,
                          const float* advantage, const int32_t* kl_mask, int32_t n_samples, int64_t elems_per_sample,
                          int32_t dtype, float a_max, float beta, float lambda_kl, float* loss, float* grad_v_theta,
                          void* hip_stream) {
  size_t need = 0;
  if (workspace_bytes_of(n_samples, elems_per_sample, &need) != ASTRO_OK) return ASTRO_ERR_INVALID_ARG;
  if (need > kStaticScratchBytes) return ASTRO_ERR_WORKSPACE;  // more partial sums than the static array holds
  void* ws = nullptr;
  const int rc = static_scratch_of_current_device(&ws);
  if (rc != ASTRO_OK) return rc;
  return run_nft_loss(v_theta, v_old, v_ref, target, advantage, kl_mask, n_samples, elems_per_sample, dtype, a_max, beta,
                      lambda_kl, loss, grad_v_theta, ws, kStaticScratchBytes, static_cast<hipStream_t>(hip_stream), false);
}

}  // extern "C"
