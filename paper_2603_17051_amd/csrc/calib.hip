// Machine calibration for the roofline context: what this GPU sustains on nothing but bf16
// MFMAs (with the operand values the caller supplies: the sustained clock depends on them)
// and on a plain streaming copy.  Timed like every other launch, through astro_profile_*.
#include "kernels.hpp"
#include "mfma_common.hpp"

namespace astro {
namespace {

constexpr int kOperandSets = 4;

// Each wave keeps 4 A and 4 B operand fragments in registers and issues independent
// 16x16x32 MFMAs (the shape the attention kernels use) into 8 accumulators, pairing the
// fragments differently each time so that the multiplier inputs change between consecutive
// instructions as they do in a real tile loop.  32 MFMAs of 16384 flop per iteration.
__global__ void __launch_bounds__(256, 2) calib_mfma_kernel(const bf16x8* __restrict__ operands, float* __restrict__ sink,
                                                            int iters) {
  bf16x8 a[kOperandSets], b[kOperandSets];
#pragma unroll
  for (int j = 0; j < kOperandSets; ++j) {
    a[j] = operands[(2 * j) * 256 + threadIdx.x];
    b[j] = operands[(2 * j + 1) * 256 + threadIdx.x];
  }
  f32x4 c[2 * kOperandSets];
#pragma unroll
  for (int j = 0; j < 2 * kOperandSets; ++j) c[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int u = 0; u < kOperandSets; ++u)
#pragma unroll
      for (int j = 0; j < 2 * kOperandSets; ++j) c[j] = mfma16(a[(j + u) % kOperandSets], b[j % kOperandSets], c[j]);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 2 * kOperandSets; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) s += c[j][r];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Four 16-byte loads in flight per lane, cache-bypassing loads and stores: the fastest of the
// plain copies tried on this chip (6.0 TB/s read + write at 1 GiB; one load at a time with
// default cache policy: 4.5 TB/s).
__global__ void __launch_bounds__(256) calib_copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, size_t n16) {
  constexpr int kUnroll = 4;
  const size_t span = (size_t)kUnroll * 256;
  for (size_t base = (size_t)blockIdx.x * span; base < n16; base += (size_t)gridDim.x * span) {
    f32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t i = base + (size_t)u * 256 + threadIdx.x;
      if (i < n16) v[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const size_t i = base + (size_t)u * 256 + threadIdx.x;
      if (i < n16) __builtin_nontemporal_store(v[u], dst + i);
    }
  }
}

}  // namespace
}  // namespace astro

using namespace astro;

extern "C" {

int astro_calib_mfma(const void* operands, int32_t workgroups, int32_t iters, float* sink, void* hip_stream) {
  if (!operands || !sink || workgroups <= 0 || workgroups > (1 << 16) || iters <= 0 || iters > (1 << 20)) return ASTRO_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  {
    ProfileScope prof("calib_mfma_bf16", stream);
    calib_mfma_kernel<<<dim3(workgroups), dim3(256), 0, stream>>>(static_cast<const bf16x8*>(operands), sink, iters);
  }
  return hipGetLastError() == hipSuccess ? ASTRO_OK : ASTRO_ERR_HIP;
}

int astro_calib_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
  if (!src || !dst || bytes == 0 || bytes % 16 != 0) return ASTRO_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  {
    ProfileScope prof("calib_copy", stream);
    calib_copy_kernel<<<dim3(256 * 16), dim3(256), 0, stream>>>(static_cast<const f32x4*>(src), static_cast<f32x4*>(dst), bytes / 16);
  }
  return hipGetLastError() == hipSuccess ? ASTRO_OK : ASTRO_ERR_HIP;
}

}  // extern "C"
