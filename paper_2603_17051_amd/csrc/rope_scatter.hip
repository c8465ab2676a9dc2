// 3-axis rotary embedding fused with the layout change token-major -> head-major.
// Used by the KV append (keys rotated into their ring slot, values copied; Sec. 3.2)
// and by the attention pre-pass (queries and chunk keys rotated into the workspace).
// HBM-bound: every element is read once and written once, 16 bytes per lane.
#include "kernels.hpp"
#include "ring_state.hpp"

namespace astro {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kMaxBlockPairs = 64;  // n_t + n_h <= D/2 <= 64

__device__ __forceinline__ int ring_slot(int n, int C, int S) {
  return n < C ? n : S + (n - S) % (C - S);
}

// Block-constant (cos, sin): temporal pairs computed here in fp64 from the absolute
// frame index, row pairs read from the table.
__device__ __forceinline__ void fill_block_table(float2* tab, const DevGeom& g, int frame, int row) {
  const int t = threadIdx.x;
  if (t < g.n_t) {
    double s, c;
    sincos((double)frame * g.inv_freq_t[t], &s, &c);
    tab[t] = make_float2((float)c, (float)s);
  } else if (t < g.n_t + g.n_h) {
    tab[t] = g.tab_h[row * g.n_h + (t - g.n_t)];
  }
  __syncthreads();
}

__device__ __forceinline__ float2 pair_cs(const float2* tab, const DevGeom& g, int w, int pair) {
  const int nb = g.n_t + g.n_h;
  return pair < nb ? tab[pair] : g.tab_w[w * g.n_w + (pair - nb)];
}

// grid: x = n_frames * gh (frame in chunk, row), y = head, z = stream
template <typename Elem, bool kRotateB>
__global__ void __launch_bounds__(kThreads) rope_scatter_kernel(DevGeom g, const Elem* __restrict__ a_in,
                                                                const Elem* __restrict__ b_in, Elem* __restrict__ a_out,
                                                                Elem* __restrict__ b_out, int64_t rows_per_head, int ring,
                                                                int n_frames, StreamInts first_frame, StreamInts next_n,
                                                                float2* __restrict__ tab_t_out, float a_scale) {
  constexpr int EPC = 16 / sizeof(Elem);  // elements per 16-byte chunk
  __shared__ float2 tab[kMaxBlockPairs];
  const int fi = blockIdx.x / g.gh, row = blockIdx.x % g.gh;
  const int h = blockIdx.y, b = blockIdx.z;
  const bool rope = (g.n_t + g.n_h + g.n_w) != 0;
  const int cpr = g.D / EPC;  // chunks per token row of one head
  const int dst_frame_row = ring ? ring_slot(next_n.v[b] + fi, g.C, g.S) * g.T : fi * g.T;
  const int64_t in_tok0 = ((int64_t)b * n_frames + fi) * g.T + (int64_t)row * g.gw;
  const int64_t out_row0 = ((int64_t)b * g.H + h) * rows_per_head + dst_frame_row + (int64_t)row * g.gw;
  if constexpr (sizeof(Elem) == 2) {
    // kUnroll chunks of each tensor per lane and trip: all their loads are issued before the
    // first is used (2 * kUnroll 16-byte loads in flight per lane), and every element is
    // touched once, so the loads (and the append's stores) bypass the caches' keep-for-reuse policy.
    // Measured on a plain copy of 1 GiB: 6.0 TB/s this way against 4.5 TB/s one chunk at a time.
    // The first trip's loads are issued before the block's (cos, sin) table is built, so the
    // fp64 sincos of the temporal pairs runs under their latency.
    constexpr int kUnroll = 4;
    const int n_chunks = g.gw * cpr;
    for (int base = 0; base < n_chunks; base += kUnroll * kThreads) {
      bf16x8 xa[kUnroll], xb[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int idx = base + u * kThreads + threadIdx.x;
        if (idx < n_chunks) {
          const int w = idx / cpr, c = idx % cpr;
          const int64_t in_off = ((in_tok0 + w) * g.H + h) * g.D + c * EPC;
          xa[u] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(a_in + in_off));
          xb[u] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(b_in + in_off));
        }
      }
      if (rope && base == 0) {
        fill_block_table(tab, g, first_frame.v[b] + fi, row);
        // one block per (stream, frame) leaves the temporal pairs' (cos, sin) for the backward's epilogues
        if (tab_t_out && row == 0 && h == 0 && (int)threadIdx.x < g.n_t)
          tab_t_out[((int64_t)b * n_frames + fi) * g.n_t + threadIdx.x] = tab[threadIdx.x];
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const int idx = base + u * kThreads + threadIdx.x;
        if (idx >= n_chunks) continue;
        const int w = idx / cpr, c = idx % cpr;
        const int64_t out_off = (out_row0 + w) * g.D + c * EPC;
        if (rope) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const float2 cs = pair_cs(tab, g, w, c * 4 + v);
            const float a0 = (float)xa[u][2 * v], a1 = (float)xa[u][2 * v + 1];
            xa[u][2 * v] = (__bf16)((a0 * cs.x - a1 * cs.y) * a_scale);
            xa[u][2 * v + 1] = (__bf16)((a0 * cs.y + a1 * cs.x) * a_scale);
            if (kRotateB) {
              const float b0 = (float)xb[u][2 * v], b1 = (float)xb[u][2 * v + 1];
              xb[u][2 * v] = (__bf16)(b0 * cs.x - b1 * cs.y);
              xb[u][2 * v + 1] = (__bf16)(b0 * cs.y + b1 * cs.x);
            }
          }
        }
        if (!rope && a_scale != 1.f) {
#pragma unroll
          for (int v = 0; v < 8; ++v) xa[u][v] = (__bf16)((float)xa[u][v] * a_scale);
        }
        if constexpr (kRotateB) {  // staged Q~, K~: read again at once by the attention launch
          *reinterpret_cast<bf16x8*>(a_out + out_off) = xa[u];
          *reinterpret_cast<bf16x8*>(b_out + out_off) = xb[u];
        } else {
          __builtin_nontemporal_store(xa[u], reinterpret_cast<bf16x8*>(a_out + out_off));
          __builtin_nontemporal_store(xb[u], reinterpret_cast<bf16x8*>(b_out + out_off));
        }
      }
    }
    return;
  } else {
    // fp32 debug path: one chunk at a time
    if (rope) fill_block_table(tab, g, first_frame.v[b] + fi, row);
    for (int idx = threadIdx.x; idx < g.gw * cpr; idx += kThreads) {
      const int w = idx / cpr, c = idx % cpr;
      const int64_t in_off = ((in_tok0 + w) * g.H + h) * g.D + c * EPC;
      const int64_t out_off = (out_row0 + w) * g.D + c * EPC;
      f32x4 xa = *reinterpret_cast<const f32x4*>(a_in + in_off);
      f32x4 xb = *reinterpret_cast<const f32x4*>(b_in + in_off);
      if (rope) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const float2 cs = pair_cs(tab, g, w, c * 2 + u);
          const float a0 = xa[2 * u], a1 = xa[2 * u + 1];
          xa[2 * u] = a0 * cs.x - a1 * cs.y;
          xa[2 * u + 1] = a0 * cs.y + a1 * cs.x;
          if (kRotateB) {
            const float b0 = xb[2 * u], b1 = xb[2 * u + 1];
            xb[2 * u] = b0 * cs.x - b1 * cs.y;
            xb[2 * u + 1] = b0 * cs.y + b1 * cs.x;
          }
        }
      }
      *reinterpret_cast<f32x4*>(a_out + out_off) = xa;
      *reinterpret_cast<f32x4*>(b_out + out_off) = xb;
    }
  }
}

// Gradient w.r.t. the un-rotated tensor = R(phi)^T * gradient w.r.t. the rotated one.
// One block = one token row of one frame: src head-major rows [.][H][rows_per_head][D] -> dst
// token-major [., rows_per_head, H, D]; tok0 = first token of the row within its stream.
__device__ __forceinline__ void unrotate_row(const DevGeom& g, const float2* tab, bool rope, const float* __restrict__ src,
                                             float* __restrict__ dst, int b, int h, int64_t tok0, int64_t rows_per_head) {
  const int cpr = g.D / 4;
  for (int idx = threadIdx.x; idx < g.gw * cpr; idx += kThreads) {
    const int w = idx / cpr, c = idx % cpr;
    const int64_t src_off = (((int64_t)b * g.H + h) * rows_per_head + tok0 + w) * g.D + c * 4;
    const int64_t dst_off = (((int64_t)b * rows_per_head + tok0 + w) * g.H + h) * g.D + c * 4;
    f32x4 x = *reinterpret_cast<const f32x4*>(src + src_off);
    if (rope) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float2 cs = pair_cs(tab, g, w, c * 2 + u);
        const float x0 = x[2 * u], x1 = x[2 * u + 1];
        x[2 * u] = x0 * cs.x + x1 * cs.y;
        x[2 * u + 1] = -x0 * cs.y + x1 * cs.x;
      }
    }
    *reinterpret_cast<f32x4*>(dst + dst_off) = x;
  }
}

// chunk gradients: frame fi of the chunk sits at absolute index first_frame + fi
__global__ void __launch_bounds__(kThreads) rope_unscatter_f32_kernel(DevGeom g, const float* __restrict__ src,
                                                                      float* __restrict__ dst, int n_frames,
                                                                      StreamInts first_frame) {
  __shared__ float2 tab[kMaxBlockPairs];
  const int fi = blockIdx.x / g.gh, row = blockIdx.x % g.gh;
  const int h = blockIdx.y, b = blockIdx.z;
  const bool rope = (g.n_t + g.n_h + g.n_w) != 0;
  if (rope) fill_block_table(tab, g, first_frame.v[b] + fi, row);
  unrotate_row(g, tab, rope, src, dst, b, h, (int64_t)fi * g.T + (int64_t)row * g.gw, (int64_t)n_frames * g.T);
}

// gradients of the ring rows: slot s of stream b holds the frame the closed form names; empty
// slots are skipped (their rows of dst are not written)
__global__ void __launch_bounds__(kThreads) rope_unscatter_ring_f32_kernel(DevGeom g, const float* __restrict__ src,
                                                                           float* __restrict__ dst, StreamInts start,
                                                                           StreamInts next_n, StreamInts sink_shift) {
  __shared__ float2 tab[kMaxBlockPairs];
  const int slot = blockIdx.x / g.gh, row = blockIdx.x % g.gh;
  const int h = blockIdx.y, b = blockIdx.z;
  const int64_t n = frame_number_in_slot(slot, next_n.v[b], g.C, g.S);
  if (n < 0) return;  // whole block
  const bool rope = (g.n_t + g.n_h + g.n_w) != 0;
  if (rope) fill_block_table(tab, g, start.v[b] + (int)n + (slot < g.S ? sink_shift.v[b] : 0), row);
  unrotate_row(g, tab, rope, src, dst, b, h, (int64_t)slot * g.T + (int64_t)row * g.gw, (int64_t)g.C * g.T);
}

// Sink keys rotated again at a new frame position (window-relative temporal positions): one
// block = one token row of one sink frame of one head; un-rotated token-major rows in,
// head-major ring rows (slot = the sink's own number) out.  A few MB per call: one 16-byte
// chunk per lane at a time.
template <typename Elem>
__global__ void __launch_bounds__(kThreads) rope_sink_rerotate_kernel(DevGeom g, const Elem* __restrict__ sink_raw,
                                                                      Elem* __restrict__ k_cache, StreamInts first_pos,
                                                                      StreamInts count) {
  constexpr int EPC = 16 / sizeof(Elem);
  typedef Elem Chunk __attribute__((ext_vector_type(EPC)));
  __shared__ float2 tab[kMaxBlockPairs];
  const int s = blockIdx.x / g.gh, row = blockIdx.x % g.gh;
  const int h = blockIdx.y, b = blockIdx.z;
  if (s >= count.v[b]) return;  // whole block
  fill_block_table(tab, g, first_pos.v[b] + s, row);
  const int cpr = g.D / EPC;
  const int64_t in_tok0 = ((int64_t)b * g.S + s) * g.T + (int64_t)row * g.gw;
  const int64_t out_row0 = ((int64_t)b * g.H + h) * ((int64_t)g.C * g.T) + (int64_t)s * g.T + (int64_t)row * g.gw;
  for (int idx = threadIdx.x; idx < g.gw * cpr; idx += kThreads) {
    const int w = idx / cpr, c = idx % cpr;
    Chunk x = *reinterpret_cast<const Chunk*>(sink_raw + ((in_tok0 + w) * g.H + h) * g.D + c * EPC);
#pragma unroll
    for (int v = 0; v < EPC / 2; ++v) {
      const float2 cs = pair_cs(tab, g, w, c * (EPC / 2) + v);
      const float x0 = (float)x[2 * v], x1 = (float)x[2 * v + 1];
      x[2 * v] = (Elem)(x0 * cs.x - x1 * cs.y);
      x[2 * v + 1] = (Elem)(x0 * cs.y + x1 * cs.x);
    }
    *reinterpret_cast<Chunk*>(k_cache + (out_row0 + w) * g.D + c * EPC) = x;
  }
}

}  // namespace

hipError_t launch_rope_scatter(const DevGeom& g, int dtype, const void* a_in, const void* b_in, ScatterDst dst,
                               bool rotate_b, int n_frames, const StreamInts& first_frame, const StreamInts& next_n,
                               float2* tab_t_out, float a_scale, hipStream_t stream) {
  dim3 grid(n_frames * g.gh, g.H, g.B), block(kThreads);
  ProfileScope prof(dst.ring ? "kv_append_rope" : "chunk_rope_stage", stream);
  if (dtype == ASTRO_BF16) {
    auto a = static_cast<const __bf16*>(a_in);
    auto b = static_cast<const __bf16*>(b_in);
    if (rotate_b)
      rope_scatter_kernel<__bf16, true><<<grid, block, 0, stream>>>(g, a, b, (__bf16*)dst.a, (__bf16*)dst.b,
                                                                   dst.rows_per_head, dst.ring, n_frames, first_frame, next_n, tab_t_out, a_scale);
    else
      rope_scatter_kernel<__bf16, false><<<grid, block, 0, stream>>>(g, a, b, (__bf16*)dst.a, (__bf16*)dst.b,
                                                                    dst.rows_per_head, dst.ring, n_frames, first_frame, next_n, tab_t_out, a_scale);
  } else {
    auto a = static_cast<const float*>(a_in);
    auto b = static_cast<const float*>(b_in);
    if (rotate_b)
      rope_scatter_kernel<float, true><<<grid, block, 0, stream>>>(g, a, b, (float*)dst.a, (float*)dst.b,
                                                                  dst.rows_per_head, dst.ring, n_frames, first_frame, next_n, tab_t_out, a_scale);
    else
      rope_scatter_kernel<float, false><<<grid, block, 0, stream>>>(g, a, b, (float*)dst.a, (float*)dst.b,
                                                                   dst.rows_per_head, dst.ring, n_frames, first_frame, next_n, tab_t_out, a_scale);
  }
  return hipGetLastError();
}

hipError_t launch_rope_unscatter_f32(const DevGeom& g, const float* src, float* dst, int n_frames,
                                     const StreamInts& first_frame, hipStream_t stream) {
  dim3 grid(n_frames * g.gh, g.H, g.B), block(kThreads);
  ProfileScope prof("grad_rope_unstage", stream);
  rope_unscatter_f32_kernel<<<grid, block, 0, stream>>>(g, src, dst, n_frames, first_frame);
  return hipGetLastError();
}

hipError_t launch_rope_unscatter_ring_f32(const DevGeom& g, const float* src, float* dst, const StreamInts& start,
                                          const StreamInts& next_n, const StreamInts& sink_shift, hipStream_t stream) {
  dim3 grid(g.C * g.gh, g.H, g.B), block(kThreads);
  ProfileScope prof("grad_rope_unstage_ring", stream);
  rope_unscatter_ring_f32_kernel<<<grid, block, 0, stream>>>(g, src, dst, start, next_n, sink_shift);
  return hipGetLastError();
}

hipError_t launch_rope_sink_rerotate(const DevGeom& g, int dtype, const void* sink_raw, void* k_cache,
                                     const StreamInts& first_pos, const StreamInts& count, hipStream_t stream) {
  dim3 grid(g.S * g.gh, g.H, g.B), block(kThreads);
  ProfileScope prof("sink_rerotate", stream);
  if (dtype == ASTRO_BF16)
    rope_sink_rerotate_kernel<__bf16><<<grid, block, 0, stream>>>(g, (const __bf16*)sink_raw, (__bf16*)k_cache, first_pos, count);
  else
    rope_sink_rerotate_kernel<float><<<grid, block, 0, stream>>>(g, (const float*)sink_raw, (float*)k_cache, first_pos, count);
  return hipGetLastError();
}

}  // namespace astro
