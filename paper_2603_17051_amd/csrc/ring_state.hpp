// Host-side state of the rolling KV cache: descriptor validation and the
// per-stream slot / position tables (Sec. 3.2, rolling cache with frame sinks).
// Pure C++, no HIP: compiled into the library and usable without a GPU.
#pragma once

#include <cstdint>
#include <vector>

#include "../../include/astro.h"

namespace astro {

struct RingGeometry {
  int B, H, D, gh, gw, T, C, S, Lw, max_chunk;
  int block_frames;  // causal block size inside a chunk, 0 = the whole chunk
  int n_t, n_h, n_w;
  int dtype;
  bool host_only;
  bool window_relative;  // temporal positions by rank in the attended sequence
  bool reuse_staged;     // a backward may pick up the rotated Q / K_chunk the forward before it staged
  double rope_base;
  size_t elem_bytes() const { return dtype == ASTRO_BF16 ? 2 : 4; }
  size_t rows_per_head() const { return (size_t)C * (size_t)T; }
  size_t storage_bytes() const { return (size_t)B * H * rows_per_head() * D * elem_bytes(); }
  // the sinks' keys move only under window-relative positions, and only if the frame axis has rotary pairs
  bool sinks_move() const { return window_relative && S > 0 && n_t > 0; }
  size_t sink_bytes() const { return sinks_move() ? (size_t)B * S * T * H * D * elem_bytes() : 0; }
};

// Checks every field of the descriptor; fills `g` only on success.
inline int validate_desc(const astro_kvcache_desc_t* d, RingGeometry* g) {
  if (!d) return ASTRO_ERR_INVALID_ARG;
  if (d->batch < 1 || d->batch > ASTRO_MAX_BATCH) return ASTRO_ERR_INVALID_ARG;
  if (d->heads < 1 || d->heads > 1024) return ASTRO_ERR_INVALID_ARG;
  if (d->head_dim != 64 && d->head_dim != 128) return ASTRO_ERR_UNSUPPORTED;
  if (d->grid_h < 1 || d->grid_w < 1 || d->grid_h > 4096 || d->grid_w > 4096) return ASTRO_ERR_INVALID_ARG;
  if ((int64_t)d->grid_h * d->grid_w > (1 << 20)) return ASTRO_ERR_INVALID_ARG;
  if (d->capacity_frames < 1 || d->capacity_frames > ASTRO_MAX_CAPACITY_FRAMES) return ASTRO_ERR_INVALID_ARG;
  if (d->sink_frames < 0 || d->sink_frames >= d->capacity_frames) return ASTRO_ERR_INVALID_ARG;
  const int Lw = d->capacity_frames - d->sink_frames;
  if (d->max_chunk_frames < 1 || d->max_chunk_frames > Lw) return ASTRO_ERR_INVALID_ARG;
  if (d->rope_pairs_t < 0 || d->rope_pairs_h < 0 || d->rope_pairs_w < 0) return ASTRO_ERR_INVALID_ARG;
  const int npairs = d->rope_pairs_t + d->rope_pairs_h + d->rope_pairs_w;
  if (npairs != 0 && npairs != d->head_dim / 2) return ASTRO_ERR_INVALID_ARG;
  if (npairs != 0 && !(d->rope_base > 1.0)) return ASTRO_ERR_INVALID_ARG;
  if (d->dtype != ASTRO_BF16 && d->dtype != ASTRO_F32) return ASTRO_ERR_UNSUPPORTED;
  if (d->flags & ~(ASTRO_FLAG_HOST_ONLY | ASTRO_FLAG_WINDOW_RELATIVE | ASTRO_FLAG_REUSE_STAGED)) return ASTRO_ERR_INVALID_ARG;
  if (d->block_frames < 0) return ASTRO_ERR_INVALID_ARG;
  const bool host_only = (d->flags & ASTRO_FLAG_HOST_ONLY) != 0;
  if (!host_only && (!d->k_storage || !d->v_storage)) return ASTRO_ERR_INVALID_ARG;
  const bool sinks_move = (d->flags & ASTRO_FLAG_WINDOW_RELATIVE) && d->sink_frames > 0 && d->rope_pairs_t > 0;
  if (!host_only && sinks_move && !d->k_sink_storage) return ASTRO_ERR_INVALID_ARG;
  // token rows of one head's ring plus one chunk must index with int32
  const int64_t rows = (int64_t)(d->capacity_frames + d->max_chunk_frames) * d->grid_h * d->grid_w;
  if (rows > (int64_t)1 << 30) return ASTRO_ERR_UNSUPPORTED;
  g->B = d->batch; g->H = d->heads; g->D = d->head_dim;
  g->gh = d->grid_h; g->gw = d->grid_w; g->T = d->grid_h * d->grid_w;
  g->C = d->capacity_frames; g->S = d->sink_frames; g->Lw = Lw;
  g->max_chunk = d->max_chunk_frames;
  g->block_frames = d->block_frames;
  g->n_t = d->rope_pairs_t; g->n_h = d->rope_pairs_h; g->n_w = d->rope_pairs_w;
  g->dtype = d->dtype; g->host_only = host_only; g->rope_base = d->rope_base;
  g->window_relative = (d->flags & ASTRO_FLAG_WINDOW_RELATIVE) != 0;
  g->reuse_staged = (d->flags & ASTRO_FLAG_REUSE_STAGED) != 0;
  return ASTRO_OK;
}

#if defined(__HIPCC__)
#define ASTRO_HOST_DEVICE __host__ __device__
#else
#define ASTRO_HOST_DEVICE
#endif

// Ring slot of the n-th frame appended to a stream since its reset: the first C
// frames fill slots in order (so residents are always a prefix of the slots while
// the ring fills); afterwards the sliding part wraps over slots S .. C-1, which
// overwrites frame n - Lw, the oldest non-sink frame.
ASTRO_HOST_DEVICE inline int slot_of_frame_number(int64_t n, int C, int S) {
  if (n < C) return (int)n;
  return S + (int)((n - S) % (C - S));
}

// The inverse: number (since the reset) of the frame slot s holds once next_n frames have been
// appended, or -1 for an empty slot.  While the ring fills, slot s holds frame s; afterwards a
// sink slot keeps its frame and sliding slot S + j holds the newest frame n with (n - S) mod Lw = j.
ASTRO_HOST_DEVICE inline int64_t frame_number_in_slot(int s, int64_t next_n, int C, int S) {
  if (s < S || next_n <= C) return s < next_n ? s : -1;
  const int Lw = C - S, j = s - S;
  return S + j + ((next_n - 1 - S - j) / Lw) * Lw;
}

class RingTables {
 public:
  RingTables(int B, int C, int S)
      : B_(B), C_(C), S_(S), start_(B, 0), next_n_(B, 0) {}

  void reset(int stream, int32_t start_frame) {
    for (int b = (stream < 0 ? 0 : stream); b < (stream < 0 ? B_ : stream + 1); ++b) {
      start_[b] = start_frame;
      next_n_[b] = 0;
    }
  }
  // true if appending n_frames to every stream keeps every absolute frame index in int32
  bool can_append(int n_frames) const {
    for (int b = 0; b < B_; ++b)
      if ((int64_t)start_[b] + next_n_[b] + n_frames > INT32_MAX) return false;
    return true;
  }
  void append(int n_frames) {
    for (int b = 0; b < B_; ++b) next_n_[b] += n_frames;
  }
  int32_t start(int b) const { return start_[b]; }
  int32_t next_n(int b) const { return next_n_[b]; }
  int32_t resident(int b) const { return next_n_[b] < C_ ? next_n_[b] : C_; }
  // frames evicted so far = how far the sinks sit ahead of their own index under window-relative positions
  int32_t evicted(int b) const { return next_n_[b] > C_ ? next_n_[b] - C_ : 0; }
  // rank of every slot's frame among the residents in stream order, [B][C], -1 = empty
  std::vector<int32_t> slot_rank() const {
    std::vector<int32_t> t((size_t)B_ * C_, -1);
    for (int b = 0; b < B_; ++b)
      for (int s = 0; s < C_; ++s) {
        const int64_t n = frame_number_in_slot(s, next_n_[b], C_, S_);
        if (n >= 0) t[(size_t)b * C_ + s] = (int32_t)(n < S_ ? n : n - evicted(b));
      }
    return t;
  }
  // absolute frame index held by every slot, [B][C], -1 = empty (closed form; the kernels that
  // need a slot's frame use the same function)
  std::vector<int32_t> slot_frame() const {
    std::vector<int32_t> t((size_t)B_ * C_, -1);
    for (int b = 0; b < B_; ++b)
      for (int s = 0; s < C_; ++s) {
        const int64_t n = frame_number_in_slot(s, next_n_[b], C_, S_);
        if (n >= 0) t[(size_t)b * C_ + s] = (int32_t)(start_[b] + n);
      }
    return t;
  }

 private:
  int B_, C_, S_;
  std::vector<int32_t> start_, next_n_;
};

}  // namespace astro
