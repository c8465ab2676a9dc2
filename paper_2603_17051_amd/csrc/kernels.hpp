// Launch interfaces between the C-ABI layer and the HIP kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

#include "../../include/astro.h"

namespace astro {

// Times the launches made during its lifetime when profiling is on (astro_profile_begin).
class ProfileScope {
 public:
  ProfileScope(const char* name, hipStream_t stream, bool enabled = true);
  ~ProfileScope();
  ProfileScope(const ProfileScope&) = delete;
  ProfileScope& operator=(const ProfileScope&) = delete;

 private:
  hipStream_t stream_;
  int index_;
};

// Per-stream integers handed to kernels by value (the host tables are authoritative).
struct StreamInts {
  int32_t v[ASTRO_MAX_BATCH];
};

// Geometry and rotary tables every kernel needs.
struct DevGeom {
  int B, H, D, gh, gw, T, C, S;
  int n_cus;  // compute units of the device the cache lives on
  int n_t, n_h, n_w;
  const double* inv_freq_t;  // [n_t]  frequency of each temporal pair (fp64)
  const float2* tab_h;       // [gh][n_h] (cos, sin) of row position * frequency
  const float2* tab_w;       // [gw][n_w] (cos, sin) of column position * frequency
};

// Where a rotated / copied chunk tensor goes: head-major rows [B][H][rows_per_head][D];
// frame i of stream b starts at row slot(b, i) * T when `ring` is set (slot from the
// closed form over next_n), else at row i * T.
struct ScatterDst {
  void* a;
  void* b;
  int64_t rows_per_head;
  int ring;
};

// a_in, b_in: [B, n_frames*T, H, D].  a is always rotated (if the geometry has rotary
// pairs); b is rotated iff rotate_b.  first_frame.v[b] = absolute index of the chunk's
// first frame, next_n.v[b] = its stream-local number.
// tab_t_out (may be null): [B][n_frames][n_t] (cos, sin) of the temporal pairs at each chunk frame's
// position, exactly the values this launch rotates with, for the kernels that rotate gradients back.
// a_scale: factor applied to the rotated `a` before it is rounded for storage (1 = none).
hipError_t launch_rope_scatter(const DevGeom& g, int dtype, const void* a_in, const void* b_in,
                               ScatterDst dst, bool rotate_b, int n_frames,
                               const StreamInts& first_frame, const StreamInts& next_n,
                               float2* tab_t_out, float a_scale, hipStream_t stream);

// Inverse rotation of fp32 gradients: src head-major [B][H][n_frames*T][D] (rotated frame)
// -> dst [B, n_frames*T, H, D] (un-rotated frame).
hipError_t launch_rope_unscatter_f32(const DevGeom& g, const float* src, float* dst, int n_frames,
                                     const StreamInts& first_frame, hipStream_t stream);

// The same for gradients of the ring rows: src [B][H][C*T][D] (rotated frame) -> dst
// [B, C*T, H, D] w.r.t. the un-rotated keys; the frame a slot holds follows from start and
// next_n (frames appended); rows of empty slots are not written.  sink_shift.v[b] = how far
// ahead of their own frame index stream b's sink slots are rotated (0 with absolute positions).
hipError_t launch_rope_unscatter_ring_f32(const DevGeom& g, const float* src, float* dst,
                                          const StreamInts& start, const StreamInts& next_n,
                                          const StreamInts& sink_shift, hipStream_t stream);

// Window-relative temporal positions: rotate the sink frames' keys again from their un-rotated
// copy sink_raw [B, S*T, H, D] into ring slots 0 .. S-1 of k_cache [B][H][C*T][D]; sink s of
// stream b is rotated at frame position first_pos.v[b] + s, and only the first count.v[b]
// sinks of stream b are touched (0 = leave the stream alone).
hipError_t launch_rope_sink_rerotate(const DevGeom& g, int dtype, const void* sink_raw, void* k_cache,
                                     const StreamInts& first_pos, const StreamInts& count,
                                     hipStream_t stream);

// Keys / values visible to a chunk: the resident ring rows (a prefix of the ring) and
// the chunk's own rows.  With group > 1 the chunk tensors hold `group` candidate chunks per
// cache stream (candidate c = b*group + g, DevGeom::B counts candidates); all candidates of
// stream b see that stream's ring rows and only their own chunk rows.
struct AttnOperands {
  const void* q_rot;    // [B][H][Nq][D] rotated queries (workspace); bf16 path: times log2(e)/sqrt(D)
  const void* kc_rot;   // [B][H][Nq][D] rotated chunk keys (workspace)
  const void* v_chunk;  // [B, Nq, H, D] caller's chunk values
  const void* k_cache;  // [B][H][C*T][D]
  const void* v_cache;  // [B][H][C*T][D]
  const float2* tab_t;  // [B][n_frames][n_t] (cos, sin) of the temporal pairs at the chunk's frames (workspace)
  int Nq;
  int group;             // candidates per cache stream (1 = plain chunk attention)
  int block_rows;        // causal block inside the chunk, in token rows; 0 = none (whole chunk)
  StreamInts hist_rows;  // resident ring rows per CACHE stream
};

// ---- fp32 debug path -------------------------------------------------------
size_t f32_fwd_workspace_floats(const DevGeom& g, int Nq);  // beyond q_rot / kc_rot
size_t f32_bwd_workspace_floats(const DevGeom& g, int Nq);
hipError_t launch_attn_fwd_f32(const DevGeom& g, const AttnOperands& op, float* out, float* lse,
                               float* scratch, hipStream_t stream);
hipError_t launch_attn_bwd_f32(const DevGeom& g, const AttnOperands& op, const float* out,
                               const float* lse, const float* dout, float* dq_rot, float* dk_rot,
                               float* dv, float* scratch, hipStream_t stream);

// ---- bf16 MFMA path ----------------------------------------------------------
// `parts`: bf16_fwd_split_bytes() bytes of scratch for the per-split results of a launch that is
// split over the keys (0 bytes when the shape fills the chip without), or null = never split.
size_t bf16_fwd_split_bytes(const DevGeom& g, int Nq);
int bf16_fwd_splits(const DevGeom& g, const AttnOperands& op, bool have_parts);
hipError_t launch_attn_fwd_bf16(const DevGeom& g, const AttnOperands& op, void* out, float* lse, void* parts,
                                hipStream_t stream);
size_t bf16_bwd_workspace_bytes(const DevGeom& g, int Nq);  // beyond q_rot / kc_rot
// dq, dk, dv: [B, Nq, H, D] fp32 w.r.t. the UN-rotated inputs (the kernels turn dQ~ and dK~ back in
// their epilogues with the tables of `g` and op.tab_t)
hipError_t launch_attn_bwd_bf16(const DevGeom& g, const AttnOperands& op, const void* out,
                                const float* lse, const void* dout, float* dq, float* dk,
                                float* dv, void* scratch, hipStream_t stream);
// Gradients of the ring rows (the non-detached backward): dk_hist_rot [B][H][C*T][D] w.r.t. the
// rotated keys as cached, dv_hist [B, C*T, H, D]; rows of empty slots are not written.  Needs
// the row terms launch_attn_bwd_bf16 left in `scratch` (same call sequence, same stream);
// group must be 1.
hipError_t launch_attn_bwd_hist_bf16(const DevGeom& g, const AttnOperands& op, const float* lse,
                                     const void* dout, float* dk_hist_rot, float* dv_hist,
                                     const void* scratch, hipStream_t stream);

}  // namespace astro
