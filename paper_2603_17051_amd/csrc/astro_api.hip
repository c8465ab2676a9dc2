// C-ABI layer: argument validation, host tables, workspace carving, kernel launches.
// Every step of the path runs in the HIP kernels; there is no CPU fallback.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/astro.h"
#include "kernels.hpp"
#include "ring_state.hpp"

using namespace astro;

struct astro_kvcache {
  RingGeometry geo;
  RingTables tables;
  void* k_storage;
  void* v_storage;
  void* k_sink_storage = nullptr;  // un-rotated sink keys (window-relative positions only)
  // small library-owned device tables
  double* d_inv_freq_t = nullptr;
  float2* d_tab_h = nullptr;
  float2* d_tab_w = nullptr;
  int device = -1;
  int n_cus = 256;
  // What the last rotation pre-pass left in a caller's workspace (ASTRO_FLAG_REUSE_STAGED): the
  // call's chunk pointers, workspace, sizes and the state of the tables it was made in.
  struct Staged {
    const void* q = nullptr;
    const void* k = nullptr;
    const void* ws = nullptr;
    int n_frames = 0, group = 0;
    uint64_t epoch = 0;
    bool valid = false;
  } staged;
  uint64_t epoch = 0;  // bumped by every reset and append: chunk positions may have changed
  // An append whose launches failed half way leaves ring rows that the tables do not describe:
  // the handle then refuses work until every stream is reset.
  bool ring_undefined = false;
  astro_kvcache(const RingGeometry& g, void* k, void* v) : geo(g), tables(g.B, g.C, g.S), k_storage(k), v_storage(v) {}
};

namespace {

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// group > 1: the chunk tensors hold `group` candidates per cache stream; the kernels then see
// B * group streams of chunk data
DevGeom dev_geom(const astro_kvcache* c, int group = 1) {
  const RingGeometry& g = c->geo;
  DevGeom d;
  d.B = g.B * group; d.H = g.H; d.D = g.D; d.gh = g.gh; d.gw = g.gw; d.T = g.T; d.C = g.C; d.S = g.S;
  d.n_t = g.n_t; d.n_h = g.n_h; d.n_w = g.n_w;
  d.n_cus = c->n_cus;
  d.inv_freq_t = c->d_inv_freq_t;
  d.tab_h = c->d_tab_h;
  d.tab_w = c->d_tab_w;
  return d;
}

struct Workspace {
  size_t q_rot, kc_rot, tab_t, staged_end, dq_rot, dk_rot, scratch, dk_hist_rot, total;
};

Workspace carve(const astro_kvcache* c, int n_frames, bool bwd, int group, bool ring_grads = false) {
  const RingGeometry& g = c->geo;
  const size_t nq = (size_t)n_frames * g.T;
  const size_t rot = align256((size_t)g.B * group * g.H * nq * g.D * g.elem_bytes());
  const size_t grad = align256((size_t)g.B * group * g.H * nq * g.D * sizeof(float));
  const DevGeom d = dev_geom(c, group);
  Workspace w{};
  size_t off = 0;
  // what the rotation pre-pass leaves: the same bytes at the same offsets for a forward and a
  // backward of the same chunk size, so a backward can pick up what a forward staged
  w.q_rot = off; off += rot;
  w.kc_rot = off; off += rot;
  w.tab_t = off; off += align256((size_t)g.B * group * n_frames * (g.n_t > 0 ? g.n_t : 1) * sizeof(float2));
  w.staged_end = off;
  // rotated-frame gradients: the fp32 path turns them back in a pass of its own, the bf16
  // kernels do it in their epilogues
  if (bwd && g.dtype == ASTRO_F32) {
    w.dq_rot = off; off += grad;
    w.dk_rot = off; off += grad;
  }
  w.scratch = off;
  if (g.dtype == ASTRO_F32)
    off += align256(sizeof(float) * (bwd ? f32_bwd_workspace_floats(d, (int)nq) : f32_fwd_workspace_floats(d, (int)nq)));
  else if (bwd)
    off += align256(bf16_bwd_workspace_bytes(d, (int)nq));
  else
    off += align256(bf16_fwd_split_bytes(d, (int)nq));
  w.dk_hist_rot = off;
  if (ring_grads) off += align256((size_t)g.B * g.H * g.rows_per_head() * g.D * sizeof(float));
  w.total = off;
  return w;
}

int check_group(const astro_kvcache* c, int group) {
  if (!c) return ASTRO_ERR_INVALID_ARG;
  if (group < 1 || (int64_t)c->geo.B * group > ASTRO_MAX_BATCH) return ASTRO_ERR_INVALID_ARG;
  return ASTRO_OK;
}

int check_chunk_call(const astro_kvcache* c, int n_frames, int group) {
  if (!c) return ASTRO_ERR_INVALID_ARG;
  if (c->geo.host_only || c->ring_undefined) return ASTRO_ERR_BAD_STATE;
  if (n_frames < 1 || n_frames > c->geo.max_chunk) return ASTRO_ERR_INVALID_ARG;
  if (check_group(c, group) != ASTRO_OK) return ASTRO_ERR_INVALID_ARG;
  if (!c->tables.can_append(n_frames)) return ASTRO_ERR_BAD_STATE;
  // the kernels address one stream's chunk tensor and one head's ring with 32-bit byte offsets
  const RingGeometry& g = c->geo;
  const int64_t chunk_bytes = (int64_t)n_frames * g.T * g.H * g.D * 4;
  const int64_t ring_bytes = (int64_t)g.C * g.T * g.D * 4;
  if (chunk_bytes >= ((int64_t)1 << 31) || ring_bytes >= ((int64_t)1 << 31)) return ASTRO_ERR_UNSUPPORTED;
  return ASTRO_OK;
}

// first_frame / next_n are indexed by candidate (cache stream * group + g), hist_rows by cache stream
void stream_ints(const astro_kvcache* c, StreamInts* first_frame, StreamInts* next_n, StreamInts* hist_rows,
                 int group = 1) {
  for (int i = 0; i < ASTRO_MAX_BATCH; ++i) {
    const int b = i / group;
    const bool live = b < c->geo.B;
    if (first_frame) first_frame->v[i] = live ? c->tables.start(b) + c->tables.next_n(b) : 0;
    if (next_n) next_n->v[i] = live ? c->tables.next_n(b) : 0;
    if (hist_rows) hist_rows->v[i] = i < c->geo.B ? c->tables.resident(i) * c->geo.T : 0;
  }
}

AttnOperands attn_operands(const astro_kvcache* c, char* ws, const Workspace& w, const void* v_chunk, int n_frames,
                           int group) {
  AttnOperands op;
  op.q_rot = ws + w.q_rot;
  op.kc_rot = ws + w.kc_rot;
  op.v_chunk = v_chunk;
  op.k_cache = c->k_storage;
  op.v_cache = c->v_storage;
  op.tab_t = (const float2*)(ws + w.tab_t);
  op.Nq = n_frames * c->geo.T;
  op.group = group;
  // a block size that covers the chunk is no mask at all
  const int bf = c->geo.block_frames;
  op.block_rows = (bf > 0 && bf < n_frames) ? bf * c->geo.T : 0;
  stream_ints(c, nullptr, nullptr, &op.hist_rows);
  return op;
}

// rotate Q and K_chunk into the workspace (head-major), unless the handle may reuse staged copies
// and the last pre-pass was made for exactly this call's chunk, workspace and table state
hipError_t stage_chunk(astro_kvcache* c, const void* q, const void* k_chunk, char* ws, const Workspace& w,
                       int n_frames, int group, hipStream_t stream) {
  astro_kvcache::Staged& st = c->staged;
  if (c->geo.reuse_staged && st.valid && st.q == q && st.k == k_chunk && st.ws == ws && st.n_frames == n_frames &&
      st.group == group && st.epoch == c->epoch)
    return hipSuccess;
  st.valid = false;
  StreamInts first, next;
  stream_ints(c, &first, &next, nullptr, group);
  ScatterDst dst{ws + w.q_rot, ws + w.kc_rot, (int64_t)n_frames * c->geo.T, 0};
  // The bf16 kernels take the queries pre-multiplied by log2(e)/sqrt(D) (applied in fp32 to the
  // rotated value, before its one rounding to bf16): Q~' K~^T is then directly the exponent of 2,
  // and the row's reference or log-sum-exp enters as the start value of the MFMA accumulators, so
  // no multiply-add per score is left in front of the exponential.
  const float q_scale = c->geo.dtype == ASTRO_BF16 ? 1.4426950408889634f / std::sqrt((float)c->geo.D) : 1.f;
  const hipError_t e = launch_rope_scatter(dev_geom(c, group), c->geo.dtype, q, k_chunk, dst, true, n_frames, first, next,
                                           (float2*)(ws + w.tab_t), q_scale, stream);
  if (e == hipSuccess) st = astro_kvcache::Staged{q, k_chunk, ws, n_frames, group, c->epoch, true};
  return e;
}

}  // namespace

extern "C" {

int astro_kvcache_bytes(const astro_kvcache_desc_t* desc, size_t* k_bytes, size_t* v_bytes) {
  astro_kvcache_desc_t d;
  if (!desc) return ASTRO_ERR_INVALID_ARG;
  d = *desc;
  d.flags |= ASTRO_FLAG_HOST_ONLY;  // storage pointers are not needed to size the cache
  RingGeometry g;
  const int rc = validate_desc(&d, &g);
  if (rc != ASTRO_OK) return rc;
  if (k_bytes) *k_bytes = g.storage_bytes();
  if (v_bytes) *v_bytes = g.storage_bytes();
  return ASTRO_OK;
}

int astro_kvcache_sink_bytes(const astro_kvcache_desc_t* desc, size_t* bytes) {
  astro_kvcache_desc_t d;
  if (!desc || !bytes) return ASTRO_ERR_INVALID_ARG;
  d = *desc;
  d.flags |= ASTRO_FLAG_HOST_ONLY;
  RingGeometry g;
  const int rc = validate_desc(&d, &g);
  if (rc != ASTRO_OK) return rc;
  *bytes = g.sink_bytes();
  return ASTRO_OK;
}

int astro_kvcache_create(const astro_kvcache_desc_t* desc, astro_kvcache_t** out) {
  if (!out) return ASTRO_ERR_INVALID_ARG;
  RingGeometry g;
  const int rc = validate_desc(desc, &g);
  if (rc != ASTRO_OK) return rc;
  astro_kvcache* c = new (std::nothrow) astro_kvcache(g, desc->k_storage, desc->v_storage);
  if (!c) return ASTRO_ERR_INVALID_ARG;
  c->k_sink_storage = desc->k_sink_storage;
  if (!g.host_only) {
    // rotary tables in fp64, rounded once to fp32
    std::vector<double> inv_t(g.n_t > 0 ? g.n_t : 1, 0.0);
    for (int j = 0; j < g.n_t; ++j) inv_t[j] = std::pow(g.rope_base, -(double)j / g.n_t);
    std::vector<float2> th((size_t)g.gh * (g.n_h > 0 ? g.n_h : 1)), tw((size_t)g.gw * (g.n_w > 0 ? g.n_w : 1));
    for (int r = 0; r < g.gh; ++r)
      for (int j = 0; j < g.n_h; ++j) {
        const double a = (double)r * std::pow(g.rope_base, -(double)j / g.n_h);
        th[(size_t)r * g.n_h + j] = make_float2((float)std::cos(a), (float)std::sin(a));
      }
    for (int w = 0; w < g.gw; ++w)
      for (int j = 0; j < g.n_w; ++j) {
        const double a = (double)w * std::pow(g.rope_base, -(double)j / g.n_w);
        tw[(size_t)w * g.n_w + j] = make_float2((float)std::cos(a), (float)std::sin(a));
      }
    bool ok = hipGetDevice(&c->device) == hipSuccess;
    ok = ok && hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && c->n_cus > 0;
    ok = ok && hipMalloc((void**)&c->d_inv_freq_t, inv_t.size() * sizeof(double)) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->d_tab_h, th.size() * sizeof(float2)) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->d_tab_w, tw.size() * sizeof(float2)) == hipSuccess;
    ok = ok && hipMemcpy(c->d_inv_freq_t, inv_t.data(), inv_t.size() * sizeof(double), hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(c->d_tab_h, th.data(), th.size() * sizeof(float2), hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(c->d_tab_w, tw.data(), tw.size() * sizeof(float2), hipMemcpyHostToDevice) == hipSuccess;
    if (!ok) {
      (void)hipGetLastError();
      astro_kvcache_destroy(c);
      return ASTRO_ERR_HIP;
    }
  }
  *out = c;
  return ASTRO_OK;
}

int astro_kvcache_destroy(astro_kvcache_t* cache) {
  if (!cache) return ASTRO_ERR_INVALID_ARG;
  int rc = ASTRO_OK;
  if (cache->d_inv_freq_t && hipFree(cache->d_inv_freq_t) != hipSuccess) rc = ASTRO_ERR_HIP;
  if (cache->d_tab_h && hipFree(cache->d_tab_h) != hipSuccess) rc = ASTRO_ERR_HIP;
  if (cache->d_tab_w && hipFree(cache->d_tab_w) != hipSuccess) rc = ASTRO_ERR_HIP;
  delete cache;
  return rc;
}

int astro_kvcache_reset(astro_kvcache_t* cache, int32_t stream, int32_t start_frame) {
  if (!cache) return ASTRO_ERR_INVALID_ARG;
  if (stream < -1 || stream >= cache->geo.B || start_frame < 0) return ASTRO_ERR_INVALID_ARG;
  if (cache->ring_undefined && stream != -1) return ASTRO_ERR_BAD_STATE;  // only emptying every stream helps
  cache->ring_undefined = false;
  cache->tables.reset(stream, start_frame);
  ++cache->epoch;
  return ASTRO_OK;
}

int astro_kvcache_append(astro_kvcache_t* cache, const void* k, const void* v, int32_t n_frames, void* hip_stream) {
  if (!cache) return ASTRO_ERR_INVALID_ARG;
  const RingGeometry& g = cache->geo;
  if (n_frames < 1 || n_frames > g.max_chunk || n_frames > g.Lw) return ASTRO_ERR_INVALID_ARG;
  if (cache->ring_undefined || !cache->tables.can_append(n_frames)) return ASTRO_ERR_BAD_STATE;
  if (!g.host_only) {
    if (!k || !v) return ASTRO_ERR_INVALID_ARG;
    // Everything is validated; from here on a failing launch leaves ring rows (or sinks) that the
    // tables do not describe, so it marks the handle instead of pretending nothing happened.
    StreamInts first, next;
    stream_ints(cache, &first, &next, nullptr);
    ScatterDst dst{cache->k_storage, cache->v_storage, (int64_t)g.C * g.T, 1};
    hipStream_t stream = (hipStream_t)hip_stream;
    bool ok = true;
    if (g.sinks_move()) {
      // Window-relative positions, before the ring is touched: sink frames that arrive in this
      // call keep an un-rotated copy of their keys (written again unchanged if the call is repeated).
      const size_t frame_bytes = (size_t)g.T * g.H * g.D * g.elem_bytes();
      for (int b = 0; b < g.B && ok; ++b) {
        const int n0 = cache->tables.next_n(b), n1 = n0 + n_frames;
        if (n0 >= g.S) continue;
        const int cnt = n1 < g.S ? n_frames : g.S - n0;
        const char* src = (const char*)k + (size_t)b * n_frames * frame_bytes;
        char* dstp = (char*)cache->k_sink_storage + ((size_t)b * g.S + n0) * frame_bytes;
        ok = hipMemcpyAsync(dstp, src, cnt * frame_bytes, hipMemcpyDeviceToDevice, stream) == hipSuccess;
      }
      if (!ok) {  // the ring is untouched: nothing has changed that the tables describe
        (void)hipGetLastError();
        return ASTRO_ERR_HIP;
      }
    }
    ok = launch_rope_scatter(dev_geom(cache), g.dtype, k, v, dst, false, n_frames, first, next, nullptr, 1.f, stream) == hipSuccess;
    if (ok && g.sinks_move()) {
      // Streams whose eviction count changes: rotate their sinks again, at their own index plus the
      // frames evicted once this call's frames are in.  An append holds at most Lw frames, so a
      // call never both receives sinks and evicts for one stream.
      StreamInts first_pos, count;
      bool any = false;
      for (int b = 0; b < ASTRO_MAX_BATCH; ++b) {
        first_pos.v[b] = count.v[b] = 0;
        if (b >= g.B) continue;
        const int n0 = cache->tables.next_n(b), n1 = n0 + n_frames;
        const int ev0 = n0 > g.C ? n0 - g.C : 0, ev1 = n1 > g.C ? n1 - g.C : 0;
        if (ev1 != ev0) {
          first_pos.v[b] = cache->tables.start(b) + ev1;
          count.v[b] = g.S;
          any = true;
        }
      }
      if (any)
        ok = launch_rope_sink_rerotate(dev_geom(cache), g.dtype, cache->k_sink_storage, cache->k_storage, first_pos, count,
                                       stream) == hipSuccess;
    }
    if (!ok) {
      (void)hipGetLastError();
      cache->ring_undefined = true;
      cache->staged.valid = false;
      return ASTRO_ERR_HIP;
    }
  }
  cache->tables.append(n_frames);
  ++cache->epoch;
  return ASTRO_OK;
}

int astro_kvcache_tables(const astro_kvcache_t* cache, int32_t* slot_frame, int32_t* slot_pos, int32_t* next_n) {
  if (!cache) return ASTRO_ERR_INVALID_ARG;
  const std::vector<int32_t> sf = cache->tables.slot_frame();
  // the temporal rotary position of a resident frame is its absolute frame index, or with
  // window-relative positions its rank among the residents
  const std::vector<int32_t> sp = cache->geo.window_relative ? cache->tables.slot_rank() : sf;
  if (slot_frame) std::memcpy(slot_frame, sf.data(), sf.size() * sizeof(int32_t));
  if (slot_pos) std::memcpy(slot_pos, sp.data(), sp.size() * sizeof(int32_t));
  if (next_n)
    for (int b = 0; b < cache->geo.B; ++b) next_n[b] = cache->tables.next_n(b);
  return ASTRO_OK;
}

int astro_group_attn_workspace_bytes(const astro_kvcache_t* cache, int32_t n_frames, int32_t group, size_t* fwd_bytes,
                                     size_t* bwd_bytes) {
  if (!cache) return ASTRO_ERR_INVALID_ARG;
  if (n_frames < 1 || n_frames > cache->geo.max_chunk) return ASTRO_ERR_INVALID_ARG;
  if (check_group(cache, group) != ASTRO_OK) return ASTRO_ERR_INVALID_ARG;
  if (fwd_bytes) *fwd_bytes = carve(cache, n_frames, false, group).total;
  if (bwd_bytes) *bwd_bytes = carve(cache, n_frames, true, group).total;
  return ASTRO_OK;
}

int astro_group_attn_fwd(astro_kvcache_t* cache, const void* q, const void* k_chunk, const void* v_chunk,
                         int32_t n_frames, int32_t group, void* out, float* lse, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  const int rc = check_chunk_call(cache, n_frames, group);
  if (rc != ASTRO_OK) return rc;
  if (!q || !k_chunk || !v_chunk || !out || !lse) return ASTRO_ERR_INVALID_ARG;
  const Workspace w = carve(cache, n_frames, false, group);
  if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255)) return ASTRO_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  hipStream_t stream = (hipStream_t)hip_stream;
  if (stage_chunk(cache, q, k_chunk, ws, w, n_frames, group, stream) != hipSuccess) return ASTRO_ERR_HIP;
  const AttnOperands op = attn_operands(cache, ws, w, v_chunk, n_frames, group);
  const DevGeom d = dev_geom(cache, group);
  hipError_t e;
  if (cache->geo.dtype == ASTRO_F32)
    e = launch_attn_fwd_f32(d, op, (float*)out, lse, (float*)(ws + w.scratch), stream);
  else
    e = launch_attn_fwd_bf16(d, op, out, lse, w.total > w.scratch ? ws + w.scratch : nullptr, stream);
  return e == hipSuccess ? ASTRO_OK : ASTRO_ERR_HIP;
}

int astro_group_attn_bwd(astro_kvcache_t* cache, const void* q, const void* k_chunk, const void* v_chunk,
                         const void* out, const float* lse, const void* dout, int32_t n_frames, int32_t group,
                         float* dq, float* dk_chunk, float* dv_chunk, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  const int rc = check_chunk_call(cache, n_frames, group);
  if (rc != ASTRO_OK) return rc;
  if (!q || !k_chunk || !v_chunk || !out || !lse || !dout || !dq || !dk_chunk || !dv_chunk) return ASTRO_ERR_INVALID_ARG;
  const Workspace w = carve(cache, n_frames, true, group);
  if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255)) return ASTRO_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  hipStream_t stream = (hipStream_t)hip_stream;
  if (stage_chunk(cache, q, k_chunk, ws, w, n_frames, group, stream) != hipSuccess) return ASTRO_ERR_HIP;
  const AttnOperands op = attn_operands(cache, ws, w, v_chunk, n_frames, group);
  const DevGeom d = dev_geom(cache, group);
  if (cache->geo.dtype == ASTRO_BF16)  // gradients leave the kernels un-rotated and token-major
    return launch_attn_bwd_bf16(d, op, out, lse, dout, dq, dk_chunk, dv_chunk, ws + w.scratch, stream) == hipSuccess
               ? ASTRO_OK
               : ASTRO_ERR_HIP;
  float* dq_rot = (float*)(ws + w.dq_rot);
  float* dk_rot = (float*)(ws + w.dk_rot);
  if (launch_attn_bwd_f32(d, op, (const float*)out, lse, (const float*)dout, dq_rot, dk_rot, dv_chunk,
                          (float*)(ws + w.scratch), stream) != hipSuccess)
    return ASTRO_ERR_HIP;
  // gradients w.r.t. the un-rotated Q and K_chunk: inverse rotation, back to token-major
  StreamInts first;
  stream_ints(cache, &first, nullptr, nullptr, group);
  if (launch_rope_unscatter_f32(d, dq_rot, dq, n_frames, first, stream) != hipSuccess) return ASTRO_ERR_HIP;
  if (launch_rope_unscatter_f32(d, dk_rot, dk_chunk, n_frames, first, stream) != hipSuccess) return ASTRO_ERR_HIP;
  return ASTRO_OK;
}

int astro_chunk_attn_bwd_full_workspace_bytes(const astro_kvcache_t* cache, int32_t n_frames, size_t* bytes) {
  if (!cache || !bytes) return ASTRO_ERR_INVALID_ARG;
  if (n_frames < 1 || n_frames > cache->geo.max_chunk) return ASTRO_ERR_INVALID_ARG;
  if (cache->geo.dtype != ASTRO_BF16) return ASTRO_ERR_UNSUPPORTED;
  *bytes = carve(cache, n_frames, true, 1, true).total;
  return ASTRO_OK;
}

int astro_chunk_attn_bwd_full(astro_kvcache_t* cache, const void* q, const void* k_chunk, const void* v_chunk,
                              const void* out, const float* lse, const void* dout, int32_t n_frames, float* dq,
                              float* dk_chunk, float* dv_chunk, float* dk_cache, float* dv_cache, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  const int rc = check_chunk_call(cache, n_frames, 1);
  if (rc != ASTRO_OK) return rc;
  if (cache->geo.dtype != ASTRO_BF16) return ASTRO_ERR_UNSUPPORTED;
  if (!dk_cache || !dv_cache) return ASTRO_ERR_INVALID_ARG;
  const Workspace w = carve(cache, n_frames, true, 1, true);
  if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255)) return ASTRO_ERR_WORKSPACE;
  // the detached backward first (it also leaves the row terms the ring-row kernels need) ...
  const int rc2 = astro_group_attn_bwd(cache, q, k_chunk, v_chunk, out, lse, dout, n_frames, 1, dq, dk_chunk, dv_chunk,
                                       workspace, workspace_bytes, hip_stream);
  if (rc2 != ASTRO_OK) return rc2;
  // ... then dK~, dV of the resident ring rows, and the inverse rotation at each slot's frame
  char* ws = (char*)workspace;
  hipStream_t stream = (hipStream_t)hip_stream;
  const AttnOperands op = attn_operands(cache, ws, w, v_chunk, n_frames, 1);
  const DevGeom d = dev_geom(cache);
  float* dk_hist_rot = (float*)(ws + w.dk_hist_rot);
  if (launch_attn_bwd_hist_bf16(d, op, lse, dout, dk_hist_rot, dv_cache, ws + w.scratch, stream) != hipSuccess)
    return ASTRO_ERR_HIP;
  StreamInts start, next, sink_shift;
  for (int b = 0; b < ASTRO_MAX_BATCH; ++b) {
    start.v[b] = b < cache->geo.B ? cache->tables.start(b) : 0;
    next.v[b] = b < cache->geo.B ? cache->tables.next_n(b) : 0;
    sink_shift.v[b] = b < cache->geo.B && cache->geo.sinks_move() ? cache->tables.evicted(b) : 0;
  }
  if (launch_rope_unscatter_ring_f32(d, dk_hist_rot, dk_cache, start, next, sink_shift, stream) != hipSuccess)
    return ASTRO_ERR_HIP;
  return ASTRO_OK;
}

int astro_chunk_attn_workspace_bytes(const astro_kvcache_t* cache, int32_t n_frames, size_t* fwd_bytes,
                                     size_t* bwd_bytes) {
  return astro_group_attn_workspace_bytes(cache, n_frames, 1, fwd_bytes, bwd_bytes);
}

int astro_chunk_attn_fwd(astro_kvcache_t* cache, const void* q, const void* k_chunk, const void* v_chunk,
                         int32_t n_frames, void* out, float* lse, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  return astro_group_attn_fwd(cache, q, k_chunk, v_chunk, n_frames, 1, out, lse, workspace, workspace_bytes, hip_stream);
}

int astro_chunk_attn_bwd(astro_kvcache_t* cache, const void* q, const void* k_chunk, const void* v_chunk,
                         const void* out, const float* lse, const void* dout, int32_t n_frames, float* dq,
                         float* dk_chunk, float* dv_chunk, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return astro_group_attn_bwd(cache, q, k_chunk, v_chunk, out, lse, dout, n_frames, 1, dq, dk_chunk, dv_chunk, workspace,
                              workspace_bytes, hip_stream);
}

const char* astro_strerror(int err) {
  switch (err) {
    case ASTRO_OK: return "ok";
    case ASTRO_ERR_INVALID_ARG: return "invalid argument";
    case ASTRO_ERR_BAD_STATE: return "call not possible in the current cache state";
    case ASTRO_ERR_UNSUPPORTED: return "unsupported configuration";
    case ASTRO_ERR_HIP: return "HIP runtime error";
    case ASTRO_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    default: return "unknown astro error";
  }
}

}  // extern "C"
