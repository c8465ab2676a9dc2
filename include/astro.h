/*
 * astro.h -- C ABI of the rolling-KV-cache chunk-attention library for MI355X (gfx950).
 *
 * The library implements the attention hot path of the streaming RL scheme of
 * arXiv 2603.17051: a stream of video frames is generated chunk by chunk; each
 * new chunk attends to a bounded context (a few permanent "sink" frames plus a
 * rolling window of the most recent frames, Sec. 3.2) held in a ring-buffer KV
 * cache, and in the RL update the cached context is a constant while gradients
 * flow through the chunk only (Sec. 3.3, "Streaming Long Tuning").
 *
 * Conventions
 *   B streams (independent caches), H heads, D head dim, frames of
 *   T = grid_h * grid_w tokens, ring capacity C frames of which the first S
 *   appended after a reset are sinks, window Lw = C - S.
 *   Chunk tensors are [B, n_frames*T, H, D], D contiguous, token index
 *   n = (frame_in_chunk * grid_h + row) * grid_w + col.
 *   "device" pointers are HIP device memory owned by the CALLER (e.g. torch
 *   tensors); the library never frees them and keeps none of them beyond the
 *   call, except k_storage / v_storage, which it uses until destroy.
 *   All launches are asynchronous on the caller's HIP stream (`hip_stream` is a
 *   hipStream_t cast to void*; NULL = the default stream).  Calls on one cache
 *   handle must be made from one host thread at a time.
 *   Every function returns ASTRO_OK (0) or a negative astro error.  Arguments and state are
 *   checked before anything else: ASTRO_ERR_INVALID_ARG, _BAD_STATE, _UNSUPPORTED and _WORKSPACE
 *   mean that nothing was launched and no state has changed.  ASTRO_ERR_HIP means the HIP runtime
 *   refused a launch or a copy of a call that was valid: launches before it may be enqueued, the
 *   call's output buffers and workspace contents are undefined, and the tables are not advanced.
 *   If that happens to astro_kvcache_append after the ring was touched, the ring rows no longer
 *   match the tables: the handle then answers every call but astro_kvcache_tables and
 *   astro_kvcache_destroy with ASTRO_ERR_BAD_STATE until astro_kvcache_reset(cache, -1, ...)
 *   has emptied all streams.
 *
 * Rotary embedding (the paper names none; this layout is fixed by the library):
 *   adjacent pairs (x[2i], x[2i+1]), i < D/2; pairs [0, n_t) turn with the
 *   absolute frame index, [n_t, n_t+n_h) with the row, the rest with the column;
 *   pair j of an axis with n pairs has frequency rope_base^(-j/n).  Keys are
 *   cached after rotation; values are never rotated.  All three counts 0 = no
 *   rotary embedding.
 *
 * Window-relative temporal positions (ASTRO_FLAG_WINDOW_RELATIVE).  Sec. 4.3 runs models
 *   trained on short clips for long videos through a positional-extrapolation method it
 *   only cites; the library's reading: the temporal position of a frame is its RANK in the
 *   sequence a chunk attends to -- sinks 0 .. S-1, then the resident window frames from
 *   oldest to newest, then the chunk's frames -- so no position exceeds C + n_frames - 1
 *   however long the stream runs, and start_frame no longer matters.  Rows and columns
 *   are unchanged.  Since rotary scores depend on position differences only, and window
 *   and chunk frames are consecutive in both numberings, this equals keeping absolute
 *   indices for them and moving the SINKS forward by the number of frames evicted so
 *   far.  That is how it is stored: every append that evicts rotates the sinks' keys
 *   again, from an un-rotated copy kept in k_sink_storage (one rounding, however often
 *   they move), to their new position; the attention calls are unchanged.
 */
#ifndef ASTRO_H_
#define ASTRO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ASTRO_OK 0
#define ASTRO_ERR_INVALID_ARG (-1) /* null pointer, size or shape out of range        */
#define ASTRO_ERR_BAD_STATE (-2)   /* call not possible in the handle's current state */
#define ASTRO_ERR_UNSUPPORTED (-3) /* valid request the kernels do not cover          */
#define ASTRO_ERR_HIP (-4)         /* a HIP runtime call failed                       */
#define ASTRO_ERR_WORKSPACE (-5)   /* workspace missing or too small                  */

#define ASTRO_BF16 0 /* bf16 tensors, bf16 MFMA, fp32 accumulation (production path)  */
#define ASTRO_F32 1  /* fp32 tensors and arithmetic (slow debug path)                 */

/* desc.flags */
#define ASTRO_FLAG_HOST_ONLY 1 /* no device work at all: the handle only plans slots  */
#define ASTRO_FLAG_WINDOW_RELATIVE 2 /* temporal rotary positions by rank in the window   */
#define ASTRO_FLAG_REUSE_STAGED 4 /* a backward may reuse what the forward before it staged */

#define ASTRO_MAX_BATCH 64
#define ASTRO_MAX_CAPACITY_FRAMES 256

typedef struct astro_kvcache astro_kvcache_t; /* opaque */

typedef struct astro_kvcache_desc {
  int32_t batch, heads, head_dim;     /* B in [1,64], H >= 1, D in {64, 128}              */
  int32_t grid_h, grid_w;             /* T = grid_h * grid_w tokens per frame             */
  int32_t capacity_frames;            /* C in [1,256]: frames resident before a chunk     */
  int32_t sink_frames;                /* S, 0 <= S < C                                    */
  int32_t max_chunk_frames;           /* largest n_frames of any call, 1 .. C - S         */
  int32_t rope_pairs_t, rope_pairs_h, rope_pairs_w; /* sum == D/2, or all three 0         */
  int32_t dtype;                      /* ASTRO_BF16 or ASTRO_F32                          */
  int32_t flags;                      /* bit set of ASTRO_FLAG_*                          */
  int32_t block_frames;               /* block size of the causal mask inside a chunk, in */
                                      /* frames; 0 = the whole chunk is one block         */
  double rope_base;                   /* > 1, e.g. 10000                                  */
  void *k_storage, *v_storage;        /* device, sizes from astro_kvcache_bytes; layout   */
                                      /* [B][H][C*T][D] of dtype; may be NULL iff         */
                                      /* ASTRO_FLAG_HOST_ONLY                             */
  void *k_sink_storage;               /* device, astro_kvcache_sink_bytes: un-rotated     */
                                      /* keys of the sink frames, [B, S*T, H, D] of dtype;*/
                                      /* needed iff ASTRO_FLAG_WINDOW_RELATIVE with S > 0 */
                                      /* and rotary pairs on the frame axis (not HOST_ONLY)*/
} astro_kvcache_desc_t;

/* Bytes of device storage the cache of `desc` needs for keys and for values
 * (Sec. 3.2: constant in the video length).  Host only. */
int astro_kvcache_bytes(const astro_kvcache_desc_t *desc, size_t *k_bytes, size_t *v_bytes);

/* Bytes of k_sink_storage for `desc` (0 when it is not needed).  Host only. */
int astro_kvcache_sink_bytes(const astro_kvcache_desc_t *desc, size_t *bytes);

/* Create a cache handle: all B streams empty, start frame 0.  Validates `desc`,
 * builds the per-row / per-column rotary tables in fp64 and uploads them (small,
 * library-owned device memory; the only allocation the library makes).
 * Host-synchronous.  *out is untouched on error. */
int astro_kvcache_create(const astro_kvcache_desc_t *desc, astro_kvcache_t **out);

/* Free the handle and its small tables (not k_storage / v_storage).  The caller
 * must have synchronised every stream that still uses the cache. */
int astro_kvcache_destroy(astro_kvcache_t *cache);

/* Empty stream `stream` (or all streams if -1) and set the absolute index of the
 * next appended frame to `start_frame` (>= 0).  Host only; storage is not cleared. */
int astro_kvcache_reset(astro_kvcache_t *cache, int32_t stream, int32_t start_frame);

/* Sec. 3.2, rolling cache with frame sinks: commit `n_frames` new frames per
 * stream.  k, v: device, un-rotated, [B, n_frames*T, H, D].  Frame number n of a
 * stream (0-based since reset) goes to ring slot n if n < C, else
 * S + (n - S) mod Lw, overwriting -- evicting -- frame n - Lw; keys are rotated
 * at absolute frame index start_frame + n and stored, values copied.
 * With ASTRO_FLAG_WINDOW_RELATIVE the un-rotated keys of arriving sink frames are also
 * copied to k_sink_storage, and once frames are evicted the sinks' keys in the ring are
 * rotated again at start_frame + s + (frames evicted so far) in the same call.
 * 1 <= n_frames <= min(max_chunk_frames, Lw).  Advances the tables. */
int astro_kvcache_append(astro_kvcache_t *cache, const void *k, const void *v, int32_t n_frames,
                         void *hip_stream);

/* Host copies of the integer tables: slot_frame[B*C] = absolute index of the
 * frame resident in each ring slot (-1 = empty), slot_pos[B*C] = its temporal
 * rotary position (-1 = empty): the absolute index, or with ASTRO_FLAG_WINDOW_RELATIVE
 * its rank among the resident frames; next_n[B] = frames appended since reset.  Any
 * output pointer may be NULL.  Host only (tables are host-authoritative). */
int astro_kvcache_tables(const astro_kvcache_t *cache, int32_t *slot_frame, int32_t *slot_pos,
                         int32_t *next_n);

/* Bytes of caller-provided device workspace the two attention calls need for a
 * chunk of n_frames (rotated copies of Q and K_chunk; for backward also the
 * row terms and rotated-gradient staging).  Either output may be NULL. */
int astro_chunk_attn_workspace_bytes(const astro_kvcache_t *cache, int32_t n_frames,
                                     size_t *fwd_bytes, size_t *bwd_bytes);

/* Block-causal chunk attention over the rolling cache (Sec. 3.1 / 3.2: the new
 * chunk is conditioned on the KV cache of the context window only).  For every
 * stream, the chunk's queries (rotated at frame indices start_frame + next_n ...)
 * attend to all resident cache frames and to all keys of the chunk itself:
 *   out = softmax(Q~ K~^T / sqrt(D)) V,  lse = log-sum-exp of the scaled scores.
 * With desc.block_frames = k > 0 the chunk's frames form blocks of k frames (the last
 * may be shorter) and a query sees, of the chunk, only the keys of its own and of
 * earlier blocks (block-causal attention at that block size; k = 1 is the frame-by-
 * frame factorisation p(x_i | x_<i) of Sec. 3.1 evaluated for several frames in one
 * call); resident frames stay visible to every query.  Every attention call of the
 * handle (chunk, group, both backwards) uses the same mask.
 * q, k_chunk, v_chunk: device, un-rotated, [B, n_frames*T, H, D];
 * out: device [B, n_frames*T, H, D] (dtype of the cache); lse: device fp32
 * [B, H, n_frames*T].  Does not modify the cache or its tables (append does).
 * workspace: device, >= fwd_bytes, 256-byte aligned; contents undefined after. */
int astro_chunk_attn_fwd(astro_kvcache_t *cache, const void *q, const void *k_chunk,
                         const void *v_chunk, int32_t n_frames, void *out, float *lse,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/* Backward of astro_chunk_attn_fwd with the cached context detached (Sec. 3.3):
 * given dout = dL/dout, writes dL/dq, dL/dk_chunk, dL/dv_chunk (fp32, device,
 * [B, n_frames*T, H, D], w.r.t. the UN-rotated inputs).  Cached keys / values get
 * no gradient.  q, k_chunk, v_chunk, out, lse must be those of a forward call on
 * the same cache state.  dout has the cache dtype.
 * workspace: device, >= bwd_bytes, 256-byte aligned.
 * With ASTRO_FLAG_REUSE_STAGED (the re-forward + backward of gradient checkpointing, Table S1):
 * an attention call whose q, k_chunk, workspace pointer, n_frames and group equal those of the
 * handle's previous attention call, with no reset or append in between, skips the rotation
 * pre-pass and reads the rotated copies that call left at the start of the workspace.  The
 * caller promises that q, k_chunk and the workspace were not written in between (by anything
 * but this library's attention calls on this handle).  The decision is taken on the host when
 * the call is made: a call recorded into a HIP graph skips (or runs) the pre-pass on every
 * replay as it did at capture, so capture the forward together with the backward that reuses it. */
int astro_chunk_attn_bwd(astro_kvcache_t *cache, const void *q, const void *k_chunk,
                         const void *v_chunk, const void *out, const float *lse,
                         const void *dout, int32_t n_frames, float *dq, float *dk_chunk,
                         float *dv_chunk, void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/* The non-detached backward ("Clip + Full BP" of the paper's streaming-training ablation,
 * Sec. 4.5, Table 4(a)): everything astro_chunk_attn_bwd writes, plus the gradients the detach drops,
 *   dk_cache, dv_cache: device fp32 [B, C*T, H, D], row = slot*T + token, w.r.t. the keys
 *   (UN-rotated, as they were appended) and values of the frames resident in the ring.
 * Rows of slots that hold no frame are not written.  bf16 caches only (ASTRO_ERR_UNSUPPORTED
 * for ASTRO_F32).  workspace: >= astro_chunk_attn_bwd_full_workspace_bytes, 256-byte aligned. */
int astro_chunk_attn_bwd_full_workspace_bytes(const astro_kvcache_t *cache, int32_t n_frames,
                                              size_t *bytes);
int astro_chunk_attn_bwd_full(astro_kvcache_t *cache, const void *q, const void *k_chunk,
                              const void *v_chunk, const void *out, const float *lse,
                              const void *dout, int32_t n_frames, float *dq, float *dk_chunk,
                              float *dv_chunk, float *dk_cache, float *dv_cache, void *workspace,
                              size_t workspace_bytes, void *hip_stream);

/* Group-wise candidates over one shared, frozen cache (Sec. 3.2, clip-level group
 * sampling: G candidate continuations are generated from the same rolling KV cache and
 * compared; Sec. 3.3 for the backward).  The chunk tensors hold `group` candidate chunks
 * per cache stream: q, k_chunk, v_chunk, out, dout, dq, dk_chunk, dv_chunk are
 * [B*group, n_frames*T, H, D] and lse is [B*group, H, n_frames*T], candidate
 * c = b*group + g.  Every candidate of stream b sits at the chunk position of stream b
 * (frames start_frame + next_n ...), attends to stream b's resident frames and to its OWN
 * chunk keys only, never to another candidate's.  Otherwise exactly as the chunk calls
 * (which are these with group = 1): same dtypes, workspace rules, errors; the cache is not
 * modified (append the chosen candidate's k_chunk, v_chunk afterwards).
 * group >= 1 and B*group <= ASTRO_MAX_BATCH, else ASTRO_ERR_INVALID_ARG. */
int astro_group_attn_workspace_bytes(const astro_kvcache_t *cache, int32_t n_frames, int32_t group,
                                     size_t *fwd_bytes, size_t *bwd_bytes);
int astro_group_attn_fwd(astro_kvcache_t *cache, const void *q, const void *k_chunk,
                         const void *v_chunk, int32_t n_frames, int32_t group, void *out,
                         float *lse, void *workspace, size_t workspace_bytes, void *hip_stream);
int astro_group_attn_bwd(astro_kvcache_t *cache, const void *q, const void *k_chunk,
                         const void *v_chunk, const void *out, const float *lse, const void *dout,
                         int32_t n_frames, int32_t group, float *dq, float *dk_chunk,
                         float *dv_chunk, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Clip-level forward-process RL loss and its gradient (Sec. 3.1 eq. (1)-(2); Sec. 3.3 reward
 * normalisation; Sec. 3.4 selective KL; Alg. 1, Phase 2), one fused pass.  For sample i of
 * n_samples, each of elems_per_sample elements:
 *   r~_i = clip(A_i / a_max, -1, 1) / 2 + 0.5
 *   v+ = (1 - beta) v_old + beta v_theta,   v- = (1 + beta) v_old - beta v_theta
 *   L_policy = (1/n) sum_i [ r~_i |v+ - target|^2 + (1 - r~_i) |v- - target|^2 ]   (|.|^2 = sum over the sample)
 *   L_KL     = (1/|M|) sum_{i : kl_mask_i != 0} |v_theta - v_ref|^2               (0 if no sample is masked)
 *   loss[0] = L_policy + lambda_kl L_KL, loss[1] = L_policy, loss[2] = L_KL
 *   grad_v_theta = d loss[0] / d v_theta (fp32, same shape).
 * v_theta, v_old, v_ref, target: device, [n_samples, elems_per_sample] of `dtype` (ASTRO_BF16
 * or ASTRO_F32), 16-byte aligned; elems_per_sample a multiple of 8 (bf16) / 4 (fp32), else
 * ASTRO_ERR_UNSUPPORTED.  advantage: device fp32 [n_samples]; kl_mask: device int32
 * [n_samples]; loss: device fp32 [3]; grad_v_theta: device fp32, 16-byte aligned.
 * n_samples in 1 .. 65535; a_max > 0.  workspace: device, >= the reported bytes, 256-byte
 * aligned.  Arithmetic in fp32, the final sums in fp64; results do not depend on timing. */
int astro_nft_loss_workspace_bytes(int32_t n_samples, int64_t elems_per_sample, size_t *bytes);
int astro_nft_loss(const void *v_theta, const void *v_old, const void *v_ref, const void *target,
                   const float *advantage, const int32_t *kl_mask, int32_t n_samples,
                   int64_t elems_per_sample, int32_t dtype, float a_max, float beta, float lambda_kl,
                   float *loss, float *grad_v_theta, void *workspace, size_t workspace_bytes,
                   void *hip_stream);

/* astro_nft_loss for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation,
 * arguments, results and errors as astro_nft_loss without the workspace: r~, the masked count and
 * the per-block partial sums live in a static device array of astro_nft_loss_static_bytes() bytes
 * (1 MiB) that every GPU the library runs on holds until the process ends.  The call allocates and
 * frees nothing and calls no allocating routine (its launches are never timed by astro_profile_*,
 * which would create events).  A size whose workspace
 * (astro_nft_loss_workspace_bytes) exceeds the array is rejected with ASTRO_ERR_WORKSPACE and
 * nothing is launched.  All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams or host threads) race; calls on one stream are ordered and safe, and
 * no call depends on what an earlier one left in the array. */
int astro_nft_loss_static_bytes(size_t *bytes);
int astro_nft_loss_static(const void *v_theta, const void *v_old, const void *v_ref, const void *target,
                          const float *advantage, const int32_t *kl_mask, int32_t n_samples,
                          int64_t elems_per_sample, int32_t dtype, float a_max, float beta,
                          float lambda_kl, float *loss, float *grad_v_theta, void *hip_stream);

/* Measurement aid (Sec. 3.2 / 3.3 name no kernels; this times the library's own):
 * between begin and end every kernel launch is bracketed by HIP events recorded on
 * the stream it is launched on.  end() waits for those events (host-synchronous),
 * aggregates by kernel name into out[0 .. *n_entries) (at most max_entries names)
 * and switches timing off.  Process-wide, one host thread. */
typedef struct astro_kernel_time {
  char name[48];     /* kernel name, NUL-terminated */
  int32_t launches;  /* launches seen                */
  float total_ms;    /* summed event time            */
} astro_kernel_time_t;
int astro_profile_begin(void);
int astro_profile_end(astro_kernel_time_t *out, int32_t max_entries, int32_t *n_entries);

/* Machine calibration for the roofline the attention kernels are priced against (no
 * operation of the paper; both are timed through astro_profile_* under the names
 * "calib_mfma_bf16" and "calib_copy").
 * astro_calib_mfma: `workgroups` workgroups of 4 waves issue nothing but bf16 16x16x32
 *   MFMAs (the shape the attention kernels use): iters * 32 per wave, 16384 flop each.  operands: device, 8 * 256 * 16 bytes of
 *   bf16 (4 A and 4 B fragments per lane); the clock the chip sustains depends on their
 *   values (all zero vs N(0,1)).  sink: device, workgroups * 256 floats, overwritten.
 *   workgroups in 1 .. 65536, iters in 1 .. 2^20.
 * astro_calib_copy: dst[0 .. bytes) = src[0 .. bytes), device pointers, 16-byte aligned,
 *   bytes a multiple of 16; moves 2 * bytes through HBM when bytes exceeds the caches. */
int astro_calib_mfma(const void *operands, int32_t workgroups, int32_t iters, float *sink, void *hip_stream);
int astro_calib_copy(const void *src, void *dst, size_t bytes, void *hip_stream);

/* Static, never-NULL description of an error code. */
const char *astro_strerror(int err);

#ifdef __cplusplus
}
#endif
#endif /* ASTRO_H_ */
