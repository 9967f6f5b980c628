/* ovggt.h -- C ABI of the MI355X (gfx950) OVGGT streaming hot path.
 *
 * One handle holds L independent per-layer KV caches of fixed budget B.  For
 * every incoming frame (M tokens) and layer the caller issues, in this order,
 *
 *     ovggt_global_attn  ->  ovggt_score_select  ->  ovggt_cache_compact
 *
 * which together implement: append the frame's K/V to the cache (paper Eq. 2),
 * temporal causal attention of the frame's queries over every resident entry
 * (Sec. 3.1), Activation Value Rating of the new tokens (Eq. 5), Dynamic
 * Anchor Protection's exemption of flagged tokens (Sec. 3.3), fixed-budget
 * top-k retention (Eq. 8), and the in-place removal of evicted entries.
 *
 * General rules
 *  - All `*_dev` / "device" pointers are HIP device memory owned by the caller
 *    and must outlive the handle; "host" pointers are ordinary host memory.
 *    The library allocates no device memory and frees none.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *    Hot-path calls only enqueue work on it and never synchronise; inputs must
 *    stay valid until the stream has executed the call.  Calls on one handle
 *    must be issued on streams that order them (normally the same stream).
 *  - A handle keeps host-side state and is not synchronised: use it from one
 *    thread at a time.  Different handles are independent.  The device that is
 *    current when a handle is created must be current for every call on it.
 *  - Every function returns OVGGT_OK (0) or a negative error code.  Arguments
 *    and call order are validated on the host before anything is launched; a
 *    failed call changes no state.  Conditions only the device can see set bits
 *    in a per-layer status word (ovggt_cache_status).
 *  - `layer` is in [0, n_layers) or OVGGT_ALL_LAYERS (-1): one launch covers
 *    all layers and every tensor argument carries a leading [n_layers]
 *    dimension; all layers must then be at the same point of the call order.
 *  - Tensors are dense row-major: Q, K, V, O are [M, n_heads, head_dim] (token-
 *    major), residuals are [M, resid_dim], in the handle's dtype.  Pointers
 *    must be 16-byte aligned.
 *  - The physical layout of the cache buffers is private; use
 *    ovggt_cache_export for a defined logical view.
 */
#ifndef OVGGT_H
#define OVGGT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ovggt_cache ovggt_cache;     /* opaque host object */

enum { OVGGT_F32 = 0, OVGGT_BF16 = 1 };
enum { OVGGT_ALL_LAYERS = -1 };
enum {
  OVGGT_OK = 0,
  OVGGT_ERR_ARG = -1,      /* NULL / misaligned pointer, bad layer, bad config value   */
  OVGGT_ERR_STATE = -2,    /* call out of order for that layer                          */
  OVGGT_ERR_NOMEM = -3,    /* host memory for the handle could not be allocated         */
  OVGGT_ERR_HIP = -4,      /* a HIP runtime call failed (launch, copy, query)            */
  OVGGT_ERR_TOO_LARGE = -5 /* ovggt_global_attn_static_ws: the launch needs more than the fixed workspace */
};
/* bits of the device status word */
enum {
  OVGGT_STATUS_BUDGET = 1, /* |P| > B at a selection: Eq. 8's k would be negative; the
                              frame's surplus slots were dropped instead (cache invalid) */
  OVGGT_STATUS_NONFINITE = 2, /* a NaN (or negative) score was seen; it ranks lowest     */
  OVGGT_STATUS_VRANGE = 4  /* bf16 handle: a K or V element was NaN or beyond +-65504 (both
                              are cached as IEEE half; such values were saturated)       */
};

typedef struct {
  int32_t n_layers;          /* L >= 1 independent caches                                  */
  int32_t n_heads;           /* N_h >= 1                                                   */
  int32_t head_dim;          /* d; must be 64                                              */
  int32_t tokens_per_frame;  /* M = 1 + 4 + N_p in the paper (Sec. 3.1); any M >= 1        */
  int32_t resid_dim;         /* C: width of the FFN-residual rows, 1..4096                 */
  int32_t budget;            /* B tokens per layer, protected tokens included; B >= M      */
  int32_t dtype;             /* OVGGT_F32 or OVGGT_BF16: Q/K/V/O/residual and cache storage */
  int32_t score_mode;        /* 0 = every entry keeps the Eq. 5 score it entered with;
                                1 = hybrid scoring (Eq. 7), see hybrid_beta below           */
  float   softmax_scale;     /* 0 => 1/sqrt(head_dim)                                      */
  int32_t out_dtype;         /* type of the attention output O: OVGGT_F32, or OVGGT_BF16
                                (bf16 handles only).  bf16 handles accumulate O in fp32
                                either way; OVGGT_BF16 rounds it once (RNE) on store     */
  /* Activation smoothing (Eq. 6).  smooth_alpha = 0 turns it off and every field below is
   * ignored; the rank key of a token is then ss = s^2.  With 0 < alpha <= 1 a frame is
   * n_special aux tokens followed by a patch_h x patch_w map in row-major order
   * (n_special + patch_h*patch_w = M), s = sqrt(ss) in fp32 (correctly rounded), the patch
   * scores are replaced by alpha*(G*S) + (1-alpha)*S and the aux tokens keep s; that value is
   * the token's rank key (what `ss` of export then holds).  G is the 3x3 kernel below, row-major,
   * applied with the border replicated; the paper fixes neither its size nor its width, so the
   * caller supplies the weights (they should sum to 1).  All of it in fp32 without fused
   * multiply-adds: products g*s are rounded, added left to right in kernel order starting from
   * the first product, then fl(fl(alpha*conv) + fl(fl(1-alpha)*s)).                           */
  float   smooth_alpha;
  int32_t patch_h, patch_w, n_special;
  float   smooth_kernel[9];
  /* Hybrid scoring (Eq. 7), score_mode 1, bf16 handles with n_heads <= 64 only.  Whenever a
   * selection has to evict (n > B after the append), every evictable entry is ranked by
   *   r = (1 - beta) * minmax(d_i),  d_i = 1 - cos(k_i, kbar)   for the entries of earlier frames,
   *   r = beta * minmax(s_i)                                     for the current frame's tokens
   * (s_i = sqrt(ss_i), or Eq. 6's smoothed value when smoothing is on), and r replaces the
   * entry's stored score (`ss` of export); protected entries keep theirs.  k_i is the cached
   * (half precision) key of all heads concatenated, kbar the centroid of the evictable earlier
   * entries, summed exactly in 64-bit fixed point (units of 2^-24) and rounded to fp32 via fp64;
   * dot products and squared norms are fp32 balanced trees over the index h*d + e (zero-padded
   * to a power of two); cos = dot / (sqrt(|k_i|^2) * sqrt(|kbar|^2)), 0 when that product is 0;
   * minmax(x) = (x - min) / (max - min) over the evictable entries of the same source, 0 when
   * max = min.  Every step is one correctly rounded fp32 operation.  Which tokens form the
   * centroid, the concatenation over heads and the degenerate cases are not fixed by the paper.
   * Frames that fit the budget are not ranked at all.  0 <= beta <= 1; ignored in score_mode 0. */
  float   hybrid_beta;
} ovggt_config;

/* Sizes (bytes) of the three caller-allocated device buffers for `cfg`:
 * K/V storage (Eq. 2's cache, capacity B+M per layer, 2*N_h*d elements per
 * token as in the paper's footprint formula), per-slot metadata, and kernel
 * workspace.  Pure host arithmetic.  ERR_ARG on a bad config. */
int ovggt_cache_query_bytes(const ovggt_config* cfg, size_t* kv_bytes, size_t* meta_bytes, size_t* ws_bytes);

/* Create a handle over caller-allocated device buffers of at least the queried
 * sizes (256-byte aligned).  Enqueues zero-fill kernels for all three buffers on
 * `hip_stream`; the cache starts empty (Sec. 3.1: C_{-1} is empty).  *out is
 * host memory freed by ovggt_cache_destroy.  ERR_ARG / ERR_NOMEM / ERR_HIP. */
int ovggt_cache_init(ovggt_cache** out, const ovggt_config* cfg,
                     void* kv_dev, void* meta_dev, void* ws_dev, void* hip_stream);

/* Eq. 2 + Sec. 3.1's temporal causal attention.  Appends (k_new, v_new) as slots
 * [n, n+M) with token ids t*M+i, then out = softmax(q K^T * scale) V over all
 * n+M resident slots (frame-level causality: the frame sees itself entirely).
 * q, k_new, v_new: device, read-only, [M, N_h, d] in the handle's dtype; out:
 * device, written, [M, N_h, d] in the handle's out_dtype.  bf16 runs compute both
 * Q K^T and P V on the f16 MFMA with fp32 accumulation (K and V are cached as IEEE
 * half, the queries are multiplied by scale*log2(e) and rounded to half, softmax
 * weights are rounded to half) and an fp32 online softmax; f32 runs compute in
 * fp32.  Accuracy of bf16 runs: the rounded query makes a logit of magnitude x
 * (after the scale, in units of ln 2) uncertain by about x * 2^-12, so the
 * output error relative to the output's RMS is a few 1e-3 for logits of unit
 * spread and approaches 2e-2 when their spread reaches 16.  Range of bf16 runs: K
 * and V elements beyond +-65504 saturate when cached (OVGGT_STATUS_VRANGE); a query
 * element whose product with scale*log2(e) lies beyond +-65504 is clamped to that
 * bound without a status bit (a finite result instead of NaN; such logits are far
 * outside what the rounding above resolves).  ERR_STATE unless the layer expects a
 * new frame. */
int ovggt_global_attn(ovggt_cache* c, int layer, const void* q, const void* k_new, const void* v_new,
                      void* out, void* hip_stream);

/* ovggt_global_attn for callers that cannot allocate device memory at all (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc) and therefore have no workspace
 * buffer to hand to ovggt_cache_init for the attention's partial results: the same call, same
 * arguments, same kernels and same results, but the partial (O, m, l) records of the launch go to a
 * device array that is part of the library (51 904 512 bytes, held by every GPU the library runs on
 * until the process ends) instead of the handle's workspace.  Calls no allocating routine; nothing
 * in the array has to be cleared between calls (every record the merge pass reads is written by the
 * same launch).  Limit: a launch over more than 16 (layer, head) pairs (layers in the call times
 * n_heads) whose heads cannot be handed out as whole (head pair, query block) items -- the head
 * pairs do not divide among the chip's 8 XCDs, or there are fewer items than workgroups -- needs
 * more records than the array holds, returns OVGGT_ERR_TOO_LARGE and changes nothing; f32 handles
 * use no workspace and behave as ovggt_global_attn.  Every call on a GPU shares that GPU's array: calls that may overlap
 * on one GPU (different streams, different handles) race and must be ordered by the caller. */
int ovggt_global_attn_static_ws(ovggt_cache* c, int layer, const void* q, const void* k_new, const void* v_new,
                                void* out, void* hip_stream);

/* Eq. 5 + Sec. 3.3 + Eq. 8.  Scores the M tokens appended by the preceding
 * ovggt_global_attn from their FFN-residual rows `resid` (device, [M, C]):
 * ss_i = fp32 balanced-tree sum of the fp32 squares (s_i = sqrt(ss_i) is Eq. 5's
 * norm; ranking on ss gives the same order).  `anchor_flags` (device, uint8[M],
 * nonzero = protected, may be NULL = none) marks new members of the protected
 * set P.  If more than B entries are resident, keeps P and the B-|P| best
 * evictable entries under the total order (ss descending, token id ascending)
 * and writes the move list consumed by ovggt_cache_compact.  ERR_STATE unless
 * ovggt_global_attn was the previous call for the layer. */
int ovggt_score_select(ovggt_cache* c, int layer, const void* resid, const uint8_t* anchor_flags,
                       void* hip_stream);

/* Eq. 8's "evict the rest", applied to the layout: after the selection the layer holds
 * min(n+M, B) entries.  Stream rule first: this call enqueues nothing on `hip_stream`.  It closes
 * the frame on the host; the copy itself is enqueued by the next call that touches the layer's
 * cache, on THAT call's stream -- normally the next ovggt_global_attn, whose append overwrites
 * exactly the moved entries' old slots and carries them to their destinations in the same pass
 * (one launch and one pass over those slots less per frame); export, import, set_protect and
 * ovggt_cache_flush apply it first, on their own stream.  A caller that orders work by the
 * stream passed here must therefore order the next call on the layer as well (the general rule:
 * calls on one handle are issued on streams that order them), or call ovggt_cache_flush on the
 * stream it wants the copy on.  Through this interface the cache always reads as compacted.
 * Layout rule (the paper only says that the rest is evicted; this is the build's own choice,
 * unpinned by the paper): the r-th vacated slot below B (ascending) receives the r-th surviving
 * slot at or above B (ascending), for K, V, ids, scores and flags.  At most M entries move,
 * sources and destinations are disjoint, so the rewrite is in place.  Slot order is then not
 * chronological; attention does not depend on it.  ERR_STATE unless ovggt_score_select was the
 * previous call for the layer. */
int ovggt_cache_compact(ovggt_cache* c, int layer, void* hip_stream);

/* Replaying a step from a HIP graph.  The three hot-path calls of a frame only launch kernels
 * (no memset or copy nodes, no host synchronisation, no allocation) and no kernel argument depends
 * on the frame number -- the frame's first token id t*M (Eq. 2's arrival order) is kept in device
 * memory -- so once the cache is full a step may be captured into a graph (hipStreamBeginCapture
 * on the stream passed to the calls; kernel timing off) and replayed for every later frame, with
 * the frame's inputs copied into the captured buffers before each replay.  The capture requires
 * the steady state: at least one evicting frame completed, nothing that flushes the compaction
 * (export, set_protect, ...) since.  The captured calls update the host-side state as if they had
 * run, so the capture accounts for the first replay; BEFORE every further replay call
 * ovggt_cache_advance(c, layer, 1) (or once with the count before a run of replays): it checks
 * that the handle is still in the state the graph was captured in and counts the frames.  If it
 * fails, do not replay; issue the frame through the three calls instead.  Host arithmetic only.
 * ERR_STATE unless the layer is in that steady state and expects a new frame; ERR_ARG if
 * frames < 1 or the token ids would leave 32 bits. */
int ovggt_cache_advance(ovggt_cache* c, int layer, int64_t frames);

/* Enqueues any compaction of `layer` (or OVGGT_ALL_LAYERS) that has not been
 * applied yet, as a launch of its own on `hip_stream`.  No-op otherwise. */
int ovggt_cache_flush(ovggt_cache* c, int layer, void* hip_stream);

/* Frees the host handle (device buffers stay with the caller). */
int ovggt_cache_destroy(ovggt_cache* c);

/* Sec. 3.3, historical anchors: grant (on != 0) or withdraw (on == 0) protection of tokens
 * that are already cached.  Affects the still-resident tokens of frame `frame` (token ids
 * frame*M .. frame*M + M - 1) whose byte in `mask` (device, uint8[M]) is nonzero; mask NULL =
 * every token of the frame.  Tokens of the frame that were evicted earlier stay evicted: a late
 * registration covers what is left.  A released token returns to the evictable set with the
 * score it holds.  `layer` may be OVGGT_ALL_LAYERS (one mask for all).  Enqueues on `hip_stream`;
 * no host synchronisation.  With hybrid scoring the running centroid sum follows the change.
 * ERR_STATE unless the layer expects a new frame (after ovggt_cache_compact, before the next
 * ovggt_global_attn); ERR_ARG for a frame not yet seen.  |P| > B shows at the next selection
 * (OVGGT_STATUS_BUDGET). */
int ovggt_cache_set_protect(ovggt_cache* c, int layer, int64_t frame, const uint8_t* mask, int on,
                            void* hip_stream);

/* ---- helpers, not on the hot path ------------------------------------- */

/* Resident entries of `layer` (host arithmetic, no synchronisation): after a
 * completed frame this is min((t+1)*M, B); between global_attn and compact it
 * still counts the frame's M pending slots. */
int ovggt_cache_size(const ovggt_cache* c, int layer, int32_t* n);

/* Frames fully processed by `layer`. */
int ovggt_cache_frames(const ovggt_cache* c, int layer, int64_t* t);

/* Synchronises `hip_stream`, reads the layer's device status word into
 * *status (host) and clears it on the device. */
int ovggt_cache_status(ovggt_cache* c, int layer, int32_t* status, void* hip_stream);

/* Synchronises `hip_stream` and copies the layer's n resident entries to host
 * buffers in slot order: ids uint32[n], k and v [n, N_h, d] in the handle's
 * dtype, ss float[n], flags uint8[n].  Any output pointer may be NULL.  Serves
 * tests and checkpointing.  For bf16 handles K and V come back as bf16(half(x)):
 * equal to the appended value whenever that is a normal half number. */
int ovggt_cache_export(ovggt_cache* c, int layer, uint32_t* ids, void* k, void* v, float* ss,
                       uint8_t* flags, void* hip_stream);

/* Inverse of export: replaces the layer's contents by n <= B entries given in
 * host buffers (all required) and sets its processed-frame count to `frames`
 * (the next frame's token ids start at frames*M).  Synchronous. */
int ovggt_cache_import(ovggt_cache* c, int layer, int32_t n, int64_t frames, const uint32_t* ids,
                       const void* k, const void* v, const float* ss, const uint8_t* flags,
                       void* hip_stream);

/* Copies the most recent move list of `layer` to host (dst, src: uint32[M]) and
 * its length to *n_moves.  Synchronises `hip_stream`.  For tests/diagnostics. */
int ovggt_cache_last_moves(ovggt_cache* c, int layer, uint32_t* dst, uint32_t* src, int32_t* n_moves,
                           void* hip_stream);

/* Kernel timing for benchmarks (off by default; the hot path records nothing
 * when off).  level 1: bracket the attention kernel of every `every`-th
 * ovggt_global_attn call with HIP events on the call's stream; level 2: bracket
 * every kernel of every call.  ovggt_profile_read synchronises `hip_stream`,
 * returns per kernel class the summed elapsed milliseconds and the number of
 * bracketed launches since the last read (host arrays of OVGGT_PROF_CLASSES
 * entries), and resets them. */
enum { OVGGT_PROF_APPEND = 0, OVGGT_PROF_ATTN = 1, OVGGT_PROF_COMBINE = 2, OVGGT_PROF_SELECT = 3,
       OVGGT_PROF_COMPACT = 4, OVGGT_PROF_CLASSES = 5 };
int ovggt_profile_enable(ovggt_cache* c, int level, int every);
int ovggt_profile_read(ovggt_cache* c, double* ms_sum, int64_t* count, void* hip_stream);
/* What an event bracket reports beyond the bracketed kernel's own execution: the mean elapsed
 * milliseconds of the same bracket around `reps` launches of a kernel that runs for a known time
 * (one wave that watches the device's constant-rate wall clock for 0.1 ms, about as long as the
 * kernels the brackets are used on), minus that time.  Touches no buffer of the handle.
 * Synchronises `hip_stream`. */
int ovggt_profile_overhead(ovggt_cache* c, int reps, double* ms_mean, void* hip_stream);

/* ---- Dynamic Anchor Protection: which frames become anchors (Sec. 3.3) ------------------
 * Host-only bookkeeping; no device work, usable without a GPU.  The model's outputs are inputs:
 * the coverage ratio rho_t (fraction of the latest anchor's points that project inside the
 * current image) and the per-patch confidences of the point head.
 * Frame 0 is the global initial anchor: the caller protects all of its tokens when it inserts
 * them (anchor_flags of ovggt_score_select); it is never demoted, does not count towards k_max,
 * and is the reference of the first coverage test and of the spacing rule.  At frame t > 0 a
 * new anchor is registered when rho_t < tau and t - (last registration) >= min_gap.  Of its
 * n_patches patch tokens the ceil(eta * n_patches) (in double precision) with the highest
 * confidence are protected, equal confidences going to the lower patch index; the n_special
 * aux tokens are not.  When k_max anchors are active, the oldest is demoted (FIFO).  The
 * protected set then obeys |P| <= M + k_max * ceil(eta * n_patches) (Eq. 9). */
typedef struct ovggt_dap ovggt_dap;
/* ERR_ARG unless k_max >= 1, min_gap >= 1, 0 < eta <= 1, n_patches >= 1, n_special >= 0 and tau is a number. */
int ovggt_dap_create(ovggt_dap** out, int32_t k_max, int32_t min_gap, double tau, double eta,
                     int32_t n_special, int32_t n_patches);
/* Decision for frame t (frames must be fed in increasing order; ERR_ARG otherwise).  conf: host,
 * float[n_patches], finite; may be NULL when the frame cannot become an anchor anyway.
 * *register_frame = t and mask_out (host, uint8[n_special + n_patches], written in full) when
 * frame t becomes an anchor, else -1 and mask_out untouched.  *demote_frame = the frame to
 * release (pass it to ovggt_cache_set_protect with on = 0 and mask NULL), else -1. */
int ovggt_dap_step(ovggt_dap* d, int64_t t, double rho, const float* conf, int64_t* register_frame,
                   uint8_t* mask_out, int64_t* demote_frame);
/* Active historical anchors, oldest first: writes up to cap frame numbers, *n = how many are active. */
int ovggt_dap_active(const ovggt_dap* d, int64_t* frames, int32_t cap, int32_t* n);
int ovggt_dap_destroy(ovggt_dap* d);

/* Host-only: how the bf16 attention launch of `layers_in_launch` layers (1 or cfg->n_layers) over
 * n_total resident slots would be divided among n_wgs workgroups (the library uses one per compute
 * unit).  Walks the plan as the kernel does and checks that every (head, query block, key tile) is
 * covered exactly once and that no workgroup needs more partial records than it owns.
 * out[0..7] = workgroups, rounds per workgroup, tile segments, 1 if chunks are cost-balanced, most
 * pieces given to one workgroup, fewest and most tiles given to one workgroup, work items in which
 * both halves of a workgroup take two query blocks of one head (they fetch that head's K/V tiles
 * once for both; the walk also checks that items and halves cover every query block of every head
 * exactly once); cost[0..1] = largest and mean estimated cost per workgroup in tiles (tiles + a
 * fixed charge per piece).
 * OVGGT_OK, ERR_ARG (bad config or sizes), ERR_STATE (inconsistent plan: a bug). */
int ovggt_attn_plan_stats(const ovggt_config* cfg, int32_t layers_in_launch, int32_t n_total, int32_t n_wgs,
                          int32_t* out, float* cost);

const char* ovggt_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* OVGGT_H */
