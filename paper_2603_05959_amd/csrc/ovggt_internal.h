// Internal layout description and kernel launchers shared by the HIP
// translation units of libovggt.  Nothing here is part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

// Timing builds (-DOVGGT_TRACE) keep cycle stamps of the kernels' phases; in product builds the
// statements inside OVGGT_TRACE_ONLY(...) do not exist.
#ifdef OVGGT_TRACE
#define OVGGT_TRACE_ONLY(...) __VA_ARGS__
#else
#define OVGGT_TRACE_ONLY(...)
#endif

namespace ovggt {

constexpr int kSlotTile = 128;      // attention consumes the cache in 128-slot tiles
constexpr int kQueryTile = 128;     // queries per attention work item
constexpr int kMaxAttnWgs = 256;    // upper bound on attention workgroups (one per CU; sizes the workspace)

// Per-layer control block kept in the metadata buffer.
struct Ctrl {
  uint32_t status;     // OVGGT_STATUS_* bits
  uint32_t n_moves;    // length of the move list written by the last selection
  uint32_t arrive;     // arrival counter of the score kernel's workgroups
  uint32_t gid_next;   // token id of the next frame's first token (t * M): read by the append, advanced by M by
                       // the frame's selection, so a step's launches carry no per-frame argument
  uint32_t pad[60];
};
static_assert(sizeof(Ctrl) == 256, "Ctrl is one 256-byte block");

// Geometry of one handle.  Device K/V storage per layer is
//   K[H][cap][d] followed by V[H][cap][d]   (head-major, slot rows of d elements)
// so one head's 128-slot tile is a contiguous 128*d*esize block.
struct Geom {
  int L, H, d, M, C, B;
  int cap;                 // slots per layer: round_up(B + M, kSlotTile)
  int esize;               // 2 (bf16) or 4 (f32)
  int hybrid;              // 1: hybrid scoring (Eq. 7), the handle maintains the centroid of its evictable keys
  size_t kv_layer_bytes;   // 2 * H * cap * d * esize
  size_t meta_layer_bytes;
  size_t off_ids, off_ss, off_flags, off_ctrl, off_mvdst, off_mvsrc;   // byte offsets in a layer's metadata
  size_t off_csum;         // H*d 64-bit sums of the evictable resident keys, units of 2^-24 (hybrid scoring)
  size_t off_evbits;       // evict bit per slot of the last selection, 32 slots per word (hybrid scoring)
  size_t off_dval;         // d_i = 1 - cos(k_i, centroid) of the slots below n_old, one fp32 per slot (hybrid scoring)
  size_t off_cvec;         // the sum as H*d fp32 values, refreshed by each frame's append (hybrid scoring)
  size_t off_dpart;        // (min, max) of d_i over the evictable slots of each wave of the diversity pass (hybrid scoring)
  size_t off_mvmap;        // per slot B + j (j < M): the slot below B it moves to under the last selection, or kNoMove
  size_t off_hist;         // kSelHistBins counters: the selection's first-level histogram of the cached entries' score
                           // words, filled by all workgroups of a launch and zeroed again by the one that selects
};

constexpr int kSelHistBins = 2048;  // the 11 bits below the sign of a score word
constexpr uint32_t kNoMove = 0xFFFFFFFFu;

__host__ __device__ inline char* layer_k(char* kv, const Geom& g, int layer) {
  return kv + (size_t)layer * g.kv_layer_bytes;
}
__host__ __device__ inline char* layer_v(char* kv, const Geom& g, int layer) {
  return kv + (size_t)layer * g.kv_layer_bytes + (size_t)g.H * g.cap * g.d * g.esize;
}
__host__ __device__ inline char* layer_meta(char* meta, const Geom& g, int layer) {
  return meta + (size_t)layer * g.meta_layer_bytes;
}

// ---- launchers (each only enqueues on `s`) ---------------------------------
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
// One wave that runs for `ticks` ticks of the device's constant-rate wall clock (timing aid).
hipError_t launch_spin(unsigned long long ticks, hipStream_t s);

// Eq. 2: copy the frame's K/V rows into slots [n, n+M) of layers [layer0, layer0+nl)
// and initialise their ids (the layer's gid_next + i), scores (0) and flags (0).  apply_moves: the previous
// frame's compaction is still outstanding (n == B then): every entry that the last selection
// moves out of a slot the new frame overwrites is carried to its destination first.
hipError_t launch_append(const Geom& g, char* kv, char* meta, int layer0, int nl,
                         const void* k_new, const void* v_new, int n, bool apply_moves, hipStream_t s);

// Attention of M queries over n_total resident slots.
hipError_t launch_attn_f32(const Geom& g, char* kv, int layer0, int nl, const void* q, void* out,
                           int n_total, float scale, hipStream_t s);
// `ev` (optional, 3 events) are recorded before the main kernel, between it and
// the combine kernel, and after the combine kernel.
hipError_t launch_attn_bf16(const Geom& g, char* kv, int layer0, int nl, const void* q, void* out,
                            int n_total, float scale, char* ws, size_t ws_bytes, int n_wgs, bool out_f32,
                            hipStream_t s, hipEvent_t* ev = nullptr);
size_t attn_ws_bytes(int layer_heads, int query_blocks);
bool attn_whole_items(int layer_heads, int query_blocks, int n_wgs);
// The library's own workspace for the attention's partial records (a device array of fixed size, one
// copy per GPU): its device address on the current device and its size.  Looks the address up on the
// first call per device; allocates nothing.
hipError_t attn_static_ws(char** ptr, size_t* bytes);
// What the attention launch over nl layers and n_total resident slots hands to its workgroups (host-side walk of
// the plan; false: the plan is inconsistent).  cost = tiles + a fixed charge per piece, in tiles.
struct AttnPlanStats {
  int n_wgs, rounds, segments, balanced, pieces_max, tiles_min, tiles_max;
  int shared_items;           // items whose two wave sets take two query blocks of one head (one fetch of its K/V tiles for both)
  float cost_max, cost_mean;
};
bool attn_plan_stats(const Geom& g, int nl, int n_total, int n_wgs, size_t ws_bytes, AttnPlanStats* st);

// Eq. 6: activation smoothing of a frame's patch scores (alpha = 0: off).
struct SmoothParams {
  float alpha;
  int ph, pw, n_special;
  float g[9];
};

// Eq. 7: how the selection ranks (on = 0: every entry by the score it entered with).
struct HybridParams {
  int on;
  float beta;
  int n_part;              // waves of the frame's diversity pass = (min, max) pairs it left per layer
};

// Slots per workgroup and workgroups per layer of the diversity pass (a wave takes 8 slots at a time).
constexpr int kDivSlotsPerWg = 32;
constexpr int kDivWavesPerWg = 4;
inline int diversity_grid_x(int n_hist, int nl) {
  long gx = (n_hist + kDivSlotsPerWg - 1) / kDivSlotsPerWg;
  const long cap_x = 8192 / nl > 0 ? 8192 / nl : 1;      // 24 layers: 155 us at 8192 workgroups, 159 at 4096, 160 at 12288
  return (int)(gx > cap_x ? cap_x : gx);
}

// Eq. 7, history side (bf16 handles only: the cache holds K as half).  The handle keeps the exact sum of
// its evictable resident keys per layer:
//   launch_diversity        d_i = 1 - cos(k_i, centroid) written to the d_i array for the evictable slots below n_hist
//   launch_centroid_update  after the frame's selection: add the frame's evictable tokens that stay, subtract
//                           the evicted entries of earlier frames (reads the hole list and the evict bitmap)
//   launch_centroid_rebuild zero the sum and add every evictable slot below n (after an import)
hipError_t launch_diversity(const Geom& g, char* kv, char* meta, int layer0, int nl, int n_hist, hipStream_t s);
hipError_t launch_centroid_update(const Geom& g, char* kv, char* meta, int layer0, int nl, int n_total, hipStream_t s);
hipError_t launch_centroid_rebuild(const Geom& g, char* kv, char* meta, int layer, int n, hipStream_t s);

// Eq. 5 + anchor flags for the M slots [n_total-M, n_total), Eq. 6's smoothing of
// their scores when enabled, then (when n_total > B) Eq. 8's selection and the
// move list.
hipError_t launch_score_select(const Geom& g, const SmoothParams& sm, const HybridParams& hy, char* meta, int layer0, int nl, const void* resid,
                               const uint8_t* anchors, int n_total, hipStream_t s);

// Sec. 3.3: set or clear the protection flag of the resident tokens with ids in [gid_lo, gid_lo + M) whose mask
// byte is set (mask may be null: all).  launch_centroid_protect adjusts the hybrid-scoring sum for the same change
// and must run first (it reads the flags as they were).
hipError_t launch_centroid_protect(const Geom& g, char* kv, char* meta, int layer0, int nl, int n, uint32_t gid_lo,
                                   const uint8_t* mask, int on, hipStream_t s);
hipError_t launch_set_protect(const Geom& g, char* meta, int layer0, int nl, int n, uint32_t gid_lo,
                              const uint8_t* mask, int on, hipStream_t s);

// Apply the move list to K, V and the per-slot metadata.
hipError_t launch_compact(const Geom& g, char* kv, char* meta, int layer0, int nl, hipStream_t s);

}  // namespace ovggt
