// Host side of the C ABI declared in include/ovggt.h: argument validation, the
// per-layer call-order state machine, size arithmetic (the resident count of a
// layer is known on the host without reading the device: it grows by M per
// frame and is clipped to B by Eq. 8) and the kernel launches.
#include "../../include/ovggt.h"
#include "ovggt_internal.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

using namespace ovggt;

struct ovggt_cache {
  ovggt_config cfg;
  Geom g;
  char* kv;
  char* meta;
  char* ws;
  float scale;
  int n_wgs;                       // attention workgroups (1 per CU, 8 waves each)
  SmoothParams smooth;             // Eq. 6 parameters (alpha = 0: off)
  std::vector<int32_t> n;          // resident (incl. pending) slots per layer
  std::vector<int64_t> frames;     // completed frames per layer
  std::vector<int8_t> phase;       // 0: expects global_attn, 1: score_select, 2: compact
  std::vector<int8_t> pending;     // 1: the layer's last move list has not been applied yet (n == B); the next
                                   // append applies it, anything else that touches the cache flushes it first
  // optional kernel timing (ovggt_profile_*): event pairs per kernel class
  int prof_level = 0, prof_every = 1;
  int64_t prof_calls = 0;
  std::vector<hipEvent_t> prof_free;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_pending[OVGGT_PROF_CLASSES];
};

namespace {

// ---- host conversions between the bf16 interface and the half K/V storage ----
inline float bf16_bits_to_float(uint16_t b) { uint32_t u = (uint32_t)b << 16; float f; std::memcpy(&f, &u, 4); return f; }
inline uint16_t float_to_bf16_bits(float f) {
  uint32_t u; std::memcpy(&u, &f, 4);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
inline float half_bits_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h & 0x8000u) << 16, exp = (h >> 10) & 31u, man = h & 1023u;
  float f;
  if (exp == 0) f = std::ldexp((float)man, -24);
  else if (exp == 31) f = man ? NAN : INFINITY;
  else f = std::ldexp((float)(man | 1024u), (int)exp - 25);
  uint32_t u; std::memcpy(&u, &f, 4); u |= sign; std::memcpy(&f, &u, 4);
  return f;
}
// round-to-nearest-even float -> half, saturating at +-65504 like the append kernel
inline uint16_t float_to_half_bits_sat(float f) {
  if (f != f) return 0x7E00;
  uint16_t sign = std::signbit(f) ? 0x8000 : 0;
  float a = std::fabs(f);
  if (a > 65504.f) a = 65504.f;
  if (a < 5.9604645e-8f * 0.5f) return sign;                       // below half the smallest subnormal
  int e; (void)std::frexp(a, &e);                                   // a = m * 2^e, m in [0.5, 1)
  int shift = e - 1 < -14 ? -24 : e - 11;                           // exponent of one ulp
  const float q = std::ldexp(a, -shift);                            // in ulps
  float r = std::nearbyint(q);                                      // default rounding mode: nearest even
  float v = std::ldexp(r, shift);
  if (v >= 65520.f) v = 65504.f;
  if (v < 6.1035156e-5f) return (uint16_t)(sign | (uint16_t)std::lround(std::ldexp(v, 24)));
  int e2; const float m2 = std::frexp(v, &e2);                      // v = m2 * 2^e2
  const uint32_t man = (uint32_t)std::lround(std::ldexp(m2, 11)) - 1024u;
  return (uint16_t)(sign | (uint16_t)((e2 - 1 + 15) << 10) | (uint16_t)man);
}

inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

bool valid_config(const ovggt_config* c) {
  if (!c) return false;
  if (c->n_layers < 1 || c->n_layers > 4096) return false;
  if (c->n_heads < 1 || c->n_heads > 1024) return false;
  if (c->head_dim != 64) return false;
  if (c->tokens_per_frame < 1) return false;
  if (c->resid_dim < 1 || c->resid_dim > 4096) return false;
  if (c->budget < c->tokens_per_frame) return false;
  if ((int64_t)c->budget + c->tokens_per_frame > 128 * 1024) return false;   // selection handles <= 2^17 slots
  if (c->dtype != OVGGT_F32 && c->dtype != OVGGT_BF16) return false;
  if (c->score_mode != 0 && c->score_mode != 1) return false;
  if (c->score_mode == 1) {
    if (c->dtype != OVGGT_BF16 || c->n_heads > 64) return false;       // the key pass reads the half-precision cache
    if (!(c->hybrid_beta >= 0.f && c->hybrid_beta <= 1.f)) return false;
  }
  if (c->out_dtype != OVGGT_F32 && c->out_dtype != OVGGT_BF16) return false;
  if (c->dtype == OVGGT_F32 && c->out_dtype != OVGGT_F32) return false;
  if (!(c->softmax_scale >= 0.f) || !std::isfinite(c->softmax_scale)) return false;
  if (!(c->smooth_alpha >= 0.f && c->smooth_alpha <= 1.f)) return false;
  if (c->smooth_alpha > 0.f) {
    if (c->patch_h < 1 || c->patch_w < 1 || c->n_special < 0) return false;
    if ((int64_t)c->n_special + (int64_t)c->patch_h * c->patch_w != c->tokens_per_frame) return false;
    for (float w : c->smooth_kernel)
      if (!std::isfinite(w)) return false;
  }
  return true;
}

void make_geom(const ovggt_config& c, Geom* g) {
  g->L = c.n_layers; g->H = c.n_heads; g->d = c.head_dim; g->M = c.tokens_per_frame;
  g->C = c.resid_dim; g->B = c.budget;
  g->cap = (c.budget + c.tokens_per_frame + kSlotTile - 1) / kSlotTile * kSlotTile;
  g->esize = c.dtype == OVGGT_BF16 ? 2 : 4;
  g->kv_layer_bytes = up256((size_t)2 * g->H * g->cap * g->d * g->esize);
  size_t off = 0;
  g->off_ids = off;   off += up256((size_t)4 * g->cap);
  g->off_ss = off;    off += up256((size_t)4 * g->cap);
  g->off_flags = off; off += up256((size_t)g->cap);
  g->off_ctrl = off;  off += sizeof(Ctrl);
  g->off_mvdst = off; off += up256((size_t)4 * g->M);
  g->off_mvsrc = off; off += up256((size_t)4 * g->M);
  g->off_csum = off;  off += up256((size_t)8 * g->H * g->d);
  g->off_evbits = off; off += up256((size_t)g->cap / 8);
  g->off_cvec = off;  off += up256((size_t)4 * g->H * g->d);
  g->off_dval = off;  off += c.score_mode == 1 ? up256((size_t)4 * g->cap) : 0;
  g->off_dpart = off; off += c.score_mode == 1 ? up256((size_t)8 * kDivWavesPerWg * diversity_grid_x(g->cap, 1)) : 0;
  g->off_mvmap = off; off += up256((size_t)4 * g->M);
  g->off_hist = off;  off += up256((size_t)4 * kSelHistBins);
  g->hybrid = c.score_mode == 1 ? 1 : 0;
  g->meta_layer_bytes = off;
}

int query_blocks(const ovggt_config& c) { return (c.tokens_per_frame + kQueryTile - 1) / kQueryTile; }

// the larger of what a single-layer launch and an all-layers launch need
size_t ws_bytes_for(const ovggt_config& c) {
  if (c.dtype != OVGGT_BF16) return 256;
  const size_t one = attn_ws_bytes(c.n_heads, query_blocks(c)), all = attn_ws_bytes(c.n_layers * c.n_heads, query_blocks(c));
  return up256(one > all ? one : all);
}

bool aligned16(const void* p) { return p && ((uintptr_t)p & 15) == 0; }

// resolves `layer` to [l0, l0+nl); false if out of range
bool layer_range(const ovggt_cache* c, int layer, int* l0, int* nl) {
  if (layer == OVGGT_ALL_LAYERS) { *l0 = 0; *nl = c->g.L; return true; }
  if (layer < 0 || layer >= c->g.L) return false;
  *l0 = layer; *nl = 1;
  return true;
}

bool uniform(const ovggt_cache* c, int l0, int nl, int phase) {
  for (int l = l0; l < l0 + nl; ++l)
    if (c->phase[l] != phase || c->n[l] != c->n[l0] || c->frames[l] != c->frames[l0]) return false;
  return true;
}

hipEvent_t prof_event(ovggt_cache* c) {
  if (!c->prof_free.empty()) { hipEvent_t e = c->prof_free.back(); c->prof_free.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

// Returns every pending event to the free list (an event shared by two
// intervals is returned once).
void prof_recycle(ovggt_cache* c) {
  std::vector<hipEvent_t> seen;
  for (int k = 0; k < OVGGT_PROF_CLASSES; ++k) {
    for (auto& pr : c->prof_pending[k])
      for (hipEvent_t e : {pr.first, pr.second}) {
        bool dup = false;
        for (hipEvent_t x : seen) if (x == e) { dup = true; break; }
        if (!dup) seen.push_back(e);
      }
    c->prof_pending[k].clear();
  }
  for (hipEvent_t e : seen) c->prof_free.push_back(e);
}

// Brackets one launch with events when profiling asks for this kernel class.
struct ProfScope {
  ovggt_cache* c; int cls; hipStream_t s; hipEvent_t e0 = nullptr, e1 = nullptr;
  ProfScope(ovggt_cache* c_, int cls_, hipStream_t s_, bool on) : c(c_), cls(cls_), s(s_) {
    if (!on) return;
    e0 = prof_event(c); e1 = prof_event(c);
    if (e0 && e1) (void)hipEventRecord(e0, s); else e0 = e1 = nullptr;
  }
  ~ProfScope() {
    if (!e0) return;
    (void)hipEventRecord(e1, s);
    c->prof_pending[cls].push_back({e0, e1});
  }
};

// Applies the outstanding compactions of layers [l0, l0+nl) with the stand-alone kernel.
int flush_pending(ovggt_cache* c, int l0, int nl, hipStream_t s) {
  for (int l = l0; l < l0 + nl;) {
    if (!c->pending[l]) { ++l; continue; }
    int e = l;
    while (e < l0 + nl && c->pending[e]) ++e;
    ProfScope ps(c, OVGGT_PROF_COMPACT, s, c->prof_level >= 2);
    if (launch_compact(c->g, c->kv, c->meta, l, e - l, s) != hipSuccess) return OVGGT_ERR_HIP;
    for (; l < e; ++l) c->pending[l] = 0;
  }
  return OVGGT_OK;
}

inline Ctrl* ctrl_of(const ovggt_cache* c, int layer) {
  return (Ctrl*)(layer_meta(c->meta, c->g, layer) + c->g.off_ctrl);
}

}  // namespace

extern "C" {

int ovggt_cache_query_bytes(const ovggt_config* cfg, size_t* kv_bytes, size_t* meta_bytes, size_t* ws_bytes) {
  if (!valid_config(cfg)) return OVGGT_ERR_ARG;
  Geom g;
  make_geom(*cfg, &g);
  if (kv_bytes) *kv_bytes = g.kv_layer_bytes * g.L;
  if (meta_bytes) *meta_bytes = g.meta_layer_bytes * g.L;
  if (ws_bytes) *ws_bytes = ws_bytes_for(*cfg);
  return OVGGT_OK;
}

int ovggt_cache_init(ovggt_cache** out, const ovggt_config* cfg, void* kv_dev, void* meta_dev,
                     void* ws_dev, void* hip_stream) {
  if (!out || !valid_config(cfg)) return OVGGT_ERR_ARG;
  if (!kv_dev || !meta_dev || !ws_dev) return OVGGT_ERR_ARG;
  if (((uintptr_t)kv_dev | (uintptr_t)meta_dev | (uintptr_t)ws_dev) & 255) return OVGGT_ERR_ARG;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return OVGGT_ERR_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return OVGGT_ERR_HIP;
  ovggt_cache* c = new (std::nothrow) ovggt_cache();
  if (!c) return OVGGT_ERR_NOMEM;
  c->cfg = *cfg;
  make_geom(*cfg, &c->g);
  c->smooth.alpha = cfg->smooth_alpha;
  c->smooth.ph = cfg->patch_h; c->smooth.pw = cfg->patch_w; c->smooth.n_special = cfg->n_special;
  for (int i = 0; i < 9; ++i) c->smooth.g[i] = cfg->smooth_kernel[i];
  c->kv = (char*)kv_dev; c->meta = (char*)meta_dev; c->ws = (char*)ws_dev;
  c->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  int wgs = cus;
  wgs = (wgs + 7) & ~7;
  if (wgs < 8) wgs = 8;
  if (wgs > kMaxAttnWgs) wgs = kMaxAttnWgs;
  c->n_wgs = wgs;
  c->n.assign(c->g.L, 0);
  c->frames.assign(c->g.L, 0);
  c->phase.assign(c->g.L, 0);
  c->pending.assign(c->g.L, 0);
  hipStream_t s = (hipStream_t)hip_stream;
  if (launch_fill_zero(c->kv, c->g.kv_layer_bytes * c->g.L, s) != hipSuccess ||
      launch_fill_zero(c->meta, c->g.meta_layer_bytes * c->g.L, s) != hipSuccess ||
      launch_fill_zero(c->ws, ws_bytes_for(*cfg), s) != hipSuccess) {
    delete c;
    return OVGGT_ERR_HIP;
  }
  *out = c;
  return OVGGT_OK;
}

// ovggt_global_attn, with the attention's partial records in the handle's workspace (static_ws =
// false) or in the library's own device array.
static int global_attn_impl(ovggt_cache* c, int layer, const void* q, const void* k_new, const void* v_new,
                            void* out, void* hip_stream, bool static_ws) {
  if (!c) return OVGGT_ERR_ARG;
  int l0, nl;
  if (!layer_range(c, layer, &l0, &nl)) return OVGGT_ERR_ARG;
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out)) return OVGGT_ERR_ARG;
  if (!uniform(c, l0, nl, 0)) return OVGGT_ERR_STATE;
  const Geom& g = c->g;
  char* ws = c->ws;
  size_t ws_bytes = ws_bytes_for(c->cfg);
  if (static_ws && g.esize == 2) {
    if (attn_static_ws(&ws, &ws_bytes) != hipSuccess) return OVGGT_ERR_HIP;
    if (attn_ws_bytes(nl * g.H, query_blocks(c->cfg)) > ws_bytes) return OVGGT_ERR_TOO_LARGE;   // before anything is launched
  }
  const int n = c->n[l0];
  const int64_t gid0 = c->frames[l0] * (int64_t)g.M;
  if (gid0 + g.M > 0xFFFFFFFFLL) return OVGGT_ERR_ARG;          // token ids are 32-bit
  if (n + g.M > g.cap) return OVGGT_ERR_STATE;
  hipStream_t s = (hipStream_t)hip_stream;
  const bool prof_attn = c->prof_level >= 1 && (c->prof_calls++ % c->prof_every) == 0;
  const bool prof_all = c->prof_level >= 2;
  // an outstanding compaction rides along with the append when every layer of the call has one
  bool all_pending = true, any_pending = false;
  for (int l = l0; l < l0 + nl; ++l) { all_pending = all_pending && c->pending[l]; any_pending = any_pending || c->pending[l]; }
  if (any_pending && !all_pending) {
    if (flush_pending(c, l0, nl, s) != OVGGT_OK) return OVGGT_ERR_HIP;
    all_pending = false;
  }
  {
    ProfScope ps(c, OVGGT_PROF_APPEND, s, prof_all);
    if (launch_append(g, c->kv, c->meta, l0, nl, k_new, v_new, n, all_pending, s) != hipSuccess)
      return OVGGT_ERR_HIP;
  }
  for (int l = l0; l < l0 + nl; ++l) c->pending[l] = 0;
  hipError_t e;
  if (g.esize == 2) {
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    bool have = false;
    if (prof_attn) {
      for (auto& x : ev) x = prof_event(c);
      have = ev[0] && ev[1] && ev[2];
      if (!have)                                       // out of events: this call goes untimed
        for (hipEvent_t x : ev)
          if (x) c->prof_free.push_back(x);
    }
    e = launch_attn_bf16(g, c->kv, l0, nl, q, out, n + g.M, c->scale, ws, ws_bytes, c->n_wgs,
                         c->cfg.out_dtype == OVGGT_F32, s, have ? ev : nullptr);
    if (have) {
      c->prof_pending[OVGGT_PROF_ATTN].push_back({ev[0], ev[1]});
      c->prof_pending[OVGGT_PROF_COMBINE].push_back({ev[1], ev[2]});   // shares ev[1] as its start
    }
  } else {
    ProfScope ps(c, OVGGT_PROF_ATTN, s, prof_attn);
    e = launch_attn_f32(g, c->kv, l0, nl, q, out, n + g.M, c->scale, s);
  }
  if (e != hipSuccess) return OVGGT_ERR_HIP;
  for (int l = l0; l < l0 + nl; ++l) { c->n[l] = n + g.M; c->phase[l] = 1; }
  return OVGGT_OK;
}

int ovggt_global_attn(ovggt_cache* c, int layer, const void* q, const void* k_new, const void* v_new,
                      void* out, void* hip_stream) {
  return global_attn_impl(c, layer, q, k_new, v_new, out, hip_stream, false);
}

int ovggt_global_attn_static_ws(ovggt_cache* c, int layer, const void* q, const void* k_new, const void* v_new,
                                void* out, void* hip_stream) {
  return global_attn_impl(c, layer, q, k_new, v_new, out, hip_stream, true);
}

int ovggt_score_select(ovggt_cache* c, int layer, const void* resid, const uint8_t* anchor_flags,
                       void* hip_stream) {
  if (!c) return OVGGT_ERR_ARG;
  int l0, nl;
  if (!layer_range(c, layer, &l0, &nl)) return OVGGT_ERR_ARG;
  if (!aligned16(resid)) return OVGGT_ERR_ARG;
  if (!uniform(c, l0, nl, 1)) return OVGGT_ERR_STATE;
  {
    ProfScope ps(c, OVGGT_PROF_SELECT, (hipStream_t)hip_stream, c->prof_level >= 2);
    const HybridParams hy = {c->cfg.score_mode == 1 ? 1 : 0, c->cfg.hybrid_beta,
                             kDivWavesPerWg * diversity_grid_x(c->n[l0] - c->g.M, nl)};
    if (hy.on && c->n[l0] > c->g.B &&
        launch_diversity(c->g, c->kv, c->meta, l0, nl, c->n[l0] - c->g.M, (hipStream_t)hip_stream) != hipSuccess)
      return OVGGT_ERR_HIP;
    if (launch_score_select(c->g, c->smooth, hy, c->meta, l0, nl, resid, anchor_flags, c->n[l0], (hipStream_t)hip_stream) != hipSuccess)
      return OVGGT_ERR_HIP;
    if (hy.on && launch_centroid_update(c->g, c->kv, c->meta, l0, nl, c->n[l0], (hipStream_t)hip_stream) != hipSuccess)
      return OVGGT_ERR_HIP;
  }
  for (int l = l0; l < l0 + nl; ++l) c->phase[l] = 2;
  return OVGGT_OK;
}

int ovggt_cache_compact(ovggt_cache* c, int layer, void* hip_stream) {
  if (!c) return OVGGT_ERR_ARG;
  int l0, nl;
  if (!layer_range(c, layer, &l0, &nl)) return OVGGT_ERR_ARG;
  if (!uniform(c, l0, nl, 2)) return OVGGT_ERR_STATE;
  const Geom& g = c->g;
  // The move list is applied by the next frame's append (same pass over the same slots), or by the
  // stand-alone kernel as soon as anything else reads or changes the cache.
  for (int l = l0; l < l0 + nl; ++l) {
    if (c->n[l] > g.B) { c->n[l] = g.B; c->pending[l] = 1; }
    c->frames[l] += 1;
    c->phase[l] = 0;
  }
  return OVGGT_OK;
}

int ovggt_cache_advance(ovggt_cache* c, int layer, int64_t frames) {
  if (!c || frames < 1) return OVGGT_ERR_ARG;
  int l0, nl;
  if (!layer_range(c, layer, &l0, &nl)) return OVGGT_ERR_ARG;
  const Geom& g = c->g;
  // a replayed step is the steady-state step: full cache, the last selection's moves outstanding
  for (int l = l0; l < l0 + nl; ++l)
    if (c->phase[l] != 0 || c->n[l] != g.B || !c->pending[l]) return OVGGT_ERR_STATE;
  for (int l = l0; l < l0 + nl; ++l)
    if ((c->frames[l] + frames) * (int64_t)g.M > 0xFFFFFFFFLL) return OVGGT_ERR_ARG;   // token ids are 32-bit
  for (int l = l0; l < l0 + nl; ++l) c->frames[l] += frames;
  return OVGGT_OK;
}

int ovggt_cache_flush(ovggt_cache* c, int layer, void* hip_stream) {
  if (!c) return OVGGT_ERR_ARG;
  int l0, nl;
  if (!layer_range(c, layer, &l0, &nl)) return OVGGT_ERR_ARG;
  return flush_pending(c, l0, nl, (hipStream_t)hip_stream);
}

int ovggt_cache_set_protect(ovggt_cache* c, int layer, int64_t frame, const uint8_t* mask, int on,
                            void* hip_stream) {
  if (!c) return OVGGT_ERR_ARG;
  int l0, nl;
  if (!layer_range(c, layer, &l0, &nl)) return OVGGT_ERR_ARG;
  if (!uniform(c, l0, nl, 0)) return OVGGT_ERR_STATE;
  if (frame < 0 || frame >= c->frames[l0]) return OVGGT_ERR_ARG;
  const Geom& g = c->g;
  const uint32_t gid_lo = (uint32_t)(frame * (int64_t)g.M);          // fits: the frame has been appended
  hipStream_t s = (hipStream_t)hip_stream;
  if (flush_pending(c, l0, nl, s) != OVGGT_OK) return OVGGT_ERR_HIP;
  if (g.hybrid && launch_centroid_protect(g, c->kv, c->meta, l0, nl, c->n[l0], gid_lo, mask, on, s) != hipSuccess)
    return OVGGT_ERR_HIP;
  if (launch_set_protect(g, c->meta, l0, nl, c->n[l0], gid_lo, mask, on, s) != hipSuccess) return OVGGT_ERR_HIP;
  return OVGGT_OK;
}

int ovggt_cache_destroy(ovggt_cache* c) {
  if (!c) return OVGGT_ERR_ARG;
  prof_recycle(c);
  for (hipEvent_t e : c->prof_free) (void)hipEventDestroy(e);
  delete c;
  return OVGGT_OK;
}

int ovggt_cache_size(const ovggt_cache* c, int layer, int32_t* n) {
  if (!c || !n || layer < 0 || layer >= c->g.L) return OVGGT_ERR_ARG;
  *n = c->n[layer];
  return OVGGT_OK;
}

int ovggt_cache_frames(const ovggt_cache* c, int layer, int64_t* t) {
  if (!c || !t || layer < 0 || layer >= c->g.L) return OVGGT_ERR_ARG;
  *t = c->frames[layer];
  return OVGGT_OK;
}

int ovggt_cache_status(ovggt_cache* c, int layer, int32_t* status, void* hip_stream) {
  if (!c || !status || layer < 0 || layer >= c->g.L) return OVGGT_ERR_ARG;
  if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return OVGGT_ERR_HIP;
  uint32_t st = 0, zero = 0;
  Ctrl* ctrl = ctrl_of(c, layer);
  if (hipMemcpy(&st, &ctrl->status, 4, hipMemcpyDeviceToHost) != hipSuccess) return OVGGT_ERR_HIP;
  if (hipMemcpy(&ctrl->status, &zero, 4, hipMemcpyHostToDevice) != hipSuccess) return OVGGT_ERR_HIP;
  *status = (int32_t)st;
  return OVGGT_OK;
}

int ovggt_cache_export(ovggt_cache* c, int layer, uint32_t* ids, void* k, void* v, float* ss,
                       uint8_t* flags, void* hip_stream) {
  if (!c || layer < 0 || layer >= c->g.L) return OVGGT_ERR_ARG;
  if (flush_pending(c, layer, 1, (hipStream_t)hip_stream) != OVGGT_OK) return OVGGT_ERR_HIP;
  if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return OVGGT_ERR_HIP;
  const Geom& g = c->g;
  const int n = c->n[layer];
  if (n == 0) return OVGGT_OK;
  char* mb = layer_meta(c->meta, g, layer);
  if (ids && hipMemcpy(ids, mb + g.off_ids, (size_t)4 * n, hipMemcpyDeviceToHost) != hipSuccess) return OVGGT_ERR_HIP;
  if (ss && hipMemcpy(ss, mb + g.off_ss, (size_t)4 * n, hipMemcpyDeviceToHost) != hipSuccess) return OVGGT_ERR_HIP;
  if (flags && hipMemcpy(flags, mb + g.off_flags, (size_t)n, hipMemcpyDeviceToHost) != hipSuccess) return OVGGT_ERR_HIP;
  const size_t row = (size_t)g.d * g.esize;
  std::vector<char> tmp;
  for (int which = 0; which < 2; ++which) {
    char* dst = (char*)(which ? v : k);
    if (!dst) continue;
    const char* src = which ? layer_v(c->kv, g, layer) : layer_k(c->kv, g, layer);
    tmp.resize((size_t)n * row);
    for (int h = 0; h < g.H; ++h) {
      if (hipMemcpy(tmp.data(), src + (size_t)h * g.cap * row, (size_t)n * row, hipMemcpyDeviceToHost) != hipSuccess)
        return OVGGT_ERR_HIP;
      if (g.esize == 2) {                      // K and V are stored as half: hand them back as bf16
        uint16_t* t16 = (uint16_t*)tmp.data();
        for (size_t j = 0; j < (size_t)n * g.d; ++j) t16[j] = float_to_bf16_bits(half_bits_to_float(t16[j]));
      }
      for (int i = 0; i < n; ++i) std::memcpy(dst + ((size_t)i * g.H + h) * row, tmp.data() + (size_t)i * row, row);
    }
  }
  return OVGGT_OK;
}

int ovggt_cache_import(ovggt_cache* c, int layer, int32_t n, int64_t frames, const uint32_t* ids,
                       const void* k, const void* v, const float* ss, const uint8_t* flags,
                       void* hip_stream) {
  if (!c || layer < 0 || layer >= c->g.L) return OVGGT_ERR_ARG;
  const Geom& g = c->g;
  if (n < 0 || n > g.B || frames < 0 || (n > 0 && (!ids || !k || !v || !ss || !flags))) return OVGGT_ERR_ARG;
  if ((frames + 1) * (int64_t)g.M > 0xFFFFFFFFLL) return OVGGT_ERR_ARG;
  if (c->phase[layer] != 0) return OVGGT_ERR_STATE;
  if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return OVGGT_ERR_HIP;
  c->pending[layer] = 0;                               // the contents it would have rearranged are replaced
  char* mb = layer_meta(c->meta, g, layer);
  if (n > 0) {
    if (hipMemcpy(mb + g.off_ids, ids, (size_t)4 * n, hipMemcpyHostToDevice) != hipSuccess) return OVGGT_ERR_HIP;
    if (hipMemcpy(mb + g.off_ss, ss, (size_t)4 * n, hipMemcpyHostToDevice) != hipSuccess) return OVGGT_ERR_HIP;
    if (hipMemcpy(mb + g.off_flags, flags, (size_t)n, hipMemcpyHostToDevice) != hipSuccess) return OVGGT_ERR_HIP;
    const size_t row = (size_t)g.d * g.esize;
    std::vector<char> tmp((size_t)n * row);
    for (int which = 0; which < 2; ++which) {
      const char* src = (const char*)(which ? v : k);
      char* dst = which ? layer_v(c->kv, g, layer) : layer_k(c->kv, g, layer);
      for (int h = 0; h < g.H; ++h) {
        for (int i = 0; i < n; ++i) std::memcpy(tmp.data() + (size_t)i * row, src + ((size_t)i * g.H + h) * row, row);
        if (g.esize == 2) {                    // bf16 in, half stored
          uint16_t* t16 = (uint16_t*)tmp.data();
          for (size_t j = 0; j < (size_t)n * g.d; ++j) t16[j] = float_to_half_bits_sat(bf16_bits_to_float(t16[j]));
        }
        if (hipMemcpy(dst + (size_t)h * g.cap * row, tmp.data(), (size_t)n * row, hipMemcpyHostToDevice) != hipSuccess)
          return OVGGT_ERR_HIP;
      }
    }
  }
  if (c->cfg.score_mode == 1) {
    if (launch_centroid_rebuild(g, c->kv, c->meta, layer, n, (hipStream_t)hip_stream) != hipSuccess) return OVGGT_ERR_HIP;
    if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return OVGGT_ERR_HIP;
  }
  const uint32_t gid_next = (uint32_t)(frames * (int64_t)g.M);
  if (hipMemcpy(&ctrl_of(c, layer)->gid_next, &gid_next, 4, hipMemcpyHostToDevice) != hipSuccess) return OVGGT_ERR_HIP;
  c->n[layer] = n;
  c->frames[layer] = frames;
  return OVGGT_OK;
}

int ovggt_cache_last_moves(ovggt_cache* c, int layer, uint32_t* dst, uint32_t* src, int32_t* n_moves,
                           void* hip_stream) {
  if (!c || !n_moves || layer < 0 || layer >= c->g.L) return OVGGT_ERR_ARG;
  if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return OVGGT_ERR_HIP;
  const Geom& g = c->g;
  char* mb = layer_meta(c->meta, g, layer);
  uint32_t nm = 0;
  if (hipMemcpy(&nm, &ctrl_of(c, layer)->n_moves, 4, hipMemcpyDeviceToHost) != hipSuccess) return OVGGT_ERR_HIP;
  if (nm > (uint32_t)g.M) nm = (uint32_t)g.M;
  if (dst && nm && hipMemcpy(dst, mb + g.off_mvdst, (size_t)4 * nm, hipMemcpyDeviceToHost) != hipSuccess) return OVGGT_ERR_HIP;
  if (src && nm && hipMemcpy(src, mb + g.off_mvsrc, (size_t)4 * nm, hipMemcpyDeviceToHost) != hipSuccess) return OVGGT_ERR_HIP;
  *n_moves = (int32_t)nm;
  return OVGGT_OK;
}

int ovggt_profile_enable(ovggt_cache* c, int level, int every) {
  if (!c || level < 0 || level > 2 || every < 1) return OVGGT_ERR_ARG;
  c->prof_level = level;
  c->prof_every = every;
  c->prof_calls = 0;
  return OVGGT_OK;
}

int ovggt_profile_read(ovggt_cache* c, double* ms_sum, int64_t* count, void* hip_stream) {
  if (!c || !ms_sum || !count) return OVGGT_ERR_ARG;
  if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess) return OVGGT_ERR_HIP;
  for (int k = 0; k < OVGGT_PROF_CLASSES; ++k) {
    ms_sum[k] = 0.0; count[k] = 0;
    for (auto& pr : c->prof_pending[k]) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, pr.first, pr.second) != hipSuccess) return OVGGT_ERR_HIP;
      ms_sum[k] += ms; count[k] += 1;
    }
  }
  prof_recycle(c);
  return OVGGT_OK;
}

int ovggt_profile_overhead(ovggt_cache* c, int reps, double* ms_mean, void* hip_stream) {
  if (!c || !ms_mean || reps < 1 || reps > 1024) return OVGGT_ERR_ARG;
  hipStream_t s = (hipStream_t)hip_stream;
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0)
    return OVGGT_ERR_HIP;
  const double spin_ms = 0.1;                          // as long as the kernels the brackets are used on
  const unsigned long long ticks = (unsigned long long)(spin_ms * khz + 0.5);
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev;
  bool failed = false;
  for (int i = 0; i < reps; ++i) {
    hipEvent_t e0 = prof_event(c), e1 = prof_event(c);
    bool ok = e0 && e1;
    // the same bracket as around a timed kernel, around a kernel whose own duration is known
    ok = ok && hipEventRecord(e0, s) == hipSuccess && launch_spin(ticks, s) == hipSuccess &&
         hipEventRecord(e1, s) == hipSuccess;
    if (e0) ev.push_back({e0, e1});                  // returned to the free list below, also after a failure
    else if (e1) c->prof_free.push_back(e1);
    if (!ok) { failed = true; break; }
  }
  if (hipStreamSynchronize(s) != hipSuccess) failed = true;
  double sum = 0.0;
  for (auto& pr : ev) {
    float ms = 0.f;
    if (!failed && hipEventElapsedTime(&ms, pr.first, pr.second) != hipSuccess) failed = true;
    sum += ms;
    c->prof_free.push_back(pr.first);
    if (pr.second) c->prof_free.push_back(pr.second);
  }
  if (failed) return OVGGT_ERR_HIP;
  *ms_mean = sum / reps - spin_ms;
  return OVGGT_OK;
}

int ovggt_attn_plan_stats(const ovggt_config* cfg, int32_t layers_in_launch, int32_t n_total, int32_t n_wgs,
                          int32_t* out, float* cost) {
  if (!valid_config(cfg) || !out || !cost || cfg->dtype != OVGGT_BF16) return OVGGT_ERR_ARG;
  if (layers_in_launch != 1 && layers_in_launch != cfg->n_layers) return OVGGT_ERR_ARG;
  if (n_total < 1 || n_total > cfg->budget + cfg->tokens_per_frame || n_wgs < 1) return OVGGT_ERR_ARG;
  Geom g;
  make_geom(*cfg, &g);
  AttnPlanStats st;
  if (!attn_plan_stats(g, layers_in_launch, n_total, n_wgs, ws_bytes_for(*cfg), &st)) return OVGGT_ERR_STATE;
  out[0] = st.n_wgs; out[1] = st.rounds; out[2] = st.segments; out[3] = st.balanced; out[4] = st.pieces_max;
  out[5] = st.tiles_min; out[6] = st.tiles_max; out[7] = st.shared_items;
  cost[0] = st.cost_max; cost[1] = st.cost_mean;
  return OVGGT_OK;
}

const char* ovggt_strerror(int code) {
  switch (code) {
    case OVGGT_OK: return "ok";
    case OVGGT_ERR_ARG: return "invalid argument";
    case OVGGT_ERR_STATE: return "call out of order for this layer";
    case OVGGT_ERR_NOMEM: return "out of host memory";
    case OVGGT_ERR_HIP: return "HIP runtime error";
    case OVGGT_ERR_TOO_LARGE: return "launch too large for the library's static workspace";
    default: return "unknown error";
  }
}

}  // extern "C"
