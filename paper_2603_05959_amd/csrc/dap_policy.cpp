// Dynamic Anchor Protection, registration rule (paper Sec. 3.3): host-only bookkeeping of which
// frames are historical anchors and which of their patch tokens are protected.  The cache itself
// only honours per-token flags (ovggt_score_select's anchor bits, ovggt_cache_set_protect).
#include "../../include/ovggt.h"

#include <algorithm>
#include <cmath>
#include <deque>
#include <new>
#include <numeric>
#include <vector>

struct ovggt_dap {
  int32_t k_max, min_gap, n_special, n_patches;
  double tau, eta;
  int64_t last_reg = 0;          // frame 0, the global initial anchor, opens the spacing window
  int64_t last_t = -1;
  std::deque<int64_t> active;    // oldest first
};

extern "C" {

int ovggt_dap_create(ovggt_dap** out, int32_t k_max, int32_t min_gap, double tau, double eta,
                     int32_t n_special, int32_t n_patches) {
  if (!out) return OVGGT_ERR_ARG;
  if (k_max < 1 || min_gap < 1 || n_special < 0 || n_patches < 1) return OVGGT_ERR_ARG;
  if (!(eta > 0.0 && eta <= 1.0) || std::isnan(tau)) return OVGGT_ERR_ARG;
  ovggt_dap* d = new (std::nothrow) ovggt_dap();
  if (!d) return OVGGT_ERR_ARG;
  d->k_max = k_max; d->min_gap = min_gap; d->n_special = n_special; d->n_patches = n_patches;
  d->tau = tau; d->eta = eta;
  *out = d;
  return OVGGT_OK;
}

int ovggt_dap_step(ovggt_dap* d, int64_t t, double rho, const float* conf, int64_t* register_frame,
                   uint8_t* mask_out, int64_t* demote_frame) {
  if (!d || !register_frame || !demote_frame || t < 0 || t <= d->last_t) return OVGGT_ERR_ARG;
  *register_frame = -1;
  *demote_frame = -1;
  const bool wants = t > 0 && rho < d->tau && t - d->last_reg >= d->min_gap;
  if (wants && (!conf || !mask_out)) return OVGGT_ERR_ARG;      // nothing recorded: the call may be repeated
  d->last_t = t;
  if (!wants) return OVGGT_OK;
  // the ceil(eta * N_p) most confident patches; equal confidences go to the lower index
  const int n_keep = (int)std::ceil(d->eta * (double)d->n_patches);
  std::vector<int32_t> order((size_t)d->n_patches);
  std::iota(order.begin(), order.end(), 0);
  std::partial_sort(order.begin(), order.begin() + n_keep, order.end(), [conf](int32_t a, int32_t b) {
    return conf[a] > conf[b] || (conf[a] == conf[b] && a < b);
  });
  std::fill(mask_out, mask_out + d->n_special + d->n_patches, (uint8_t)0);
  for (int i = 0; i < n_keep; ++i) mask_out[d->n_special + order[(size_t)i]] = 1;
  if ((int32_t)d->active.size() == d->k_max) {
    *demote_frame = d->active.front();
    d->active.pop_front();
  }
  d->active.push_back(t);
  d->last_reg = t;
  *register_frame = t;
  return OVGGT_OK;
}

int ovggt_dap_active(const ovggt_dap* d, int64_t* frames, int32_t cap, int32_t* n) {
  if (!d || !n || cap < 0 || (cap > 0 && !frames)) return OVGGT_ERR_ARG;
  *n = (int32_t)d->active.size();
  for (int32_t i = 0; i < cap && i < *n; ++i) frames[i] = d->active[(size_t)i];
  return OVGGT_OK;
}

int ovggt_dap_destroy(ovggt_dap* d) {
  if (!d) return OVGGT_ERR_ARG;
  delete d;
  return OVGGT_OK;
}

}  // extern "C"
