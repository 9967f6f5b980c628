// Diversity scores of the cached history (paper Eq. 7, first case): d_i = 1 - cos(k_i, kbar),
// where k_i is a token's key over all heads and kbar the centroid of the evictable history.
//
// The centroid is kept as a running sum of the evictable resident keys.  Every half is an integer
// multiple of 2^-24, so the sum is a 64-bit integer in those units: exact, independent of the
// order in which workgroups and atomics add their parts, and therefore something that can be
// maintained frame by frame (add the tokens that stay, subtract the entries that leave: O(M) rows)
// instead of re-read from the whole cache (O(B) rows).
//   centroid_update_kernel   the per-frame maintenance, after the selection
//   centroid_rebuild_kernel  the same sum from nothing, after a cache import
//   diversity_kernel  the HBM-bound pass over the layer's K cache: dot(k_i, c), |k_i|^2 and |c|^2 as
//                     fp32 balanced trees over the concatenated index h*d + e, then
//                     d_i = 1 - dot / (sqrt(|k_i|^2) * sqrt(|c|^2)), written to the layer's d_i array.
// The selection kernel min-max normalises these and blends them with the new frame's scores.
#include "ovggt_internal.h"
#include "../../include/ovggt.h"
#include <hip/hip_fp16.h>

namespace ovggt {

constexpr int kCenThreads = 256;
constexpr int kCenUnroll = 8;                 // 16-byte loads a thread keeps in flight
constexpr int kCenMaxAdds = 64;               // 64 * 2^24 < 2^31
constexpr int kDivThreads = 256;
constexpr int kDivWaves = kDivThreads / 64;

__device__ inline void unpack_halfs(const uint4& w, float f[8]) {
  const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const __half2 h = *(const __half2*)&ww[t];
    f[2 * t] = __low2float(h);
    f[2 * t + 1] = __high2float(h);
  }
}

// ---- exact centroid sum -------------------------------------------------------------------------
// A thread owns 8 consecutive elements of one head (a 16-byte piece of a slot's 128-byte row);
// 8*H threads cover a key, kCenThreads / (8*H) keys are read side by side, and kCenUnroll loads per
// thread are in flight before any is consumed.  `row(v, &slot)` names the cache slot of the
// workgroup's v-th row and returns +1 (add), -1 (subtract) or 0 (skip); each workgroup ends with
// one 64-bit atomic per key element it changed.
template <typename RowFn>
__device__ inline void accumulate_rows(const Geom& g, const char* K, unsigned long long* csum,
                                       int v0, int v1, RowFn row) {
  __shared__ long long part[kCenThreads][8];
  const int pieces = g.H * 8;                         // 16-byte pieces per key
  for (int p0 = 0; p0 < pieces; p0 += kCenThreads) {  // one trip unless the key is wider than 32 heads
    const int lanes = min(pieces - p0, kCenThreads);  // threads that hold a piece in this trip
    const int side = kCenThreads / lanes;             // keys read side by side
    const int piece = p0 + (int)threadIdx.x % lanes, sl = (int)threadIdx.x / lanes;
    const int h = piece >> 3, cg = piece & 7;
    const char* Kp = K + (size_t)h * g.cap * 128 + cg * 16;
    // value * 2^24 = hi * 2^16 + lo with |hi| < 2^24 and |lo| < 2^16; a thread adds at most
    // kCenMaxAdds of them into the 32-bit sums before they are widened
    int hi[8], lo[8];
    long long acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { hi[j] = 0; lo[j] = 0; acc[j] = 0; }
    int adds = 0;
    if (sl < side) {
      for (int base = v0 + sl; base < v1; base += side * kCenUnroll) {
        uint4 w[kCenUnroll];
        int sign[kCenUnroll];
#pragma unroll
        for (int u = 0; u < kCenUnroll; ++u) {
          const int v = base + u * side;
          int slot = 0;
          sign[u] = v < v1 ? row(v, &slot) : 0;
          w[u] = *(const uint4*)(Kp + (size_t)slot * 128);       // slot 0 when the row is skipped: in bounds
        }
#pragma unroll
        for (int u = 0; u < kCenUnroll; ++u) {
          if (sign[u] == 0) continue;
          float f[8];
          unpack_halfs(w[u], f);
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float a = f[j] * 256.0f;            // exact
            const int ih = (int)a;                    // towards zero
            const float rem = a - (float)ih;          // exact, |rem| < 1, a multiple of 2^-16
            hi[j] += sign[u] * ih;
            lo[j] += sign[u] * (int)(rem * 65536.0f);
          }
        }
        adds += kCenUnroll;
        if (adds + kCenUnroll > kCenMaxAdds) {
#pragma unroll
          for (int j = 0; j < 8; ++j) { acc[j] += (long long)hi[j] * 65536 + (long long)lo[j]; hi[j] = 0; lo[j] = 0; }
          adds = 0;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) part[threadIdx.x][j] = acc[j] + (long long)hi[j] * 65536 + (long long)lo[j];
    __syncthreads();
    // element e of the trip's pieces: sum over the keys read side by side, one atomic per element
    for (int e = threadIdx.x; e < lanes * 8; e += kCenThreads) {
      long long t = 0;
      for (int r = 0; r < side; ++r) t += part[r * lanes + (e >> 3)][e & 7];
      if (t != 0) atomicAdd(&csum[(size_t)p0 * 8 + e], (unsigned long long)t);
    }
    __syncthreads();
  }
}

// Sum of all evictable entries among slots [0, n): builds the centroid sum from nothing (after an
// import).  grid (chunks, 1); the sums must be zero on entry.
__global__ void __launch_bounds__(kCenThreads)
centroid_rebuild_kernel(Geom g, char* kv, char* meta, int layer, int n, int chunk) {
  char* mb = layer_meta(meta, g, layer);
  const uint8_t* flags = (const uint8_t*)(mb + g.off_flags);
  const int v0 = blockIdx.x * chunk, v1 = min(v0 + chunk, n);
  accumulate_rows(g, layer_k(kv, g, layer), (unsigned long long*)(mb + g.off_csum), v0, v1,
                  [&](int v, int* slot) { *slot = v; return flags[v] ? 0 : 1; });
}

// After a frame's selection: the sum gains the frame's evictable tokens that stay and loses the
// evicted entries of earlier frames, so that it again covers every evictable resident entry.
// Rows [0, M) are the frame's slots n_old + v; rows [M, 2M) walk the hole list (slots below B whose
// entry was evicted), of which the ones below n_old held earlier frames' entries.  grid (chunks, layers).
__global__ void __launch_bounds__(kCenThreads)
centroid_update_kernel(Geom g, char* kv, char* meta, int layer0, int n_total, int chunk) {
  const int layer = layer0 + blockIdx.y;
  char* mb = layer_meta(meta, g, layer);
  const uint8_t* flags = (const uint8_t*)(mb + g.off_flags);
  const uint32_t* evbits = (const uint32_t*)(mb + g.off_evbits);
  const uint32_t* holes = (const uint32_t*)(mb + g.off_mvdst);
  const int n_old = n_total - g.M;
  const bool evicting = n_total > g.B;
  const int n_holes = evicting ? (int)min(((const Ctrl*)(mb + g.off_ctrl))->n_moves, (uint32_t)g.M) : 0;
  const int v0 = blockIdx.x * chunk, v1 = min(v0 + chunk, 2 * g.M);
  accumulate_rows(g, layer_k(kv, g, layer), (unsigned long long*)(mb + g.off_csum), v0, v1,
                  [&](int v, int* slot) {
                    if (v < g.M) {
                      const int s = n_old + v;
                      if (flags[s]) return 0;
                      if (evicting && ((evbits[s >> 5] >> (s & 31)) & 1u)) return 0;
                      *slot = s;
                      return 1;
                    }
                    const int j = v - g.M;
                    if (j >= n_holes) return 0;
                    const int s = (int)holes[j];
                    if (s >= n_old) return 0;          // a token of this frame: never entered the sum
                    *slot = s;
                    return -1;
                  });
}

// ---- pass 2: d_i per history slot ----------------------------------------------------------------
// A wave takes 8 consecutive slots.  For every head one load instruction fetches the 8 slots' rows,
// 1 KiB of consecutive memory (the cache is head-major: a slot's key is H rows 2 MB apart, and
// pieces shorter than this made the pass latency- rather than bandwidth-bound): lane l holds the
// 16-byte piece l & 7 of slot l >> 3.  The balanced tree over the concatenated index h*64 + e
// (zero-padded to a power of two) is evaluated as: a pairwise tree over the lane's 8 elements, three
// butterfly steps over the 8 lanes of a slot (quad permutes and the half-row mirror: after each
// step all lanes of a group hold the group's sum, so any lane of the sibling group is a valid
// partner), and a tree over the heads folded in as they arrive (a binary counter of partial sums).
__device__ inline float dpp_f(float v, int ctrl_is) {
  // ctrl_is: 0 quad [1,0,3,2], 1 quad [2,3,0,1], 2 row half mirror
  const int x = __float_as_int(v);
  int y;
  switch (ctrl_is) {
    case 0: y = __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false); break;
    case 1: y = __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false); break;
    default: y = __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, false); break;
  }
  return __int_as_float(y);
}
__device__ inline float tree8_lanes8(const float (&p)[8]) {
  float v = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
  v = v + dpp_f(v, 0);
  v = v + dpp_f(v, 1);
  v = v + dpp_f(v, 2);
  return v;
}
constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

// dot(k, c) and |k|^2 of the 8 slots of a wave; key_of(h, k8) delivers the lane's 8 elements of head h
// (h < H).  cs: the centroid in LDS, H*64 floats.  Every lane of a slot's group returns the slot's sums.
template <int HP, typename KeyOf>
__device__ inline void slot_sums(const float* cs, int piece, int H, KeyOf key_of, float* dot, float* nk) {
#pragma clang fp contract(off)
  constexpr int LV = ilog2(HP);
  float sd[LV + 1], sn[LV + 1];
  float vd = 0.f, vn = 0.f;
#pragma unroll
  for (int h = 0; h < HP; ++h) {
    vd = 0.f; vn = 0.f;                                // heads beyond H are the tree's zero padding
    if (h < H) {
      float k8[8];
      key_of(h, k8);
      const float4 c0 = *(const float4*)(cs + h * 64 + piece * 8), c1 = *(const float4*)(cs + h * 64 + piece * 8 + 4);
      const float cc[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
      float p[8], q[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) { p[i] = k8[i] * cc[i]; q[i] = k8[i] * k8[i]; }
      vd = tree8_lanes8(p);
      vn = tree8_lanes8(q);
    }
#pragma unroll
    for (int lvl = 0; lvl < LV; ++lvl) {
      if ((h >> lvl) & 1) { vd = sd[lvl] + vd; vn = sn[lvl] + vn; }
      else { sd[lvl] = vd; sn[lvl] = vn; break; }
    }
  }
  *dot = vd; *nk = vn;
}

constexpr int kDivHeadBatch = 16;              // head rows of a round requested together (64 registers)

template <int HP>
__global__ void __launch_bounds__(kDivThreads)
diversity_kernel(Geom g, char* kv, char* meta, int layer0, int n_hist) {
#pragma clang fp contract(off)
  __shared__ float cs[HP * 64];
  const int layer = layer0 + blockIdx.y;
  char* mb = layer_meta(meta, g, layer);
  const uint8_t* flags = (const uint8_t*)(mb + g.off_flags);
  const float* cvec = (const float*)(mb + g.off_cvec);   // the fp32 centroid the frame's append left
  float* dval = (float*)(mb + g.off_dval);
  const char* K = layer_k(kv, g, layer);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sl = lane >> 3, piece = lane & 7;
  const int H = g.H;
  for (int i = threadIdx.x; i < H * 64; i += kDivThreads) cs[i] = cvec[i];
  __syncthreads();

  // |c|^2 by the same tree (the centroid plays the key)
  float nc, unused;
  slot_sums<HP>(cs, piece, H, [&](int h, float (&k8)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) k8[i] = cs[h * 64 + piece * 8 + i];
  }, &nc, &unused);
  const float root_nc = __builtin_sqrtf(nc);

  // minimum and maximum of the d_i this wave writes: the selection normalises with them and reads
  // one pair per wave of this pass instead of every d_i
  float d_lo = __builtin_inff(), d_hi = -__builtin_inff();
  const int stride = gridDim.x * kDivWaves * 8;
  for (int s0 = (blockIdx.x * kDivWaves + wave) * 8; s0 < n_hist; s0 += stride) {
    const int slot = s0 + sl;
    const int sc = min(slot, n_hist - 1);
    const uint8_t fl = flags[sc];
    const char* row0 = K + (size_t)sc * 128 + piece * 16;
    float dot, nk;
    if constexpr (HP <= kDivHeadBatch) {
      // every load is issued (heads beyond H repeat the last one): no branch between the loads, so
      // all of them are in flight before the first wait
      uint4 w[HP];
#pragma unroll
      for (int h = 0; h < HP; ++h) w[h] = *(const uint4*)(row0 + (size_t)min(h, H - 1) * g.cap * 128);
      slot_sums<HP>(cs, piece, H, [&](int h, float (&k8)[8]) { unpack_halfs(w[h], k8); }, &dot, &nk);
    } else {
      slot_sums<HP>(cs, piece, H, [&](int h, float (&k8)[8]) {
        unpack_halfs(*(const uint4*)(row0 + (size_t)h * g.cap * 128), k8);
      }, &dot, &nk);
    }
    if (piece == 0 && slot < n_hist && fl == 0) {
      const float den = __builtin_sqrtf(nk) * root_nc;
      const float cosv = den == 0.f ? 0.f : dot / den;
      const float dv = 1.0f - cosv;
      dval[slot] = dv;
      d_lo = fminf(d_lo, dv); d_hi = fmaxf(d_hi, dv);
    }
  }
  // only the first lane of each slot's eight holds values: three butterfly steps across the slots,
  // one pair per wave (no workgroup barrier: a workgroup lives for a few slot groups only)
#pragma unroll
  for (int off = 8; off < 64; off *= 2) {
    d_lo = fminf(d_lo, __shfl_xor(d_lo, off, 64));
    d_hi = fmaxf(d_hi, __shfl_xor(d_hi, off, 64));
  }
  if (lane == 0) ((float2*)(mb + g.off_dpart))[blockIdx.x * kDivWaves + wave] = make_float2(d_lo, d_hi);
}

// A change of protection (Sec. 3.3) moves tokens between P and the evictable set: the sum loses the
// keys of the newly protected tokens and regains those of the released ones.  Reads the flags as they
// were before the change; the flags themselves are rewritten by the launch that follows.
__global__ void __launch_bounds__(kCenThreads)
centroid_protect_kernel(Geom g, char* kv, char* meta, int layer0, int n, uint32_t gid_lo, const uint8_t* mask,
                        int on, int chunk) {
  const int layer = layer0 + blockIdx.y;
  char* mb = layer_meta(meta, g, layer);
  const uint8_t* flags = (const uint8_t*)(mb + g.off_flags);
  const uint32_t* ids = (const uint32_t*)(mb + g.off_ids);
  const int v0 = blockIdx.x * chunk, v1 = min(v0 + chunk, n);
  accumulate_rows(g, layer_k(kv, g, layer), (unsigned long long*)(mb + g.off_csum), v0, v1,
                  [&](int v, int* slot) {
                    const uint32_t local = ids[v] - gid_lo;
                    if (local >= (uint32_t)g.M) return 0;
                    if (mask && mask[local] == 0) return 0;
                    const int was = flags[v] ? 1 : 0, now = on ? 1 : 0;
                    if (was == now) return 0;
                    *slot = v;
                    return now ? -1 : 1;
                  });
}

hipError_t launch_centroid_protect(const Geom& g, char* kv, char* meta, int layer0, int nl, int n, uint32_t gid_lo,
                                   const uint8_t* mask, int on, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int chunk = 64;
  dim3 grid((unsigned)((n + chunk - 1) / chunk), (unsigned)nl);
  hipLaunchKernelGGL(centroid_protect_kernel, grid, dim3(kCenThreads), 0, s, g, kv, meta, layer0, n, gid_lo, mask, on,
                     chunk);
  return hipGetLastError();
}

hipError_t launch_diversity(const Geom& g, char* kv, char* meta, int layer0, int nl, int n_hist, hipStream_t s) {
  if (n_hist <= 0) return hipSuccess;
  int hp = 1;
  while (hp < g.H) hp *= 2;
  static_assert(kDivWaves * 8 == kDivSlotsPerWg && kDivWaves == kDivWavesPerWg, "a wave takes 8 slots at a time");
  dim3 dgrid((unsigned)diversity_grid_x(n_hist, nl), (unsigned)nl);
#define OVGGT_DIV_LAUNCH(HH) \
  hipLaunchKernelGGL(diversity_kernel<HH>, dgrid, dim3(kDivThreads), 0, s, g, kv, meta, layer0, n_hist)
  switch (hp) {
    case 1: OVGGT_DIV_LAUNCH(1); break;
    case 2: OVGGT_DIV_LAUNCH(2); break;
    case 4: OVGGT_DIV_LAUNCH(4); break;
    case 8: OVGGT_DIV_LAUNCH(8); break;
    case 16: OVGGT_DIV_LAUNCH(16); break;
    case 32: OVGGT_DIV_LAUNCH(32); break;
    default: OVGGT_DIV_LAUNCH(64); break;
  }
#undef OVGGT_DIV_LAUNCH
  return hipGetLastError();
}

hipError_t launch_centroid_update(const Geom& g, char* kv, char* meta, int layer0, int nl, int n_total, hipStream_t s) {
  // rows per workgroup: few enough that one layer's update is a single round of loads on many CUs,
  // more when many layers share the launch (each workgroup ends with an atomic per key element)
  int chunk = (int)(((long)2 * g.M * nl + 1023) / 1024 + 15) / 16 * 16;
  if (chunk < 16) chunk = 16;
  if (chunk > 64) chunk = 64;
  dim3 grid((unsigned)((2 * g.M + chunk - 1) / chunk), (unsigned)nl);
  hipLaunchKernelGGL(centroid_update_kernel, grid, dim3(kCenThreads), 0, s, g, kv, meta, layer0, n_total, chunk);
  return hipGetLastError();
}

hipError_t launch_centroid_rebuild(const Geom& g, char* kv, char* meta, int layer, int n, hipStream_t s) {
  hipError_t e = launch_fill_zero(layer_meta(meta, g, layer) + g.off_csum, (size_t)8 * g.H * g.d, s);
  if (e != hipSuccess || n <= 0) return e;
  const int chunk = 64;
  hipLaunchKernelGGL(centroid_rebuild_kernel, dim3((unsigned)((n + chunk - 1) / chunk)), dim3(kCenThreads), 0, s,
                     g, kv, meta, layer, n, chunk);
  return hipGetLastError();
}

}  // namespace ovggt
