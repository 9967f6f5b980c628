// Cache maintenance kernels: zero fill, append (paper Eq. 2) and the in-place
// hole-fill compaction that follows Eq. 8's selection.  All are pure copies,
// bound by HBM bandwidth; every lane moves 16-byte pieces of 128-byte-or-longer
// contiguous rows.
#include "ovggt_internal.h"
#include "../../include/ovggt.h"
#include <hip/hip_fp16.h>

namespace ovggt {

// bf16 handles keep K and V as IEEE binary16: both attention products then run
// on the f16 MFMA, P*V with 11-bit softmax weights instead of 8-bit ones and
// Q*K^T with queries that carry the softmax scale at 11 bits.  Values beyond the
// half range saturate (and are reported), values below 2^-14 round to the half
// subnormal grid.
__device__ inline uint32_t bf16pair_to_half(uint32_t w, bool* clipped) {
  float a = __uint_as_float(w << 16), b = __uint_as_float(w & 0xFFFF0000u);
  if (!(fabsf(a) <= 65504.f)) { *clipped = true; a = a != a ? a : copysignf(65504.f, a); }
  if (!(fabsf(b) <= 65504.f)) { *clipped = true; b = b != b ? b : copysignf(65504.f, b); }
  const __half2 h = __floats2half2_rn(a, b);
  return *(const uint32_t*)&h;
}

// --------------------------------------------------------------------------
__global__ void __launch_bounds__(256) fill_zero_kernel(uint4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const uint4 z = {0u, 0u, 0u, 0u};
  for (; i < n16; i += stride) p[i] = z;
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;        // buffers are sized in multiples of 256 bytes
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)p, n16);
  return hipGetLastError();
}

// --------------------------------------------------------------------------
// Timing aid: one wave that returns after `ticks` ticks of the constant-rate wall clock (or after
// a fixed number of polls, whichever comes first, so the kernel ends under all circumstances).
__global__ void __launch_bounds__(64) spin_kernel(unsigned long long ticks) {
  const unsigned long long t0 = wall_clock64();
  for (int i = 0; i < (1 << 22); ++i) {
    if (wall_clock64() - t0 >= ticks) break;
    __builtin_amdgcn_s_sleep(8);
  }
}

hipError_t launch_spin(unsigned long long ticks, hipStream_t s) {
  hipLaunchKernelGGL(spin_kernel, dim3(1), dim3(64), 0, s, ticks);
  return hipGetLastError();
}

// --------------------------------------------------------------------------
// Append.  Input rows are token-major [M][H][d]; the cache is head-major
// [H][cap][d].  One thread per 16-byte piece of K and of V.
// MOVES: the compaction that follows the previous frame's selection has not been applied yet
// (n == B).  Its sources are exactly the slots this frame overwrites, so the thread that owns a
// piece of slot B + m first carries the piece it finds there to the slot the selection assigned
// (below B, disjoint from every slot written here), then stores the new one: no other thread
// reads or writes either location.
template <bool MOVES>
__global__ void __launch_bounds__(256)
append_kernel(Geom g, char* kv, char* meta, int layer0, const char* k_new, const char* v_new, int n) {
  const int layer = layer0 + blockIdx.y;
  if (g.hybrid && blockIdx.x == 0) {
    // Hybrid scoring: the frame's diversity pass wants the centroid in fp32.  The running sum (64-bit
    // integers in units of 2^-24, final since the previous frame's update) is rounded integer -> fp64
    // -> fp32, each to nearest even, and scaled by 2^-24 exactly.
    char* mb = layer_meta(meta, g, layer);
    const long long* csum = (const long long*)(mb + g.off_csum);
    float* cvec = (float*)(mb + g.off_cvec);
    for (int e = threadIdx.x; e < g.H * g.d; e += blockDim.x)
      cvec[e] = (float)(double)csum[e] * 5.9604644775390625e-8f;
  }
  const int row_bytes = g.d * g.esize;             // 128 (bf16) or 256 (f32)
  const int pieces = row_bytes / 16;
  const size_t per_layer_in = (size_t)g.M * g.H * row_bytes;
  const size_t total = (size_t)g.M * g.H * pieces;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int piece = (int)(i % pieces);
  const int h = (int)((i / pieces) % g.H);
  const int m = (int)(i / ((size_t)pieces * g.H));
  const size_t src = (size_t)blockIdx.y * per_layer_in + ((size_t)m * g.H + h) * row_bytes + piece * 16;
  const size_t dst = ((size_t)h * g.cap + (n + m)) * row_bytes + piece * 16;
  uint4 kk = *(const uint4*)(k_new + src);
  uint4 vv = *(const uint4*)(v_new + src);
  char* mb = layer_meta(meta, g, layer);
  if constexpr (MOVES) {
    // the entry that sits in the slot is fetched together with its destination, not after it: one
    // round trip to memory less on the path of every moved piece
    const uint4 ok = *(const uint4*)(layer_k(kv, g, layer) + dst);
    const uint4 ov = *(const uint4*)(layer_v(kv, g, layer) + dst);
    const uint32_t to = ((const uint32_t*)(mb + g.off_mvmap))[m];
    if (to < (uint32_t)g.B) {                        // kNoMove, or anything out of range: nothing to carry
      const size_t mv = ((size_t)h * g.cap + to) * row_bytes + piece * 16;
      uint32_t id = 0; float sc = 0.f; uint8_t fl = 0;
      const bool meta_thread = h == 0 && piece == 0;
      if (meta_thread) {
        id = ((const uint32_t*)(mb + g.off_ids))[n + m];
        sc = ((const float*)(mb + g.off_ss))[n + m];
        fl = ((const uint8_t*)(mb + g.off_flags))[n + m];
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the old contents are in registers before anything is stored
      *(uint4*)(layer_k(kv, g, layer) + mv) = ok;
      *(uint4*)(layer_v(kv, g, layer) + mv) = ov;
      if (meta_thread) {
        ((uint32_t*)(mb + g.off_ids))[to] = id;
        ((float*)(mb + g.off_ss))[to] = sc;
        ((uint8_t*)(mb + g.off_flags))[to] = fl;
      }
    }
  }
  if (g.esize == 2) {
    bool clipped = false;
    kk.x = bf16pair_to_half(kk.x, &clipped); kk.y = bf16pair_to_half(kk.y, &clipped);
    kk.z = bf16pair_to_half(kk.z, &clipped); kk.w = bf16pair_to_half(kk.w, &clipped);
    vv.x = bf16pair_to_half(vv.x, &clipped); vv.y = bf16pair_to_half(vv.y, &clipped);
    vv.z = bf16pair_to_half(vv.z, &clipped); vv.w = bf16pair_to_half(vv.w, &clipped);
    if (clipped) atomicOr(&((Ctrl*)(mb + g.off_ctrl))->status, (uint32_t)OVGGT_STATUS_VRANGE);
  }
  *(uint4*)(layer_k(kv, g, layer) + dst) = kk;
  *(uint4*)(layer_v(kv, g, layer) + dst) = vv;
  if (h == 0 && piece == 0) {
    // ids t*M + i (Eq. 2's arrival order): the frame's first id lives in the control block, where the
    // previous frame's selection left it, so the launch is the same for every frame (graph replay)
    const uint32_t gid0 = ((const Ctrl*)(mb + g.off_ctrl))->gid_next;
    ((uint32_t*)(mb + g.off_ids))[n + m] = gid0 + (uint32_t)m;
    ((float*)(mb + g.off_ss))[n + m] = 0.f;
    ((uint8_t*)(mb + g.off_flags))[n + m] = 0;
  }
}

hipError_t launch_append(const Geom& g, char* kv, char* meta, int layer0, int nl,
                         const void* k_new, const void* v_new, int n, bool apply_moves, hipStream_t s) {
  const size_t total = (size_t)g.M * g.H * (g.d * g.esize / 16);
  dim3 grid((unsigned)((total + 255) / 256), (unsigned)nl);
  if (apply_moves && n == g.B)
    hipLaunchKernelGGL(append_kernel<true>, grid, dim3(256), 0, s, g, kv, meta, layer0,
                       (const char*)k_new, (const char*)v_new, n);
  else if (apply_moves)
    return hipErrorInvalidValue;                     // a pending compaction implies a full cache
  else
    hipLaunchKernelGGL(append_kernel<false>, grid, dim3(256), 0, s, g, kv, meta, layer0,
                       (const char*)k_new, (const char*)v_new, n);
  return hipGetLastError();
}

// --------------------------------------------------------------------------
// Compaction.  Workgroup r of a layer moves entry src[r] -> dst[r]: 2*H rows of
// d elements (K and V of every head) plus id, score and flag.  Destinations are
// slots below B, sources slots at or above B, so no ordering between moves is
// needed.  Workgroups beyond the list length exit at once.
__global__ void __launch_bounds__(256)
compact_kernel(Geom g, char* kv, char* meta, int layer0) {
  const int layer = layer0 + blockIdx.y;
  char* mb = layer_meta(meta, g, layer);
  const Ctrl* ctrl = (const Ctrl*)(mb + g.off_ctrl);
  const uint32_t n_moves = ctrl->n_moves;
  const uint32_t r = blockIdx.x;
  if (r >= n_moves) return;
  const uint32_t dst = ((const uint32_t*)(mb + g.off_mvdst))[r];
  const uint32_t src = ((const uint32_t*)(mb + g.off_mvsrc))[r];
  if (dst >= (uint32_t)g.B || src < (uint32_t)g.B || src >= (uint32_t)g.cap) return;   // never out of bounds
  const int row_bytes = g.d * g.esize;
  const int pieces = row_bytes / 16;
  const int total = 2 * g.H * pieces;
  char* kbase = layer_k(kv, g, layer);
  const size_t v_off = (size_t)g.H * g.cap * row_bytes;
  for (int i = threadIdx.x; i < total; i += blockDim.x) {
    const int piece = i % pieces;
    const int h = (i / pieces) % g.H;
    const int isv = i / (pieces * g.H);
    char* base = kbase + (isv ? v_off : 0) + (size_t)h * g.cap * row_bytes + piece * 16;
    *(uint4*)(base + (size_t)dst * row_bytes) = *(const uint4*)(base + (size_t)src * row_bytes);
  }
  if (threadIdx.x == 0) {
    uint32_t* ids = (uint32_t*)(mb + g.off_ids);
    float* ss = (float*)(mb + g.off_ss);
    uint8_t* fl = (uint8_t*)(mb + g.off_flags);
    ids[dst] = ids[src];
    ss[dst] = ss[src];
    fl[dst] = fl[src];
  }
}

// --------------------------------------------------------------------------
// Sec. 3.3: protection granted or withdrawn for resident tokens of one frame.  One thread per
// slot: ids in [gid_lo, gid_lo + M) whose mask byte is set (no mask: all of them) take the flag.
__global__ void __launch_bounds__(256)
set_protect_kernel(Geom g, char* meta, int layer0, int n, uint32_t gid_lo, const uint8_t* mask, int on) {
  char* mb = layer_meta(meta, g, layer0 + blockIdx.y);
  const int slot = blockIdx.x * blockDim.x + threadIdx.x;
  if (slot >= n) return;
  const uint32_t local = ((const uint32_t*)(mb + g.off_ids))[slot] - gid_lo;     // wraps for ids below gid_lo
  if (local >= (uint32_t)g.M) return;
  if (mask && mask[local] == 0) return;
  ((uint8_t*)(mb + g.off_flags))[slot] = on ? 1 : 0;
}

hipError_t launch_set_protect(const Geom& g, char* meta, int layer0, int nl, int n, uint32_t gid_lo,
                              const uint8_t* mask, int on, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  dim3 grid((unsigned)((n + 255) / 256), (unsigned)nl);
  hipLaunchKernelGGL(set_protect_kernel, grid, dim3(256), 0, s, g, meta, layer0, n, gid_lo, mask, on);
  return hipGetLastError();
}

hipError_t launch_compact(const Geom& g, char* kv, char* meta, int layer0, int nl, hipStream_t s) {
  dim3 grid((unsigned)g.M, (unsigned)nl);      // at most M entries move per frame
  hipLaunchKernelGGL(compact_kernel, grid, dim3(256), 0, s, g, kv, meta, layer0);
  return hipGetLastError();
}

}  // namespace ovggt
