// fp32 attention of the new frame's queries over the resident cache (paper
// Sec. 3.1), for handles whose dtype is f32.  This is the accuracy path of the
// small all-fp32 workload (tolerance 1e-4 of output RMS), not a tuned kernel:
// one workgroup per (query, head), two passes over the keys (row maximum, then
// exp / sum / weighted values), everything accumulated in fp32.
#include "ovggt_internal.h"

namespace ovggt {

constexpr int kF32Threads = 256;

__device__ inline float block_reduce_max(float v, float* tmp) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  if ((threadIdx.x & 63) == 0) tmp[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = tmp[0];
  for (int w = 1; w < kF32Threads / 64; ++w) r = fmaxf(r, tmp[w]);
  __syncthreads();
  return r;
}

__global__ void __launch_bounds__(kF32Threads)
attn_f32_kernel(Geom g, char* kv, int layer0, const float* q, float* out, int n_total, float scale) {
  __shared__ float qs[64];
  __shared__ float tmp[kF32Threads / 64];
  __shared__ float acc[kF32Threads / 64][65];
  const int m = blockIdx.x, h = blockIdx.y, li = blockIdx.z;
  const int layer = layer0 + li;
  const int tid = threadIdx.x;
  const float* kbase = (const float*)layer_k(kv, g, layer) + (size_t)h * g.cap * 64;
  const float* vbase = (const float*)layer_v(kv, g, layer) + (size_t)h * g.cap * 64;
  const size_t qoff = (((size_t)li * g.M + m) * g.H + h) * 64;
  if (tid < 64) qs[tid] = q[qoff + tid];
  __syncthreads();

  // pass 1: maximum logit
  float mx = -INFINITY;
  for (int j = tid; j < n_total; j += kF32Threads) {
    const float* kr = kbase + (size_t)j * 64;
    float s = 0.f;
#pragma unroll 16
    for (int e = 0; e < 64; ++e) s = fmaf(qs[e], kr[e], s);
    mx = fmaxf(mx, s * scale);
  }
  mx = block_reduce_max(mx, tmp);

  // pass 2: thread t owns output element e = t & 63 and every 4th key
  const int e = tid & 63, grp = tid >> 6;
  float l = 0.f, o = 0.f;
  for (int j = grp; j < n_total; j += kF32Threads / 64) {
    const float* kr = kbase + (size_t)j * 64;
    float s = 0.f;
#pragma unroll 16
    for (int c = 0; c < 64; ++c) s = fmaf(qs[c], kr[c], s);
    const float p = __expf(s * scale - mx);
    l += p;
    o = fmaf(p, vbase[(size_t)j * 64 + e], o);
  }
  acc[grp][e] = o;
  if (e == 0) acc[grp][64] = l;
  __syncthreads();
  if (tid < 64) {
    float os = 0.f, ls = 0.f;
    for (int w = 0; w < kF32Threads / 64; ++w) { os += acc[w][tid]; ls += acc[w][64]; }
    out[qoff + tid] = os / ls;
  }
}

hipError_t launch_attn_f32(const Geom& g, char* kv, int layer0, int nl, const void* q, void* out,
                           int n_total, float scale, hipStream_t s) {
  dim3 grid((unsigned)g.M, (unsigned)g.H, (unsigned)nl);
  hipLaunchKernelGGL(attn_f32_kernel, grid, dim3(kF32Threads), 0, s, g, kv, layer0,
                     (const float*)q, (float*)out, n_total, scale);
  return hipGetLastError();
}

}  // namespace ovggt
