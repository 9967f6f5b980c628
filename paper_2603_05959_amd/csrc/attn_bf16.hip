// bf16 flash-style attention of one frame's queries over the bounded KV cache
// (paper Sec. 3.1: the temporal causal attention CA; cost O(M*B) per step once
// the cache is bounded).  gfx950 MFMA kernel.
//
// Formulation (chosen so the softmax statistics of one query live in one lane):
//   S^T = K Q^T      A = K tile rows from LDS,      B = Q^T fragments in registers
//   O^T = V^T P^T    A = V^T via LDS transpose reads, B = P^T straight from the
//                    S^T accumulators (the contraction index may be permuted
//                    freely as long as both operands agree)
// S^T uses v_mfma_f32_32x32x16_bf16 on the bf16 Q and K.  The cache holds V as
// IEEE half and the softmax weights are rounded to half, so O^T uses
// v_mfma_f32_32x32x16_f16: 11-bit weights keep the output within 1e-3 of its RMS
// where 8-bit (bf16) weights reach 4e-2 on rows with one dominant key.  Both
// accumulate in fp32; the online softmax runs in fp32 in the exp2 domain with a
// lazily applied running maximum (accumulators are rescaled only when the
// maximum grows by more than 2^8) and weights biased by 2^7 to sit in the middle
// of the half range.
//
// Work split.  An item is (layer, head, 128-query block); its work is T =
// ceil(n/128) slot tiles.  The flat list of item x tile units is cut into equal
// chunks, one per workgroup (persistent, stream-K style), so all CUs finish
// together whatever M, n and H are.  A workgroup that covers an item completely
// writes the output; otherwise it writes an unnormalised partial (O, m, l) that
// attn_combine_kernel merges.  Chunks are handed to workgroups so that each
// XCD's L2 sees as few heads as possible.
//
// A workgroup is 4 waves: wave = (query half, slot half) of the 128x128 tile;
// the two slot halves are merged through LDS at the end of an item.  K and V
// tiles are streamed global->LDS with 16-byte direct-to-LDS loads, double
// buffered, one barrier per tile.  LDS rows are 128 bytes; 16-byte pieces are
// XOR-swizzled with the row index so both the K operand reads and the V
// transpose reads are bank-conflict free.
#include "ovggt_internal.h"

namespace ovggt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// XOR swizzle of the 16-byte piece index within a 128-byte LDS row (measured against
// variants keyed on higher row bits: this one has the fewest bank conflicts).
__device__ __forceinline__ int swz(int row) { return row & 7; }

#ifndef OVGGT_ABLATE
#define OVGGT_ABLATE 0          // timing experiments only: bit 0 no exp, 1 no softmax, 2 no PV, 3 no QK, 4 no loads, 5 no barrier
#endif

constexpr int kTileBytes = kSlotTile * 128;

// 16-byte direct-to-LDS load: lane i's 16 bytes land at lds_base + 16*i.  Issued as inline
// assembly on purpose: the compiler cannot tell which LDS bytes an LDS-DMA load writes and
// would make every later LDS read wait for ALL outstanding loads (vmcnt(0)), i.e. for the
// prefetch of the next tile.  The kernel orders these loads itself: one explicit
// s_waitcnt vmcnt(0) in front of the barrier that publishes a tile.
template <int IMM>
__device__ __forceinline__ void load16_to_lds(const char* base, uint32_t lane_off, const char* lds_base) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(const char, lds_base));
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3"
               : : "s"(m0), "v"(lane_off), "s"(base), "n"(IMM) : "memory", "m0");
}

// One 128-slot K tile and V tile, global -> LDS: wave w fills rows [32w, 32w+32) of both with
// four loads each (8 rows of 128 bytes per load); piece p of row r goes to LDS piece p ^ swz(r).
// The instruction's immediate offset advances the memory address and the LDS address alike.
__device__ __forceinline__ void issue_tile_loads(const char* kbase, const char* vbase, int tile, char* buf,
                                                 int wave, int lane) {
  const int ld_row = lane >> 3;
  const uint32_t off = (uint32_t)((tile * kSlotTile + wave * 32 + ld_row) * 128 + (((lane & 7) ^ swz(ld_row)) << 4));
  char* lk = buf + wave * 4096;
  char* lv = lk + kTileBytes;
  load16_to_lds<0>(kbase, off, lk);
  load16_to_lds<0>(vbase, off, lv);
  load16_to_lds<1024>(kbase, off, lk);
  load16_to_lds<1024>(vbase, off, lv);
  load16_to_lds<2048>(kbase, off, lk);
  load16_to_lds<2048>(vbase, off, lv);
  load16_to_lds<3072>(kbase, off, lk);
  load16_to_lds<3072>(vbase, off, lv);
}

constexpr int kPartialFloats = kQueryTile * 64 + 2 * kQueryTile;
constexpr float kWeightBias = 7.0f;                    // weights are stored as 2^7 * p (half max 65504)
constexpr float kWeightSumLimit = 32768.0f;            // a lane's weight sum below 2^15 proves no weight overflowed

size_t attn_ws_bytes() { return (size_t)kMaxAttnWgs * 2 * kPartialFloats * sizeof(float); }

struct AttnParams {
  const char* q;
  char* out;
  const char* kv0;            // K of the first layer of this launch
  size_t kv_layer_bytes;
  size_t v_off;               // bytes from a layer's K to its V
  float* ws;
  int H, M, cap, n_total, nl;
  int QB;                     // query blocks per (layer, head)
  int T;                      // slot tiles
  int chunk;                  // units per workgroup
  int total_units;
  float c;                    // softmax scale * log2(e)
  int out_f32;                // output element type: 1 = fp32, 0 = bf16
};

// Lanes l and l+32 hold the two slot groups of the same query.  The swap
// instruction leaves each lane with both values in (r[0], r[1]) in some order,
// so symmetric combinations need no lane test.
__device__ inline float pair_max(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float pair_sum(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ inline f16x8 join4(const f16x2* p) {
  const f16x4 a = __builtin_shufflevector(p[0], p[1], 0, 1, 2, 3);
  const f16x4 b = __builtin_shufflevector(p[2], p[3], 0, 1, 2, 3);
  return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Softmax weights of one query block of a tile: p = exp2(s*c - mcb) for the 32 scores a lane
// holds (two 32-slot accumulators), rounded to half in pairs; returns the lane's fp32 sum of the
// weights.
__device__ __forceinline__ float tile_weights(const f32x16& s0, const f32x16& s1, float c, float mcb,
                                              f16x2 (&p0)[8], f16x2 (&p1)[8]) {
  float ls[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float a = sb ? s1[2 * j] : s0[2 * j], b = sb ? s1[2 * j + 1] : s0[2 * j + 1];
#if OVGGT_ABLATE & 2
      const float e0 = a, e1 = b;
      if (j > 0) { (sb ? p1 : p0)[j] = (sb ? p1 : p0)[0]; continue; }
#elif OVGGT_ABLATE & 1
      const float e0 = __builtin_fmaf(a, c, -mcb), e1 = __builtin_fmaf(b, c, -mcb);
#else
      const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(a, c, -mcb));
      const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(b, c, -mcb));
#endif
      f16x2 pk;
      pk[0] = (_Float16)e0;
      pk[1] = (_Float16)e1;
      // plain fp32 adds: v_dot2c_f32_f16 runs on the matrix pipe and serialises with the other
      // wave's MFMAs (measured), v_add_f32 co-executes with them
      ls[j & 3] += e0;
      ls[(j + 2) & 3] += e1;
      (sb ? p1 : p0)[j] = pk;
    }
  return (ls[0] + ls[1]) + (ls[2] + ls[3]);
}

// One 64-slot x 64-query tile of one wave: S^T = K Q^T, online softmax, O^T += V^T P^T.
// tail: the tile extends past n_total (only the last tile can); weights of the
// absent slots are cleared after the softmax (their rows hold zeros or stale but
// finite keys, so their scores are finite and merely move the reference maximum).
//
// Softmax fast path: weights are formed against the running reference maximum
// m without looking for this tile's maximum; p = 2^7 * exp2((s - m) * c) is
// rounded to half and summed.  If the lane's sum stays below 2^15 no weight can
// have overflowed half.  Otherwise (first tile, or the maximum grew by about 2^8)
// the wave takes the slow path: true tile maximum, rescale O and l, redo the
// weights.  The reference maximum therefore lags the true one by < 2^8, which
// costs no accuracy in fp32/half arithmetic.
__device__ __forceinline__ void process_tile(const char* ldsK, const int (&koff)[4], const int (&voff)[2][2],
                                             const bf16x8 (&qf)[2][4], f32x16 (&O)[2][2], float (&mrun)[2],
                                             float (&lrun)[2], float c, int sbase, int n_total, bool tail) {
  const char* ldsV = ldsK + kTileBytes;
  f32x16 S[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[a][b][i] = 0.f;
#if OVGGT_ABLATE & 8
  for (int a = 0; a < 2; ++a) for (int b = 0; b < 2; ++b) for (int i = 0; i < 16; ++i) S[a][b][i] = mrun[b] + i * 0.01f + (float)qf[a][b][0];
#else
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
#if OVGGT_ABLATE & 512
    const bf16x8 k0 = qf[1][ks], k1 = qf[0][(ks + 1) & 3];
#else
    const bf16x8 k0 = *LDS_PTR(const bf16x8, ldsK + koff[ks]);
    const bf16x8 k1 = *LDS_PTR(const bf16x8, ldsK + koff[ks] + 32 * 128);
#endif
    S[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[0][ks], S[0][0], 0, 0, 0);
    S[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[1][ks], S[0][1], 0, 0, 0);
    S[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[0][ks], S[1][0], 0, 0, 0);
    S[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[1][ks], S[1][1], 0, 0, 0);
  }
#endif
  f16x2 P[2][2][8];
  float lsum[2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
    lsum[qb] = tile_weights(S[0][qb], S[1][qb], c, mrun[qb] * c - kWeightBias, P[0][qb], P[1][qb]);

  // one overflow test for both query blocks, after all fast-path work has been issued
#if OVGGT_ABLATE & (3 | 256)
  if (false) {
#else
  if (__builtin_amdgcn_ballot_w64(!(lsum[0] <= kWeightSumLimit) || !(lsum[1] <= kWeightSumLimit)) != 0ull) {
#endif
    // rare: recompute the scores (cheaper than keeping them live past the fast path), take the
    // true maximum, rescale the accumulators and redo the weights
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 R[2];
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) R[sb][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
          R[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*LDS_PTR(const bf16x8, ldsK + koff[ks] + sb * 32 * 128),
                                                          qf[qb][ks], R[sb], 0, 0, 0);
      }
      float mx = R[0][0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, R[0][i]);
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, R[1][i]);
      mx = pair_max(mx);
      const float mnew = fmaxf(mrun[qb], mx);
      const float alpha = __builtin_amdgcn_exp2f((mrun[qb] - mnew) * c);
      mrun[qb] = mnew;
      lrun[qb] *= alpha;
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[db][qb][i] *= alpha;
      lsum[qb] = tile_weights(R[0], R[1], c, mnew * c - kWeightBias, P[0][qb], P[1][qb]);
    }
  }
  if (tail) {
    asm volatile("; tail tile: clear absent slots" ::: "memory");   // keeps this block a real branch (never if-converted)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      float ls = 0.f;
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int slot = sbase + sb * 32 + (j >> 1) * 8 + (j & 1) * 2;      // slots of accumulators 2j, 2j+1
          uint32_t w = __builtin_bit_cast(uint32_t, P[sb][qb][j]);
          w &= (slot < n_total ? 0x0000FFFFu : 0u) | (slot + 1 < n_total ? 0xFFFF0000u : 0u);
          P[sb][qb][j] = __builtin_bit_cast(f16x2, w);
          ls += (float)P[sb][qb][j][0] + (float)P[sb][qb][j][1];
        }
      lsum[qb] = ls;
    }
  }
  lrun[0] += lsum[0];
  lrun[1] += lsum[1];

  // O^T += V^T P^T; each V^T fragment feeds both query blocks
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const f16x8 pb0 = join4(P[sb][0] + 4 * s2);
      const f16x8 pb1 = join4(P[sb][1] + 4 * s2);
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        const int o = (sb * 32 + 16 * s2) * 128;
#if OVGGT_ABLATE & 1024
        const s16x4 va = __builtin_bit_cast(s16x4, __builtin_shufflevector(pb0, pb0, 0, 1, 2, 3));
        const s16x4 vb = __builtin_bit_cast(s16x4, __builtin_shufflevector(pb1, pb1, 4, 5, 6, 7));
#else
        const s16x4 va = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ldsV + voff[db][0] + o));
        const s16x4 vb = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ldsV + voff[db][1] + o));
#endif
        const __attribute__((ext_vector_type(8))) short v8 = __builtin_shufflevector(va, vb, 0, 1, 2, 3, 4, 5, 6, 7);
        const f16x8 vf = __builtin_bit_cast(f16x8, v8);
#if OVGGT_ABLATE & 4
        O[db][0][0] += (float)vf[0] * (float)pb0[0]; O[db][1][1] += (float)vf[1] * (float)pb1[1];
#else
        O[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pb0, O[db][0], 0, 0, 0);
        O[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pb1, O[db][1], 0, 0, 0);
#endif
      }
    }
}

__global__ void __launch_bounds__(256, 2) attn_bf16_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * kTileBytes];     // [buf][K|V]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int qhalf = wave & 1, khalf = wave >> 1;
  const int l32 = lane & 31, g = lane >> 5;

  const int G = gridDim.x;
  const int cidx = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);
  int u = cidx * p.chunk;
  const int u_end = min(u + p.chunk, p.total_units);
  if (u >= u_end) return;
  const int u_begin = u;
#ifdef OVGGT_DEPHASE
  if ((int)blockIdx.x >= (G >> 1)) { for (int r = 0; r < OVGGT_DEPHASE; ++r) __builtin_amdgcn_s_sleep(16); }
#endif

  // per-lane LDS offsets
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    koff[ks] = (khalf * 64 + l32) * 128 + ((((2 * ks + g) ^ swz(l32))) << 4);
  int voff[2][2];                                        // [db][second group of four slots]
  {
    const int i = lane & 15;
    const int x = 4 * g + (i >> 2);                    // row within an 8-row group (row offsets added later are multiples of 8)
    const int c0 = 2 * ((lane >> 4) & 1) + ((i & 3) >> 1);
    const int inb = (i & 1) * 8;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
        voff[db][hh] = (khalf * 64 + 8 * hh + x) * 128 + ((((c0 + 4 * db) ^ swz(8 * hh + x))) << 4) + inb;
  }
  while (u < u_end) {
    const int item = u / p.T;
    const int t0 = u - item * p.T;
    const int t1 = min(p.T, t0 + (u_end - u));
    const bool first_seg = (u == u_begin);
    const bool full = (t0 == 0 && t1 == p.T);
    const int qb_idx = item % p.QB;
    const int h = (item / p.QB) % p.H;
    const int li = item / (p.QB * p.H);
    const char* kbase = p.kv0 + (size_t)li * p.kv_layer_bytes + (size_t)h * p.cap * 128;
    const char* vbase = kbase + p.v_off;
    const int q0 = qb_idx * kQueryTile;

    // Q^T fragments: lane holds query (q0 + qhalf*64 + qb*32 + l32), d = ks*16 + 8g .. +8
    bf16x8 qf[2][4];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      int qrow = q0 + qhalf * 64 + qb * 32 + l32;
      if (qrow > p.M - 1) qrow = p.M - 1;
      const char* qp = p.q + ((((size_t)li * p.M + qrow) * p.H + h) * 64) * 2;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) qf[qb][ks] = *(const bf16x8*)(qp + (ks * 16 + 8 * g) * 2);
    }

    f32x16 O[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[a][b][i] = 0.f;
    float mrun[2] = {-1e30f, -1e30f};
    float lrun[2] = {0.f, 0.f};

    // prologue: first tile into buffer 0
    issue_tile_loads(kbase, vbase, t0, lds, wave, lane);

    for (int tt = t0; tt < ((OVGGT_ABLATE & 2048) ? t0 : t1); ++tt) {
      const int cur = (tt - t0) & 1;
      // vmcnt(0): this tile's loads have landed.  Issued through the builtin (not inline asm) so the
      // compiler also knows that every load it tracks itself (the Q fragments) is complete and puts
      // no vmcnt wait of its own inside the loop, where it would wait on the prefetch instead.
      __builtin_amdgcn_s_waitcnt(0x0F70);
#if !(OVGGT_ABLATE & 32)
      __syncthreads();
#endif
      if (tt + 1 < t1 && !(OVGGT_ABLATE & 16))
        issue_tile_loads(kbase, vbase, (OVGGT_ABLATE & 64) ? ((tt + 1) & 7) : (tt + 1),
                         lds + (cur ^ 1) * 2 * kTileBytes, wave, lane);
      const char* ldsK = lds + ((OVGGT_ABLATE & 16) ? 0 : cur) * 2 * kTileBytes;
      const int sbase = tt * kSlotTile + khalf * 64 + 4 * g;      // first slot of this lane's accumulator rows
      process_tile(ldsK, koff, voff, qf, O, mrun, lrun, p.c, sbase, p.n_total,
                   tt == p.T - 1 && (p.n_total & (kSlotTile - 1)) != 0);
    }

    // ---- merge the two slot halves through LDS
    float ltot[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) ltot[qb] = pair_sum(lrun[qb]);
    __syncthreads();                                  // all tile reads done; LDS is free
    float* mO = (float*)lds + qhalf * (64 * 64);       // [reg][lane]
    float* mML = (float*)lds + 2 * 64 * 64 + qhalf * (4 * 64);
    if (khalf == 1) {
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mO[((db * 2 + qb) * 16 + i) * 64 + lane] = O[db][qb][i];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        mML[qb * 64 + lane] = mrun[qb] * p.c;
        mML[(2 + qb) * 64 + lane] = ltot[qb];
      }
    }
    __syncthreads();
    if (khalf == 0) {
      float mfin[2], lfin[2];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const float m0 = mrun[qb] * p.c, m1 = mML[qb * 64 + lane];
        const float mt = fmaxf(m0, m1);
        const float a0 = __builtin_amdgcn_exp2f(m0 - mt), a1 = __builtin_amdgcn_exp2f(m1 - mt);
        mfin[qb] = mt;
        lfin[qb] = ltot[qb] * a0 + mML[(2 + qb) * 64 + lane] * a1;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            O[db][qb][i] = O[db][qb][i] * a0 + mO[((db * 2 + qb) * 16 + i) * 64 + lane] * a1;
      }
      if (full) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const int qrow = q0 + qhalf * 64 + qb * 32 + l32;
          if (qrow < p.M) {
            const float inv = 1.0f / lfin[qb];
            const size_t oel = (((size_t)li * p.M + qrow) * p.H + h) * 64;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
              for (int ig = 0; ig < 4; ++ig) {
                const int dcol = db * 32 + ig * 8 + 4 * g;
                if (p.out_f32) {
                  float4 w = {O[db][qb][ig * 4] * inv, O[db][qb][ig * 4 + 1] * inv,
                              O[db][qb][ig * 4 + 2] * inv, O[db][qb][ig * 4 + 3] * inv};
                  *(float4*)(p.out + (oel + dcol) * 4) = w;
                } else {
                  bf16x4 w;
#pragma unroll
                  for (int j = 0; j < 4; ++j) w[j] = (__bf16)(O[db][qb][ig * 4 + j] * inv);
                  *(bf16x4*)(p.out + (oel + dcol) * 2) = w;
                }
              }
          }
        }
      } else {
        float* rec = p.ws + (size_t)(2 * cidx + (first_seg ? 0 : 1)) * kPartialFloats;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const int r = qhalf * 64 + qb * 32 + l32;
#pragma unroll
          for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int ig = 0; ig < 4; ++ig) {
              float4 w = {O[db][qb][ig * 4], O[db][qb][ig * 4 + 1], O[db][qb][ig * 4 + 2], O[db][qb][ig * 4 + 3]};
              *(float4*)(rec + r * 64 + db * 32 + ig * 8 + 4 * g) = w;
            }
          if (g == 0) {
            rec[kQueryTile * 64 + r] = mfin[qb];
            rec[kQueryTile * 64 + kQueryTile + r] = lfin[qb];
          }
        }
      }
    }
    __syncthreads();                                  // merge scratch is reused as tile buffers
    u += t1 - t0;
  }
}

// Merge the partials of every item that was split across workgroups.
__global__ void __launch_bounds__(256) attn_combine_kernel(AttnParams p) {
  const int item = blockIdx.x;
  const long ua = (long)item * p.T, ub = ua + p.T - 1;
  const int cf = (int)(ua / p.chunk), cl = (int)(ub / p.chunk);
  if (cf == cl) return;                                // one workgroup did the whole item
  const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
  const int qb_idx = item % p.QB;
  const int h = (item / p.QB) % p.H;
  const int li = item / (p.QB * p.H);
  const int qrow = qb_idx * kQueryTile + row;
  if (qrow >= p.M) return;
  float mt = -INFINITY;
  for (int c = cf; c <= cl; ++c) {
    const float* rec = p.ws + (size_t)(2 * c + ((long)c * p.chunk < ua ? 1 : 0)) * kPartialFloats;
    mt = fmaxf(mt, rec[kQueryTile * 64 + row]);
  }
  float acc[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) acc[j] = 0.f;
  float l = 0.f;
  for (int c = cf; c <= cl; ++c) {
    const float* rec = p.ws + (size_t)(2 * c + ((long)c * p.chunk < ua ? 1 : 0)) * kPartialFloats;
    const float w = __builtin_amdgcn_exp2f(rec[kQueryTile * 64 + row] - mt);
    l += rec[kQueryTile * 64 + kQueryTile + row] * w;
    const float4* o4 = (const float4*)(rec + row * 64 + half * 32);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float4 v = o4[j];
      acc[4 * j] += v.x * w; acc[4 * j + 1] += v.y * w; acc[4 * j + 2] += v.z * w; acc[4 * j + 3] += v.w * w;
    }
  }
  const float inv = 1.0f / l;
  const size_t oel = (((size_t)li * p.M + qrow) * p.H + h) * 64 + half * 32;
  if (p.out_f32) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float4 w = {acc[4 * j] * inv, acc[4 * j + 1] * inv, acc[4 * j + 2] * inv, acc[4 * j + 3] * inv};
      *(float4*)(p.out + (oel + 4 * j) * 4) = w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x8 w;
#pragma unroll
      for (int e = 0; e < 8; ++e) w[e] = (__bf16)(acc[8 * j + e] * inv);
      *(bf16x8*)(p.out + (oel + 8 * j) * 2) = w;
    }
  }
}

hipError_t launch_attn_bf16(const Geom& g, char* kv, int layer0, int nl, const void* q, void* out,
                            int n_total, float scale, char* ws, int n_wgs, bool out_f32,
                            hipStream_t s, hipEvent_t* ev) {
  AttnParams p;
  p.q = (const char*)q;
  p.out = (char*)out;
  p.kv0 = layer_k(kv, g, layer0);
  p.kv_layer_bytes = g.kv_layer_bytes;
  p.v_off = (size_t)g.H * g.cap * g.d * g.esize;
  p.ws = (float*)ws;
  p.H = g.H; p.M = g.M; p.cap = g.cap; p.n_total = n_total; p.nl = nl;
  p.QB = (g.M + kQueryTile - 1) / kQueryTile;
  p.T = (n_total + kSlotTile - 1) / kSlotTile;
  const long total = (long)nl * g.H * p.QB * p.T;
  if (total > 0x7FFFFFFFL) return hipErrorInvalidValue;
  p.total_units = (int)total;
  if (n_wgs > kMaxAttnWgs) n_wgs = kMaxAttnWgs;
  n_wgs &= ~7;
  if (n_wgs < 8) n_wgs = 8;
  p.chunk = (int)((total + n_wgs - 1) / n_wgs);
  p.c = scale * 1.4426950408889634f;
  p.out_f32 = out_f32 ? 1 : 0;
  if (ev && hipEventRecord(ev[0], s) != hipSuccess) return hipErrorUnknown;
  hipLaunchKernelGGL(attn_bf16_kernel, dim3((unsigned)n_wgs), dim3(256), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev && hipEventRecord(ev[1], s) != hipSuccess) return hipErrorUnknown;
  const int items = nl * g.H * p.QB;
  hipLaunchKernelGGL(attn_combine_kernel, dim3((unsigned)items), dim3(256), 0, s, p);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev && hipEventRecord(ev[2], s) != hipSuccess) return hipErrorUnknown;
  return hipSuccess;
}

}  // namespace ovggt
