// Activation Value Rating (paper Eq. 5), activation smoothing (Eq. 6, optional),
// anchor flags (Sec. 3.3) and the fixed-budget selection (Eq. 8) in one launch.
//
// Phase 1 (all workgroups): one wave per new token reduces the token's residual
// row to ss = sum of squares in fp32 with a fixed balanced-tree order -- lane l
// owns E consecutive elements, sums their squares pairwise in registers, then
// six xor-butterfly steps add neighbouring lanes -- so the value is bit-for-bit
// reproducible by a plain pairwise sum on any machine.  HBM-bound: each row is
// read once with 16-byte loads.
//
// While its rows load, every workgroup also counts its share of the cached
// entries by the 11 leading bits of their score words (LDS histogram, flushed
// to per-layer counters in memory with one device-scope atomic per occupied bin).
//
// Phase 2 (the workgroup that arrives last for a layer, found with an arrival
// counter; nobody waits): if more than B entries are resident, find the E =
// n - B lowest-ranked evictable entries under the total order (ss ascending,
// token id descending) on the 64-bit key (ss bits, ~id): the counters give the
// threshold's first-level bin, one pass over the score words marks what lies
// below it and collects what lies in it, a second 11-bit level over those
// candidates leaves a handful of keys that one wave orders (ids included).
// Populations that defeat the two levels (thousands of keys in one bin, more
// than 64 equal in 22 leading bits) take a streaming 8-bit radix selection.
// Then emit the move list in ascending slot order.
#include "ovggt_internal.h"
#include "../../include/ovggt.h"

namespace ovggt {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
// Tokens scored per wave and round when many layers are batched (one round covers 24 layers of 1374
// rows with 10 workgroups each; measured 23 us with 4 rows in flight per wave, 19.5 us with 9,
// 17.8 us once the wave's scores leave in one store instruction).
constexpr int kRowsPerWave = 9;
constexpr int kMaxSelChunks = 128;          // n_total <= 128 * 1024 slots

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// ---- phase 1 ---------------------------------------------------------------
template <int E, bool BF16>
__device__ inline float row_sum_sq(const char* row, int C, int lane) {
  float p[E];
  const int first = lane * E;
  if constexpr (BF16) {
    const uint16_t* r = (const uint16_t*)row;
    if constexpr (E >= 8) {
      if ((C & 7) == 0) {
#pragma unroll
        for (int j = 0; j < E; j += 8) {
          uint4 w = {0u, 0u, 0u, 0u};
          if (first + j < C) w = *(const uint4*)(r + first + j);
          const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const float a = __uint_as_float(ww[t] << 16), b = __uint_as_float(ww[t] & 0xFFFF0000u);
            p[j + 2 * t] = __fmul_rn(a, a);
            p[j + 2 * t + 1] = __fmul_rn(b, b);
          }
        }
        goto tree;
      }
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const float a = (first + j < C) ? bf16_to_f32(r[first + j]) : 0.f;
      p[j] = __fmul_rn(a, a);
    }
  } else {
    const float* r = (const float*)row;
    if constexpr (E >= 4) {
      if ((C & 3) == 0) {
#pragma unroll
        for (int j = 0; j < E; j += 4) {
          float4 w = {0.f, 0.f, 0.f, 0.f};
          if (first + j < C) w = *(const float4*)(r + first + j);
          p[j] = __fmul_rn(w.x, w.x); p[j + 1] = __fmul_rn(w.y, w.y);
          p[j + 2] = __fmul_rn(w.z, w.z); p[j + 3] = __fmul_rn(w.w, w.w);
        }
        goto tree;
      }
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const float a = (first + j < C) ? r[first + j] : 0.f;
      p[j] = __fmul_rn(a, a);
    }
  }
tree:
#pragma unroll
  for (int w = 1; w < E; w *= 2)
#pragma unroll
    for (int j = 0; j < E; j += 2 * w) p[j] = __fadd_rn(p[j], p[j + w]);
  float v = p[0];
#pragma unroll
  for (int off = 1; off < 64; off *= 2) v = __fadd_rn(v, __shfl_xor(v, off, 64));
  return v;
}

// Phase 1 of one workgroup for a compile-time E.  A wave takes R consecutive tokens per round;
// their loads are independent, so all of them are in flight before the first reduction.  R = 1
// spreads a single layer's rows over as many CUs as possible, R = kRowsPerWave amortises the
// per-workgroup arrival when the launch covers many layers.
template <int E, bool BF16, int R>
__device__ inline void score_rows(const char* rbase, size_t row_bytes, int C, int M, const uint8_t* anchors_layer,
                                  float* ss_new, uint8_t* flags_new) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int tok0 = (blockIdx.x * kSelWaves + wave) * R; tok0 < M; tok0 += gridDim.x * kSelWaves * R) {
    float v[R];
#pragma unroll
    for (int r = 0; r < R; ++r)
      v[r] = row_sum_sq<E, BF16>(rbase + (size_t)min(tok0 + r, M - 1) * row_bytes, C, lane);
    // Every lane holds every row's sum after the butterfly: lane r publishes row r, so the wave's
    // R consecutive tokens leave in one store instruction for the scores and one for the flags.
    // Device-coherent (write-through) stores: the selection may run on another XCD, and a
    // device-scope release fence per workgroup (an L2 write-back each) would cost far more.
    float mine = v[0];
#pragma unroll
    for (int r = 1; r < R; ++r) mine = lane == r ? v[r] : mine;
    const int tok = tok0 + lane;
    if (lane < R && tok < M) {
      __hip_atomic_store(&ss_new[tok], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&flags_new[tok], (uint8_t)((anchors_layer && anchors_layer[tok]) ? 1 : 0),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// ---- activation smoothing (Eq. 6), by the workgroup that saw all scores arrive -------------
// s = sqrt(ss) for every new token; patch tokens (row-major ph x pw map behind the n_special aux
// tokens) become alpha * (G * S) + (1 - alpha) * S with the border replicated, aux tokens keep s.
// The result replaces ss as the token's rank key.  fp32 throughout, every operation rounded on its
// own (contraction off, sqrtf is the correctly rounded one: the hardware's approximate square root
// is a unit in the last place off now and then), taps added left to right in kernel order: the CPU
// reference repeats exactly this sequence.  `raw` is scratch for M floats.
__device__ inline void smooth_new_scores(const SmoothParams& sm, int M, float* key, float* raw) {
#pragma clang fp contract(off)
  for (int i = threadIdx.x; i < M; i += kSelThreads) raw[i] = __builtin_sqrtf(key[i]);
  __syncthreads();
  const float one_minus = 1.0f - sm.alpha;
  for (int i = threadIdx.x; i < M; i += kSelThreads) {
    float v = raw[i];
    if (i >= sm.n_special) {
      const int p = i - sm.n_special, y = p / sm.pw, x = p - y * sm.pw;
      float conv = 0.f;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int yy = min(max(y + t / 3 - 1, 0), sm.ph - 1), xx = min(max(x + t % 3 - 1, 0), sm.pw - 1);
        const float prod = sm.g[t] * raw[sm.n_special + yy * sm.pw + xx];
        conv = t == 0 ? prod : conv + prod;
      }
      const float blur = sm.alpha * conv, keep = one_minus * v;
      v = blur + keep;
    }
    key[i] = v;
  }
  __syncthreads();
}

// ---- phase 2 helpers ---------------------------------------------------------
constexpr int kHoleListCap = 2048;   // hole-list entries mirrored in LDS (longer lists are read back from memory)
struct SelShared {
  uint32_t hist[256][64];          // histogram selection: the candidate lists (score words, then slots); streaming
                                   // selection: one histogram column per lane id in rows 0..127 (two 16-bit bins a word)
  uint32_t level[2][kSelHistBins]; // histogram selection: first-level counts (a workgroup's share of the cache, then
                                   // the new frame's tokens) and second-level counts of the candidates
  uint32_t cnt[256];
  uint32_t evmap[kMaxSelChunks * kSelThreads / 32];   // evict bit per slot, slot order
  uint32_t candmap[kMaxSelChunks * kSelThreads / 32]; // histogram selection: slots whose key lies in the threshold's bin
  uint32_t scan_tmp[2][kSelWaves];
  uint32_t digit, rank, bucket, is_last, n_evictable, bad;
  uint32_t n_cand, n_final;        // histogram selection: entries of the candidate list, of the final list
  uint32_t final_list[64];         // candidate-list positions of the keys that the last wave step orders
  uint32_t hole_list[kHoleListCap]; // the first entries of the hole list, for the movers' look-up
};

// Histogram selection: sizes of its lists.
constexpr int kCandCap = 8192;     // candidates (keys in the threshold's first-level bin) held in LDS
constexpr int kFinalCap = 64;      // keys that still tie after the second level: ordered by one wave
static_assert(sizeof(((SelShared*)nullptr)->hist) == 2 * kCandCap * sizeof(uint32_t), "candidate lists overlay hist");

constexpr uint32_t kNotEvictable = 0xFFFFFFFFu;   // score word of protected / absent slots (no real score maps to it)

// Score word of a slot: the fp32 bit pattern of ss (order-preserving for ss >= 0);
// NaN or negative values rank lowest (0) and are reported.
__device__ inline uint32_t score_word(float ss, bool* bad) {
  uint32_t b = __float_as_uint(ss);
  if (ss != ss || (b & 0x80000000u)) { b = 0u; *bad = true; }
  return b;
}

// From the 256 bin counts in sh.cnt: the digit whose bucket holds the rank-th smallest candidate
// (sh.digit), the rank inside that bucket (sh.rank), the bucket's size (sh.bucket) and the number
// of candidates (sh.n_evictable).  Ends with a barrier.
__device__ inline void pick_digit(SelShared& sh, uint32_t rank) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (wave == 0) {
    uint32_t c4[4];
    uint32_t s = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) { c4[j] = sh.cnt[4 * lane + j]; s += c4[j]; }
    uint32_t inc = s;
#pragma unroll
    for (int off = 1; off < 64; off *= 2) {
      const uint32_t y = __shfl_up(inc, off, 64);
      if (lane >= off) inc += y;
    }
    uint32_t before = inc - s;
    if (lane == 63) sh.n_evictable = inc;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (before < rank && rank <= before + c4[j]) {
        sh.digit = 4 * lane + j; sh.rank = rank - before; sh.bucket = c4[j];
      }
      before += c4[j];
    }
  }
  __syncthreads();
}

// One radix pass of the streaming selection (keys re-read from memory): histogram of an 8-bit digit
// of the candidates (digit_of(chunk) < 0: not a candidate), then the digit whose bucket holds the
// rank-th smallest candidate.  Results in sh.digit / sh.rank / sh.bucket (and sh.n_evictable =
// number of candidates).
template <typename DigitOf>
__device__ inline void radix_pass(SelShared& sh, int n_iter, uint32_t rank, DigitOf digit_of) {
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid; i < 128 * 64; i += kSelThreads) (&sh.hist[0][0])[i] = 0u;
  __syncthreads();
  // digits of 8 chunks are fetched together so their loads overlap
  for (int c0 = 0; c0 < n_iter; c0 += 8) {
    int dg[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) dg[j] = c0 + j < n_iter ? digit_of(c0 + j) : -1;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (dg[j] >= 0) atomicAdd(&sh.hist[dg[j] >> 1][lane], 1u << (16 * (dg[j] & 1)));
  }
  __syncthreads();
  {   // column sums: thread -> (bin, quarter of the 64 columns)
    const int bin = tid >> 2, quarter = tid & 3;
    uint32_t s = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int col = quarter * 16 + ((j + (lane >> 2)) & 15);   // 64 distinct columns per wave read
      s += (sh.hist[bin >> 1][col] >> (16 * (bin & 1))) & 0xFFFFu;
    }
    s += __shfl_xor(s, 1, 64);
    s += __shfl_xor(s, 2, 64);
    if (quarter == 0) sh.cnt[bin] = s;
  }
  __syncthreads();
  pick_digit(sh, rank);
}

// timing builds leave 10 ns timestamps of the phases in the control block's padding
#ifdef OVGGT_TRACE
#define TSTAMP(k) do { if (tid == 0) ctrl->pad[k] = (uint32_t)wall_clock64(); } while (0)
#else
#define TSTAMP(k) do { } while (0)
#endif

// The ordered move list from the evict bitmap in sh.evmap (complete, and a barrier behind it),
// and the same moves keyed by source: mvmap[j] = destination of the entry in slot B + j, or
// kNoMove (read by the append that applies an outstanding compaction).
// Holes (evicted slots below B) are sparse: a thread takes PP consecutive 32-slot words of the
// bitmap below B, and one scan over the per-thread counts gives it the list position of its first
// hole.  Movers (kept slots at or above B) are dense: one slot per thread and round, positions from
// a ballot and the per-wave totals; the r-th mover looks its destination up in the hole list.
__device__ inline void emit_moves(SelShared& sh, const Geom& g, Ctrl* ctrl, uint32_t* mvdst, uint32_t* mvsrc,
                                  uint32_t* mvmap, uint32_t* evbits, int n_total, bool budget_error, int pass) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  (void)pass;
  const int n_words = (n_total + 31) >> 5;
  if (evbits)
    for (int wi = tid; wi < n_words; wi += kSelThreads) evbits[wi] = sh.evmap[wi];
  const uint32_t m_cap = (uint32_t)g.M;
  const int hole_words = (g.B + 31) >> 5;
  const int PP = (hole_words + kSelThreads - 1) / kSelThreads;   // <= 4
  uint32_t hw[4];
  uint32_t nh = 0;
  const bool wave_has_words = wave * 64 * PP < hole_words;       // the other waves only keep the barriers company
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    hw[j] = 0u;
    const int wi = tid * PP + j;
    if (j < PP && wi < hole_words) {
      const int s0 = wi << 5;
      const uint32_t below_b = s0 + 32 <= g.B ? 0xFFFFFFFFu : ((1u << (g.B - s0)) - 1u);
      hw[j] = budget_error ? 0u : sh.evmap[wi] & below_b;
      nh += __popc(hw[j]);
    }
  }
  uint32_t inc_h = nh;
  if (wave_has_words) {
#pragma unroll
    for (int off = 1; off < 64; off *= 2) {
      const uint32_t yh = __shfl_up(inc_h, off, 64);
      if (lane >= off) inc_h += yh;
    }
  }
  if (lane == 63) sh.scan_tmp[0][wave] = inc_h;
  __syncthreads();
  uint32_t base_h = 0, tot_h = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const uint32_t th = sh.scan_tmp[0][w];
    if (w < wave) base_h += th;
    tot_h += th;
  }
  if (wave_has_words) {                                          // the hole list (entries beyond M are never used)
    uint32_t hp = base_h + inc_h - nh;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t s0 = (uint32_t)(tid * PP + j) << 5;
      uint32_t b = hw[j];
      while (b) {
        const uint32_t hole = s0 + (uint32_t)__builtin_ctz(b);
        if (hp < m_cap) mvdst[hp] = hole;
        if (hp < (uint32_t)kHoleListCap) sh.hole_list[hp] = hole;
        ++hp; b &= b - 1;
      }
    }
  }
  const uint64_t lanes_below = (1ull << lane) - 1ull;
  const uint32_t n_dst = min(tot_h, m_cap);
  uint32_t tot_m = 0;
  for (int s0 = g.B; s0 < g.B + g.M; s0 += kSelThreads) {
    const int slot = s0 + tid;
    const bool mover = !budget_error && slot < n_total && !((sh.evmap[slot >> 5] >> (slot & 31)) & 1u);
    const uint64_t bl = __ballot(mover);
    __syncthreads();                     // the hole list is visible; the previous round's totals have been read
    if (lane == 0) sh.scan_tmp[1][wave] = (uint32_t)__popcll(bl);
    __syncthreads();
    uint32_t base_m = tot_m;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const uint32_t tm = sh.scan_tmp[1][w];
      if (w < wave) base_m += tm;
      tot_m += tm;
    }
    const uint32_t mp = base_m + (uint32_t)__popcll(bl & lanes_below);
    uint32_t to = kNoMove;
    if (mover && mp < n_dst) to = mp < (uint32_t)kHoleListCap ? sh.hole_list[mp] : mvdst[mp];
    if (mover && mp < m_cap) mvsrc[mp] = (uint32_t)slot;
    if (slot < g.B + g.M) mvmap[slot - g.B] = to;
  }
  const bool consistent = !budget_error && tot_h == tot_m && tot_h <= m_cap;
  if (!consistent) {                                             // uniform: nothing moves
    __syncthreads();
    for (int j = tid; j < g.M; j += kSelThreads) mvmap[j] = kNoMove;
  }
  if (tid == 0) {
    ctrl->n_moves = consistent ? tot_h : 0u;
    uint32_t st = 0;
    if (budget_error || !consistent) st |= OVGGT_STATUS_BUDGET;
    if (sh.bad) st |= OVGGT_STATUS_NONFINITE;
    if (st) atomicOr(&ctrl->status, st);
    TSTAMP(12);
    OVGGT_TRACE_ONLY(ctrl->pad[13] = (uint32_t)pass;)
  }
}

// Streaming radix selection by one workgroup, for any population of keys: 8-bit digits of the
// 64-bit key (score word, inverted id), every pass re-reads the score words (and, once equal
// scores straddle the threshold, the ids) from memory; passes stop as soon as a whole bucket goes.
// The histogram selection falls back to it when its lists overflow.
__device__ inline void select_streaming(SelShared& sh, const Geom& g, const float* ss, const uint32_t* ids,
                                        const uint8_t* flags, Ctrl* ctrl, uint32_t* mvdst, uint32_t* mvsrc,
                                        uint32_t* mvmap, uint32_t* evbits, int n_total) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_chunks = (n_total + kSelThreads - 1) / kSelThreads;
  const uint32_t n_evict = (uint32_t)(n_total - g.B);
  bool bad = false;
  auto word = [&](int c) -> uint32_t {               // branch-free so that loads of several chunks overlap
    const int i = c * kSelThreads + tid;
    const int ic = i < n_total ? i : n_total - 1;
    const uint8_t f = flags[ic];
    const uint32_t w = score_word(ss[ic], &bad);
    return (i >= n_total || f != 0) ? kNotEvictable : w;
  };
  auto idw = [&](int c) -> uint32_t {
    const int i = c * kSelThreads + tid;
    return 0xFFFFFFFFu - ids[i < n_total ? i : n_total - 1];
  };
  if (tid == 0) sh.bad = 0;
  TSTAMP(1);

  // radix select of the n_evict-th smallest (score word, inverted id) pair
  uint32_t rank = n_evict;
  int pass = 0;
  bool budget_error = false, done = false;
  uint32_t pre_hi = 0, pre_lo = 0;
#pragma nounroll
  for (; pass < 4 && !done; ++pass) {
    const int shift = 24 - 8 * pass;
    radix_pass(sh, n_chunks, rank, [&](int c) -> int {
      const uint32_t w = word(c);
      if (w == kNotEvictable) return -1;
      if (pass > 0 && (w >> (shift + 8)) != (pre_hi >> (shift + 8))) return -1;
      return (int)((w >> shift) & 255u);
    });
    if (pass == 0 && sh.n_evictable < n_evict) { budget_error = true; break; }   // |P| > B
    pre_hi |= sh.digit << shift;
    rank = sh.rank;
    done = (rank == sh.bucket);          // the whole bucket goes
    __syncthreads();
  }
  const int hi_shift = pass > 0 ? 24 - 8 * (pass - 1) : 24;
  int lo_shift = 32;                      // 32: ids did not have to be consulted
  if (!done && !budget_error) {
#pragma nounroll
    for (int p2 = 0; p2 < 4 && !done; ++p2) {
      const int shift = 24 - 8 * p2;
      radix_pass(sh, n_chunks, rank, [&](int c) -> int {
        if (word(c) != pre_hi) return -1;
        const uint32_t w = idw(c);
        if (p2 > 0 && (w >> (shift + 8)) != (pre_lo >> (shift + 8))) return -1;
        return (int)((w >> shift) & 255u);
      });
      pre_lo |= sh.digit << shift;
      rank = sh.rank;
      done = (rank == sh.bucket);
      lo_shift = shift;
      __syncthreads();
    }
  }
  if (bad) sh.bad = 1;

  // evict bit per slot, published in slot order: the ballot of one chunk over one wave covers 64
  // consecutive slots
  for (int c = 0; c < n_chunks; ++c) {
    bool ev = false;
    if (!budget_error) {
      const uint32_t w = word(c);
      if (w != kNotEvictable) {
        if (lo_shift == 32) ev = (w >> hi_shift) <= (pre_hi >> hi_shift);
        else ev = w < pre_hi || (w == pre_hi && (idw(c) >> lo_shift) <= (pre_lo >> lo_shift));
      }
    }
    const uint64_t bl = __ballot(ev);
    if (lane == 0) {
      sh.evmap[(c * kSelThreads >> 5) + 2 * wave] = (uint32_t)bl;
      sh.evmap[(c * kSelThreads >> 5) + 2 * wave + 1] = (uint32_t)(bl >> 32);
    }
  }
  __syncthreads();
  TSTAMP(11);
  emit_moves(sh, g, ctrl, mvdst, mvsrc, mvmap, evbits, n_total, budget_error, pass);
}

// ---- histogram selection -----------------------------------------------------------------------
// The first radix level (the 11 bits below the sign of a score word, kSelHistBins bins) is counted
// by every workgroup of the launch over its share of the cached entries, in an LDS histogram that
// is flushed into the layer's counters in memory with one device-scope atomic per occupied bin; the
// workgroup that selects adds the new frame's tokens, finds the threshold's bin, and then reads the
// score words once: entries in lower bins go, entries in the bin become candidates (a bitmap, then
// an LDS list) and are counted by their next 11 bits.  The second level usually leaves a handful of
// keys, which one wave orders by (score word, inverted id).  Inputs that defeat this (more than
// kCandCap keys in one first-level bin, more than kFinalCap keys equal in their leading 22 bits at
// the threshold) take the streaming radix selection instead.  One CU executes this phase: 1024
// threads cost 16 cycles per instruction slot, which is what bounds the pass over the score words.

// Inclusive scan over the 2 * 1024 bin counts (thread t owns bins 2t and 2t+1): the bin that holds
// the rank-th smallest key (sh.digit), the rank inside it (sh.rank), its size (sh.bucket) and the
// total (sh.n_evictable).  rank > total leaves the first three unwritten.  Ends with a barrier.
__device__ inline void pick_bin(SelShared& sh, uint32_t c0, uint32_t c1, uint32_t rank) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t s = c0 + c1;
  uint32_t inc = s;
#pragma unroll
  for (int off = 1; off < 64; off *= 2) {
    const uint32_t y = __shfl_up(inc, off, 64);
    if (lane >= off) inc += y;
  }
  if (lane == 63) sh.scan_tmp[0][wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const uint32_t t = sh.scan_tmp[0][w];
    if (w < wave) base += t;
    tot += t;
  }
  uint32_t before = base + inc - s;
  if (before < rank && rank <= before + c0) { sh.digit = 2 * tid; sh.rank = rank - before; sh.bucket = c0; }
  before += c0;
  if (before < rank && rank <= before + c1) { sh.digit = 2 * tid + 1; sh.rank = rank - before; sh.bucket = c1; }
  if (tid == 0) sh.n_evictable = tot;
  __syncthreads();
}

// Every workgroup, before it announces its arrival, counts its share of the cached entries
// [0, n_old) by first-level bin into `lh` (LDS, zero, a barrier behind the clearing).  Protected
// entries do not take part.  The share's first two entries per thread are requested before the
// frame's rows are scored (hist_share_load) and counted afterwards, so their latency hides there.
struct HistShare { uint32_t w[2]; int next, end; };

__device__ inline uint32_t evictable_word(float ssv, uint8_t flag) {
  bool bad = false;                                     // bad scores are reported by the workgroup that selects
  const uint32_t w = score_word(ssv, &bad);
  return flag ? kNotEvictable : w;
}

__device__ inline HistShare hist_share_load(const float* ss, const uint8_t* flags, int n_old) {
  HistShare h;
  const int per = (n_old + (int)gridDim.x - 1) / (int)gridDim.x;
  const int i0 = blockIdx.x * per + threadIdx.x;
  h.end = min(((int)blockIdx.x + 1) * per, n_old);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int i = i0 + j * kSelThreads;
    const int ic = min(i, n_old - 1);                   // n_old >= 1 whenever a selection runs
    const uint32_t w = evictable_word(ss[ic], flags[ic]);
    h.w[j] = i < h.end ? w : kNotEvictable;
  }
  h.next = i0 + 2 * kSelThreads;
  return h;
}

__device__ inline void hist_share_count(uint32_t* lh, const HistShare& h, const float* ss, const uint8_t* flags) {
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if (h.w[j] != kNotEvictable) atomicAdd(&lh[h.w[j] >> 20], 1u);
  for (int i = h.next; i < h.end; i += kSelThreads) {
    const uint32_t w = evictable_word(ss[i], flags[i]);
    if (w != kNotEvictable) atomicAdd(&lh[w >> 20], 1u);
  }
}

// Adds the occupied bins of `lh` to the layer's counters and leaves `lh` zero (a barrier in front).
__device__ inline void hist_flush(uint32_t* lh, uint32_t* ghist) {
  __syncthreads();
#pragma unroll
  for (int b = threadIdx.x; b < kSelHistBins; b += kSelThreads) {
    const uint32_t v = lh[b];
    if (v) {
      __hip_atomic_fetch_add(&ghist[b], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      lh[b] = 0u;
    }
  }
}

constexpr int kQuadBatch = 6;       // 16-byte score loads (4 slots each) a thread keeps in flight
struct QuadBatch { float4 sv[kQuadBatch]; uint32_t fl[kQuadBatch]; };

__device__ inline void select_hist(SelShared& sh, const Geom& g, const float* ss, const uint32_t* ids,
                                   const uint8_t* flags, Ctrl* ctrl, uint32_t* mvdst, uint32_t* mvsrc,
                                   uint32_t* mvmap, uint32_t* evbits, uint32_t* ghist, int n_total) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_old = n_total - g.M;
  const uint32_t n_evict = (uint32_t)(n_total - g.B);
  uint32_t* lh = sh.level[0];                           // first level, zero on entry
  uint32_t* h2 = sh.level[1];                           // second level, zero on entry
  uint32_t* cand_w = &sh.hist[0][0];                    // candidates: score word and slot
  uint32_t* cand_slot = cand_w + kCandCap;
  bool bad = false;
  TSTAMP(1);
  // first level: the other workgroups' counts of the cached entries, plus the frame's own tokens
  const uint2 gh = *(const uint2*)(ghist + 2 * tid);
  const int n_quads = (n_total + 3) >> 2;
  auto load_batch = [&](QuadBatch& qb, int q0) {
#pragma unroll
    for (int j = 0; j < kQuadBatch; ++j) {
      const int q = min(q0 + j * kSelThreads + tid, n_quads - 1);
      qb.sv[j] = ((const float4*)ss)[q];
      qb.fl[j] = ((const uint32_t*)flags)[q];
    }
  };
  QuadBatch qb0;
  if (tid == 0) { sh.bad = 0; sh.n_cand = 0; sh.n_final = 0; }
  for (int wi = tid; wi < (n_total + 31) >> 5; wi += kSelThreads) sh.evmap[wi] = sh.candmap[wi] = 0u;   // a barrier follows below
  for (int i0 = n_old + tid; i0 < n_total; i0 += 2 * kSelThreads) {    // two loads in flight per thread
    uint32_t w[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int i = i0 + j * kSelThreads;
      const int ic = min(i, n_total - 1);
      const uint32_t x = evictable_word(ss[ic], flags[ic]);
      w[j] = i < n_total ? x : kNotEvictable;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
      if (w[j] != kNotEvictable) atomicAdd(&lh[w[j] >> 20], 1u);
  }
  load_batch(qb0, 0);                                   // in flight while the bin is picked
  __syncthreads();
  pick_bin(sh, gh.x + lh[2 * tid], gh.y + lh[2 * tid + 1], n_evict);
  // the counters start the next frame at zero (written through; the values above are in registers)
  __hip_atomic_store(&ghist[2 * tid], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(&ghist[2 * tid + 1], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const bool budget_error = sh.n_evictable < n_evict;   // |P| > B
  const uint32_t bin1 = sh.digit, rank1 = sh.rank;
  const bool all1 = rank1 == sh.bucket;                 // the whole bin goes
  TSTAMP(2);
  // One pass over the score words, four consecutive slots per thread and load, in batches of
  // kQuadBatch loads per thread; the next batch is requested before the current one is used (the
  // first one before the bin was picked).  Two bitmaps: "below the bin" (w < thr_lo: the entry
  // goes) and "in the bin" (thr_lo <= w < thr_hi: a candidate).  Protected and absent slots carry
  // the all-ones word, which is neither.
  const uint32_t thr_lo = budget_error ? 0u : (all1 ? bin1 + 1u : bin1) << 20;
  const uint32_t thr_hi = (budget_error || all1) ? thr_lo : thr_lo + (1u << 20);   // at most 2^31
  auto use_batch = [&](const QuadBatch& qb, int q0) {
#pragma unroll
    for (int j = 0; j < kQuadBatch; ++j) {
      const int q = q0 + j * kSelThreads + tid;
      if (q < n_quads) {
        const int base = q << 2, n_valid = n_total - base;
        uint32_t w[4] = {__float_as_uint(qb.sv[j].x), __float_as_uint(qb.sv[j].y), __float_as_uint(qb.sv[j].z),
                         __float_as_uint(qb.sv[j].w)};
        const uint32_t w_max = max(max(w[0], w[1]), max(w[2], w[3]));
        if (qb.fl[j] != 0u || n_valid < 4 || w_max > 0x7F800000u) {   // rare: protected, tail, NaN or negative
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bool in_range = e < n_valid;
            const bool odd = w[e] > 0x7F800000u;        // ranks lowest, reported
            if (odd && in_range) bad = true;
            if (odd) w[e] = 0u;
            if (!in_range || ((qb.fl[j] >> (8 * e)) & 255u) != 0u) w[e] = kNotEvictable;
          }
        }
        uint32_t nib_lo = 0, nib_hi = 0;
#pragma unroll
        for (int e = 3; e >= 0; --e) {
          nib_lo = 2u * nib_lo + (w[e] < thr_lo ? 1u : 0u);
          nib_hi = 2u * nib_hi + (w[e] < thr_hi ? 1u : 0u);
        }
        const uint32_t sft = base & 31;
        if (nib_lo) atomicOr(&sh.evmap[base >> 5], nib_lo << sft);
        if (nib_hi != nib_lo) atomicOr(&sh.candmap[base >> 5], (nib_hi ^ nib_lo) << sft);
      }
    }
  };
  constexpr int kStep = kQuadBatch * kSelThreads;
  for (int q0 = 0; q0 < n_quads; q0 += 2 * kStep) {
    QuadBatch qb1;
    if (q0 + kStep < n_quads) load_batch(qb1, q0 + kStep);          // uniform
    use_batch(qb0, q0);
    if (q0 + 2 * kStep < n_quads) load_batch(qb0, q0 + 2 * kStep);
    if (q0 + kStep < n_quads) use_batch(qb1, q0 + kStep);
  }
  if (bad) sh.bad = 1;
  __syncthreads();
  TSTAMP(5);
  // the candidates (few) to a list, with their score words, and counted by their next 11 bits
  for (int wi = tid; wi < (n_total + 31) >> 5; wi += kSelThreads) {
    uint32_t bits = sh.candmap[wi];
    while (bits) {
      const uint32_t slot = ((uint32_t)wi << 5) + (uint32_t)__builtin_ctz(bits);
      bits &= bits - 1;
      const uint32_t b = __float_as_uint(ss[slot]);
      const uint32_t w = b > 0x7F800000u ? 0u : b;
      const uint32_t pos = atomicAdd(&sh.n_cand, 1u);
      if (pos < (uint32_t)kCandCap) { cand_w[pos] = w; cand_slot[pos] = slot; }
      atomicAdd(&h2[(w >> 9) & (kSelHistBins - 1)], 1u);
    }
  }
  __syncthreads();
  TSTAMP(3);
  const uint32_t n_cand = sh.n_cand;
  bool fallback = n_cand > (uint32_t)kCandCap;
  if (!fallback && n_cand > 0) {
    // second level over the candidates (n_cand = the bin's size, rank1 of them go)
    pick_bin(sh, h2[2 * tid], h2[2 * tid + 1], rank1);
    const uint32_t bin2 = sh.digit, rank2 = sh.rank;
    const bool all2 = rank2 == sh.bucket;
    for (uint32_t e = tid; e < n_cand; e += kSelThreads) {
      const uint32_t d2 = (cand_w[e] >> 9) & (kSelHistBins - 1), slot = cand_slot[e];
      if (d2 < bin2 || (all2 && d2 == bin2)) atomicOr(&sh.evmap[slot >> 5], 1u << (slot & 31));
      else if (d2 == bin2) {
        const uint32_t pos = atomicAdd(&sh.n_final, 1u);
        if (pos < (uint32_t)kFinalCap) sh.final_list[pos] = e;
      }
    }
    __syncthreads();
    TSTAMP(4);
    const uint32_t n_final = sh.n_final;
    fallback = n_final > (uint32_t)kFinalCap;
    if (!fallback && n_final > 0 && wave == 0) {
      // rank2 of these keys go: a key's position in the order is the number of smaller keys
      uint32_t w = 0xFFFFFFFFu, inv = 0xFFFFFFFFu, slot = 0;
      if ((uint32_t)lane < n_final) {
        const uint32_t e = sh.final_list[lane];
        w = cand_w[e]; slot = cand_slot[e];
        inv = 0xFFFFFFFFu - ids[slot];
      }
      const uint64_t key = ((uint64_t)w << 32) | inv;
      uint32_t below = 0;
      for (uint32_t j = 0; j < n_final; ++j) {
        const uint64_t kj = ((uint64_t)(uint32_t)__shfl((int)w, (int)j, 64) << 32) | (uint32_t)__shfl((int)inv, (int)j, 64);
        below += kj < key ? 1u : 0u;
      }
      if ((uint32_t)lane < n_final && below < rank2) atomicOr(&sh.evmap[slot >> 5], 1u << (slot & 31));
    }
  }
  if (fallback) {                                       // uniform: decided from shared counters behind a barrier
    select_streaming(sh, g, ss, ids, flags, ctrl, mvdst, mvsrc, mvmap, evbits, n_total);
    return;
  }
  __syncthreads();
  TSTAMP(11);
  emit_moves(sh, g, ctrl, mvdst, mvsrc, mvmap, evbits, n_total, budget_error, 2);
}

// ---- Eq. 7: rank values of the evictable slots ----------------------------------------------------
// Each source is min-max normalised over its evictable slots (all zeros when max = min) and
// weighted: (1 - beta) * d^ for history, beta * s^ for the new frame.  One fp32 operation at a
// time, in this order; the CPU reference repeats it.
//
// Workgroup-wide minimum and maximum of value_of(i), i in [0, n), over the unflagged slots.
template <typename ValueOf>
__device__ inline void block_min_max(SelShared& sh, const uint8_t* flags, int n, ValueOf value_of,
                                     float* lo_out, float* hi_out) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float inf = __builtin_inff();
  float lo = inf, hi = -inf;
  for (int i = tid; i < n; i += kSelThreads) {
    if (flags[i]) continue;
    const float x = value_of(i);
    lo = fminf(lo, x); hi = fmaxf(hi, x);
  }
#pragma unroll
  for (int off = 1; off < 64; off *= 2) {
    lo = fminf(lo, __shfl_xor(lo, off, 64));
    hi = fmaxf(hi, __shfl_xor(hi, off, 64));
  }
  float* red = (float*)sh.cnt;                               // 2 values per wave
  __syncthreads();
  if (lane == 0) { red[wave * 2] = lo; red[wave * 2 + 1] = hi; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) { lo = fminf(lo, red[w * 2]); hi = fmaxf(hi, red[w * 2 + 1]); }
  __syncthreads();                                           // sh.cnt is reused afterwards
  *lo_out = lo; *hi_out = hi;
}

// History side, spread over every workgroup of the layer's launch.  `dval` holds d_i of the slots
// below n_old, `part` the (minimum, maximum) over the evictable slots of each wave of this
// frame's diversity pass (both read-only here).  Every workgroup folds the few thousand pairs into
// the same minimum and maximum (reading all d_i and flags instead, 80 KB per workgroup, made this
// phase take 13.5 us instead of 4.8), then writes the rank values of its own share of slots over
// their scores, written through like the scores of phase 1, and counts them by first-level bin
// into `lh`, which is zero and has a barrier behind its clearing.
__device__ inline void hybrid_history_values(SelShared& sh, const HybridParams& hy, const float* dval,
                                             const float2* part, float* ss, const uint8_t* flags, int n_old,
                                             uint32_t* lh) {
#pragma clang fp contract(off)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float lo = __builtin_inff(), hi = -__builtin_inff();
  for (int i = tid; i < hy.n_part; i += kSelThreads) {
    const float2 p = part[i];
    lo = fminf(lo, p.x); hi = fmaxf(hi, p.y);
  }
#pragma unroll
  for (int off = 1; off < 64; off *= 2) {
    lo = fminf(lo, __shfl_xor(lo, off, 64));
    hi = fmaxf(hi, __shfl_xor(hi, off, 64));
  }
  float* red = (float*)sh.cnt;                               // 2 values per wave
  __syncthreads();
  if (lane == 0) { red[wave * 2] = lo; red[wave * 2 + 1] = hi; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) { lo = fminf(lo, red[w * 2]); hi = fmaxf(hi, red[w * 2 + 1]); }
  __syncthreads();                                           // sh.cnt is reused afterwards
  const float weight = 1.0f - hy.beta, range = hi - lo;
  const int per = (n_old + (int)gridDim.x - 1) / (int)gridDim.x;
  const int i1 = min(((int)blockIdx.x + 1) * per, n_old);
  for (int i = blockIdx.x * per + threadIdx.x; i < i1; i += kSelThreads) {
    if (flags[i]) continue;
    const float unit = hi == lo ? 0.f : (dval[i] - lo) / range;
    const float rv = weight * unit;
    __hip_atomic_store(&ss[i], rv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    bool bad = false;                                        // first-level count of this share
    atomicAdd(&lh[score_word(rv, &bad) >> 20], 1u);
  }
}

// New frame's side, by the workgroup that runs the selection: the slots [n_old, n_total) hold ss, or
// Eq. 6's smoothed s.
__device__ inline void hybrid_new_values(SelShared& sh, const HybridParams& hy, bool smoothed, float* ss,
                                         const uint8_t* flags, int n_old, int n_total) {
#pragma clang fp contract(off)
  float lo, hi;
  float* sn = ss + n_old;
  const uint8_t* fn = flags + n_old;
  auto value_of = [&](int i) { return smoothed ? sn[i] : __builtin_sqrtf(sn[i]); };
  block_min_max(sh, fn, n_total - n_old, value_of, &lo, &hi);
  const float range = hi - lo;
  for (int i = threadIdx.x; i < n_total - n_old; i += kSelThreads) {
    if (fn[i]) continue;
    const float unit = hi == lo ? 0.f : (value_of(i) - lo) / range;
    sn[i] = hy.beta * unit;
  }
  __syncthreads();
}

template <bool BF16>
__global__ void __launch_bounds__(kSelThreads)
score_select_kernel(Geom g, SmoothParams sm, HybridParams hy, char* meta, int layer0, const char* resid, const uint8_t* anchors,
                    int n_total, int e_per_lane) {
  __shared__ SelShared sh;
  const int layer = layer0 + blockIdx.y;
  const int li = blockIdx.y;
  char* mb = layer_meta(meta, g, layer);
  uint32_t* ids = (uint32_t*)(mb + g.off_ids);
  float* ss = (float*)(mb + g.off_ss);
  uint8_t* flags = (uint8_t*)(mb + g.off_flags);
  Ctrl* ctrl = (Ctrl*)(mb + g.off_ctrl);
  const int tid = threadIdx.x;
  const int n_old = n_total - g.M;

  OVGGT_TRACE_ONLY(if (blockIdx.x == 0 && tid == 0) ctrl->pad[15] = (uint32_t)wall_clock64();)
  // The two histogram levels start at zero in every workgroup (each counts its share of the cache
  // into the first, and whichever selects uses both); cleared in the shadow of phase 1's loads.
  const bool selecting = n_total > g.B;
  HistShare share = {};
  if (selecting) {
    const uint4 z = {0u, 0u, 0u, 0u};
    ((uint4*)&sh.level[0][0])[tid] = z;
    if (!hy.on) share = hist_share_load(ss, flags, n_old);     // used after the rows are scored
  }
  // ---- phase 1: scores and flags of the M new slots
  {
    const size_t row_bytes = (size_t)g.C * g.esize;
    const char* rbase = resid + (size_t)li * g.M * row_bytes;
    const uint8_t* al = anchors ? anchors + (size_t)li * g.M : nullptr;
    float* sn = ss + n_old;
    uint8_t* fn = flags + n_old;
    const bool many = gridDim.x * kSelWaves < (unsigned)g.M;       // the launch packs several tokens per wave
    switch (e_per_lane) {
      case 1: if (many) score_rows<1, BF16, kRowsPerWave>(rbase, row_bytes, g.C, g.M, al, sn, fn); else score_rows<1, BF16, 1>(rbase, row_bytes, g.C, g.M, al, sn, fn); break;
      case 2: if (many) score_rows<2, BF16, kRowsPerWave>(rbase, row_bytes, g.C, g.M, al, sn, fn); else score_rows<2, BF16, 1>(rbase, row_bytes, g.C, g.M, al, sn, fn); break;
      case 4: if (many) score_rows<4, BF16, kRowsPerWave>(rbase, row_bytes, g.C, g.M, al, sn, fn); else score_rows<4, BF16, 1>(rbase, row_bytes, g.C, g.M, al, sn, fn); break;
      case 8: if (many) score_rows<8, BF16, kRowsPerWave>(rbase, row_bytes, g.C, g.M, al, sn, fn); else score_rows<8, BF16, 1>(rbase, row_bytes, g.C, g.M, al, sn, fn); break;
      case 16: if (many) score_rows<16, BF16, kRowsPerWave>(rbase, row_bytes, g.C, g.M, al, sn, fn); else score_rows<16, BF16, 1>(rbase, row_bytes, g.C, g.M, al, sn, fn); break;
      case 32: if (many) score_rows<32, BF16, kRowsPerWave>(rbase, row_bytes, g.C, g.M, al, sn, fn); else score_rows<32, BF16, 1>(rbase, row_bytes, g.C, g.M, al, sn, fn); break;
      default: if (many) score_rows<64, BF16, kRowsPerWave>(rbase, row_bytes, g.C, g.M, al, sn, fn); else score_rows<64, BF16, 1>(rbase, row_bytes, g.C, g.M, al, sn, fn); break;
    }
  }
  // first histogram level of this workgroup's share of the cached entries, added to the layer's counters
  uint32_t* lh = sh.level[0];
  uint32_t* ghist = (uint32_t*)(mb + g.off_hist);
  if (selecting) {
    if (hy.on)
      hybrid_history_values(sh, hy, (const float*)(mb + g.off_dval), (const float2*)(mb + g.off_dpart), ss, flags, n_old, lh);
    else {
      __syncthreads();                         // the histogram was cleared when the kernel started
      hist_share_count(lh, share, ss, flags);
    }
    hist_flush(lh, ghist);
  }
  const bool smoothing = sm.alpha > 0.f;
  if (n_total <= g.B && !smoothing) {        // under budget and no smoothing: nothing needs the whole frame
    if (blockIdx.x == 0 && tid == 0) { ctrl->n_moves = 0; ctrl->gid_next += (uint32_t)g.M; }
    return;
  }
  // Publish this workgroup's scores and count its arrival.  The scores were written through to
  // device-coherent memory, so every wave only waits for its own stores to be acknowledged; the
  // arrival counter is a relaxed device-scope atomic, and the one workgroup that arrives last
  // invalidates its caches (acquire) before it reads what the others wrote.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0) {
    const uint32_t prev = __hip_atomic_fetch_add(&ctrl->arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = prev == gridDim.x - 1;
    if (last) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      __hip_atomic_store(&ctrl->arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      OVGGT_TRACE_ONLY(ctrl->pad[0] = (uint32_t)wall_clock64();)
    }
    sh.is_last = last ? 1u : 0u;
  }
  __syncthreads();
  if (!sh.is_last) return;

  // ---- phase 2: this workgroup saw every other one arrive
  if (tid == 0) ctrl->gid_next += (uint32_t)g.M;       // once per layer and frame: the next frame's first token id
  uint32_t* mvdst = (uint32_t*)(mb + g.off_mvdst);
  uint32_t* mvsrc = (uint32_t*)(mb + g.off_mvsrc);
  if (smoothing) {
    smooth_new_scores(sm, g.M, ss + n_old, (float*)mvdst);     // the move list is not written yet: scratch
    if (n_total <= g.B) {
      if (tid == 0) ctrl->n_moves = 0;
      return;
    }
  }
  if (hy.on) hybrid_new_values(sh, hy, smoothing, ss, flags, n_old, n_total);
  // hybrid scoring keeps the evict bitmap: the centroid's maintenance reads it
  uint32_t* evbits = hy.on ? (uint32_t*)(mb + g.off_evbits) : nullptr;
  select_hist(sh, g, ss, ids, flags, ctrl, mvdst, mvsrc, (uint32_t*)(mb + g.off_mvmap), evbits, ghist, n_total);
}

template <bool BF16>
static void launch_variant(const Geom& g, const SmoothParams& sm, const HybridParams& hy, char* meta, int layer0, int nl, const void* resid,
                           const uint8_t* anchors, int n_total, int e, hipStream_t s) {
  // One workgroup fits a CU (1024 threads and the selection's LDS set the footprint), so the
  // launch stays within one round of the chip: a single layer spreads its rows one per wave, a
  // batch of layers gives each workgroup several rounds of kRowsPerWave rows per wave.
  static const int n_cus = [] {                       // once per process (thread-safe initialisation)
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      return v;
    return 256;
  }();
  int gx = (g.M + kSelWaves - 1) / kSelWaves;
  if ((long)gx * nl > n_cus) gx = n_cus / nl > 0 ? n_cus / nl : 1;
  dim3 grid((unsigned)gx, (unsigned)nl);
  hipLaunchKernelGGL((score_select_kernel<BF16>), grid, dim3(kSelThreads), 0, s, g, sm, hy, meta,
                     layer0, (const char*)resid, anchors, n_total, e);
}

hipError_t launch_score_select(const Geom& g, const SmoothParams& sm, const HybridParams& hy, char* meta, int layer0, int nl, const void* resid,
                               const uint8_t* anchors, int n_total, hipStream_t s) {
  int cp = 1;
  while (cp < g.C) cp *= 2;
  const int e = cp >= 64 ? cp / 64 : 1;
  if (g.esize == 2) launch_variant<true>(g, sm, hy, meta, layer0, nl, resid, anchors, n_total, e, s);
  else launch_variant<false>(g, sm, hy, meta, layer0, nl, resid, anchors, n_total, e, s);
  return hipGetLastError();
}

}  // namespace ovggt
