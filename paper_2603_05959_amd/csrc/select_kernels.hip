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
// Phase 2 (the workgroup that arrives last for a layer, found with an arrival
// counter; nobody waits): if more than B entries are resident, find the E =
// n - B lowest-ranked evictable entries under the total order (ss ascending,
// token id descending) by an 8-bit-digit radix select on the 64-bit key
// (ss bits, ~id) held in registers, with a per-lane-column LDS histogram (no
// bank or address conflicts); passes stop as soon as a whole bucket is evicted,
// and the id half is only consulted when equal scores straddle the threshold.
// Then emit the move list in ascending slot order.
#include "ovggt_internal.h"
#include <type_traits>
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
struct SelShared {
  uint32_t hist[256][64];          // one column per lane id; rows 0..127 are cleared and read (streaming passes pack
                                   // two 16-bit bins per word there), rows above only absorb the marker word
  uint32_t wave_hist[kSelWaves][256];   // later passes over register-resident keys; zero between uses
  uint32_t cnt[256];
  uint32_t evmap[kMaxSelChunks * kSelThreads / 32];   // evict bit per slot, slot order
  uint32_t scan_tmp[2][kSelWaves];
  uint32_t totals[2];
  uint32_t digit, rank, bucket, is_last, n_evictable, bad;
};

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
__device__ inline void radix_pass(SelShared& sh, int n_iter, uint32_t rank, DigitOf digit_of, uint32_t* ts = nullptr) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 128 * 64; i += kSelThreads) (&sh.hist[0][0])[i] = 0u;
  __syncthreads();
#ifdef OVGGT_TRACE
  if (ts && tid == 0) ts[0] = (uint32_t)wall_clock64();
#endif
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
#ifdef OVGGT_TRACE
  if (ts && tid == 0) ts[1] = (uint32_t)wall_clock64();
#endif
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
#ifdef OVGGT_TRACE
  if (ts && tid == 0) ts[2] = (uint32_t)wall_clock64();
#endif
  pick_digit(sh, rank);
}

// First pass over register-resident keys: every key of the thread is counted by its leading byte
// into the per-lane-column histogram, which the workgroup cleared when the kernel started.  Real
// score words are non-negative floats, so their leading byte is below 128; the word that marks a
// protected or absent slot has 255 and lands in a row that nobody clears or reads -- no test per key.
template <int KPT>
__device__ inline void first_pass_registers(SelShared& sh, const uint32_t (&kw)[KPT > 0 ? KPT : 1], uint32_t rank, uint32_t* ts) {
  const int tid = threadIdx.x, lane = tid & 63;
  uint32_t* col = &sh.hist[0][0] + lane;
#pragma unroll
  for (int c = 0; c < KPT; ++c) {
    atomicAdd(col + (kw[c] >> 24) * 64u, 1u);
  }
  __syncthreads();
#ifdef OVGGT_TRACE
  if (ts && tid == 0) ts[1] = (uint32_t)wall_clock64();
#endif
  {   // column sums: thread -> (bin, eighth of the 64 columns); a wave's 64 reads hit 64 distinct columns
    const int bin = tid >> 3, part = tid & 7;
    uint32_t s = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += sh.hist[bin][part * 8 + ((j + (lane >> 3)) & 7)];
    s += __shfl_xor(s, 1, 64);
    s += __shfl_xor(s, 2, 64);
    s += __shfl_xor(s, 4, 64);
    if (part == 0) sh.cnt[bin] = s;
    if (tid < 128) sh.cnt[128 + tid] = 0u;
  }
  __syncthreads();
#ifdef OVGGT_TRACE
  if (ts && tid == 0) ts[2] = (uint32_t)wall_clock64();
#endif
  pick_digit(sh, rank);
}

// One bit per register-resident key of a thread.  Indices are compile-time constants once the loops
// over the keys are unrolled, so the words stay in registers.
template <int N>
struct KeyBits {
  uint32_t w[(N + 31) / 32];
  __device__ inline void clear() {
#pragma unroll
    for (int i = 0; i < (N + 31) / 32; ++i) w[i] = 0u;
  }
  __device__ inline bool test(int c) const { return (w[c >> 5] >> (c & 31)) & 1u; }
  __device__ inline void set(int c) { w[c >> 5] |= 1u << (c & 31); }
  __device__ inline void reset(int c) { w[c >> 5] &= ~(1u << (c & 31)); }
  __device__ inline void merge(const KeyBits& o) {
#pragma unroll
    for (int i = 0; i < (N + 31) / 32; ++i) w[i] |= o.w[i];
  }
};

// Light pass for keys held in registers: `cand` has a bit per key of this thread that is still a
// candidate (usually few after the first pass).  Each candidate is first settled against the digit
// the previous pass chose (prev_of(c) below it: evicted; not equal: no candidate any more), the
// rest are counted by digit_of(c).  Counts go to one 256-bin histogram per wave with LDS atomics (a
// wave's lanes can collide on a bin, which costs at most 64 turns per instruction whatever the
// data; no clearing and column-summing of the big per-lane histogram).
template <int KPT, typename PrevOf, typename DigitOf>
__device__ inline void radix_pass_light(SelShared& sh, KeyBits<KPT>& cand, KeyBits<KPT>& evm, uint32_t prev_chosen,
                                        uint32_t rank, PrevOf prev_of, DigitOf digit_of) {
  const int tid = threadIdx.x, wave = tid >> 6;
  uint32_t* mine = sh.wave_hist[wave];                // zero on entry: cleared at kernel start and after every use
#pragma unroll
  for (int c = 0; c < KPT; ++c)
    if (cand.test(c)) {
      const uint32_t pv = (uint32_t)prev_of(c);
      if (pv != prev_chosen) {
        cand.reset(c);
        if (pv < prev_chosen) evm.set(c);
      } else {
        atomicAdd(&mine[digit_of(c)], 1u);
      }
    }
  __syncthreads();
  if (tid < 256) {
    uint32_t t = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) { t += sh.wave_hist[w][tid]; sh.wave_hist[w][tid] = 0u; }
    sh.cnt[tid] = t;
  }
  __syncthreads();
  pick_digit(sh, rank);
}

// Selection by one workgroup.  KPT > 0: the score words (and, if IDREG, the
// inverted ids) of up to KPT*1024 slots live in registers, so the radix passes
// touch LDS only.  KPT == 0: every pass re-reads them from memory (any size).
template <int KPT, bool IDREG>
__device__ inline void select_phase(SelShared& sh, const Geom& g, const float* ss, const uint32_t* ids,
                                    const uint8_t* flags, Ctrl* ctrl, uint32_t* mvdst, uint32_t* mvsrc,
                                    uint32_t* evbits, int n_total) {
  constexpr int NREG = KPT > 0 ? KPT : 1;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_chunks = (n_total + kSelThreads - 1) / kSelThreads;
  const int n_iter = KPT > 0 ? KPT : n_chunks;
  const uint32_t n_evict = (uint32_t)(n_total - g.B);
  bool bad = false;
  uint32_t kw[NREG], kid[(KPT > 0 && IDREG) ? KPT : 1];
  auto load_word = [&](int c) -> uint32_t {          // branch-free so that loads of several chunks overlap
    const int i = c * kSelThreads + tid;
    const int ic = i < n_total ? i : n_total - 1;
    const uint8_t f = flags[ic];
    const uint32_t w = score_word(ss[ic], &bad);
    return (i >= n_total || f != 0) ? kNotEvictable : w;
  };
  auto load_id = [&](int c) -> uint32_t {
    const int i = c * kSelThreads + tid;
    return 0xFFFFFFFFu - ids[i < n_total ? i : n_total - 1];
  };
  if constexpr (KPT > 0) {
    // every load is unconditional (indices are clamped), so a batch of them is in flight together
    constexpr int kBatch = KPT <= 20 ? KPT : 18;
#pragma unroll
    for (int c0 = 0; c0 < KPT; c0 += kBatch) {
      uint8_t fl[kBatch];
      float sv[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int c = c0 + j;
        if (c < KPT) {
          const int i = c * kSelThreads + tid;
          const int ic = i < n_total ? i : n_total - 1;
          fl[j] = flags[ic];
          sv[j] = ss[ic];
          if constexpr (IDREG) kid[c] = ids[ic];
        }
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int c = c0 + j;
        if (c < KPT) {
          const int i = c * kSelThreads + tid;
          const uint32_t w = score_word(sv[j], &bad);
          kw[c] = (i >= n_total || fl[j] != 0) ? kNotEvictable : w;
          if constexpr (IDREG) kid[c] = 0xFFFFFFFFu - kid[c];
        }
      }
    }
  }
  auto word = [&](int c) -> uint32_t { if constexpr (KPT > 0) return kw[c]; else return load_word(c); };
  auto idw = [&](int c) -> uint32_t { if constexpr (KPT > 0 && IDREG) return kid[c]; else return load_id(c); };
  if (tid == 0) sh.bad = 0;
  // timing builds leave 10 ns timestamps of the phases in the control block's padding
#ifdef OVGGT_TRACE
#define TSTAMP(k) do { if (tid == 0) ctrl->pad[k] = (uint32_t)wall_clock64(); } while (0)
#else
#define TSTAMP(k) do { } while (0)
#endif
  TSTAMP(1);

  // radix select of the n_evict-th smallest (score word, inverted id) pair
  uint32_t rank = n_evict;
  int pass = 0;
  bool budget_error = false, done = false;
  if constexpr (KPT > 0) {
    // Keys in registers: two bit masks per thread follow the selection, `cand` (keys that still tie
    // with the threshold on every digit seen so far) and `evm` (keys already known to go).  The
    // first pass looks at every key (most share a handful of leading digits: per-lane histogram
    // columns); after it only the candidates are touched, and in the end the masks are the answer.
    KeyBits<KPT> cand, evm;
    cand.clear(); evm.clear();
#pragma unroll
    for (int c = 0; c < KPT; ++c)
      if (kw[c] != kNotEvictable) cand.set(c);
    // settles the candidates against the digit the last pass chose: below it goes, above it stays
    auto narrow = [&](auto digit_of) {
      const uint32_t chosen = sh.digit;
#pragma unroll
      for (int c = 0; c < KPT; ++c)
        if (cand.test(c)) {
          const uint32_t dg = (uint32_t)digit_of(c);
          if (dg < chosen) evm.set(c);
          if (dg != chosen) cand.reset(c);
        }
    };
    uint32_t chosen = 0;                               // digit of the last pass (its candidates are settled by the next one)
    {
      first_pass_registers<KPT>(sh, kw, rank, &ctrl->pad[20]);
      if (sh.n_evictable < n_evict) budget_error = true;          // |P| > B
      else {
        chosen = sh.digit;
        rank = sh.rank;
        done = (rank == sh.bucket);                   // the whole bucket goes
      }
      pass = 1;                                       // (the next pass runs two barriers before it writes these again)
      TSTAMP(2);
    }
    int last_shift = 24;                               // where the last pass took its digit from
    bool last_id = false;
#pragma nounroll
    for (; pass < 4 && !done && !budget_error; ++pass) {
      const int shift = 24 - 8 * pass;
      radix_pass_light<KPT>(sh, cand, evm, chosen, rank,
                                  [&](int c) -> int { return (int)((kw[c] >> (shift + 8)) & 255u); },
                                  [&](int c) -> int { return (int)((kw[c] >> shift) & 255u); });
      chosen = sh.digit;
      rank = sh.rank;
      done = (rank == sh.bucket);
      last_shift = shift;
      TSTAMP(2 + pass);
    }
    if (!done && !budget_error) {
      // equal scores straddle the threshold: the ids decide (all candidates share the score word)
#pragma nounroll
      for (int p2 = 0; p2 < 4 && !done; ++p2) {
        const int shift = 24 - 8 * p2;
        if (p2 == 0)
          radix_pass_light<KPT>(sh, cand, evm, chosen, rank,
                                      [&](int c) -> int { return (int)(kw[c] & 255u); },
                                      [&](int c) -> int { return (int)(idw(c) >> 24); });
        else
          radix_pass_light<KPT>(sh, cand, evm, chosen, rank,
                                      [&](int c) -> int { return (int)((idw(c) >> (shift + 8)) & 255u); },
                                      [&](int c) -> int { return (int)((idw(c) >> shift) & 255u); });
        chosen = sh.digit;
        rank = sh.rank;
        done = (rank == sh.bucket);
        last_shift = shift;
        last_id = true;
      }
    }
    // the last pass's candidates are still unsettled
    if (!budget_error) {
      if (last_id) narrow([&](int c) -> int { return (int)((idw(c) >> last_shift) & 255u); });
      else narrow([&](int c) -> int { return (int)((kw[c] >> last_shift) & 255u); });
      (void)chosen;
    }
    if (done) evm.merge(cand);
    if (budget_error) evm.clear();
    if (bad) sh.bad = 1;
    TSTAMP(10);
    // evict bit per slot, published in slot order: the ballot of one chunk over one wave covers 64
    // consecutive slots
#pragma unroll
    for (int c = 0; c < KPT; ++c)
      if (c < n_chunks) {
        const uint64_t bl = __ballot(evm.test(c));
        if (lane == 0) {
          sh.evmap[(c * kSelThreads >> 5) + 2 * wave] = (uint32_t)bl;
          sh.evmap[(c * kSelThreads >> 5) + 2 * wave + 1] = (uint32_t)(bl >> 32);
        }
      }
  } else {
  uint32_t pre_hi = 0, pre_lo = 0;
#pragma nounroll
  for (; pass < 4 && !done; ++pass) {
    const int shift = 24 - 8 * pass;
    radix_pass(sh, n_iter, rank, [&](int c) -> int {
      const uint32_t w = word(c);
      if (w == kNotEvictable) return -1;
      if (pass > 0 && (w >> (shift + 8)) != (pre_hi >> (shift + 8))) return -1;
      return (int)((w >> shift) & 255u);
    }, pass == 0 ? &ctrl->pad[20] : nullptr);
    if (pass == 0 && sh.n_evictable < n_evict) { budget_error = true; break; }   // |P| > B
    pre_hi |= sh.digit << shift;
    rank = sh.rank;
    done = (rank == sh.bucket);          // the whole bucket goes
    __syncthreads();
    TSTAMP(2 + pass);
  }
  const int hi_shift = pass > 0 ? 24 - 8 * (pass - 1) : 24;
  int lo_shift = 32;                      // 32: ids did not have to be consulted
  if (!done && !budget_error) {
#pragma nounroll
    for (int p2 = 0; p2 < 4 && !done; ++p2) {
      const int shift = 24 - 8 * p2;
      radix_pass(sh, n_iter, rank, [&](int c) -> int {
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
  TSTAMP(10);

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
  }
  __syncthreads();
  TSTAMP(11);
  // holes (evicted slot below B) and movers (kept slot at or above B), in slot order: a thread
  // takes PP consecutive 32-slot words of the bitmap, one scan over the per-thread (holes, movers)
  // counts gives it the list position of its first hole and first mover
  const int n_words = (n_total + 31) >> 5;
  const int PP = (n_words + kSelThreads - 1) / kSelThreads;      // <= 4
  uint32_t hw[4], mw[4];
  uint32_t nh = 0, nm = 0;
  const bool wave_has_words = wave * 64 * PP < n_words;          // the other waves only keep the barriers company
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    hw[j] = mw[j] = 0u;
    const int wi = tid * PP + j;
    if (j < PP && wi < n_words) {
      const int s0 = wi << 5;
      const uint32_t e = sh.evmap[wi];
      if (evbits) evbits[wi] = e;
      const uint32_t below_b = s0 + 32 <= g.B ? 0xFFFFFFFFu : (s0 >= g.B ? 0u : ((1u << (g.B - s0)) - 1u));
      const uint32_t below_n = s0 + 32 <= n_total ? 0xFFFFFFFFu : ((1u << (n_total - s0)) - 1u);
      hw[j] = e & below_b;
      mw[j] = ~e & ~below_b & below_n;
      nh += __popc(hw[j]);
      nm += __popc(mw[j]);
    }
  }
  bool consistent = false;
  {
    uint32_t inc_h = nh, inc_m = nm;
    if (wave_has_words) {
#pragma unroll
      for (int off = 1; off < 64; off *= 2) {
        const uint32_t yh = __shfl_up(inc_h, off, 64), ym = __shfl_up(inc_m, off, 64);
        if (lane >= off) { inc_h += yh; inc_m += ym; }
      }
    }
    if (lane == 63) { sh.scan_tmp[0][wave] = inc_h; sh.scan_tmp[1][wave] = inc_m; }
    __syncthreads();
    if (wave_has_words) {
      uint32_t base_h = 0, base_m = 0, tot_h = 0, tot_m = 0;
#pragma unroll
      for (int w = 0; w < kSelWaves; ++w) {
        const uint32_t th = sh.scan_tmp[0][w], tm = sh.scan_tmp[1][w];
        if (w < wave) { base_h += th; base_m += tm; }
        tot_h += th; tot_m += tm;
      }
      consistent = !budget_error && tot_h == tot_m && tot_h <= (uint32_t)g.M;
      if (tid == 0) sh.totals[0] = tot_h;
      if (consistent) {
        uint32_t hp = base_h + inc_h - nh, mp = base_m + inc_m - nm;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t s0 = (uint32_t)(tid * PP + j) << 5;
          uint32_t b = hw[j];
          while (b) { mvdst[hp++] = s0 + (uint32_t)__builtin_ctz(b); b &= b - 1; }
          b = mw[j];
          while (b) { mvsrc[mp++] = s0 + (uint32_t)__builtin_ctz(b); b &= b - 1; }
        }
      }
    }
  }
  __syncthreads();
  if (tid == 0) {
    ctrl->n_moves = consistent ? sh.totals[0] : 0u;
    uint32_t st = 0;
    if (budget_error || !consistent) st |= OVGGT_STATUS_BUDGET;
    if (sh.bad) st |= OVGGT_STATUS_NONFINITE;
    if (st) atomicOr(&ctrl->status, st);
    TSTAMP(12);
#ifdef OVGGT_TRACE
    ctrl->pad[13] = (uint32_t)pass;
#endif
  }
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
// their scores, written through like the scores of phase 1.
__device__ inline void hybrid_history_values(SelShared& sh, const HybridParams& hy, const float* dval,
                                             const float2* part, float* ss, const uint8_t* flags, int n_old) {
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
    __hip_atomic_store(&ss[i], weight * unit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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

template <bool BF16, int KPT, bool IDREG>
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

#ifdef OVGGT_TRACE
  if (blockIdx.x == 0 && tid == 0) ctrl->pad[15] = (uint32_t)wall_clock64();
#endif
  // Whichever workgroup ends up running the selection wants its histograms cleared: every
  // workgroup does that now, in the shadow of phase 1's loads.
  if (n_total > g.B) {
    uint4* h4 = (uint4*)&sh.hist[0][0];
    const uint4 z = {0u, 0u, 0u, 0u};
    h4[tid] = z; h4[tid + kSelThreads] = z;                       // rows 0..127
    ((uint4*)&sh.wave_hist[0][0])[tid] = z;
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
  if (hy.on && n_total > g.B)
    hybrid_history_values(sh, hy, (const float*)(mb + g.off_dval), (const float2*)(mb + g.off_dpart), ss, flags, n_old);
  const bool smoothing = sm.alpha > 0.f;
  if (n_total <= g.B && !smoothing) {        // under budget and no smoothing: nothing needs the whole frame
    if (blockIdx.x == 0 && tid == 0) ctrl->n_moves = 0;
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
#ifdef OVGGT_TRACE
      ctrl->pad[0] = (uint32_t)wall_clock64();
#endif
    }
    sh.is_last = last ? 1u : 0u;
  }
  __syncthreads();
  if (!sh.is_last) return;

  // ---- phase 2: this workgroup saw every other one arrive
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
  select_phase<KPT, IDREG>(sh, g, ss, ids, flags, ctrl, mvdst, mvsrc,
                           hy.on ? (uint32_t*)(mb + g.off_evbits) : nullptr, n_total);
}

template <bool BF16>
static void launch_variant(const Geom& g, const SmoothParams& sm, const HybridParams& hy, char* meta, int layer0, int nl, const void* resid,
                           const uint8_t* anchors, int n_total, int e, hipStream_t s) {
  // One workgroup fits a CU (the selection's register-resident keys set the footprint), so the
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
  const int n_chunks = (n_total + kSelThreads - 1) / kSelThreads;
#define OVGGT_SEL_LAUNCH(KPT, IDREG)                                                                  \
  hipLaunchKernelGGL((score_select_kernel<BF16, KPT, IDREG>), grid, dim3(kSelThreads), 0, s, g, sm, hy, meta, \
                     layer0, (const char*)resid, anchors, n_total, e)
  // the variant only matters when a selection will run (n_total > B)
  if (n_total <= g.B || n_chunks <= 8) OVGGT_SEL_LAUNCH(8, true);
  else if (n_chunks <= 20) OVGGT_SEL_LAUNCH(20, true);
  else if (n_chunks <= 36) OVGGT_SEL_LAUNCH(36, false);      // ids stay in memory: fetched only for keys whose equal scores straddle the threshold
  else OVGGT_SEL_LAUNCH(0, false);                           // (72 keys per thread in registers measured slower than streaming)
#undef OVGGT_SEL_LAUNCH
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
