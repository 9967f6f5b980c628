// bf16 flash-style attention of one frame's queries over the bounded KV cache
// (paper Sec. 3.1: the temporal causal attention CA; cost O(M*B) per step once
// the cache is bounded).  gfx950 MFMA kernel.
//
// Formulation (chosen so the softmax statistics of one query live in one lane):
//   S^T = K Q^T      A = K tile rows from LDS,      B = Q^T fragments in registers
//   O^T = V^T P^T    A = V^T via LDS transpose reads, B = P^T straight from the
//                    S^T accumulators (the contraction index may be permuted
//                    freely as long as both operands agree)
// Both products run on v_mfma_f32_32x32x16_f16 with fp32 accumulation.  The cache
// holds K and V as IEEE half (exact images of the bf16 inputs inside the half
// range) and the softmax weights are rounded to half: 11-bit weights keep the
// output within 1e-3 of its RMS where 8-bit (bf16) weights reach 4e-2 on rows with
// one dominant key.  The queries are scaled by c = scale * log2(e) and rounded to
// half when a work item starts (relative error 2^-12 per element, below the
// weights' own rounding), and the running reference of every query enters S^T as
// a fifth contraction step, so the accumulators leave the matrix pipe as the
// exponents x = s*c - ref and the softmax is exp2, convert, add and nothing else.
// The reference is applied lazily (accumulators are rescaled only when the
// maximum grows by more than 2^8) and sits 7 below the maximum, so weights are
// stored as 2^7 * p in the middle of the half range.
//
// Schedule.  On this chip the softmax of a tile (64 x {exp, add} + 32
// conversions per lane) costs more VALU time than the tile's 32 MFMAs cost matrix
// time, a wave never overlaps its own MFMAs with its own VALU work, and two free
// running waves on a SIMD starve the younger one.  So a workgroup is 8 waves =
// two sets of 4, one wave of each set per SIMD, and the sets alternate between a
// matrix phase (P V of the previous tile, then Q K^T of the current one; LDS
// reads, no VALU instruction) and a vector phase (the softmax; no MFMA), with one
// workgroup barrier per phase.  Set B starts one barrier late, so while one set
// is in its matrix phase the other is in its vector phase and both pipes stay
// busy.  Every wave executes the same sequence of barriers.
//
// Work split.  A work item is one of the QB items of a (layer, head) pair; its work is
// T = ceil(n/128) slot tiles for both wave sets, which share control flow (same tile range).
// Where a head has two query blocks left, an item is two neighbouring 128-query blocks of ONE
// head, one per set, and both sets read the same K/V tiles from set A's LDS buffers: set A
// requests the K tiles, set B the V tiles, so a tile travels from L2 into LDS once for 256 queries
// (work_of_item).  The odd last block of the pair's two heads makes up the last item, one head
// per set, each with its own tile buffers (also the only form when the launch has an odd number
// of heads).  The flat list of item x tile units is cut into chunks, one per workgroup (one
// workgroup per CU, persistent, stream-K style).  A set that covers its block completely writes
// the output; otherwise it writes an unnormalised partial (O, m, l) that attn_combine_kernel
// merges.  Chunks are handed to workgroups so that each XCD's L2 sees as few heads as possible.
//
// Inside a set, wave = (query half, slot half) of the 128x128 tile; the two slot
// halves are merged through LDS at the end of an item.  K and V tiles stream
// global->LDS with 16-byte direct-to-LDS loads, double buffered: K of tile t+1 is
// requested at the start of the matrix phase of tile t, V of tile t+1 at the
// start of its vector phase, and both are awaited (vmcnt) just before the barrier
// that precedes their first use.  With shared tiles the same two requests come from
// set A (K, matrix phase) and set B (V, vector phase: the same moment, B being a phase
// behind), B awaits its V rows one phase earlier (A multiplies by them first), and a
// wave that has to redo a tile's exponents re-reads K from memory, because set A's next
// request may already be filling the buffer set B's tile came from.  LDS rows are 128 bytes; 16-byte pieces are
// XOR-swizzled with the row index so both the K operand reads and the V
// transpose reads are bank-conflict free.
#include "ovggt_internal.h"
#include <algorithm>
#include <mutex>
#include <vector>

namespace ovggt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// XOR swizzle of the 16-byte piece index within a 128-byte LDS row (measured against
// variants keyed on higher row bits: this one has the fewest bank conflicts).
__device__ __forceinline__ int swz(int row) { return row & 7; }

// Wave priority in the two phases.  The vector phase is the longer one and its VALU stream loses
// issue slots to the other set's MFMAs; giving it the higher priority shortens the younger set's
// vector phase by a tenth (measured) at no cost to the matrix phase that runs beside it.
constexpr int kPrioMatrix = 0, kPrioVector = 3;
constexpr int kTileBytes = kSlotTile * 128;            // one K (or V) tile: 128 slots x 64 16-bit elements
constexpr int kSetBytes = 4 * kTileBytes;              // LDS of one wave set: [parity][K | V]
constexpr int kMergeBytes = 2 * 64 * 64 * 4 + 2 * 4 * 64 * 4;   // a set's slot-half merge area: O of two query halves, then (ref, l)
static_assert((kSetBytes & (kSetBytes - 1)) == 0 && kMergeBytes <= kSetBytes, "region arithmetic of the tile loop");
constexpr int kAttnThreads = 512;
constexpr int kPartialFloats = kQueryTile * 64 + 2 * kQueryTile;
// Float offset, inside a partial record's O part, of the 256-float block that holds the values
// O[db][qb][4*ig .. 4*ig+3] of all 64 lanes of the waves of query half `qhalf` (lane * 4 + j inside
// the block): element (row = 64*qhalf + 32*qb + lane % 32, column = 32*db + 8*ig + 4*(lane / 32) + j).
__host__ __device__ constexpr int partial_block_offset(int qhalf, int db, int qb, int ig) {
  return (((qhalf * 2 + db) * 2 + qb) * 4 + ig) * 256;
}
constexpr float kWeightBias = 7.0f;                    // weights are stored as 2^7 * p (half max 65504)
constexpr float kWeightSumLimit = 32768.0f;            // a lane's weight sum below 2^15 proves no weight overflowed

// s_waitcnt immediates (gfx9 encoding: vmcnt [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8])
constexpr int kWaitVm0 = 0x0F70;                       // vmcnt(0), nothing else
constexpr int kWaitVm4 = 0x0F74;                       // vmcnt(4)
constexpr int kWaitLgkm0 = 0xC07F;                     // lgkmcnt(0), nothing else

constexpr int kSegRecs = 3;                            // partial records per workgroup and wave set
// Workspace: kSegRecs partial records per chunk and wave set.  A launch over few (layer, head)
// pairs has one chunk per workgroup, and so has one that hands out whole items (only its last round
// leaves records); a launch whose head pairs are dealt out to the XCDs round by round has
// kMaxAttnWgs / 8 chunks per head pair.
// Launches over many head pairs hand whole items (head pair x query block) to the workgroups when
// the head pairs divide among the 8 XCDs and every workgroup gets at least one whole item.
bool attn_whole_items(int layer_heads, int query_blocks, int n_wgs) {
  const int pairs = (layer_heads + 1) / 2;
  return pairs > 8 && pairs % 8 == 0 && (long)(pairs / 8) * query_blocks >= n_wgs / 8;
}

size_t attn_ws_bytes(int layer_heads, int query_blocks) {
  const long pairs = (layer_heads + 1) / 2;
  long chunks = pairs * (kMaxAttnWgs / 8) > kMaxAttnWgs ? pairs * (kMaxAttnWgs / 8) : kMaxAttnWgs;
  if (attn_whole_items(layer_heads, query_blocks, kMaxAttnWgs)) chunks = kMaxAttnWgs;   // holds for fewer workgroups too
  size_t bytes = (size_t)chunks * kSegRecs * 2 * kPartialFloats * sizeof(float);
  OVGGT_TRACE_ONLY(bytes += (size_t)kMaxAttnWgs * 8 * 64;)   // timing builds: one 64-byte record per wave behind the partials
  return bytes;
}

// ---- workspace for callers that cannot allocate ---------------------------------------------------
// The partial records of a launch of up to kMaxAttnWgs chunks (one layer of any head count the
// one-round plan covers), as a device array of the library itself: every GPU the library runs on
// holds it until the process ends.  In host code the array's name is only a stand-in; its device
// address is looked up once per device, with that device current, and kept.
constexpr size_t kStaticWsBytes = (size_t)kMaxAttnWgs * kSegRecs * 2 * kPartialFloats * sizeof(float);   // 51 904 512 bytes
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_static_ws_mutex;
static char* g_static_ws_ptr[kMaxDevices];

hipError_t attn_static_ws(char** ptr, size_t* bytes) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_ws_mutex);
  if (!g_static_ws_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_ws_ptr[dev] = (char*)p;
  }
  *ptr = g_static_ws_ptr[dev];
  *bytes = kStaticWsBytes;
  return hipSuccess;
}

constexpr int kMaxChunksPerPair = 64;
constexpr int kMaxTableItems = 16, kMaxTableRecs = 12;  // query blocks, and partial records of one, in the merge pass's table
constexpr uint8_t kWholeItem = 255;
struct AttnParams {
  const char* q;
  char* out;
  const char* kv0;            // K of the first layer of this launch
  size_t kv_layer_bytes;
  size_t v_off;               // bytes from a layer's K to its V
  float* ws;
  int H, M, cap, n_total;
  int LH;                     // (layer, head) count of this launch
  int QB;                     // query blocks per (layer, head)
  int T;                      // slot tiles
  int chunk;                  // units per workgroup
  int NS, L0;                 // tile segments per item and their length (the last one takes the rest)
  int PP;                     // unit slots per head pair: QB * T, or that rounded up to whole chunks
  int rounds;                 // chunks per workgroup (chunk index = round * workgroups + workgroup's index)
  int cpp;                    // > 0: every head pair is cut into cpp chunks at the unit offsets in cstart
  int cstart[kMaxChunksPerPair + 1];   // (chunks of unequal tile counts but equal estimated cost); 0: equal chunks of `chunk` units
  // With cpp > 0 and few enough query blocks, the merge pass finds an item's partial records in a
  // table instead of working them out (the same table for every head pair): query block qb has
  // rec_count[qb] entries, each chunk-in-pair + 256 * record-in-chunk; kWholeItem: one workgroup
  // did the whole item and wrote the output itself.  rec_table_on = 0: no table.
  int rec_table_on;
  uint8_t rec_count[kMaxTableItems];
  uint16_t rec_table[kMaxTableItems][kMaxTableRecs];
  // Whole items (launches over many head pairs): an XCD's workgroups (per_xcd of them) own ppx
  // consecutive head pairs = ppx * QB items; in each of the first rf rounds a workgroup takes one
  // whole item (all T tiles, no partial record, no merge), and the items left over are cut evenly
  // into per_xcd chunks of lo_chunk units for one last round.  item_mode = 0: off.
  int item_mode, per_xcd, ppx, rf, lo_chunk;
  // share = 1: the two wave sets of a workgroup take two query blocks of ONE head wherever a head
  // has two left, and read the same K/V tiles (see item_of_block); 0: always two heads, one block.
  int share;
  size_t trace_off;           // floats from ws to the end of the record area (timing builds)
  int total_units;            // ceil(LH / 2) * PP
  float c;                    // softmax scale * log2(e)
  int out_f32;                // output element type: 1 = fp32, 0 = bf16
};

// Order of the work units.  Inside one (layer, head) pair the T tiles of every query block are cut
// into NS segments (L0 tiles each, the last one takes the rest), and the units run segment by
// segment, query block by query block, tile by tile.  With L0 equal to a workgroup's chunk,
// neighbouring workgroups (same XCD, same L2) start on the same tile of neighbouring query blocks
// and walk the same K/V tiles side by side, so a tile is fetched into the L2 once instead of once
// per query block.  NS = 1 is the plain order (query block, tile).  A head pair's units may be
// followed by empty slots up to a whole number of chunks, which keeps chunk and segment boundaries
// aligned in every head pair (one piece per workgroup in all but the last segment).
struct UnitPos {
  bool valid;                 // false: an empty slot behind the head pair's last unit
  int hp, s, qb;              // head pair, segment, item within the head pair (called query block in the plan: see work_of_item)
  int tile;                   // first tile of the unit's run
  int seg_end;                // end of the segment (exclusive)
  int combo;                  // running index of (hp, s, qb)
};
// What the two wave sets of a workgroup do with item j (0 .. QB-1) of head pair hp.  The plan only
// knows items; which query blocks they stand for is decided here.  Without sharing, item j is query
// block j of both heads, one head per wave set.  With sharing, a head's blocks are taken two at a
// time by one workgroup -- items 0 .. QB/2-1 are block pairs of the first head, the next QB/2 those
// of the second, both wave sets on the same head and the same K/V tiles, which are then fetched
// into LDS once for 256 queries instead of once for 128 -- and an odd last block of the two heads
// makes up the last item, one head per wave set as before.  The item count per head pair is QB
// either way.
struct SetWork {
  int lh, qb;                 // (layer, head) index and query block of this wave set
  bool shared;                // both sets read one head's tiles
};
__host__ __device__ inline SetWork work_of_item(int hp, int j, int set, int QB, int share) {
  const int nsh = QB >> 1;
  if (share && j < 2 * nsh) {
    const int second = j >= nsh ? 1 : 0;
    return {2 * hp + second, 2 * (j - second * nsh) + set, true};
  }
  return {2 * hp + set, j, false};
}
// The inverse: the item (within its head pair) and the wave set that handle query block qb of lh.
struct ItemOfBlock { int j, set; };
__host__ __device__ inline ItemOfBlock item_of_block(int lh, int qb, int QB, int share) {
  const int nsh = QB >> 1;
  if (share && qb < 2 * nsh) return {(lh & 1) * nsh + (qb >> 1), qb & 1};
  return {qb, lh & 1};
}

__host__ __device__ inline UnitPos decode_unit(long u, int T, int QB, int NS, int L0, int PP) {
  UnitPos r;
  r.hp = (int)(u / PP);
  int rem = (int)(u - (long)r.hp * PP);
  r.valid = rem < QB * T;
  if (!r.valid) rem = QB * T - 1;
  r.s = NS == 1 ? 0 : min(rem / (QB * L0), NS - 1);
  const int seg0 = r.s * L0;
  r.seg_end = r.s == NS - 1 ? T : seg0 + L0;
  const int len = r.seg_end - seg0;
  const int r2 = rem - QB * seg0;
  r.qb = r2 / len;
  r.tile = seg0 + r2 - r.qb * len;
  r.combo = (r.hp * NS + r.s) * QB + r.qb;
  return r;
}

// First unit of chunk c (c may be one past the last chunk), and the chunk a unit belongs to.
__host__ __device__ inline long chunk_first_unit(const AttnParams& p, int c) {
  if (p.cpp == 0) return min((long)c * p.chunk, (long)p.total_units);
  const int hp = c / p.cpp;
  return (long)hp * p.PP + p.cstart[c - hp * p.cpp];
}
__host__ __device__ inline int chunk_of_unit(const AttnParams& p, long u) {
  if (p.cpp == 0) return (int)(u / p.chunk);
  const int hp = (int)(u / p.PP);
  const int r = (int)(u - (long)hp * p.PP);
  int lc = 0;
  while (lc + 1 < p.cpp && p.cstart[lc + 1] <= r) ++lc;
  return hp * p.cpp + lc;
}

// Units [u0, u1) that workgroup `cidx` (XCD-major index: cidx / per_xcd is its XCD) works on in
// round `rnd` of a launch of G workgroups, and the chunk number its partial records are filed under.
struct ChunkRange { long u0, u1; int rec_chunk; };
__host__ __device__ inline ChunkRange chunk_range(const AttnParams& p, int rnd, int cidx, int G) {
  ChunkRange r;
  if (!p.item_mode) {
    const int c = rnd * G + cidx;
    r.u0 = chunk_first_unit(p, c);
    r.u1 = chunk_first_unit(p, c + 1);
    r.rec_chunk = c;
    return r;
  }
  const int x = cidx / p.per_xcd, j = cidx - x * p.per_xcd;
  const long base = (long)x * p.ppx * p.PP;              // the XCD's first unit (PP = QB * T units per head pair)
  r.rec_chunk = cidx;
  if (rnd < p.rf) {
    r.u0 = base + ((long)rnd * p.per_xcd + j) * p.T;
    r.u1 = r.u0 + p.T;
  } else {
    const long lo0 = base + (long)p.rf * p.per_xcd * p.T, lo1 = base + (long)p.ppx * p.PP;
    r.u0 = min(lo0 + (long)j * p.lo_chunk, lo1);
    r.u1 = min(r.u0 + p.lo_chunk, lo1);
  }
  return r;
}

// Half a tile pair, global -> LDS: the calling wave fills 32 rows (4 KiB) of a K or V tile with four
// 16-byte-per-lane direct-to-LDS loads (8 rows of 128 bytes each); lane i's 16 bytes land at
// lds_addr + 16*i, and the immediate offset advances the memory address and the LDS address alike.
// Inline assembly on purpose: the compiler cannot tell which LDS bytes an LDS-DMA load writes and
// would make every later LDS read wait for all outstanding loads.  The kernel orders these loads
// itself with explicit vmcnt waits in front of the barrier that publishes a tile.
__device__ __forceinline__ void load_rows_to_lds(const char* gtile, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\t"
               "s_nop 0\n\t"
               "global_load_lds_dwordx4 %1, %2 offset:0\n\t"
               "global_load_lds_dwordx4 %1, %2 offset:1024\n\t"
               "global_load_lds_dwordx4 %1, %2 offset:2048\n\t"
               "global_load_lds_dwordx4 %1, %2 offset:3072"
               : : "s"(lds_addr), "v"(lane_off), "s"(gtile) : "memory", "m0");
}

// One of the four loads of load_rows_to_lds (rows 8*I .. 8*I+7 of the wave's 32).  The vector phase
// issues its four V loads one in front of each batch of sixteen exp2 instead of together at its
// start (a direct-to-LDS load keeps its wave from issuing anything else for about 44 cycles;
// measured: 1-2 % of the kernel on one layer, nothing on 24).
template <int I>
__device__ __forceinline__ void load_row_group_to_lds(const char* gtile, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\t"
               "s_nop 0\n\t"
               "global_load_lds_dwordx4 %1, %2 offset:%3"
               : : "s"(lds_addr), "v"(lane_off), "s"(gtile), "n"(I * 1024) : "memory", "m0");
}
// The V loads of the next tile as a hook the softmax calls in front of its four batches (I = 0..3);
// NoLoads does nothing (a piece's last tile, the redone weights of the slow path).
struct NoLoads {
  template <int I> __device__ __forceinline__ void at() const {}
};
struct TileLoads {
  bool on; const char* gtile; uint32_t lane_off, lds_addr;
  template <int I> __device__ __forceinline__ void at() const { if (on) load_row_group_to_lds<I>(gtile, lane_off, lds_addr); }
};

// Workgroup barrier that neither memory accesses nor ALU work may be moved across.
__device__ __forceinline__ void phase_barrier() {
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("s_barrier" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

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

__device__ inline f16x8 join4(const uint32_t* p) {
  const u32x4 v = {p[0], p[1], p[2], p[3]};
  return __builtin_bit_cast(f16x8, v);
}

// Softmax weights of one query block of a tile: p = exp2(x + d) for the 32 exponents a lane holds
// (two 32-slot accumulators; the matrix phase already delivered x = s*c - reference), rounded to
// half in pairs (kept as the 32-bit pattern of the pair); returns the lane's fp32 sum of the
// weights.  SHIFT: d is added first (slow path only; the fast path has d = 0 and no instruction
// for it).
//
// Issued in batches of 16 (all exp, then conversions and adds) with scheduling fences between
// them: an instruction that consumes the result of the one issued just before it stalls about four
// cycles (measured for exp -> add), and left to itself the scheduler emits exactly such dependent
// pairs to save registers.
template <bool SHIFT, int QB, class Loads>
__device__ __forceinline__ float tile_weights(const f32x16& s0, const f32x16& s1, float d,
                                              uint32_t (&p0)[8], uint32_t (&p1)[8], const Loads& loads) {
  // The row sum is taken over the weights as the matrix unit will see them (rounded to half), with
  // packed half adds: one instruction per two weights instead of two fp32 adds, on the pipe that
  // co-executes with the other set's MFMAs (v_dot2c_f32_f16 would be exact but runs on the matrix
  // pipe and serialises with them: measured).  Four independent packed accumulators of 8 terms
  // each (the first four pairs start them, no zero to add to), joined pairwise in half and widened
  // once: 32 terms, five levels of half rounding, near 2^-11 relative and unbiased.  An
  // overflowing weight or partial sum becomes +inf and trips the caller's limit test (sums
  // beyond 2^15 take the slow path anyway).
  f16x2 ls[4];
#pragma unroll
  for (int sb = 0; sb < 2; ++sb) {
    float e[16];
    if (sb == 0) loads.template at<2 * QB>(); else loads.template at<2 * QB + 1>();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float x = sb ? s1[i] : s0[i];
      e[i] = __builtin_amdgcn_exp2f(SHIFT ? x + d : x);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      f16x2 pk;
      pk[0] = (_Float16)e[2 * j];
      pk[1] = (_Float16)e[2 * j + 1];
      if (sb == 0 && j < 4) ls[j] = pk; else ls[j & 3] += pk;
      (sb ? p1 : p0)[j] = __builtin_bit_cast(uint32_t, pk);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  const f16x2 t = (ls[0] + ls[1]) + (ls[2] + ls[3]);
  return (float)t[0] + (float)t[1];

}

// The reference of a query block as the B operand of the bias step of S^T (a 32x32x8 MFMA, whose
// operands are four halves per lane): -ref (exact in half) at contraction index 0, which only the
// lanes of the first 4-index group hold.
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
__device__ __forceinline__ f16x4 bias_operand(float ref, int g) {
  const f16x2 h = {(_Float16)(-ref), (_Float16)0.f};
  const u32x2 v = {g == 0 ? __builtin_bit_cast(uint32_t, h) : 0u, 0u};
  return __builtin_bit_cast(f16x4, v);
}

// Matrix phase, first part: O^T += V^T P^T for one 64-slot x 64-query tile of one wave; each V^T
// fragment feeds both query blocks.  P is indexed [slot block][query block][pair].
template <int PAR>
__device__ __forceinline__ void pv_tile(const char* lds, const int (&voff)[2][2], const uint32_t (&P)[2][2][8],
                                        f32x16 (&O)[2][2]) {
  const char* ldsV = lds + PAR * 2 * kTileBytes + kTileBytes;
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const f16x8 pb0 = join4(P[sb][0] + 4 * s2);
      const f16x8 pb1 = join4(P[sb][1] + 4 * s2);
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        const int o = (sb * 32 + 16 * s2) * 128;
        const s16x4 va = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ldsV + voff[db][0] + o));
        const s16x4 vb = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, ldsV + voff[db][1] + o));
        const __attribute__((ext_vector_type(8))) short v8 = __builtin_shufflevector(va, vb, 0, 1, 2, 3, 4, 5, 6, 7);
        const f16x8 vf = __builtin_bit_cast(f16x8, v8);
        O[db][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pb0, O[db][0], 0, 0, 0);
        O[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pb1, O[db][1], 0, 0, 0);
      }
    }
}

// Matrix phase, second part: S^T = K Q'^T - ref, S indexed [slot block][query block].  Q' is the
// query scaled by c = scale * log2(e) and rounded to half, K is cached as half, and the reference of
// each query enters as one more step of the contraction (a column of ones on the K side times a
// row holding -ref on the Q side), so the accumulators leave the matrix pipe as the exponents the
// softmax needs and the vector phase spends no instruction on scaling or subtracting.  The bias
// step goes first: it needs no LDS operand and covers the latency of the first K reads.
template <int PAR>
__device__ __forceinline__ void k_frags(const char* lds, const int (&koff)[4], f16x8 (&kf)[4][2]) {
  const char* ldsK = lds + PAR * 2 * kTileBytes;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    kf[ks][0] = *LDS_PTR(const f16x8, ldsK + koff[ks]);
    kf[ks][1] = *LDS_PTR(const f16x8, ldsK + koff[ks] + 32 * 128);
  }
}
__device__ __forceinline__ void qk_tile(const f16x8 (&kf)[4][2], const f16x8 (&qf)[2][4], const f16x4 (&qbias)[2],
                                        f16x4 kones, f32x16 (&S)[2][2]) {
  f32x16 zero;
#pragma unroll
  for (int i = 0; i < 16; ++i) zero[i] = 0.f;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) S[a][b] = __builtin_amdgcn_mfma_f32_32x32x8f16(kones, qbias[b], zero, 0, 0, 0);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    S[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[ks][0], qf[0][ks], S[0][0], 0, 0, 0);
    S[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[ks][0], qf[1][ks], S[0][1], 0, 0, 0);
    S[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[ks][1], qf[0][ks], S[1][0], 0, 0, 0);
    S[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[ks][1], qf[1][ks], S[1][1], 0, 0, 0);
  }
}

// The lane number, read where it is needed.  For the rarely taken paths of the tile loop (the tail
// tile, the redone exponents of a shared piece): a value derived from the lane number at the start
// of the kernel would have to be kept, or spilled, across every loop; the statement is volatile so
// that it is not moved out of the path either.
__device__ __forceinline__ int lane_number_here() {
  int ln;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ln));
  return ln;
}

// Tail tile: accumulator i of slot block sb belongs to slot sbase + 4*(lane/32) + 32*sb + 8*(i/4) + i%4
// (sbase: the first slot of the wave's 64, uniform).  Exponents of slots at or beyond n_total become -inf: exp2
// gives them weight 0 and a maximum ignores them.  A lane (or a whole wave) left without any real
// slot ends with the reference -65504 and a zero sum, which the merges treat as an empty part.
__device__ __forceinline__ void mask_absent_slots(f32x16 (&S)[2][2], int sbase, int n_total) {
  // The lane's share of the slot index is read here: it keeps the caller's test a real branch and
  // the 32 comparisons below inside it (the tail tile is the last one, so from values known at the
  // start of the kernel the compiler works them out once and carries 64 scalar registers of masks
  // through every loop).
  sbase += 4 * (lane_number_here() >> 5);
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const bool absent = sbase + sb * 32 + (i >> 2) * 8 + (i & 3) >= n_total;
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) S[sb][qb][i] = absent ? -INFINITY : S[sb][qb][i];
    }
}

// Vector phase: online softmax of one 64-slot x 64-query tile of one wave.
// S holds x = s*c - ref for the reference ref the query block had when the matrix phase ran; ref
// is (a half-representable value near) the running maximum of s*c minus 7, so weights are stored
// as 2^7 * p and sit in the middle of the half range.
// tail: the tile extends past n_total (only the last tile can); the exponents of the absent slots
// are set to -inf before anything looks at them, so they neither move the reference nor carry
// weight (their rows hold zeros or stale but finite values, so 0 * V stays finite).
//
// Fast path: weights are formed against the current reference without looking for this tile's
// maximum; p = exp2(x) is rounded to half and summed.  If the lane's sum stays below 2^15 no
// weight can have overflowed half.  Otherwise (the maximum grew by about 2^8), and always on the
// first tile of a segment (force: the reference starts at 0 and must be set from real scores so
// that small weights do not underflow), the wave takes the slow path: exponents again, true tile maximum, new
// reference, rescale O and l, redo the weights.  The reference therefore lags the true maximum
// by < 2^8, which costs no accuracy in fp32/half arithmetic; any value of it is consistent as long
// as every weight since the last rescale used the same one, which the exact half value guarantees.
// O holds the tiles before this one (their P V products were issued in the preceding matrix
// phase), so rescaling it here is consistent.
template <int PAR, bool force, class Loads>
__device__ __forceinline__ void softmax_tile(f32x16 (&S)[2][2], uint32_t (&P)[2][2][8], f32x16 (&O)[2][2],
                                             float (&ref)[2], f16x4 (&qbias)[2], float (&lrun)[2], int g,
                                             int sbase, int n_total, bool tail, const char* lds,
                                             const int (&koff)[4], const f16x8 (&qf)[2][4], f16x4 kones,
                                             const char* ktile_mem, int kfrag_row0, const Loads& loads) {
  float lsum[2];
  bool overflow = false;
  if (__builtin_expect(tail, 0)) mask_absent_slots(S, sbase, n_total);
  if constexpr (!force) {
    lsum[0] = tile_weights<false, 0>(S[0][0], S[1][0], 0.f, P[0][0], P[1][0], loads);
    lsum[1] = tile_weights<false, 1>(S[0][1], S[1][1], 0.f, P[0][1], P[1][1], loads);

    // one overflow test for both query blocks; the compare is issued before the conversions to half
    // are forced out, so the branch does not wait for the VALU pipeline to drain
    overflow =
        __builtin_amdgcn_ballot_w64(!(lsum[0] <= kWeightSumLimit) || !(lsum[1] <= kWeightSumLimit)) != 0ull;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < 8; ++j) asm volatile("" : "+v"(P[a][b][j]));
  }
  if (__builtin_expect(overflow || force, 0)) {
    // rare: the exponents are recomputed from the K tile (still resident in this phase) rather than
    // kept alive through the fast path, which frees their registers for the weights.  The first tile
    // of a segment comes here directly: its exponents (taken against the reference 0) are still in S.
    if constexpr (!force) {
      // (a piece whose tiles are shared by both wave sets reads them from memory instead: set B
      // comes here while set A's request for the tile after next is already filling this buffer)
      f16x8 kf[4][2];
      if (ktile_mem) {
        // uniform base; this lane's offset is worked out here from the lane number (row kfrag_row0 +
        // lane % 32, 16-byte piece lane / 32 of each 32-byte step): kept from the start of the
        // kernel it would be one more value to spill around the tile loop
        const int ln = lane_number_here();
        const uint32_t kfrag_off = (uint32_t)((kfrag_row0 + (ln & 31)) * 128 + (ln >> 5) * 16);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          kf[ks][0] = *(const f16x8*)(ktile_mem + (kfrag_off + ks * 32));
          kf[ks][1] = *(const f16x8*)(ktile_mem + (kfrag_off + ks * 32 + 32 * 128));
        }
      } else {
        k_frags<PAR>(lds, koff, kf);
      }
      qk_tile(kf, qf, qbias, kones, S);
      if (tail) mask_absent_slots(S, sbase, n_total);
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      float mx = S[0][qb][0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, S[0][qb][i]);
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[1][qb][i]);
      mx = pair_max(mx);
      // the tile's maximum of s*c is mx + ref; the new reference is that minus 7, rounded to half
      const float want = fminf(fmaxf(mx + ref[qb] - kWeightBias, -65504.f), 65504.f);
      const float cand = (float)(_Float16)want;
      const float rnew = force ? cand : fmaxf(ref[qb], cand);
      const float d = ref[qb] - rnew;
      const float alpha = force ? 1.f : __builtin_amdgcn_exp2f(d);     // nothing accumulated yet when forced
      ref[qb] = rnew;
      qbias[qb] = bias_operand(rnew, g);
      lrun[qb] *= alpha;
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[db][qb][i] *= alpha;
      // (the forced first tile comes here without the fast path: its loads are issued here)
      if (force && qb == 0) lsum[qb] = tile_weights<true, 0>(S[0][qb], S[1][qb], d, P[0][qb], P[1][qb], loads);
      else if (force) lsum[qb] = tile_weights<true, 1>(S[0][qb], S[1][qb], d, P[0][qb], P[1][qb], loads);
      else lsum[qb] = tile_weights<true, 0>(S[0][qb], S[1][qb], d, P[0][qb], P[1][qb], NoLoads());
    }
  }
  lrun[0] += lsum[0];
  lrun[1] += lsum[1];
}

// State a wave carries through one segment (a run of tiles of one item).
struct TileCtx {
  const char* lds;            // base of the LDS array
  const char* kbase;          // K rows of this set's (layer, head)
  const char* vbase;
  uint32_t lane_off;          // this lane's byte offset inside a tile for the direct-to-LDS loads
  uint32_t lds_ld;            // LDS byte address of this wave's 32 rows in K buffer 0 of its set
  int t1, T, n_total, slot0;  // slot0: first slot of this wave's accumulator rows within a tile
  int g;                      // which 8-index group of the contraction this lane holds
  bool active;
  // which of a tile's loads this wave set issues, and where it awaits them.  Two heads: each set
  // loads its own K (matrix phase) and V (vector phase) and awaits K at the end of the vector phase.
  // One head, shared tiles: set A loads K for both (awaited at the end of its vector phase), set B
  // loads V for both at the start of its vector phase -- when set A, a phase ahead, has finished
  // with the V tile two back -- and awaits it at the end of its next matrix phase, one phase before
  // set A multiplies by it.
  bool shared, ldk, ldv;
  int kfrag_row0;             // first of this wave's 64 rows inside a K tile (slow path of shared pieces)
  OVGGT_TRACE_ONLY(unsigned long long tr_m, tr_x, tr_v, tr_y, tr_w;)   // cycles in matrix phase, at its barrier, in vector phase, at its barrier
};

// Per-wave attention state of one segment.
struct SegState {
  f16x8 qf[2][4];             // Q'^T fragments: c * q rounded to half
  f16x4 qbias[2];             // bias operand of each query block (-ref at contraction index 0)
  f16x4 kones;                // K-side operand of the bias step (1 at contraction index 0)
  f32x16 S[2][2], O[2][2];
  uint32_t P[2][2][8];
  float ref[2], lrun[2];
};

// One tile: matrix phase, barrier, vector phase, barrier.  PAR is the parity of the tile within the
// segment and selects the LDS buffers at compile time (no address arithmetic on the VALU).
template <int PAR, bool FIRST>
__device__ __forceinline__ void tile_step(TileCtx& x, int tt, const int (&koff)[4],
                                          const int (&voff)[2][2], SegState& z) {
  const bool more = tt + 1 < x.t1;
  OVGGT_TRACE_ONLY(
    const unsigned long long tr0 = clock64();
    __builtin_amdgcn_sched_barrier(0);
  )
  // ---- matrix phase
  __builtin_amdgcn_s_setprio(kPrioMatrix);
  if (x.active) {
    if (more && x.ldk)
      load_rows_to_lds(x.kbase + (size_t)(tt + 1) * kTileBytes, x.lane_off, x.lds_ld + (PAR ^ 1) * 2 * kTileBytes);
    f16x8 kf[4][2];
    if (!FIRST) pv_tile<PAR ^ 1>(x.lds, voff, z.P, z.O);
    k_frags<PAR>(x.lds, koff, kf);
    qk_tile(kf, z.qf, z.qbias, z.kones, z.S);
    if (!FIRST) {
      // Issue order of this phase (one scheduling region: 24 LDS reads, 34 MFMAs).  Left alone the
      // scheduler saves registers by reading each operand right before the MFMA that needs it and
      // exposes the LDS latency every time; instead: two V^T fragment groups up front, then each
      // group of four P V MFMAs is followed by the four reads the MFMAs two groups later need
      // (the rest of V^T, then K in two halves), so the Q K^T MFMAs find their operands in registers.
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
      for (int grp = 0; grp < 3; ++grp) {
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);      // last P V group and the two bias steps
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);      // second half of K
      __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
    }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) asm volatile("" : "+v"(z.S[a][b]));      // issued before the barrier
  }
  __builtin_amdgcn_s_setprio(kPrioVector);
  // shared tiles: the V rows this set requested a phase ago are multiplied by the other set next
  if (x.shared && x.ldv) __builtin_amdgcn_s_waitcnt(kWaitVm0);
  OVGGT_TRACE_ONLY(
    __builtin_amdgcn_sched_barrier(0);
    const unsigned long long tr1 = clock64();
  )
  phase_barrier();
  OVGGT_TRACE_ONLY(
    const unsigned long long tr2 = clock64();
    __builtin_amdgcn_sched_barrier(0);
  )
  // ---- vector phase
  if (x.active) {
    const TileLoads vl{more && x.ldv, x.vbase + (size_t)(tt + 1) * kTileBytes, x.lane_off,
                       x.lds_ld + (PAR ^ 1) * 2 * kTileBytes + kTileBytes};
    softmax_tile<PAR, FIRST>(z.S, z.P, z.O, z.ref, z.qbias, z.lrun, x.g, tt * kSlotTile + x.slot0, x.n_total,
                             tt == x.T - 1 && (x.n_total & (kSlotTile - 1)) != 0, x.lds, koff, z.qf, z.kones,
                             x.shared ? x.kbase + (size_t)tt * kTileBytes : nullptr, x.kfrag_row0, vl);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < 8; ++j) asm volatile("" : "+v"(z.P[a][b][j]));   // computed before the barrier
  }
  OVGGT_TRACE_ONLY(
    __builtin_amdgcn_sched_barrier(0);
    const unsigned long long tr2b = clock64();
    __builtin_amdgcn_sched_barrier(0);
  )
  // K of tile tt+1 (and everything older) has landed; only V of tile tt+1 may still be in flight
  // (a set that requests one kind only has four loads in flight at most: it awaits them all)
  if (more && x.ldk && x.ldv) __builtin_amdgcn_s_waitcnt(kWaitVm4);
  else if (x.ldk) __builtin_amdgcn_s_waitcnt(kWaitVm0);
  OVGGT_TRACE_ONLY(
    __builtin_amdgcn_sched_barrier(0);
    const unsigned long long tr3 = clock64();
  )
  phase_barrier();
  OVGGT_TRACE_ONLY(
    const unsigned long long tr4 = clock64();
    x.tr_m += tr1 - tr0; x.tr_x += tr2 - tr1; x.tr_v += tr2b - tr2; x.tr_y += tr4 - tr3; x.tr_w += tr3 - tr2b;
  )
}

// Touches every 64-byte line of the kernel's argument block (the explicit arguments and the
// launch dimensions behind them) with one scalar load each, all in flight together, and waits for
// them once.  The plan in AttnParams is read piecemeal and in dependent steps (grid size, chunk
// table, unit decoding, tile addresses); left cold, each step is a round trip to memory of its own
// at the start of every workgroup (measured: 4.5 thousand cycles before the first tile is
// requested).  The wait is part of the same statement: the compiler does not know that these are
// loads, so nothing of them may still be in flight when it reuses the register.
__device__ __forceinline__ void warm_kernel_arguments() {
  static_assert(sizeof(AttnParams) + 64 <= 14 * 64, "one load per 64-byte line of the argument block");
  const char __attribute__((address_space(4)))* ka =
      (const char __attribute__((address_space(4)))*)__builtin_amdgcn_kernarg_segment_ptr();
  uint32_t sink;
  asm volatile("s_load_dword %0, %1, 0x0\n\ts_load_dword %0, %1, 0x40\n\ts_load_dword %0, %1, 0x80\n\t"
               "s_load_dword %0, %1, 0xc0\n\ts_load_dword %0, %1, 0x100\n\ts_load_dword %0, %1, 0x140\n\t"
               "s_load_dword %0, %1, 0x180\n\ts_load_dword %0, %1, 0x1c0\n\ts_load_dword %0, %1, 0x200\n\t"
               "s_load_dword %0, %1, 0x240\n\ts_load_dword %0, %1, 0x280\n\ts_load_dword %0, %1, 0x2c0\n\t"
               "s_load_dword %0, %1, 0x300\n\ts_load_dword %0, %1, 0x340\n\t"
               "s_waitcnt lgkmcnt(0)"
               : "=&s"(sink) : "s"(ka) : "memory");
}

__global__ void __launch_bounds__(kAttnThreads, 1) attn_bf16_kernel(AttnParams p) {
  warm_kernel_arguments();
  // [set][parity][K | V]; behind them room for the second slot-half merge area of a piece whose tiles
  // both sets share (such a piece keeps its tiles in set A's region and merges in set B's and behind)
  __shared__ __attribute__((aligned(1024))) char lds[kSetBytes + 2 * kMergeBytes];
  const int tid = threadIdx.x, lane0 = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int set = wave >> 2, wv = wave & 3;
  const int qhalf = wv & 1, khalf = wv >> 1;
  const int lane = lane0, l32 = lane0 & 31, g = lane0 >> 5;   // for the set-up below; every piece forms its own

  const int G = gridDim.x;
  const int cidx = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);
  if (!p.item_mode && chunk_first_unit(p, cidx) >= p.total_units) return;   // whole workgroup: no barrier has been executed yet
  OVGGT_TRACE_ONLY(
    const unsigned long long tr_w0 = wall_clock64(), tr_c0 = clock64();
    unsigned long long tr_n = 0;
  )

  // per-lane LDS offsets (the set's region included; set B's move to set A's region and back when
  // a piece with shared tiles begins or ends: kSetBytes is a power of two, the move is one XOR)
  int region = set * kSetBytes;                        // where this set's tiles are at the moment
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    koff[ks] = set * kSetBytes + (khalf * 64 + l32) * 128 + ((((2 * ks + g) ^ swz(l32))) << 4);
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
        voff[db][hh] = set * kSetBytes + (khalf * 64 + 8 * hh + x) * 128 + ((((c0 + 4 * db) ^ swz(8 * hh + x))) << 4) + inb;
  }

  TileCtx x;
  OVGGT_TRACE_ONLY(x.tr_m = x.tr_x = x.tr_v = x.tr_y = x.tr_w = 0;)
  x.lds = lds;
  x.T = p.T;
  x.n_total = p.n_total;
  x.g = g;
  x.slot0 = khalf * 64;
  {
    const int ld_row = lane >> 3;
    x.lane_off = (uint32_t)((wv * 32 + ld_row) * 128 + (((lane & 7) ^ swz(ld_row)) << 4));
    x.kfrag_row0 = khalf * 64;
  }

  // Set B runs one barrier behind set A, so that its matrix phases coincide with A's vector phases:
  // it executes one barrier more than A before its first tile (below, once its first piece's loads
  // are on their way) and A makes up for it at the end.  `started` is uniform over the workgroup.
  bool started = false;

  // Head pairs are dealt out round by round: in every round an XCD's workgroups share one head
  // pair (its K/V tiles then live in that XCD's L2 while all its query blocks pass over them).
  for (int rnd = 0; rnd < p.rounds; ++rnd) {
  const ChunkRange cr = chunk_range(p, rnd, cidx, G);
  const int chunk_idx = cr.rec_chunk;
  int u = (int)cr.u0;
  const int u_end = (int)cr.u1;
  const int u_begin = u;
  int n_piece = 0;
  while (u < u_end) {
    const UnitPos up = decode_unit(u, p.T, p.QB, p.NS, p.L0, p.PP);
    if (!up.valid) break;                                // the rest of the chunk is empty slots
    const int t0 = up.tile;
    const int t1 = min(up.seg_end, t0 + (u_end - u));
    // plain order: only the first and the last piece of a chunk can be partial (records 0 and 1);
    // segmented order: every piece is partial and takes the next record
    const int rec_ord = p.NS == 1 ? (u == u_begin ? 0 : 1) : n_piece;
    ++n_piece;
    const bool full = (p.NS == 1 && t0 == 0 && t1 == p.T);
    // What a piece needs of the lane number (query rows, operand constants, record offsets) is worked
    // out again from an opaque copy at its start and at its end: carried from the start of the kernel,
    // or across the tile loop, these values are what the register allocator spills to memory.
    int lane_p = lane0;
    asm volatile("" : "+v"(lane_p));
    const int l32 = lane_p & 31, g = lane_p >> 5;
    const SetWork sw = work_of_item(up.hp, up.qb, set, p.QB, p.share);
    const int qb_idx = sw.qb;
    const int lh = sw.lh;                                // this set's (layer, head)
    const bool active = lh < p.LH;
    x.shared = sw.shared;
    x.ldk = !sw.shared || set == 0;
    x.ldv = !sw.shared || set == 1;
    {
      const int want = sw.shared ? 0 : set * kSetBytes;
      if (want != region) {                              // uniform over the wave set
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) koff[ks] ^= kSetBytes;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) voff[db][hh] ^= kSetBytes;
        region = want;
      }
      x.lds_ld = (uint32_t)(uintptr_t)LDS_PTR(char, lds) + (uint32_t)(region + wv * 4096);
    }
    // slot-half merge area: the set's own tile region once its tiles are done with; pieces with
    // shared tiles (all in set A's region, still read by set B while A merges) use set B's region
    // and the space behind it
    char* const lset = lds + (sw.shared ? kSetBytes + set * kMergeBytes : set * kSetBytes);
    const int li = active ? lh / p.H : 0;
    const int h = active ? lh - li * p.H : 0;
    x.active = active;
    x.t1 = t1;
    x.kbase = p.kv0 + (size_t)li * p.kv_layer_bytes + (size_t)h * p.cap * 128;
    x.vbase = x.kbase + p.v_off;
    const int q0 = qb_idx * kQueryTile;

    // prologue: first tile of the segment into the parity-0 buffers
    if (active) {
      if (x.ldk) load_rows_to_lds(x.kbase + (size_t)t0 * kTileBytes, x.lane_off, x.lds_ld);
      if (x.ldv) load_rows_to_lds(x.vbase + (size_t)t0 * kTileBytes, x.lane_off, x.lds_ld + kTileBytes);
    }

    // Q'^T fragments: lane holds query (q0 + qhalf*64 + qb*32 + l32), d = ks*16 + 8g .. +8, as
    // half(c * q): the scores then leave the matrix pipe already in the exp2 domain
    SegState z;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      int qrow = q0 + qhalf * 64 + qb * 32 + l32;
      if (qrow > p.M - 1) qrow = p.M - 1;
      const char* qp = p.q + ((((size_t)li * p.M + qrow) * p.H + h) * 64) * 2;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const u32x4 w = *(const u32x4*)(qp + (ks * 16 + 8 * g) * 2);
        u32x4 r;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          f16x2 hh;
          // c * q beyond the half range is clamped to +-65504 (it would turn into +-inf and the row into NaN)
          hh[0] = (_Float16)__builtin_amdgcn_fmed3f(__uint_as_float(w[e] << 16) * p.c, -65504.f, 65504.f);
          hh[1] = (_Float16)__builtin_amdgcn_fmed3f(__uint_as_float(w[e] & 0xFFFF0000u) * p.c, -65504.f, 65504.f);
          r[e] = __builtin_bit_cast(uint32_t, hh);
        }
        z.qf[qb][ks] = __builtin_bit_cast(f16x8, r);
      }
    }
    {
      const u32x2 one = {g == 0 ? 0x00003C00u : 0u, 0u};                  // half 1.0 at contraction index 0
      z.kones = __builtin_bit_cast(f16x4, one);
    }
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      z.ref[a] = 0.f;                                    // replaced on the first tile (forced slow path)
      z.lrun[a] = 0.f;
      z.qbias[a] = bias_operand(0.f, g);
#pragma unroll
      for (int b = 0; b < 2; ++b) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { z.O[a][b][i] = 0.f; z.S[a][b][i] = 0.f; }
#pragma unroll
        for (int j = 0; j < 8; ++j) z.P[a][b][j] = 0u;
      }
    }

    // set B's extra barrier comes behind its first requests, not in front of them: both sets' cold
    // loads of the first tiles and queries are in flight together instead of one after the other
    if (!started && set == 1) phase_barrier();
    started = true;
    // the builtin wait also tells the compiler that the loads it tracks itself (Q) are complete, so
    // it adds no vmcnt waits of its own inside the tile loop
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
    phase_barrier();

    // the first tile has no predecessor to multiply by V and always sets the reference
    tile_step<0, true>(x, t0, koff, voff, z);
    int tt = t0 + 1;
    for (; tt + 1 < t1; tt += 2) {
      tile_step<1, false>(x, tt, koff, voff, z);
      tile_step<0, false>(x, tt + 1, koff, voff, z);
    }
    const bool odd = tt >= t1;                           // an odd number of tiles: the last one had parity 0
    if (!odd) tile_step<1, false>(x, tt, koff, voff, z);
    OVGGT_TRACE_ONLY(tr_n += t1 - t0;)

    // (end of the piece: the lane-derived values again, from a second opaque copy)
    int lane_e = lane0;
    asm volatile("" : "+v"(lane_e));
    const int l32e = lane_e & 31, ge = lane_e >> 5;
    // P V of the last tile
    if (active) {
      if (odd) pv_tile<0>(lds, voff, z.P, z.O);
      else pv_tile<1>(lds, voff, z.P, z.O);
    }
    f32x16 (&O)[2][2] = z.O;
    float (&lrun)[2] = z.lrun;

    // ---- merge the two slot halves through the set's LDS
    float ltot[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) ltot[qb] = pair_sum(lrun[qb]);
    __syncthreads();                                  // all tile reads done; the set's LDS is free
    float* mO = (float*)lset + qhalf * (64 * 64);      // [reg][lane]
    float* mML = (float*)lset + 2 * 64 * 64 + qhalf * (4 * 64);
    if (active && khalf == 1) {
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mO[((db * 2 + qb) * 16 + i) * 64 + lane_e] = O[db][qb][i];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        mML[qb * 64 + lane_e] = z.ref[qb];
        mML[(2 + qb) * 64 + lane_e] = ltot[qb];
      }
    }
    __syncthreads();
    if (active && khalf == 0) {
      float mfin[2], lfin[2];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const float m0 = z.ref[qb], m1 = mML[qb * 64 + lane_e];
        const float mt = fmaxf(m0, m1);
        const float a0 = __builtin_amdgcn_exp2f(m0 - mt), a1 = __builtin_amdgcn_exp2f(m1 - mt);
        mfin[qb] = mt;
        lfin[qb] = ltot[qb] * a0 + mML[(2 + qb) * 64 + lane_e] * a1;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            O[db][qb][i] = O[db][qb][i] * a0 + mO[((db * 2 + qb) * 16 + i) * 64 + lane_e] * a1;
      }
      if (full) {
        // same rule as below: offsets first, then nothing but stores
        size_t oo[2];
        float inv[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const int qrow = q0 + qhalf * 64 + qb * 32 + l32e;
          oo[qb] = ((size_t)qrow * p.H) * 64 + 4 * ge;
          inv[qb] = 1.0f / lfin[qb];
        }
        asm volatile("" : "+v"(oo[0]), "+v"(oo[1]), "+v"(inv[0]), "+v"(inv[1]));
        const size_t obase = ((size_t)li * p.M * p.H + h) * 64;          // uniform
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const int qrow = q0 + qhalf * 64 + qb * 32 + l32e;
          if (qrow < p.M) {
            if (p.out_f32) {
              float* op = (float*)p.out + obase + oo[qb];
#pragma unroll
              for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int ig = 0; ig < 4; ++ig) {
                  float4 w = {O[db][qb][ig * 4] * inv[qb], O[db][qb][ig * 4 + 1] * inv[qb],
                              O[db][qb][ig * 4 + 2] * inv[qb], O[db][qb][ig * 4 + 3] * inv[qb]};
                  *(float4*)(op + db * 32 + ig * 8) = w;
                }
            } else {
              __bf16* op = (__bf16*)p.out + obase + oo[qb];
#pragma unroll
              for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int ig = 0; ig < 4; ++ig) {
                  bf16x4 w;
#pragma unroll
                  for (int j = 0; j < 4; ++j) w[j] = (__bf16)(O[db][qb][ig * 4 + j] * inv[qb]);
                  *(bf16x4*)(op + db * 32 + ig * 8) = w;
                }
            }
          }
        }
      } else {
        // Every address is formed before the first store: a register reloaded from scratch between
        // two stores would have to wait for all stores before it (one counter covers loads and
        // stores), about a thousand cycles each time.
        // The O part of a record is laid out the way the accumulators sit in registers -- block
        // (query half, db, qb, ig), then lane, then the lane's four values -- so every store
        // instruction writes 1 KiB of consecutive memory (partial_block_offset; the merge pass
        // reads it back the same way and transposes on its way out).
        float* rec = p.ws + (size_t)((kSegRecs * chunk_idx + rec_ord) * 2 + set) * kPartialFloats;
        uint32_t ro = (uint32_t)(partial_block_offset(qhalf, 0, 0, 0) + lane_e * 4);
        uint32_t mo = (uint32_t)(kQueryTile * 64 + qhalf * 64 + l32e);
        asm volatile("" : "+v"(ro), "+v"(mo));
        float* rp0 = rec + ro;
        float* mp = rec + mo;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
          for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int ig = 0; ig < 4; ++ig) {
              float4 w = {O[db][qb][ig * 4], O[db][qb][ig * 4 + 1], O[db][qb][ig * 4 + 2], O[db][qb][ig * 4 + 3]};
              *(float4*)(rp0 + partial_block_offset(0, db, qb, ig)) = w;
            }
        }
        if (ge == 0) {
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) {
            mp[qb * 32] = mfin[qb];
            mp[kQueryTile + qb * 32] = lfin[qb];
          }
        }
      }
    }
    // the merge scratch is reused as tile buffers: everybody's LDS reads must be done, while the
    // stores of the result may still be on their way
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    phase_barrier();
    u += t1 - t0;
  }
  }
  if (started && set == 0) phase_barrier();            // set A: the barrier set B executed before its first tile
  OVGGT_TRACE_ONLY(
    if (lane0 == 0) {
      unsigned long long* tr = (unsigned long long*)(p.ws + p.trace_off) - (size_t)(cidx * 8 + wave + 1) * 8;
      tr[0] = x.tr_w; tr[1] = wall_clock64() - tr_w0; tr[2] = clock64() - tr_c0; tr[5] = tr_n;
      tr[3] = x.tr_m; tr[4] = x.tr_x; tr[6] = x.tr_v; tr[7] = x.tr_y;
    }
  )
}

// One round of the merge: up to kMaxParts partial records of a row are fetched together (all loads
// in flight at once) and folded into the running (acc, l, mt) of the thread's two float4 pieces.
constexpr int kMaxParts = 4;
__device__ __forceinline__ void combine_round(const AttnParams& p, const uint32_t (&recs)[kMaxParts], int n, int row,
                                              int off0, int off1, float4& acc0, float4& acc1, float& l, float& mt) {
  float m[kMaxParts], lp[kMaxParts];
  float4 o0[kMaxParts], o1[kMaxParts];
#pragma unroll
  for (int j = 0; j < kMaxParts; ++j) {
    const float* rec = p.ws + (size_t)recs[j] * kPartialFloats;       // entries beyond n repeat the last one
    m[j] = rec[kQueryTile * 64 + row];
    lp[j] = rec[kQueryTile * 64 + kQueryTile + row];
    o0[j] = *(const float4*)(rec + off0);
    o1[j] = *(const float4*)(rec + off1);
  }
  float mn = mt;
#pragma unroll
  for (int j = 0; j < kMaxParts; ++j)
    if (j < n) mn = fmaxf(mn, m[j]);
  const float rs = __builtin_amdgcn_exp2f(mt - mn);      // 0 in the first round (mt = -inf)
  acc0.x *= rs; acc0.y *= rs; acc0.z *= rs; acc0.w *= rs;
  acc1.x *= rs; acc1.y *= rs; acc1.z *= rs; acc1.w *= rs;
  l *= rs;
  mt = mn;
#pragma unroll
  for (int j = 0; j < kMaxParts; ++j)
    if (j < n) {
      const float w = __builtin_amdgcn_exp2f(m[j] - mt);
      l += lp[j] * w;
      acc0.x += o0[j].x * w; acc0.y += o0[j].y * w; acc0.z += o0[j].z * w; acc0.w += o0[j].w * w;
      acc1.x += o1[j].x * w; acc1.y += o1[j].y * w; acc1.z += o1[j].z * w; acc1.w += o1[j].w * w;
    }
}

// Merge the partials of every item that was split across workgroups.  A workgroup takes the 32 query
// rows of one (query half, qb) group of one item: 8 blocks of 256 floats in every record, two per
// wave, read the way they were written (lane * 4 + j: 1 KiB of consecutive memory per wave and
// load); the merged rows are transposed through LDS so that the output leaves in whole 256-byte rows.
constexpr int kCombineRows = 32;
constexpr int kCombinePitch = 68;                      // floats per LDS row (64 + 4: the transposing stores spread over the banks)
__global__ void __launch_bounds__(256) attn_combine_kernel(AttnParams p) {
  const int item = blockIdx.x / (kQueryTile / kCombineRows);     // (layer-head, query block)
  const int rgrp = blockIdx.x % (kQueryTile / kCombineRows);     // 2 * query half + qb
  const int qb_out = item % p.QB;                                // the query block whose rows are written
  const int lh = item / p.QB;
  const ItemOfBlock ib = item_of_block(lh, qb_out, p.QB, p.share);
  const int qb_idx = ib.j;                                       // the plan's item within the head pair
  const int set = ib.set;
  const int hp = lh >> 1;
  const int lane = threadIdx.x & 63, blk = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int row = rgrp * kCombineRows + l32;                     // this thread's row within the query block
  const int li = lh / p.H;
  const int h = lh - li * p.H;
  const int qrow0 = qb_out * kQueryTile + rgrp * kCombineRows;   // the workgroup's first query
  if (qrow0 >= p.M) return;                                      // whole workgroup, before any barrier
  // this thread's two pieces: blocks 2*blk and 2*blk+1 of the group (block = 4*db + ig)
  const int b0 = 2 * blk, b1 = 2 * blk + 1;
  const int off0 = partial_block_offset(rgrp >> 1, b0 >> 2, rgrp & 1, b0 & 3) + lane * 4;
  const int off1 = partial_block_offset(rgrp >> 1, b1 >> 2, rgrp & 1, b1 & 3) + lane * 4;
  constexpr int kSegGroup = 64;                        // segments whose records are listed at a time
  __shared__ uint32_t rec_list[kSegGroup * kSegRecs];
  __shared__ int n_list;
  __shared__ __attribute__((aligned(16))) float tile[kCombineRows * kCombinePitch];
  float4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f, mt = -INFINITY;
  if (p.rec_table_on) {
    // table of the item's records: no list to build, every thread walks the same few entries
    const int n = p.rec_count[qb_idx];
    if (n == kWholeItem) return;
    for (int i0 = 0; i0 < n; i0 += kMaxParts) {
      uint32_t recs[kMaxParts];
#pragma unroll
      for (int j = 0; j < kMaxParts; ++j) {
        const uint32_t e = p.rec_table[qb_idx][min(i0 + j, n - 1)];
        recs[j] = (uint32_t)((kSegRecs * (hp * p.cpp + (int)(e & 255u)) + (int)(e >> 8)) * 2 + set);
      }
      combine_round(p, recs, min(kMaxParts, n - i0), row, off0, off1, acc0, acc1, l, mt);
    }
  } else if (p.item_mode) {
    // whole-item launches: only the items of an XCD's last round were cut, each over a few of the
    // XCD's chunks (plain order: a chunk's first piece is record 0, a later one record 1)
    const int x = hp / p.ppx;
    const int i = (hp - x * p.ppx) * p.QB + qb_idx;
    if (i < p.rf * p.per_xcd) return;
    const long ua = (long)(i - p.rf * p.per_xcd) * p.T, ub = ua + p.T - 1;
    const int cf = (int)(ua / p.lo_chunk), cl = (int)(ub / p.lo_chunk);
    if (cf == cl) return;                                  // one workgroup did the whole item and wrote it
    for (int c0 = cf; c0 <= cl; c0 += kMaxParts) {
      uint32_t recs[kMaxParts];
#pragma unroll
      for (int j = 0; j < kMaxParts; ++j) {
        const int c = min(c0 + j, cl);
        const int ord = (long)c * p.lo_chunk < ua ? 1 : 0;
        recs[j] = (uint32_t)((kSegRecs * (x * p.per_xcd + c) + ord) * 2 + set);
      }
      combine_round(p, recs, min(kMaxParts, cl - c0 + 1), row, off0, off1, acc0, acc1, l, mt);
    }
  } else
  for (int sg0 = 0; sg0 < p.NS; sg0 += kSegGroup) {
    // The first wave lists the records that hold pieces of this item (integer divisions, done once).
    // With a table of chunk starts, lane l holds the start of the head pair's chunk l and one ballot
    // finds the chunk of a unit: the last one that starts at or before it.
    __syncthreads();
    if (threadIdx.x < 64) {
      const int cs_l = (p.cpp > 0 && lane < p.cpp) ? p.cstart[lane] : 0x7FFFFFFF;
      auto chunk_of = [&](long u) -> int {
        if (p.cpp == 0) return (int)(u / p.chunk);
        const int hp2 = (int)(u / p.PP);
        const int r = (int)(u - (long)hp2 * p.PP);
        const unsigned long long m = __ballot(cs_l <= r);             // never empty: the first chunk starts at 0
        return hp2 * p.cpp + 63 - __builtin_clzll(m);
      };
      int n = 0;
      for (int sg = sg0; sg < min(sg0 + kSegGroup, p.NS); ++sg) {
        const int seg0 = sg * p.L0;
        const int len = (sg == p.NS - 1 ? p.T : seg0 + p.L0) - seg0;
        const long ua = (long)hp * p.PP + (long)p.QB * seg0 + (long)qb_idx * len, ub = ua + len - 1;
        const int cf = chunk_of(ua), cl = chunk_of(ub);
        if (p.NS == 1 && cf == cl) { n = -1; break; }          // one workgroup did the whole item and wrote it
        const int combo = (hp * p.NS + sg) * p.QB + qb_idx;
        for (int c = cf; c <= cl && n < kSegGroup * kSegRecs; ++c) {
          // which of the chunk's records: plain order, 0 if the chunk starts with this item, else
          // 1; segmented order, the pieces of a chunk are numbered in unit order
          const long cu = chunk_first_unit(p, c);
          if (cu >= chunk_first_unit(p, c + 1)) continue;       // an empty chunk holds nothing
          int ord;
          if (p.NS == 1) ord = cu < ua ? 1 : 0;
          else ord = combo - decode_unit(cu, p.T, p.QB, p.NS, p.L0, p.PP).combo;
          if (lane == 0) rec_list[n] = (uint32_t)((kSegRecs * c + ord) * 2 + set);
          ++n;
        }
      }
      if (lane == 0) n_list = n;
    }
    __syncthreads();
    if (n_list < 0) return;
    const int n = n_list;
    for (int i0 = 0; i0 < n; i0 += kMaxParts) {
      uint32_t recs[kMaxParts];
#pragma unroll
      for (int j = 0; j < kMaxParts; ++j) recs[j] = rec_list[min(i0 + j, n - 1)];
      combine_round(p, recs, min(kMaxParts, n - i0), row, off0, off1, acc0, acc1, l, mt);
    }
  }
  // normalise, transpose through LDS, store whole rows
  const float inv = 1.0f / l;
  {
    float* t0 = tile + l32 * kCombinePitch + 4 * g;
    const float4 w0 = {acc0.x * inv, acc0.y * inv, acc0.z * inv, acc0.w * inv};
    const float4 w1 = {acc1.x * inv, acc1.y * inv, acc1.z * inv, acc1.w * inv};
    *(float4*)(t0 + (b0 >> 2) * 32 + (b0 & 3) * 8) = w0;
    *(float4*)(t0 + (b1 >> 2) * 32 + (b1 & 3) * 8) = w1;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int r = (threadIdx.x >> 4) + 16 * k, piece = threadIdx.x & 15;
    const int qrow = qrow0 + r;
    if (qrow >= p.M) continue;
    const float4 w = *(const float4*)(tile + r * kCombinePitch + piece * 4);
    const size_t oel = (((size_t)li * p.M + qrow) * p.H + h) * 64 + piece * 4;
    if (p.out_f32) {
      *(float4*)(p.out + oel * 4) = w;
    } else {
      bf16x4 wb = {(__bf16)w.x, (__bf16)w.y, (__bf16)w.z, (__bf16)w.w};
      *(bf16x4*)(p.out + oel * 2) = wb;
    }
  }
}

// Cost of starting and finishing a piece (Q fragments, the first tile's reference, the merge of the
// slot halves, the partial record, the two wave sets falling out of step), in tiles: workgroups with
// one and with two pieces fit time = 3.6 thousand cycles per tile + 25 thousand per piece.
constexpr float kPieceCostTiles = 7.0f;

// Cut one head pair's QB * T units into `cpp` chunks of equal estimated cost (tiles + kPieceCostTiles
// per piece) and fill p.NS, p.L0, p.PP, p.cpp, p.cstart.  Segments before the last are L0 tiles long
// and give one whole run (one piece) to a chunk each, so neighbouring workgroups still walk the same
// K/V tiles side by side; the runs of the last segment are dealt out greedily.  With equal tile
// counts instead, the workgroups that hold two or three pieces finish 10-20 % after the others.
// False (p untouched) when the shape does not fit the table or a chunk would need more than
// kSegRecs records.
static bool plan_balanced_chunks(AttnParams& p, int cpp) {
  if (cpp < 1 || cpp > kMaxChunksPerPair) return false;
  const int QB = p.QB, T = p.T;
  const float ov = kPieceCostTiles;
  int L0 = (int)(((float)QB * T + ov * (QB - 1)) / cpp + 0.5f);
  if (L0 < 1) L0 = 1;
  int NS = (T + L0 - 1) / L0;
  while (NS > 1 && (NS - 1) * QB >= cpp) {                                // the last segment needs a chunk too
    ++L0;
    NS = (T + L0 - 1) / L0;
  }
  if (NS > 1 && (T - (NS - 1) * L0) + ov < (L0 + ov) * 0.5f) --NS;      // a short remainder joins the segment before it
  if (NS <= 1) { NS = 1; L0 = T; }
  const int lead = (NS - 1) * QB;                 // chunks that are one whole run each
  const int n_rem = cpp - lead;
  const int R = T - (NS - 1) * L0;                // run length of the last segment
  int cs[kMaxChunksPerPair + 1];
  for (int c = 0; c < lead; ++c) cs[c] = c * L0;
  const int base = lead * L0, total_last = QB * R;
  // Last segment: QB runs of R tiles over n_rem chunks.  A chunk is filled run by run up to a cost
  // limit (a piece of x tiles costs ov + x; the rest of a run is split off when at least one more
  // tile fits); the smallest limit that needs no more than n_rem chunks is found by bisection.
  auto fill = [&](float limit, int* starts) -> int {
    int pos = 0, used = 0;
    while (pos < total_last) {
      if (starts && used < n_rem) starts[used] = base + pos;
      ++used;
      float cost = 0.f;
      while (pos < total_last) {
        const int run_left = R - pos % R;
        int x = (int)(limit - cost - ov);
        if (x < 1) {
          if (cost > 0.f) break;
          x = 1;                                   // an empty chunk takes at least one tile
        }
        if (x > run_left) x = run_left;
        pos += x;
        cost += ov + x;
      }
    }
    return used;
  };
  float lo = ((float)total_last + ov * QB) / n_rem, hi = (float)total_last + ov * QB + 1.f;
  if (fill(lo, nullptr) <= n_rem) hi = lo;
  for (int it = 0; it < 24 && hi - lo > 0.05f; ++it) {
    const float mid = 0.5f * (lo + hi);
    if (fill(mid, nullptr) <= n_rem) hi = mid; else lo = mid;
  }
  const int used = fill(hi, cs + lead);
  if (used > n_rem) return false;
  for (int c = used; c < n_rem; ++c) cs[lead + c] = QB * T;          // chunks left over stay empty
  cs[cpp] = QB * T;
  // every chunk within kSegRecs pieces?
  for (int c = lead; c < cpp; ++c) {
    const int a = cs[c] - base, b = cs[c + 1] - base;
    if (b > a && (b - 1) / R - a / R + 1 > kSegRecs) return false;
  }
  // walk one head pair the way the kernel will (all pairs are cut alike): the pieces must tile
  // QB * T units without crossing a segment end, within the records a chunk owns
  long covered = 0;
  for (int c = 0; c < cpp; ++c) {
    if (cs[c] > cs[c + 1]) return false;
    int u = cs[c], partial = 0;
    while (u < cs[c + 1]) {
      const UnitPos up = decode_unit(u, T, QB, NS, L0, QB * T);
      const int t1 = min(up.seg_end, up.tile + (cs[c + 1] - u));
      if (!up.valid || t1 <= up.tile) return false;
      if (!(NS == 1 && up.tile == 0 && t1 == T)) ++partial;
      covered += t1 - up.tile;
      u += t1 - up.tile;
    }
    if (NS > 1 ? partial > kSegRecs : partial > 2) return false;
  }
  if (covered != (long)QB * T) return false;
  p.NS = NS; p.L0 = L0; p.PP = QB * T; p.cpp = cpp;
  for (int c = 0; c <= cpp; ++c) p.cstart[c] = cs[c];
  // which records hold the pieces of query block qb: the same in every head pair
  p.rec_table_on = 0;
  if (QB <= kMaxTableItems) {
    bool ok = true;
    for (int qb = 0; qb < QB && ok; ++qb) {
      int n = 0;
      for (int sg = 0; sg < NS && ok; ++sg) {
        const int seg0 = sg * L0, len = (sg == NS - 1 ? T : seg0 + L0) - seg0;
        const int ua = QB * seg0 + qb * len, ub = ua + len - 1;
        const int cf = chunk_of_unit(p, ua), cl = chunk_of_unit(p, ub);
        if (NS == 1 && cf == cl) { n = kWholeItem; break; }
        const int combo = sg * QB + qb;
        for (int c = cf; c <= cl; ++c) {
          if (cs[c] >= cs[c + 1]) continue;
          const int ord = NS == 1 ? (cs[c] < ua ? 1 : 0) : combo - decode_unit(cs[c], T, QB, NS, L0, QB * T).combo;
          if (n == kMaxTableRecs || ord < 0 || ord >= kSegRecs) { ok = false; break; }
          p.rec_table[qb][n++] = (uint16_t)(c + 256 * ord);
        }
      }
      p.rec_count[qb] = (uint8_t)n;
    }
    p.rec_table_on = ok ? 1 : 0;
  }
  return true;
}

// How a launch is cut into chunks: fills the planning fields of p (LH, QB, T, chunk, NS, L0, PP,
// rounds, cpp, cstart, total_units) and the grid size.  Host only.
static hipError_t plan_attn(AttnParams& p, const Geom& g, int nl, int n_total, size_t ws_bytes, int* n_wgs_io) {
  int n_wgs = *n_wgs_io;
  p.H = g.H; p.M = g.M; p.cap = g.cap; p.n_total = n_total;
  p.LH = nl * g.H;
  p.QB = (g.M + kQueryTile - 1) / kQueryTile;
  p.T = (n_total + kSlotTile - 1) / kSlotTile;
  p.share = (p.LH % 2 == 0 && p.QB >= 2) ? 1 : 0;      // every head pair whole, and at least one pair of blocks
  const long total = (long)((p.LH + 1) / 2) * p.QB * p.T;
  if (total > 0x7FFFFFFFL) return hipErrorInvalidValue;
  p.total_units = (int)total;
  if (n_wgs > kMaxAttnWgs) n_wgs = kMaxAttnWgs;
  n_wgs &= ~7;
  if (n_wgs < 8) n_wgs = 8;
  *n_wgs_io = n_wgs;
  p.chunk = (int)((total + n_wgs - 1) / n_wgs);
  // Tile segments of the chunk's length, so that neighbouring workgroups walk the same tiles of
  // neighbouring query blocks together; a short remainder joins the segment before it, which
  // bounds the pieces of a chunk by kSegRecs (chunk - 1 <= 2 * shortest segment).
  p.NS = (p.T + p.chunk - 1) / p.chunk;
  p.L0 = p.chunk;
  if (p.NS > 1 && p.T - (p.NS - 1) * p.L0 < (p.chunk + 1) / 2) --p.NS;
  if (p.NS <= 1) { p.NS = 1; p.L0 = p.T; }
  p.PP = p.QB * p.T;
  if (p.NS > 1) {                                        // whole chunks per head pair, if the grid has room
    const long padded = (long)((p.PP + p.chunk - 1) / p.chunk) * p.chunk;
    if ((long)((p.LH + 1) / 2) * padded <= (long)n_wgs * p.chunk) p.PP = (int)padded;
  }
  p.total_units = ((p.LH + 1) / 2) * p.PP;
  p.rounds = 1;
  p.cpp = 0;
  p.rec_table_on = 0;
  const int pairs = (p.LH + 1) / 2;
  // one launch round and the workgroups divide evenly among the head pairs: chunks of equal cost
  if (n_wgs % pairs == 0 && plan_balanced_chunks(p, n_wgs / pairs)) {
    p.chunk = 0;
    p.total_units = pairs * p.PP;
  }
  // Many head pairs: deal them out to the XCDs round by round, one head pair per XCD and round, cut
  // into as many chunks as the XCD has workgroups.  The plain split above would hand a workgroup a
  // run of whole items, and the query blocks of a head would re-read its K/V from memory one after
  // the other.
  p.item_mode = 0; p.per_xcd = n_wgs / 8; p.ppx = 0; p.rf = 0; p.lo_chunk = 1;
  if (attn_whole_items(p.LH, p.QB, n_wgs)) {
    // Many head pairs: every workgroup takes whole items, round after round (no partial records, no
    // merge, 7 tiles' worth of piece overhead per 139-tile item instead of per 48-tile chunk), an
    // XCD's workgroups staying on a few consecutive head pairs whose K/V tiles they walk side by
    // side; only the items left over after the last full round are cut.
    const int per_xcd = n_wgs / 8;
    p.item_mode = 1;
    p.ppx = pairs / 8;
    const int ipx = p.ppx * p.QB;
    p.rf = ipx / per_xcd;
    const int lo = ipx - p.rf * per_xcd;
    p.lo_chunk = lo > 0 ? (int)(((long)lo * p.T + per_xcd - 1) / per_xcd) : 1;
    p.rounds = p.rf + (lo > 0 ? 1 : 0);
    p.cpp = 0; p.rec_table_on = 0; p.chunk = 0;
    p.NS = 1; p.L0 = p.T; p.PP = p.QB * p.T;
    p.total_units = pairs * p.PP;
  } else {
    const int per_xcd = n_wgs / 8;
    const long chunks = (long)pairs * per_xcd;
    if (pairs > 8 && pairs % 8 == 0 && p.QB * p.T >= per_xcd &&
        (size_t)chunks * kSegRecs * 2 * kPartialFloats * sizeof(float) <= ws_bytes) {
      if (plan_balanced_chunks(p, per_xcd)) {
        p.chunk = 0;
      } else {
        p.cpp = 0;
        p.rec_table_on = 0;
        p.chunk = (p.QB * p.T + per_xcd - 1) / per_xcd;
        p.NS = (p.T + p.chunk - 1) / p.chunk;
        p.L0 = p.chunk;
        if (p.NS > 1 && p.T - (p.NS - 1) * p.L0 < (p.chunk + 1) / 2) --p.NS;
        if (p.NS <= 1) { p.NS = 1; p.L0 = p.T; }
        p.PP = per_xcd * p.chunk;
      }
      p.total_units = pairs * p.PP;
      p.rounds = pairs / 8;
    }
  }
  return hipSuccess;
}

// Walks a plan the way the kernel does and reports what the workgroups would be given.  Returns
// false when the plan is inconsistent: a tile of some (head pair, query block) covered twice or not
// at all, a piece crossing a segment end, or a chunk with more partial pieces than records.
bool attn_plan_stats(const Geom& g, int nl, int n_total, int n_wgs, size_t ws_bytes, AttnPlanStats* st) {
  AttnParams p;
  if (plan_attn(p, g, nl, n_total, ws_bytes, &n_wgs) != hipSuccess) return false;
  const int pairs = (p.LH + 1) / 2;
  const long n_chunks = (long)p.rounds * n_wgs;
  {
    // items x wave sets -> (layer-head, query block): every existing block exactly once, a shared
    // item on one head and two neighbouring blocks, and the merge pass's inverse agrees
    std::vector<uint8_t> owned((size_t)2 * pairs * p.QB, 0);
    for (int hp = 0; hp < pairs; ++hp)
      for (int j = 0; j < p.QB; ++j) {
        const SetWork a = work_of_item(hp, j, 0, p.QB, p.share), b = work_of_item(hp, j, 1, p.QB, p.share);
        if (a.shared != b.shared) return false;
        if (a.shared && (a.lh != b.lh || b.qb != a.qb + 1 || a.lh >= p.LH)) return false;
        for (int set = 0; set < 2; ++set) {
          const SetWork& w = set ? b : a;
          if (w.lh < 0 || w.lh >= 2 * pairs || w.qb < 0 || w.qb >= p.QB) return false;
          if (owned[(size_t)w.lh * p.QB + w.qb]++) return false;
          const ItemOfBlock ib = item_of_block(w.lh, w.qb, p.QB, p.share);
          if (ib.j != j || ib.set != set || (w.lh >> 1) != hp) return false;
        }
      }
    for (uint8_t o : owned)
      if (o != 1) return false;
    st->shared_items = p.share ? pairs * (p.QB & ~1) : 0;
  }
  std::vector<uint8_t> seen((size_t)pairs * p.QB * p.T, 0);
  std::vector<int> table_refs((size_t)pairs * p.QB, 0);                  // partial pieces seen per item
  st->n_wgs = n_wgs; st->rounds = p.rounds; st->segments = p.NS; st->balanced = p.cpp > 0 ? 1 : 0;
  st->pieces_max = 0; st->tiles_min = 0x7FFFFFFF; st->tiles_max = 0; st->cost_max = 0.f; st->cost_mean = 0.f;
  for (int w = 0; w < n_wgs; ++w) {
    int tiles = 0, pieces_wg = 0;
    for (int rnd = 0; rnd < p.rounds; ++rnd) {
      const ChunkRange cr = chunk_range(p, rnd, w, n_wgs);
      const int c = cr.rec_chunk;
      long u = cr.u0;
      const long u_end = cr.u1;
      if (u > u_end || u_end > p.total_units) return false;
      int partial = 0, n_piece = 0;
      const long u_begin = u;
      while (u < u_end) {
        const UnitPos up = decode_unit(u, p.T, p.QB, p.NS, p.L0, p.PP);
        if (!up.valid) break;
        const int t0 = up.tile, t1 = (int)std::min<long>(up.seg_end, t0 + (u_end - u));
        if (t1 <= t0 || t1 > p.T || up.hp >= pairs || up.qb >= p.QB) return false;
        const bool full = p.NS == 1 && t0 == 0 && t1 == p.T;
        if (!full) ++partial;
        for (int t = t0; t < t1; ++t) {
          uint8_t& cell = seen[((size_t)up.hp * p.QB + up.qb) * p.T + t];
          if (cell) return false;
          cell = 1;
        }
        if (!full && !p.item_mode && chunk_of_unit(p, u) != c) return false;   // the merge pass must find this chunk again
        if (p.item_mode) {                                              // ... here by the same arithmetic as the merge pass
          const int x = up.hp / p.ppx, i = (up.hp - x * p.ppx) * p.QB + up.qb;
          const bool whole_round = i < p.rf * p.per_xcd;
          if (whole_round != (rnd < p.rf) || (whole_round && !full)) return false;
          if (!whole_round) {
            const long off = (long)(i - p.rf * p.per_xcd) * p.T + t0;
            if (x * p.per_xcd + (int)(off / p.lo_chunk) != c || (full != ((off - t0) / p.lo_chunk == (off - t0 + p.T - 1) / p.lo_chunk)))
              return false;
          }
        }
        const int rec_ord = p.NS == 1 ? (u == u_begin ? 0 : 1) : n_piece;
        ++n_piece;
        if (p.rec_table_on) {                                           // ... and the table must list this record once
          const int cnt = p.rec_count[up.qb];
          int hits = 0;
          if (cnt != kWholeItem)
            for (int k = 0; k < cnt; ++k)
              if (p.rec_table[up.qb][k] == (uint16_t)((c - up.hp * p.cpp) + 256 * rec_ord)) ++hits;
          if (hits != (full ? 0 : 1)) return false;
          if (!full) ++table_refs[(size_t)up.hp * p.QB + up.qb];
        }
        tiles += t1 - t0; ++pieces_wg;
        u += t1 - t0;
      }
      if (p.NS > 1 ? partial > kSegRecs : partial > 2) return false;
      if ((size_t)(c + 1) * kSegRecs * 2 * kPartialFloats * sizeof(float) > ws_bytes && partial > 0) return false;
    }
    st->pieces_max = std::max(st->pieces_max, pieces_wg);
    st->tiles_min = std::min(st->tiles_min, tiles);
    st->tiles_max = std::max(st->tiles_max, tiles);
    const float cost = tiles + kPieceCostTiles * pieces_wg;
    st->cost_max = std::max(st->cost_max, cost);
    st->cost_mean += cost / n_wgs;
  }
  (void)n_chunks;
  for (uint8_t v : seen)
    if (!v) return false;
  if (p.rec_table_on)                                                     // no entry that no piece wrote
    for (size_t i = 0; i < table_refs.size(); ++i) {
      const int cnt = p.rec_count[i % p.QB];
      if (table_refs[i] != (cnt == kWholeItem ? 0 : cnt)) return false;
    }
  return true;
}

hipError_t launch_attn_bf16(const Geom& g, char* kv, int layer0, int nl, const void* q, void* out,
                            int n_total, float scale, char* ws, size_t ws_bytes, int n_wgs, bool out_f32,
                            hipStream_t s, hipEvent_t* ev) {
  AttnParams p;
  p.q = (const char*)q;
  p.out = (char*)out;
  p.kv0 = layer_k(kv, g, layer0);
  p.kv_layer_bytes = g.kv_layer_bytes;
  p.v_off = (size_t)g.H * g.cap * g.d * g.esize;
  p.ws = (float*)ws;
  const hipError_t pe = plan_attn(p, g, nl, n_total, ws_bytes, &n_wgs);
  if (pe != hipSuccess) return pe;
  p.trace_off = ws_bytes / sizeof(float);
  p.c = scale * 1.4426950408889634f;
  p.out_f32 = out_f32 ? 1 : 0;
  if (ev && hipEventRecord(ev[0], s) != hipSuccess) return hipErrorUnknown;
  hipLaunchKernelGGL(attn_bf16_kernel, dim3((unsigned)n_wgs), dim3(kAttnThreads), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev && hipEventRecord(ev[1], s) != hipSuccess) return hipErrorUnknown;
  const int items = p.LH * p.QB;
  hipLaunchKernelGGL(attn_combine_kernel, dim3((unsigned)(items * (kQueryTile / kCombineRows))), dim3(256), 0, s, p);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev && hipEventRecord(ev[2], s) != hipSuccess) return hipErrorUnknown;
  return hipSuccess;
}

}  // namespace ovggt
