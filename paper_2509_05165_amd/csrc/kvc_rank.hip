// kvc_head_rank: per (layer, KV head, sequence) stable descending argsort of
// the scores (Section 3.3, eq. 17) and the rank-aligned scores S'.
//
// One workgroup sorts one segment with a least-significant-digit radix sort on
// the order-preserving integer image of the fp32 scores (inverted, so that
// ascending keys are descending scores).  LSD passes are stable, which yields
// the ascending-index order of equal scores for free.
//
// The number of passes follows the data.  A first sweep over the segment counts
// the lowest digit and the top byte of every key; the span of the top bytes says
// how many key bits differ at all once the smallest top byte is subtracted.
// Scores are positive and span some tens of binades, so 26..30 bits matter:
// three passes of 9 bits (span below 2^27) or of 10 bits (below 2^30) replace
// four passes of 8; anything wider (mixed signs) takes four passes of 9 bits.
// The digit counts of pass p+1 are taken while pass p runs.
//
// Between the passes the items travel as (key, position) pairs of 8 bytes, so
// a run of equal digits is one contiguous stretch of memory, written with one
// store per item.  Within a tile every wave ranks its items with ballot-based
// digit matching and lane prefix counts; per-wave digit counters live in LDS.
//
// A segment that fits one tile (n <= 12288) never leaves the chip between the
// passes: the digit-ordered staging area of one pass is the input of the next,
// global memory sees the sweep, one read of the scores and one write of the result.
#include "kvc_internal.h"

namespace kvc {

namespace {

constexpr int RK_THREADS = 1024;
constexpr int RK_WAVES = RK_THREADS / 64;
constexpr int RK_ITEMS9 = 12;              // items per lane and tile of a long segment, 9-bit digits
constexpr int RK_ITEMS10 = 12;             // the same with 10-bit digits (twice the counters in LDS)
constexpr int RK_TILE = RK_THREADS * RK_ITEMS9;
constexpr int RK_SHORT_TILE = RK_THREADS * 4;
constexpr int RK_MAX_BINS = 1024;          // 10-bit digits at most
static_assert(RK_MAX_BINS <= RK_THREADS, "one thread per bin in the scans");

__device__ __forceinline__ uint32_t desc_key(float f) { return ~float_to_ordered(f); }
__device__ __forceinline__ float desc_key_to_float(uint32_t k) { return ordered_to_float(~k); }

// The segment pointers are the same for every lane; telling the compiler so lets
// it address global memory as scalar base + 32-bit lane offset instead of doing
// 64-bit vector arithmetic per access.
template <typename T>
__device__ __forceinline__ T* uniform_ptr(T* p) {
  const uint64_t a = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
  // rebuilt as a global-memory pointer: an integer round trip alone would leave the
  // compiler with a generic pointer and flat instead of global accesses
  typedef __attribute__((address_space(1))) T* global_ptr;
  return (T*)reinterpret_cast<global_ptr>(((uint64_t)hi << 32) | lo);
}

// Element `i` of an array of 4- or 8-byte elements through a 32-bit byte offset
// (segments are shorter than 2^29 items, so 8*i fits): scalar base + 32-bit lane
// offset addressing.
template <typename T>
__device__ __forceinline__ T& at32(T* base, uint32_t i) {
  static_assert(sizeof(T) == 4 || sizeof(T) == 8, "4- or 8-byte elements");
  return *reinterpret_cast<T*>(reinterpret_cast<char*>(base) + (i * (uint32_t)sizeof(T)));
}
template <typename T>
__device__ __forceinline__ const T& at32(const T* base, uint32_t i) {
  static_assert(sizeof(T) == 4 || sizeof(T) == 8, "4- or 8-byte elements");
  return *reinterpret_cast<const T*>(reinterpret_cast<const char*>(base) + (i * (uint32_t)sizeof(T)));
}

// Loads with the streaming (non-temporal) hint, for launches whose segments in
// flight exceed the caches.  What must stay in the L2 cache during a pass are the
// partly written lines at the ends of the digit runs, each completed by the next
// tile some microseconds later; with plain loads the tiles streaming in evict them
// half written, and the memory sees two partial writes per line (the hint took a
// three-pass sort of 256 segments of 131072 items from 0.48 to 0.41 ms).  Where
// the segments in flight fit the 256 MB memory-side cache the hint costs 5-10 %
// instead (256 segments of 32768 items, batches of shorter ones): a pass then
// finds what the pass before wrote still cached, and plain loads keep it there.
constexpr long RK_STREAM_ITEMS = 10L << 20;   // items in flight (longest sequence x workgroups resident) from which loads stream
template <bool STREAM>
__device__ __forceinline__ float load_item(const float* p) {
  return STREAM ? __builtin_nontemporal_load(p) : *p;
}
template <bool STREAM>
__device__ __forceinline__ uint2 load_item(const uint2* p) {
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  if (!STREAM) return *p;
  const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
  return make_uint2(v.x, v.y);
}

// Workgroup barrier that orders LDS traffic only: global stores still in flight
// (the scatter of the previous tile) are not waited for.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// lanes (among `valid`) whose W-bit digit (bits 0..W-1 of `skey`, the key already
// shifted down) equals mine.  Per bit: `mine` is all ones or all zeros (one signed
// bit-field extract), the lanes that agree with it are ~(ballot ^ mine); written
// on 32-bit halves as x & ~(y ^ z), which is one three-input bit operation per half
// (truth table 0x90: the encoding the compiler itself picks for that expression;
// spelled out because it otherwise splits it into an xor and a shared three-input
// and).  Four vector instructions per bit: extract, compare (the ballot), two bit
// operations.
template <int W>
__device__ __forceinline__ uint64_t match_digit(uint32_t skey, uint64_t valid) {
  uint32_t lo = (uint32_t)valid, hi = (uint32_t)(valid >> 32);
#pragma unroll
  for (int bit = 0; bit < W; ++bit) {
    // (spelled as the instruction: the builtin is lowered to a shift pair)
    uint32_t mine;
    asm("v_bfe_i32 %0, %1, %2, 1" : "=v"(mine) : "v"(skey), "n"(bit));
    const uint64_t bal = __ballot(mine != 0u);
    lo = __builtin_amdgcn_bitop3_b32(lo, (uint32_t)bal, mine, 0x90);
    hi = __builtin_amdgcn_bitop3_b32(hi, (uint32_t)(bal >> 32), mine, 0x90);
  }
  return ((uint64_t)hi << 32) | lo;
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive
// moves: shifts by 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source
// add zero), then the last lane of rows 0 and 2 is added to rows 1 and 3, and lane
// 31 to rows 2 and 3.  No index registers and no LDS crossbar traffic, unlike a
// shuffle-based scan.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);   // row_shr:1
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);   // row_shr:2
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);   // row_shr:4
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);   // row_shr:8
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1, 3
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2, 3
  return x;
}

__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(uint32_t(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(uint32_t(mask), 0));
}

// LDS of one workgroup during the passes, for digits of MAXBINS values and tiles
// of up to TILE items.  The tile is as large as LDS allows, because the length of
// a digit run in the write-out (TILE / MAXBINS items of 8 bytes) is what the
// memory system's write rate follows: (512, 12288) and (1024, 12288) take 120 and
// 144 KB, one workgroup per compute unit; the launch for batches of short
// sequences uses (512, 4096), 56 KB, so that two workgroups share a compute unit
// and hide each other's barriers and load latencies.  Per-wave digit counts never
// exceed the tile size and are kept in 16 bits.
template <int MAXBINS, int TILE>
struct RankShared {
  static constexpr int max_bins = MAXBINS;
  static constexpr int tile = TILE;
  static_assert(TILE <= 65535, "16-bit per-wave counters");
  uint2 stage[TILE];                   // the tile as (key, position) in digit order, so that
                                       // the global writes run over consecutive slots
  uint32_t hist[2][MAXBINS];           // digit counts of the running pass and of the next one
  uint32_t bucket[MAXBINS];            // next free global slot of each digit
  uint16_t wave_cnt[RK_WAVES][MAXBINS];
  uint32_t gbase[MAXBINS];             // global slot of an item = gbase[digit] + tile-local slot
  uint32_t wave_tot[RK_WAVES];
};

// LDS of the first sweep over a segment (the layout of the passes is chosen from
// its result and overlays it).
struct RankSweepShared {
  uint32_t low[RK_MAX_BINS];           // counts of the lowest 10 key bits
  uint32_t top[256 * 32];              // counts of the top byte, 32 bank-private copies
  uint32_t top_min, top_max;           // smallest / largest top byte of the segment's keys
};

enum { RK_FIRST = 0, RK_MIDDLE = 1, RK_LAST = 2 };

// One tile of a pass, from the items in registers to the tile in digit order in
// the staging area: every wave ranks its items inside their digit groups, one
// thread per digit turns the per-wave counts into slots, every item is written to
// its slot.
template <int W, int KIND, int ITEMS, typename SH>
__device__ __forceinline__ void rank_and_stage(SH& sh, const uint32_t (&key)[ITEMS],
                                               const int32_t (&val)[ITEMS], int n, int wbase,
                                               int shift, int hsel) {
  constexpr int BINS = 1 << W;
  constexpr uint32_t DMASK = BINS - 1;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  uint32_t rank2[(ITEMS + 1) / 2];   // ranks inside the wave's digit groups, two 16-bit halves per register
  // zero this wave's counters (only this wave touches them until the barrier)
#pragma unroll
  for (int i = 0; i < BINS / 128; ++i) reinterpret_cast<uint32_t*>(sh.wave_cnt[wave])[i * 64 + lane] = 0;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int e = 0; e < ITEMS; ++e) {
    const bool valid = wbase + e * 64 < n;
    const uint64_t vmask = __ballot(valid);
    const uint32_t skey = key[e] >> shift;
    const uint32_t digit = skey & DMASK;
    const uint64_t mask = match_digit<W>(skey, vmask);
    const int below = lanes_below(mask);
    uint32_t prev = 0;
    if (valid) prev = sh.wave_cnt[wave][digit];
    if (e & 1) rank2[e / 2] |= (prev + below) << 16; else rank2[e / 2] = prev + below;
    __builtin_amdgcn_wave_barrier();
    if (valid && below == 0) sh.wave_cnt[wave][digit] = uint16_t(prev + (uint32_t)__popcll(mask));
    if (KIND != RK_LAST && valid) atomicAdd(&sh.hist[hsel ^ 1][(skey >> W) & DMASK], 1u);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  lds_barrier();
  // one thread per digit: digit totals -> tile-local start slots and the global base,
  // per-wave counts -> first slot of each wave's items of the digit (conflict-free columns)
  uint32_t mine = 0, local_start = 0;
  int dtid = tid;                              // (opaque: the addresses of this step are not
  asm volatile("" : "+v"(dtid));               // worth registers across the ranking loop)
  uint32_t cnt[RK_WAVES];
  if (tid < BINS) {
#pragma unroll
    for (int w = 0; w < RK_WAVES; ++w) { cnt[w] = sh.wave_cnt[w][dtid]; mine += cnt[w]; }
    const uint32_t incl = wave_inclusive_sum(mine);
    local_start = incl - mine;                 // exclusive within the wave
    if (lane == 63) sh.wave_tot[wave] = incl;  // (not in use since the bucket scan at the start of the pass)
  }
  lds_barrier();
  if (tid < BINS) {
    uint32_t start = local_start;
    for (int w = 0; w < wave; ++w) start += sh.wave_tot[w];
    const uint32_t g = sh.bucket[dtid];
    sh.gbase[dtid] = g - start;
    sh.bucket[dtid] = g + mine;
    // the counters now become the first tile-local slot of each wave's share of the
    // digit, so that placing an item costs one LDS read
    uint32_t run = start;
#pragma unroll
    for (int w = 0; w < RK_WAVES; ++w) { sh.wave_cnt[w][dtid] = uint16_t(run); run += cnt[w]; }
  }
  lds_barrier();
  // every item goes to its tile-local slot
#pragma unroll
  for (int e = 0; e < ITEMS; ++e) {
    if (wbase + e * 64 < n) {
      const uint32_t digit = (key[e] >> shift) & DMASK;
      const uint32_t slot = sh.wave_cnt[wave][digit] + ((rank2[e / 2] >> (16 * (e & 1))) & 0xffffu);
      sh.stage[slot] = make_uint2(key[e], KIND == RK_FIRST ? uint32_t(wbase + e * 64) : uint32_t(val[e]));
    }
    if (e % 4 == 3) __builtin_amdgcn_sched_barrier(0);   // (four items' temporaries at a time)
  }
}

// One stable counting pass on the W-bit digit at bit `shift` of a segment of n
// items; hist[hsel] holds the digit counts, and unless this is the last pass the
// counts of the next digit are gathered into hist[hsel ^ 1] on the way.  The first
// pass reads the scores themselves (key = inverted ordered image minus `rebase`,
// value = position), the last one writes scores and positions; in between (key,
// value) pairs move.  Tiles are processed in order; item (wave w, slot e, lane l)
// of a tile is element base + w*64*ITEMS + e*64 + l, which is also its order
// inside the tile.
// LIN / LOUT (single-tile segments only): the pass reads its (key, value) pairs
// from / leaves them in the LDS staging area, in slot order.
template <int W, int KIND, bool LIN, bool LOUT, int ITEMS, bool STREAM, typename SH>
__device__ __forceinline__ void radix_pass(SH& sh, int n, int shift, int hsel,
                                           uint32_t rebase, const float* __restrict__ src_f,
                                           const uint2* __restrict__ src_p,
                                           uint2* __restrict__ dst_p, float* __restrict__ dst_f,
                                           int32_t* __restrict__ dst_i) {
  constexpr int BINS = 1 << W;
  constexpr uint32_t DMASK = BINS - 1;
  constexpr int TILE = RK_THREADS * ITEMS;
  static_assert(BINS <= SH::max_bins && BINS % 128 == 0 && TILE <= SH::tile, "digit width, tile size");
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  src_f = uniform_ptr(src_f); src_p = uniform_ptr(src_p);
  dst_p = uniform_ptr(dst_p); dst_i = uniform_ptr(dst_i); dst_f = uniform_ptr(dst_f);
  // exclusive scan of hist[hsel] -> bucket (one thread per bin); the other
  // histogram is cleared for the counts of the next digit
  if (tid < BINS) {
    const uint32_t c = sh.hist[hsel][tid];
    const uint32_t incl = wave_inclusive_sum(c);
    if (lane == 63) sh.wave_tot[wave] = incl;
    sh.bucket[tid] = incl - c;   // exclusive within the wave
  }
  if (tid < SH::max_bins) sh.hist[hsel ^ 1][tid] = 0;
  __syncthreads();
  if (tid < BINS) {
    uint32_t add = 0;
    for (int w = 0; w < wave; ++w) add += sh.wave_tot[w];
    sh.bucket[tid] += add;
  }
  __syncthreads();

  uint32_t key[ITEMS], nkey[ITEMS];
  int32_t val[ITEMS], nval[ITEMS];
  // (opaque, so that addresses derived from it are formed where they are used instead of
  // being kept, and spilled, across the loop over the passes)
  int woff = wave * 64 * ITEMS + lane;
  asm volatile("" : "+v"(woff));
  // loads of one tile; positions past the segment re-read its last element
#define KVC_RANK_LOAD_TILE(BASE, K, V)                         \
  _Pragma("unroll") for (int e = 0; e < ITEMS; ++e) {       \
    const int pos = (BASE) + woff + e * 64;                    \
    const uint32_t cpos = uint32_t(pos < n ? pos : n - 1);     /* unsigned: 32-bit offset addressing */ \
    if (KIND == RK_FIRST) { K[e] = __float_as_uint(load_item<STREAM>(&at32(src_f, cpos))); }  /* value = position, implicit */ \
    else {                                                      \
      const uint2 kv_ = LIN ? sh.stage[cpos] : load_item<STREAM>(&at32(src_p, cpos)); \
      K[e] = kv_.x; V[e] = int32_t(kv_.y);                      \
    }                                                           \
  }
  KVC_RANK_LOAD_TILE(0, key, val)
  // (explicit, so that the loop body starts with no load the compiler still has to
  // wait for: see the wait before the scatter)
  if (!LIN) wait_vmcnt<0>();

  for (int base = 0; base < n; base += TILE) {
    // next tile's loads fly while this one is ranked and scattered
    const int nbase = base + TILE < n ? base + TILE : base;
    if (!LIN && !LOUT) { KVC_RANK_LOAD_TILE(nbase, nkey, nval) }   // a single tile has no next one
    if (KIND == RK_FIRST) {
#pragma unroll
      for (int e = 0; e < ITEMS; ++e) key[e] = desc_key(__uint_as_float(key[e])) - rebase;
    }

    const int wbase = base + woff;
    rank_and_stage<W, KIND, ITEMS>(sh, key, val, n, wbase, shift, hsel);
    lds_barrier();
    // The tile's items now live in the staging area, so the registers can take the
    // next tile.  The wait is explicit and placed before the scatter: loads and
    // stores share one in-order counter, and left to the compiler the wait for the
    // prefetched loads lands in the next tile's ranking, behind this tile's stores.
    if (!LIN && !LOUT) {
      wait_vmcnt<0>();
#pragma unroll
      for (int e = 0; e < ITEMS; ++e) { key[e] = nkey[e]; val[e] = nval[e]; }
    }
    // consecutive threads write consecutive global slots within a digit run
    // (single tile with LOUT: slot order is the order of this pass; it stays in LDS).
    // The destination is clamped into the segment: with consistent counts it never
    // needs to be, and a store can then not leave the segment whatever happens.
    const int tile_n = min(TILE, n - base);
#define KVC_RANK_WRITE_SLOT(SLOT)                                                  \
  {                                                                                \
    const uint2 kv = sh.stage[SLOT];                                               \
    uint32_t dst = sh.gbase[(kv.x >> shift) & DMASK] + (uint32_t)(SLOT);           \
    dst = min(dst, (uint32_t)(n - 1));                                             \
    if (KIND == RK_LAST) {                                                         \
      at32(dst_f, dst) = desc_key_to_float(kv.x + rebase);                         \
      at32(dst_i, dst) = int32_t(kv.y);                                            \
    } else {                                                                       \
      at32(dst_p, dst) = kv;                                                       \
    }                                                                              \
  }
    if (!LOUT) {
      // (the thread's slot base is made opaque here, so that the slot addresses
      // are formed where they are used instead of being kept, and spilled, across the
      // tile loop; four items at a time keep the temporaries of the write-out few)
      int stid = tid;
      asm volatile("" : "+v"(stid));
      if (tile_n == TILE) {              // a full tile: no per-item bounds
#pragma unroll
        for (int e = 0; e < ITEMS; ++e) {
          KVC_RANK_WRITE_SLOT(e * RK_THREADS + stid)
          if (e % 4 == 3) __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int e = 0; e < ITEMS; ++e) {
          if (e * RK_THREADS + stid < tile_n) KVC_RANK_WRITE_SLOT(e * RK_THREADS + stid)
        }
      }
    }
#undef KVC_RANK_WRITE_SLOT
  }
#undef KVC_RANK_LOAD_TILE
  // the next pass reads what this one scattered: full fence + barrier
  __threadfence_block();
  __syncthreads();
}

// All passes of one segment with W-bit digits.  Multi-tile segments ping-pong
// between the two pair arrays of the workspace; a single tile stays in LDS.
template <int W, bool ONE_TILE, int ITEMS, bool STREAM, typename SH>
__device__ __forceinline__ void radix_sort(SH& sh, int n, int passes, uint32_t rebase,
                                           const float* src_f, uint2* pa, uint2* pb, float* out_f,
                                           int32_t* out_i) {
  radix_pass<W, RK_FIRST, false, ONE_TILE, ITEMS, STREAM>(sh, n, 0, 0, rebase, src_f, nullptr, pa, nullptr, nullptr);
  int p = 1;
  for (; p < passes - 1; ++p) {
    radix_pass<W, RK_MIDDLE, ONE_TILE, ONE_TILE, ITEMS, STREAM>(sh, n, p * W, p & 1, rebase, nullptr, pa, pb, nullptr, nullptr);
    uint2* t = pa; pa = pb; pb = t;
  }
  radix_pass<W, RK_LAST, ONE_TILE, false, ITEMS, STREAM>(sh, n, p * W, p & 1, rebase, nullptr, pa, nullptr, out_f, out_i);
}

// grid: (layers * hkv, batch); block: RK_THREADS.  One workgroup sorts one segment.
// SHORT: every segment of the launch has at most RK_SHORT_TILE items (the host
// checks the longest sequence); a longer one is left alone.  STREAM: the loads of
// multi-tile segments carry the streaming hint.
template <bool SHORT, bool STREAM>
__global__ __launch_bounds__(RK_THREADS) void head_rank_kernel(
    const float* __restrict__ S, SeqTable seq, int total, int32_t* __restrict__ idx_out,
    float* __restrict__ sorted_out, uint2* __restrict__ pairs_a, uint2* __restrict__ pairs_b) {
  typedef RankShared<512, SHORT ? RK_SHORT_TILE : RK_THREADS * RK_ITEMS9> Shared9;
  typedef RankShared<1024, SHORT ? RK_SHORT_TILE : RK_THREADS * RK_ITEMS10> Shared10;
  constexpr size_t LDS_BYTES =
      SHORT ? (sizeof(Shared9) > sizeof(RankSweepShared) ? sizeof(Shared9) : sizeof(RankSweepShared))
            : (sizeof(Shared9) > sizeof(Shared10) ? sizeof(Shared9) : sizeof(Shared10));
  static_assert(LDS_BYTES >= sizeof(RankSweepShared), "the sweep's counters fit too");
  __shared__ __align__(16) unsigned char lds[LDS_BYTES];
  const int b = blockIdx.y;
  const int n = seq.cu[b + 1] - seq.cu[b];
  if (n == 0 || (SHORT && n > RK_SHORT_TILE)) return;
  const size_t seg = (size_t)blockIdx.x * total + seq.cu[b];
  const float* src_f = S + seg;
  const int tid = threadIdx.x;

  // ---- counts of the lowest 10 key bits and of the top byte, in one sweep ----
  // Eight loads in flight per thread.  The top byte (sign and high exponent bits)
  // takes a handful of values in a whole segment, so its atomics would all hit a few
  // addresses; it is counted in 32 bank-private copies instead, summed afterwards.
  RankSweepShared& sw = *reinterpret_cast<RankSweepShared*>(lds);
  sw.low[tid] = 0;
  for (int i = tid; i < 256 * 32; i += RK_THREADS) sw.top[i] = 0;
  if (tid == 0) { sw.top_min = 255u; sw.top_max = 0u; }
  __syncthreads();
  {
    const float* sweep_f = uniform_ptr(src_f);
    const int bank = tid & 31;
    for (int i0 = 0; i0 < n; i0 += RK_THREADS * 8) {
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int i = i0 + e * RK_THREADS + tid;
        x[e] = load_item<STREAM>(&at32(sweep_f, uint32_t(i < n ? i : n - 1)));   // clamped: never past the segment
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (i0 + e * RK_THREADS + tid < n) {
          const uint32_t key = desc_key(x[e]);
          atomicAdd(&sw.low[key & (RK_MAX_BINS - 1)], 1u);
          atomicAdd(&sw.top[(key >> 24) * 32 + bank], 1u);
        }
      }
    }
  }
  __syncthreads();
  if (tid < 256) {
    uint32_t sum = 0;
#pragma unroll 8
    for (int j = 0; j < 32; ++j) sum += sw.top[tid * 32 + ((j + tid) & 31)];
    if (sum != 0) { atomicMin(&sw.top_min, (uint32_t)tid); atomicMax(&sw.top_max, (uint32_t)tid); }
  }
  __syncthreads();
  // keys minus (smallest top byte << 24) are below 2^(24 + span_bits)
  const uint32_t top_min = sw.top_min, span = sw.top_max - top_min;
  const uint32_t rebase = top_min << 24;
  const int span_bits = span == 0 ? 0 : 32 - __clz((int)span);
  // 9-bit digits: three passes cover 27 bits, four cover everything; 10-bit digits:
  // three passes cover 30 bits (long segments only: a single tile always takes 9)
  const bool ten = !SHORT && n > RK_TILE && span_bits > 3 && span_bits <= 6;
  const int passes = (span_bits <= 3 || ten) ? 3 : 4;
  // the counts of the first digit move to where the layout of the passes wants them
  uint32_t first = sw.low[tid];
  if (!ten) first += sw.low[tid ^ 512];
  __syncthreads();

  float* out_f = sorted_out + seg;
  int32_t* out_i = idx_out + seg;
  if (!ten) {
    Shared9& sh = *reinterpret_cast<Shared9*>(lds);
    if (tid < 512) sh.hist[0][tid] = first;
    __syncthreads();
    // one tile: the passes hand the data on through LDS; short segments take fewer
    // items per lane (an unused item slot costs as much ranking work as a used one)
    if (n <= RK_THREADS * 2) {
      radix_sort<9, true, 2, false>(sh, n, passes, rebase, src_f, nullptr, nullptr, out_f, out_i);
    } else if (SHORT || n <= RK_THREADS * 4) {
      radix_sort<9, true, 4, false>(sh, n, passes, rebase, src_f, nullptr, nullptr, out_f, out_i);
    } else if constexpr (!SHORT) {
      if (n <= RK_THREADS * 8) {
        radix_sort<9, true, 8, false>(sh, n, passes, rebase, src_f, nullptr, nullptr, out_f, out_i);
      } else if (n <= RK_TILE) {
        radix_sort<9, true, RK_ITEMS9, false>(sh, n, passes, rebase, src_f, nullptr, nullptr, out_f, out_i);
      } else {
        radix_sort<9, false, RK_ITEMS9, STREAM>(sh, n, passes, rebase, src_f, pairs_a + seg, pairs_b + seg, out_f, out_i);
      }
    }
  } else if constexpr (!SHORT) {
    Shared10& sh = *reinterpret_cast<Shared10*>(lds);
    sh.hist[0][tid] = first;
    __syncthreads();
    radix_sort<10, false, RK_ITEMS10, STREAM>(sh, n, 3, rebase, src_f, pairs_a + seg, pairs_b + seg, out_f, out_i);
  }
}

// grid: (token blocks, layers)
__global__ void composite_kernel(const float* __restrict__ sorted, int hkv, int total,
                                 int head_max, float* __restrict__ I) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= total) return;
  const int l = blockIdx.y;
  const float* p = sorted + (size_t)l * hkv * total + c;
  float acc = p[0];
  for (int h = 1; h < hkv; ++h) {
    const float x = p[(size_t)h * total];
    acc = head_max ? fmaxf(acc, x) : acc + x;
  }
  I[(size_t)l * total + c] = head_max ? acc : acc / float(hkv);
}

// The same for HKV heads known at compile time: the loads of a thread are
// independent and in flight together; VEC consecutive ranks per thread.
template <int HKV, int VEC>
__global__ __launch_bounds__(256) void composite_plain(const float* __restrict__ sorted, int total,
                                                       int head_max, float* __restrict__ I) {
  typedef float vec_t __attribute__((ext_vector_type(VEC)));
  const int c = (blockIdx.x * 256 + threadIdx.x) * VEC;
  if (c >= total) return;                       // total is a multiple of VEC (host-checked)
  const int l = blockIdx.y;
  const float* p = sorted + (size_t)l * HKV * total + c;
  vec_t x[HKV];
#pragma unroll
  for (int h = 0; h < HKV; ++h) x[h] = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(p + (size_t)h * total));
  vec_t acc = x[0];
#pragma unroll
  for (int h = 1; h < HKV; ++h) {               // fixed head order, as in the general kernel
    if (head_max) {
#pragma unroll
      for (int j = 0; j < VEC; ++j) acc[j] = fmaxf(acc[j], x[h][j]);
    } else {
      acc += x[h];
    }
  }
  *reinterpret_cast<vec_t*>(I + (size_t)l * total + c) = head_max ? acc : acc / float(HKV);
}

}  // namespace

size_t rank_workspace_bytes(const Problem& pb) {
  // two arrays of (key, position) pairs
  const size_t lht = size_t(pb.layers) * pb.hkv * size_t(pb.total);
  return align_up(lht * 8) * 2;
}

kvc_status launch_head_rank(const Problem& pb, const float* S, int32_t* idx, float* S_sorted,
                            void* ws, hipStream_t stream) {
  const size_t lht = size_t(pb.layers) * pb.hkv * size_t(pb.total);
  // (sequences are shorter than 2^29 tokens: checked with the sequence table)
  uint2* pairs_a = static_cast<uint2*>(ws);
  uint2* pairs_b = reinterpret_cast<uint2*>(static_cast<char*>(ws) + align_up(lht * 8));
  dim3 grid(pb.layers * pb.hkv, pb.batch);
  // one workgroup of the long-segment kernels per compute unit, 256 of them: what is in flight
  const long resident = std::min<long>(long(grid.x) * grid.y, 256);
  if (pb.max_seqlen <= RK_SHORT_TILE) {
    KVC_LAUNCH("head_rank_kernel", stream, head_rank_kernel<true, false><<<grid, RK_THREADS, 0, stream>>>(S, pb.seq, int(pb.total), idx, S_sorted,
                                                      pairs_a, pairs_b));
  } else if (long(pb.max_seqlen) * resident >= RK_STREAM_ITEMS) {
    KVC_LAUNCH("head_rank_kernel", stream, head_rank_kernel<false, true><<<grid, RK_THREADS, 0, stream>>>(S, pb.seq, int(pb.total), idx, S_sorted,
                                                      pairs_a, pairs_b));
  } else {
    KVC_LAUNCH("head_rank_kernel", stream, head_rank_kernel<false, false><<<grid, RK_THREADS, 0, stream>>>(S, pb.seq, int(pb.total), idx, S_sorted,
                                                      pairs_a, pairs_b));
  }
  return KVC_OK;
}

kvc_status launch_composite(const Problem& pb, const float* S_sorted, float* I,
                            hipStream_t stream) {
  const int total = int(pb.total), head_max = pb.agg_head == KVC_AGG_MAX;
  // four ranks per thread need 16-byte aligned rows in every layer
  const bool vec4 = total % 4 == 0 &&
                    (reinterpret_cast<uintptr_t>(S_sorted) | reinterpret_cast<uintptr_t>(I)) % 16 == 0;
  if (pb.hkv == 8 && vec4) {
    dim3 grid((unsigned)((total / 4 + 255) / 256), pb.layers);
    KVC_LAUNCH("composite_kernel", stream, composite_plain<8, 4><<<grid, 256, 0, stream>>>(S_sorted, total, head_max, I));
  } else if (pb.hkv == 8) {
    dim3 grid((unsigned)((total + 255) / 256), pb.layers);
    KVC_LAUNCH("composite_kernel", stream, composite_plain<8, 1><<<grid, 256, 0, stream>>>(S_sorted, total, head_max, I));
  } else if (pb.hkv == 4 && vec4) {
    dim3 grid((unsigned)((total / 4 + 255) / 256), pb.layers);
    KVC_LAUNCH("composite_kernel", stream, composite_plain<4, 4><<<grid, 256, 0, stream>>>(S_sorted, total, head_max, I));
  } else if (pb.hkv == 4) {
    dim3 grid((unsigned)((total + 255) / 256), pb.layers);
    KVC_LAUNCH("composite_kernel", stream, composite_plain<4, 1><<<grid, 256, 0, stream>>>(S_sorted, total, head_max, I));
  } else {
    dim3 grid((unsigned)((total + 255) / 256), pb.layers);
    KVC_LAUNCH("composite_kernel", stream, composite_kernel<<<grid, 256, 0, stream>>>(S_sorted, pb.hkv, total, head_max, I));
  }
  return KVC_OK;
}

}  // namespace kvc
