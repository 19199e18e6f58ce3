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
// A segment that fits one tile (n <= 8192) never leaves the chip between the
// passes: the digit-ordered staging area of one pass is the input of the next,
// global memory sees one read of the scores and one write of the result.
#include "kvc_internal.h"

namespace kvc {

namespace {

constexpr int RK_THREADS = 1024;
constexpr int RK_WAVES = RK_THREADS / 64;
constexpr int RK_ITEMS = 8;
constexpr int RK_TILE = RK_THREADS * RK_ITEMS;
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

__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(uint32_t(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(uint32_t(mask), 0));
}

// LDS of one workgroup, for digits of up to MAXBINS values and tiles of up to TILE
// items: 148 KB for (1024, 8192), one workgroup per compute unit; 74 KB for
// (512, 4096), the launch for batches of short sequences, where two workgroups
// share a compute unit and hide each other's barriers and load latencies.
template <int MAXBINS, int TILE>
struct RankShared {
  static constexpr int max_bins = MAXBINS;
  static constexpr int tile = TILE;
  uint32_t hist[2][MAXBINS];           // digit counts of the running pass and of the next one
  uint32_t bucket[MAXBINS];            // next free global slot of each digit
  uint32_t wave_cnt[RK_WAVES][MAXBINS];
  uint32_t tstart[MAXBINS];            // first tile-local slot of each digit
  uint32_t gbase[MAXBINS];             // global slot of an item = gbase[digit] + tile-local slot
  uint32_t wave_tot[RK_WAVES];
  uint32_t top_min, top_max;           // smallest / largest top byte of the segment's keys
  uint2 stage[TILE];                   // the tile as (key, position) in digit order, so that
};                                     // the global writes run over consecutive slots

enum { RK_FIRST = 0, RK_MIDDLE = 1, RK_LAST = 2 };

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
template <int W, int KIND, bool LIN, bool LOUT, int ITEMS, typename SH>
__device__ __forceinline__ void radix_pass(SH& sh, int n, int shift, int hsel,
                                           uint32_t rebase, const float* __restrict__ src_f,
                                           const uint2* __restrict__ src_p,
                                           uint2* __restrict__ dst_p, float* __restrict__ dst_f,
                                           int32_t* __restrict__ dst_i) {
  constexpr int BINS = 1 << W;
  constexpr uint32_t DMASK = BINS - 1;
  constexpr int TILE = RK_THREADS * ITEMS;
  static_assert(BINS <= SH::max_bins && BINS % 64 == 0 && TILE <= SH::tile, "digit width, tile size");
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  src_f = uniform_ptr(src_f); src_p = uniform_ptr(src_p);
  dst_p = uniform_ptr(dst_p); dst_i = uniform_ptr(dst_i); dst_f = uniform_ptr(dst_f);
  // exclusive scan of hist[hsel] -> bucket (one thread per bin); the other
  // histogram is cleared for the counts of the next digit
  if (tid < BINS) {
    const uint32_t c = sh.hist[hsel][tid];
    uint32_t incl = c;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t o = __shfl_up(incl, off);
      if (lane >= off) incl += o;
    }
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
  const int woff = wave * 64 * ITEMS + lane;
  // loads of one tile; positions past the segment re-read its last element
#define KVC_RANK_LOAD_TILE(BASE, K, V)                         \
  _Pragma("unroll") for (int e = 0; e < ITEMS; ++e) {       \
    const int pos = (BASE) + woff + e * 64;                    \
    const uint32_t cpos = uint32_t(pos < n ? pos : n - 1);     /* unsigned: 32-bit offset addressing */ \
    if (KIND == RK_FIRST) { K[e] = __float_as_uint(at32(src_f, cpos)); V[e] = int32_t(cpos); } \
    else {                                                      \
      const uint2 kv_ = LIN ? sh.stage[cpos] : at32(src_p, cpos); \
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

    uint32_t rank[ITEMS];
    const int wbase = base + woff;
    // zero this wave's counters (only this wave touches them until the barrier)
#pragma unroll
    for (int i = 0; i < BINS / 64; ++i) sh.wave_cnt[wave][i * 64 + lane] = 0;
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
      rank[e] = prev + below;
      __builtin_amdgcn_wave_barrier();
      if (valid && below == 0) sh.wave_cnt[wave][digit] = prev + (uint32_t)__popcll(mask);
      if (KIND != RK_LAST && valid) atomicAdd(&sh.hist[hsel ^ 1][(skey >> W) & DMASK], 1u);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    lds_barrier();
    // one thread per digit: per-wave counts -> prefixes inside the digit, digit
    // totals -> tile-local start slots and the global base (conflict-free columns)
    uint32_t mine = 0, local_start = 0;
    if (tid < BINS) {
#pragma unroll
      for (int w = 0; w < RK_WAVES; ++w) {
        const uint32_t c = sh.wave_cnt[w][tid];
        sh.wave_cnt[w][tid] = mine;              // items of this digit in the waves before w
        mine += c;
      }
      uint32_t incl = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
      }
      local_start = incl - mine;                 // exclusive within the wave
      if (lane == 63) sh.wave_tot[wave] = incl;  // (free since the bucket scan of the pass start)
    }
    lds_barrier();
    if (tid < BINS) {
      uint32_t start = local_start;
      for (int w = 0; w < wave; ++w) start += sh.wave_tot[w];
      const uint32_t g = sh.bucket[tid];
      sh.tstart[tid] = start;
      sh.gbase[tid] = g - start;
      sh.bucket[tid] = g + mine;
    }
    lds_barrier();
    // every item goes to its tile-local slot
#pragma unroll
    for (int e = 0; e < ITEMS; ++e) {
      if (wbase + e * 64 < n) {
        const uint32_t digit = (key[e] >> shift) & DMASK;
        const uint32_t slot = sh.tstart[digit] + sh.wave_cnt[wave][digit] + rank[e];
        sh.stage[slot] = make_uint2(key[e], uint32_t(val[e]));
      }
    }
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
    // (single tile with LOUT: slot order is the order of this pass; it stays in LDS)
    const int tile_n = min(TILE, n - base);
    if (!LOUT) {
#pragma unroll
    for (int e = 0; e < ITEMS; ++e) {
      const int slot = e * RK_THREADS + tid;
      if (slot < tile_n) {
        const uint2 kv = sh.stage[slot];
        const uint32_t dst = sh.gbase[(kv.x >> shift) & DMASK] + (uint32_t)slot;
        if (dst < (uint32_t)n) {       // always true for consistent counts; keeps a store inside the segment regardless
          if (KIND == RK_LAST) {
            at32(dst_f, dst) = desc_key_to_float(kv.x + rebase);
            at32(dst_i, dst) = int32_t(kv.y);
          } else {
            at32(dst_p, dst) = kv;
          }
        }
      }
    }
    }
  }
#undef KVC_RANK_LOAD_TILE
  // the next pass reads what this one scattered: full fence + barrier
  __threadfence_block();
  __syncthreads();
}

// All passes of one segment with W-bit digits.  Multi-tile segments ping-pong
// between the two pair arrays of the workspace; a single tile stays in LDS.
template <int W, bool ONE_TILE, int ITEMS, typename SH>
__device__ __forceinline__ void radix_sort(SH& sh, int n, int passes, uint32_t rebase,
                                           const float* src_f, uint2* pa, uint2* pb, float* out_f,
                                           int32_t* out_i) {
  radix_pass<W, RK_FIRST, false, ONE_TILE, ITEMS>(sh, n, 0, 0, rebase, src_f, nullptr, pa, nullptr, nullptr);
  int p = 1;
  for (; p < passes - 1; ++p) {
    radix_pass<W, RK_MIDDLE, ONE_TILE, ONE_TILE, ITEMS>(sh, n, p * W, p & 1, rebase, nullptr, pa, pb, nullptr, nullptr);
    uint2* t = pa; pa = pb; pb = t;
  }
  radix_pass<W, RK_LAST, ONE_TILE, false, ITEMS>(sh, n, p * W, p & 1, rebase, nullptr, pa, nullptr, out_f, out_i);
}

// grid: (layers * hkv, batch); block: RK_THREADS.  One workgroup sorts one segment.
// SHORT: every segment of the launch has at most RK_SHORT_TILE items (the host
// checks the longest sequence); a longer one is left alone.
template <bool SHORT>
__global__ __launch_bounds__(RK_THREADS) void head_rank_kernel(
    const float* __restrict__ S, SeqTable seq, int total, int32_t* __restrict__ idx_out,
    float* __restrict__ sorted_out, uint2* __restrict__ pairs_a, uint2* __restrict__ pairs_b) {
  typedef RankShared<SHORT ? 512 : RK_MAX_BINS, SHORT ? RK_SHORT_TILE : RK_TILE> Shared;
  __shared__ Shared sh;
  const int b = blockIdx.y;
  const int n = seq.cu[b + 1] - seq.cu[b];
  if (n == 0 || (SHORT && n > RK_SHORT_TILE)) return;
  const size_t seg = (size_t)blockIdx.x * total + seq.cu[b];
  const float* src_f = S + seg;
  const int tid = threadIdx.x;

  // ---- counts of the lowest digit (as wide as the histogram allows: folded below if
  // the passes use fewer bits) and of the top byte, in one sweep ----
  // Eight loads in flight per thread.  The top byte (sign and high exponent bits)
  // takes a handful of values in a whole segment, so its atomics would all hit a few
  // addresses; it is counted in 32 bank-private copies instead, which live in the
  // staging area (unused until the first pass) and are summed afterwards.
  static_assert(Shared::tile * 2 >= 256 * 32, "staging area holds the 32 copies");
  uint32_t* top_copies = reinterpret_cast<uint32_t*>(sh.stage);
  if (tid < Shared::max_bins) sh.hist[0][tid] = 0;
  for (int i = tid; i < 256 * 32; i += RK_THREADS) top_copies[i] = 0;
  if (tid == 0) { sh.top_min = 255u; sh.top_max = 0u; }
  __syncthreads();
  {
    const float* sweep_f = uniform_ptr(src_f);
    const int bank = tid & 31;
    for (int i0 = 0; i0 < n; i0 += RK_THREADS * 8) {
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int i = i0 + e * RK_THREADS + tid;
        x[e] = at32(sweep_f, uint32_t(i < n ? i : n - 1));   // clamped: never past the segment
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (i0 + e * RK_THREADS + tid < n) {
          const uint32_t key = desc_key(x[e]);
          atomicAdd(&sh.hist[0][key & (Shared::max_bins - 1)], 1u);
          atomicAdd(&top_copies[(key >> 24) * 32 + bank], 1u);
        }
      }
    }
  }
  __syncthreads();
  if (tid < 256) {
    uint32_t sum = 0;
#pragma unroll 8
    for (int j = 0; j < 32; ++j) sum += top_copies[tid * 32 + ((j + tid) & 31)];
    if (sum != 0) { atomicMin(&sh.top_min, (uint32_t)tid); atomicMax(&sh.top_max, (uint32_t)tid); }
  }
  __syncthreads();
  // keys minus (smallest top byte << 24) are below 2^(24 + span_bits)
  const uint32_t top_min = sh.top_min, span = sh.top_max - top_min;
  const uint32_t rebase = top_min << 24;
  const int span_bits = span == 0 ? 0 : 32 - __clz((int)span);
  const bool ten = span_bits > 3 && span_bits <= 6;      // 28..30 bits: three passes of 10
  const int passes = span_bits <= 6 ? 3 : 4;             // 9-bit digits otherwise: 27 or 36 bits
  if (!SHORT && (!ten || n <= RK_TILE)) {                // (single tiles always take 9-bit digits)
    // fold the 10-bit counts into 9-bit ones (every thread reads and writes its own entries)
    if (tid < 512) sh.hist[0][tid] += sh.hist[0][tid + 512];
  }
  __syncthreads();

  float* out_f = sorted_out + seg;
  int32_t* out_i = idx_out + seg;
  // one tile: the passes hand the data on through LDS; short segments take fewer
  // items per lane (an unused item slot costs as much ranking work as a used one)
  if (n <= RK_TILE) {
    const int p1 = span_bits <= 3 ? 3 : 4;
    if (n <= RK_THREADS * 2) {
      radix_sort<9, true, 2>(sh, n, p1, rebase, src_f, nullptr, nullptr, out_f, out_i);
    } else if (SHORT || n <= RK_THREADS * 4) {
      radix_sort<9, true, 4>(sh, n, p1, rebase, src_f, nullptr, nullptr, out_f, out_i);
    } else if constexpr (!SHORT) {
      radix_sort<9, true, RK_ITEMS>(sh, n, p1, rebase, src_f, nullptr, nullptr, out_f, out_i);
    }
    return;
  }
  if constexpr (!SHORT) {
    if (ten) radix_sort<10, false, RK_ITEMS>(sh, n, 3, rebase, src_f, pairs_a + seg, pairs_b + seg, out_f, out_i);
    else radix_sort<9, false, RK_ITEMS>(sh, n, passes, rebase, src_f, pairs_a + seg, pairs_b + seg, out_f, out_i);
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
  if (pb.max_seqlen <= RK_SHORT_TILE) {
    KVC_LAUNCH("head_rank_kernel", stream, head_rank_kernel<true><<<grid, RK_THREADS, 0, stream>>>(S, pb.seq, int(pb.total), idx, S_sorted,
                                                      pairs_a, pairs_b));
  } else {
    KVC_LAUNCH("head_rank_kernel", stream, head_rank_kernel<false><<<grid, RK_THREADS, 0, stream>>>(S, pb.seq, int(pb.total), idx, S_sorted,
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
