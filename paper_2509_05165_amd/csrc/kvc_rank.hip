// kvc_head_rank: per (layer, KV head, sequence) stable descending argsort of
// the scores (Section 3.3, eq. 17) and the rank-aligned scores S'.
//
// One workgroup sorts one segment with a least-significant-digit radix sort,
// 8 bits per pass, on the order-preserving integer image of the fp32 scores
// (inverted, so that ascending keys are descending scores).  LSD passes are
// stable, which yields the ascending-index order of equal scores for free.
// Within a tile every wave ranks its items with ballot-based digit matching
// and lane prefix counts; per-wave digit counters live in LDS.
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
constexpr int RK_BINS = 256;

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

// Element `i` of a 4-byte array through a 32-bit byte offset (the library limits
// T to 2^30 tokens, so 4*i fits): scalar base + 32-bit lane offset addressing.
template <typename T>
__device__ __forceinline__ T& at32(T* base, uint32_t i) {
  static_assert(sizeof(T) == 4, "4-byte elements");
  return *reinterpret_cast<T*>(reinterpret_cast<char*>(base) + (i << 2));
}
template <typename T>
__device__ __forceinline__ const T& at32(const T* base, uint32_t i) {
  static_assert(sizeof(T) == 4, "4-byte elements");
  return *reinterpret_cast<const T*>(reinterpret_cast<const char*>(base) + (i << 2));
}

// Workgroup barrier that orders LDS traffic only: global stores still in flight
// (the scatter of the previous tile) are not waited for.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// lanes (among `valid`) whose 8-bit digit (bits SHIFT..SHIFT+7 of the key) equals
// mine.  Per bit: `mine` is all ones or all zeros (one signed bit-field extract),
// the lanes that agree with it are ~(ballot ^ mine); written on 32-bit halves as
// x & ~(y ^ z), which is one three-input bit operation per half (truth table 0x90:
// the encoding the compiler itself picks for that expression; spelled out because
// it otherwise splits it into an xor and a shared three-input and).  Four vector
// instructions per bit: extract, compare (the ballot), two bit operations.
template <int SHIFT>
__device__ __forceinline__ uint64_t match_digit(uint32_t key, uint64_t valid) {
  uint32_t lo = (uint32_t)valid, hi = (uint32_t)(valid >> 32);
#pragma unroll
  for (int bit = 0; bit < 8; ++bit) {
    // (spelled as the instruction: the builtin is lowered to a shift pair)
    uint32_t mine;
    asm("v_bfe_i32 %0, %1, %2, 1" : "=v"(mine) : "v"(key), "n"(SHIFT + bit));
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

struct RankShared {
  uint32_t hist[4][RK_BINS];
  uint32_t bucket[RK_BINS];            // next free global slot of each digit
  uint32_t wave_cnt[RK_WAVES][RK_BINS];
  uint32_t tstart[RK_BINS];            // first tile-local slot of each digit
  uint32_t gbase[RK_BINS];             // global slot of an item = gbase[digit] + tile-local slot
  uint32_t wave_tot[4];
  uint32_t stage_k[RK_TILE];           // the tile in digit order, so that the
  int32_t stage_v[RK_TILE];            // global writes run over consecutive slots
};

// One stable counting pass on digit PASS of a segment of n items.  PASS 0 reads
// the scores themselves (key = inverted ordered image, value = position), the
// last pass writes scores and positions; the others move (key, value) pairs.
// Tiles are processed in order; item (wave w, slot e, lane l) of a tile is
// element base + w*64*ITEMS + e*64 + l, which is also its order inside the tile.
// LIN / LOUT (single-tile segments only): the pass reads its (key, value) pairs
// from / leaves them in the LDS staging area, in slot order.
template <int PASS, bool LIN, bool LOUT, int ITEMS>
__device__ __forceinline__ void radix_pass(RankShared& sh, int n, const float* __restrict__ src_f,
                                           const uint32_t* __restrict__ src_k,
                                           const int32_t* __restrict__ src_i,
                                           uint32_t* __restrict__ dst_k,
                                           int32_t* __restrict__ dst_i,
                                           float* __restrict__ dst_f) {
  constexpr int shift = PASS * 8;
  constexpr int TILE = RK_THREADS * ITEMS;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  src_f = uniform_ptr(src_f); src_k = uniform_ptr(src_k); src_i = uniform_ptr(src_i);
  dst_k = uniform_ptr(dst_k); dst_i = uniform_ptr(dst_i); dst_f = uniform_ptr(dst_f);
  // exclusive scan of hist[PASS] -> bucket (first 256 threads = 4 waves)
  if (tid < RK_BINS) {
    const uint32_t c = sh.hist[PASS][tid];
    uint32_t incl = c;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t o = __shfl_up(incl, off);
      if (lane >= off) incl += o;
    }
    if (lane == 63) sh.wave_tot[wave] = incl;
    sh.bucket[tid] = incl - c;   // exclusive within the wave
  }
  __syncthreads();
  if (tid < RK_BINS) {
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
    if (PASS == 0) { K[e] = __float_as_uint(at32(src_f, cpos)); V[e] = int32_t(cpos); } \
    else if (LIN) { K[e] = sh.stage_k[cpos]; V[e] = sh.stage_v[cpos]; }  \
    else { K[e] = at32(src_k, cpos); V[e] = at32(src_i, cpos); }           \
  }
  KVC_RANK_LOAD_TILE(0, key, val)
  // (explicit, so that the loop body starts with no load the compiler still has to
  // wait for: see the wait before the scatter)
  if (!LIN) wait_vmcnt<0>();

  for (int base = 0; base < n; base += TILE) {
    // next tile's loads fly while this one is ranked and scattered
    const int nbase = base + TILE < n ? base + TILE : base;
    if (!LIN && !LOUT) { KVC_RANK_LOAD_TILE(nbase, nkey, nval) }   // a single tile has no next one
    if (PASS == 0) {
#pragma unroll
      for (int e = 0; e < ITEMS; ++e) key[e] = desc_key(__uint_as_float(key[e]));
    }

    uint32_t rank[ITEMS];
    const int wbase = base + woff;
    // zero this wave's counters (only this wave touches them until the barrier)
#pragma unroll
    for (int i = 0; i < RK_BINS / 64; ++i) sh.wave_cnt[wave][i * 64 + lane] = 0;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int e = 0; e < ITEMS; ++e) {
      const bool valid = wbase + e * 64 < n;
      const uint64_t vmask = __ballot(valid);
      const uint32_t digit = (key[e] >> shift) & 255u;
      const uint64_t mask = match_digit<shift>(key[e], vmask);
      const int below = lanes_below(mask);
      uint32_t prev = 0;
      if (valid) prev = sh.wave_cnt[wave][digit];
      rank[e] = prev + below;
      __builtin_amdgcn_wave_barrier();
      if (valid && below == 0) sh.wave_cnt[wave][digit] = prev + (uint32_t)__popcll(mask);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    lds_barrier();
    // threads 0..255 own one digit each: per-wave counts -> prefixes inside the digit,
    // digit totals -> tile-local start slots and the global base (four waves in
    // parallel, conflict-free columns; one wave doing it alone took 1 us per tile)
    uint32_t mine = 0, local_start = 0;
    if (tid < RK_BINS) {
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
    if (tid < RK_BINS) {
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
        const uint32_t digit = (key[e] >> shift) & 255u;
        const uint32_t slot = sh.tstart[digit] + sh.wave_cnt[wave][digit] + rank[e];
        sh.stage_k[slot] = key[e];
        sh.stage_v[slot] = val[e];
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
        const uint32_t k = sh.stage_k[slot];
        const int32_t v = sh.stage_v[slot];
        const uint32_t dst = sh.gbase[(k >> shift) & 255u] + (uint32_t)slot;
        if (PASS == 3) {
          at32(dst_f, dst) = desc_key_to_float(k);
          at32(dst_i, dst) = v;
        } else {
          at32(dst_k, dst) = k;
          at32(dst_i, dst) = v;
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

// grid: (layers * hkv, batch); block: RK_THREADS.  One workgroup sorts one
// segment: 4 stable passes of 8 bits, ping-pong between the workspace pair
// (tmp_keys, tmp_idx) and the output arrays.
__global__ __launch_bounds__(RK_THREADS) void head_rank_kernel(
    const float* __restrict__ S, SeqTable seq, int total, int32_t* __restrict__ idx_out,
    float* __restrict__ sorted_out, uint32_t* __restrict__ tmp_keys,
    int32_t* __restrict__ tmp_idx) {
  __shared__ RankShared sh;
  const int b = blockIdx.y;
  const int n = seq.cu[b + 1] - seq.cu[b];
  if (n == 0) return;
  const size_t seg = (size_t)blockIdx.x * total + seq.cu[b];
  const float* src_f = S + seg;
  uint32_t* a_keys = tmp_keys + seg;
  int32_t* a_idx = tmp_idx + seg;
  uint32_t* b_keys = reinterpret_cast<uint32_t*>(sorted_out) + seg;
  int32_t* b_idx = idx_out + seg;
  const int tid = threadIdx.x;

  // ---- histograms of all four digits in one sweep ----
  // Eight loads in flight per thread.  The top digit (sign and high exponent bits)
  // takes three or four values in a whole segment, so its atomics would all hit one
  // address; it is counted in 32 bank-private copies instead, which live in the
  // staging area (unused until the first pass) and are summed afterwards.
  static_assert(RK_TILE >= RK_BINS * 32, "staging area holds the 32 copies");
  uint32_t* top_copies = sh.stage_k;
  for (int i = tid; i < 3 * RK_BINS; i += RK_THREADS) (&sh.hist[0][0])[i] = 0;
  for (int i = tid; i < RK_BINS * 32; i += RK_THREADS) top_copies[i] = 0;
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
          atomicAdd(&sh.hist[0][key & 255u], 1u);
          atomicAdd(&sh.hist[1][(key >> 8) & 255u], 1u);
          atomicAdd(&sh.hist[2][(key >> 16) & 255u], 1u);
          atomicAdd(&top_copies[(key >> 24) * 32 + bank], 1u);
        }
      }
    }
  }
  __syncthreads();
  if (tid < RK_BINS) {
    uint32_t sum = 0;
#pragma unroll 8
    for (int j = 0; j < 32; ++j) sum += top_copies[tid * 32 + ((j + tid) & 31)];
    sh.hist[3][tid] = sum;
  }
  __syncthreads();

  // one tile: the passes hand the data on through LDS; short segments take fewer
  // items per lane (an unused item slot costs as much ranking work as a used one)
#define KVC_RANK_ONE_TILE(ITEMS)                                                                        \
  do {                                                                                                  \
    radix_pass<0, false, true, ITEMS>(sh, n, src_f, nullptr, nullptr, nullptr, nullptr, nullptr);       \
    radix_pass<1, true, true, ITEMS>(sh, n, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);      \
    radix_pass<2, true, true, ITEMS>(sh, n, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);      \
    radix_pass<3, true, false, ITEMS>(sh, n, nullptr, nullptr, nullptr, nullptr, b_idx, sorted_out + seg); \
  } while (0)
  if (n <= RK_THREADS * 2) { KVC_RANK_ONE_TILE(2); return; }
  if (n <= RK_THREADS * 4) { KVC_RANK_ONE_TILE(4); return; }
  if (n <= RK_TILE) { KVC_RANK_ONE_TILE(RK_ITEMS); return; }
#undef KVC_RANK_ONE_TILE
  radix_pass<0, false, false, RK_ITEMS>(sh, n, src_f, nullptr, nullptr, a_keys, a_idx, nullptr);
  radix_pass<1, false, false, RK_ITEMS>(sh, n, nullptr, a_keys, a_idx, b_keys, b_idx, nullptr);
  radix_pass<2, false, false, RK_ITEMS>(sh, n, nullptr, b_keys, b_idx, a_keys, a_idx, nullptr);
  radix_pass<3, false, false, RK_ITEMS>(sh, n, nullptr, a_keys, a_idx, nullptr, b_idx, sorted_out + seg);
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
  const size_t lht = size_t(pb.layers) * pb.hkv * size_t(pb.total);
  return align_up(lht * 4) * 2;
}

kvc_status launch_head_rank(const Problem& pb, const float* S, int32_t* idx, float* S_sorted,
                            void* ws, hipStream_t stream) {
  const size_t lht = size_t(pb.layers) * pb.hkv * size_t(pb.total);
  uint32_t* tmp_keys = static_cast<uint32_t*>(ws);
  int32_t* tmp_idx = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + align_up(lht * 4));
  dim3 grid(pb.layers * pb.hkv, pb.batch);
  KVC_LAUNCH("head_rank_kernel", stream, head_rank_kernel<<<grid, RK_THREADS, 0, stream>>>(S, pb.seq, int(pb.total), idx, S_sorted,
                                                    tmp_keys, tmp_idx));
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
