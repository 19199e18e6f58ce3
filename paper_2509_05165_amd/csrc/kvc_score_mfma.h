// bf16 matrix-core kernels of kvc_score (d = 128, window in {32,64,128,256}).
// Included by kvc_score.hip only.
//
// One workgroup (4 waves) handles one KV head x one chunk of keys x up to 256
// query rows (8 blocks of 32 rows).  A wave owns two query blocks whose
// fragments stay in registers for the whole kernel.  K streams through LDS in
// 128-key macro tiles written by direct global->LDS loads (no staging
// registers), one tile ahead of the MFMAs, in two buffers.  Inside a wave the
// MFMAs of one 32-key tile are interleaved with the softmax arithmetic of the
// previous tile (two accumulator sets), so the matrix pipe and the vector ALU
// work at the same time.
//
// v_mfma_f32_32x32x16_bf16 fragment layout (wave64): operand lane l holds, for
// row/column (l % 32), the 8 consecutive k-values 8*(l/32) .. +7; accumulator
// register r of lane l is element (row 8*(r/4) + 4*(l/32) + r%4, column l%32).
//
// LDS tile layout: row (key) r at byte 256*r, its sixteen 16-byte pieces stored
// at slot (piece ^ (r & 15)), so the fragment reads of 16 consecutive rows hit
// 16 different slots (all banks) although rows are exactly one bank-stride apart.
#pragma once

namespace kvc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int MF_D = 128;
constexpr int MF_THREADS = 256;
constexpr int MF_TILE = 128;                 // keys per LDS macro tile
constexpr int MF_RCHUNK = 256;               // query rows per workgroup
constexpr int MF_KBUF = MF_TILE * 256;       // bytes per K buffer
constexpr int MF_NBUF = 2;
constexpr int MF_DMA = MF_KBUF / 16 / MF_THREADS;   // direct loads per thread per tile (8)

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// 16 bytes per lane straight from global memory into LDS: lane i of the wave
// writes LDS bytes [lds_base + 16 i, +16).  lds_base must be wave-uniform.  The
// load is tracked by vmcnt only; the caller orders it with wait_vmcnt + barrier.
// K is read once per pass and a layer's K exceeds every cache, so the loads carry
// the streaming hint (keeps the partial results of the pass in L2 instead).
__device__ __forceinline__ void lds_dma16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_base), "v"(gptr)
               : "memory");
}
// Combine the two half-waves: both halves end up with op(lower, upper).
template <bool MAX>
__device__ __forceinline__ float cross_half(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  const float a = __uint_as_float(r[0]), b = __uint_as_float(r[1]);
  return MAX ? fmaxf(a, b) : a + b;
}

// STATS: fold one 32x32 logit tile (keys on rows) into the lane's running
// (max, sum 2^(t - max)) of its query column.
__device__ __forceinline__ void stats_fold(const f32x16& acc, float c2, float& mrun, float& srun) {
  float amax = acc[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) amax = fmaxf(amax, acc[r]);
  const float mn = fmaxf(mrun, amax * c2);
  float s = srun * fast_exp2(mrun - mn);
  const float nmn = -mn;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += fast_exp2(fmaf(acc[r], c2, nmn));
  srun = s;
  mrun = mn;
}

// The same fold for two tiles (x0, x1), cut into 16 slices so that slice i can be
// issued right behind MFMA i of the next tile.  Slices 0-1: tile maxima; slice
// 2: new running maxima and rescale; slices 3-15: the 32 exponentials.
//
// track == false (wave-uniform) freezes the reference: 2^(t - mrun) is summed
// with mrun as it stands, no maxima, no rescale.  Any reference within about
// +-100 of the true maximum (log2 units) gives the same sum to fp32 precision;
// a logit more than 127 above it overflows the sum to inf, which the caller
// detects and answers by running the chunk again with tracking on.
struct StatsCarry { float amax[2], nmn[2], s[2], e[3]; int eb[3]; };
__device__ __forceinline__ void stats_slice(int i, const f32x16& x0, const f32x16& x1, float c2,
                                            float (&mrun)[2], float (&srun)[2], StatsCarry& c,
                                            bool track) {
  if (i < 2) {
    if (track) {
      const f32x16& x = i ? x1 : x0;
      float m = fmaxf(x[0], x[1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) m = fmaxf(m, fmaxf(x[r], x[r + 1]));
      c.amax[i] = m;
    }
  } else if (i == 2) {
    if (track) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const float mn = fmaxf(mrun[b], c.amax[b] * c2);
        c.s[b] = srun[b] * fast_exp2(mrun[b] - mn);
        c.nmn[b] = -mn;
        mrun[b] = mn;
      }
    } else {
#pragma unroll
      for (int b = 0; b < 2; ++b) { c.s[b] = srun[b]; c.nmn[b] = -mrun[b]; }
    }
  } else {
    // elements 0..31 (tile 0 then tile 1): slices 3..8 take three, 9..15 take two.
    // The exponentials of a slice are summed one slice later, so the adds never
    // wait for a transcendental that has just been issued.
    const int first = i <= 8 ? 3 * (i - 3) : 18 + 2 * (i - 9);
    const int count = i <= 8 ? 3 : 2;
    const int pfirst = i == 3 ? 0 : (i - 1 <= 8 ? 3 * (i - 4) : 18 + 2 * (i - 10));
    const int pcount = i == 3 ? 0 : (i - 1 <= 8 ? 3 : 2);
    float fresh[3];
#pragma unroll
    for (int j = 0; j < count; ++j) {
      const int e = first + j, b = e >> 4, r = e & 15;
      fresh[j] = fast_exp2(fmaf(b ? x1[r] : x0[r], c2, c.nmn[b]));
    }
#pragma unroll
    for (int j = 0; j < pcount; ++j) c.s[(pfirst + j) >> 4] += c.e[j];
#pragma unroll
    for (int j = 0; j < count; ++j) c.e[j] = fresh[j];
    if (i == 15) {
#pragma unroll
      for (int j = 0; j < count; ++j) c.s[(first + j) >> 4] += c.e[j];
      srun[0] = c.s[0];
      srun[1] = c.s[1];
    }
  }
}

// EMIT: reduce one 32x32 logit tile (queries on rows) over its 32 query rows:
// max of t, or sum of 2^t, with t = logit*c2 - lse2 (nl holds -lse2 of the lane's 16
// rows).  Result in both half-waves.
//
// RECENTRE (TASK_MAX only) is the cheaper form: the accumulators start from
// -(lse2[row] - lse2[first row of the block])/c2 (nl holds that) instead of zero, so
// they are (t + lse2[first row])/c2; the maximum commutes with the positive factor c2
// and the common shift, which are applied once at the end (one FMA with base =
// -lse2[first row]) instead of once per element.  It costs accuracy in proportion to
// the start value: nothing while the rows of a block have similar log-sum-exps (those
// of one query head do), up to 2e-4 relative when they lie hundreds of units apart.
// So a workgroup uses it only if every block of its row chunk lies within
// EMIT_SPREAD_LIMIT of its first row; otherwise the workgroup is redone in the exact
// form (every element gets its own FMA; accuracy independent of the data).
constexpr float EMIT_SPREAD_LIMIT = 64.f;   // log2 units: keeps the start value's rounding below 1e-5 relative
template <bool TASK_MAX, bool RECENTRE>
__device__ __forceinline__ float emit_fold(const f32x16& acc, float c2, const float (&nl)[16],
                                           float base) {
  float v = TASK_MAX ? NEG_BIG : 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    if (TASK_MAX) v = fmaxf(v, RECENTRE ? acc[r] : fmaf(acc[r], c2, nl[r]));
    else v += fast_exp2(fmaf(acc[r], c2, nl[r]));
  }
  v = cross_half<TASK_MAX>(v);
  return (TASK_MAX && RECENTRE) ? fmaf(v, c2, base) : v;
}
// The same for two tiles in 16 slices: slice i handles elements 2(i%8), 2(i%8)+1 of
// tile i/8; the cross-half combine of a tile follows its last slice.
template <bool TASK_MAX, bool RECENTRE>
__device__ __forceinline__ void emit_slice(int i, const f32x16& x0, const f32x16& x1, float c2,
                                           const float (&nl)[2][16], const float (&base)[2],
                                           float (&v)[2]) {
  const int b = i >> 3, r = 2 * (i & 7);
  const f32x16& x = b ? x1 : x0;
  if ((i & 7) == 0) v[b] = TASK_MAX ? NEG_BIG : 0.f;
  if (TASK_MAX && RECENTRE) {
    v[b] = fmaxf(v[b], fmaxf(x[r], x[r + 1]));
  } else if (TASK_MAX) {
    v[b] = fmaxf(v[b], fmaxf(fmaf(x[r], c2, nl[b][r]), fmaf(x[r + 1], c2, nl[b][r + 1])));
  } else {
    const float t0 = fmaf(x[r], c2, nl[b][r]), t1 = fmaf(x[r + 1], c2, nl[b][r + 1]);
    v[b] += fast_exp2(t0) + fast_exp2(t1);
  }
  if ((i & 7) == 7) {
    v[b] = cross_half<TASK_MAX>(v[b]);
    if (TASK_MAX && RECENTRE) v[b] = fmaf(v[b], c2, base[b]);
  }
}

// 16 bytes per lane from (scalar base + per-lane byte offset) into LDS.
__device__ __forceinline__ void lds_dma16_s(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_base), "v"(voff), "s"(sbase)
               : "memory");
}

// grid: ((sequence, chunk) pairs, Hkv * row_chunks, Lyr), 256 threads.  WQ = waves along the query
// rows (each owns 2 blocks of 32 rows); the other 4/WQ waves split the key tiles.
// A launch covers the row chunks [rc_offset, rc_offset + row_chunks) of every KV head
// (the last, partly filled row chunk of a head may get a launch of its own with fewer
// waves along the rows).
//
// Schedule of one workgroup over its macro tiles (two K buffers, tile t in
// buffer t&1), for an even number NT of 32-key tiles per wave:
//   phase j of tile t = 16 MFMAs of key tile j into accumulator set j&1, each
//   followed by one slice of the vector work on the other set (the previous
//   key tile, possibly of tile t-1) and by the fragment reads for the next phase;
//   before the last phase of tile t all fragments of tile t are in registers, so
//   the workgroup waits for tile t+1, meets at a barrier, starts the load of
//   tile t+2 into the buffer of tile t and (EMIT) writes out tile t-1; the last
//   phase already prefetches the first fragments of tile t+1.
//
// causal != 0: task token m sits at position n - window + m of its sequence and
// sees keys at positions <= that only.  Tiles that lie wholly below position
// n - window + 1 are visible to every row and go through the pipeline; the few
// tiles above it are processed one key tile at a time with the mask applied.
//
// MODE (EMIT with TASK_MAX only; 0 otherwise): 1 = the re-centred form of emit_fold,
// with the workgroup checking its log-sum-exps first and, when they are too far apart,
// putting its block index (bx, by, bz) on the `defer` list instead of working; 2 = the
// exact form, which the list-driven kernel below runs for the listed workgroups.
// (bx, by, bz) and (gy, gz) stand for blockIdx and gridDim.y/z of the grid launch.
struct DeferList {
  uint32_t* count;        // device: number of entries appended so far
  uint64_t* entries;      // device: bx | by << 32 | bz << 56
  uint32_t capacity;
};
template <bool EMIT, bool TASK_MAX, int WQ, int MODE>
__device__ __forceinline__ void score_mfma_body(
    const PtrTable& q_tab, const PtrTable& k_tab, int batch, size_t out_layer_stride,
    const SeqTable& seq, int hq, int group, int window, int total, float c2, int chunk_keys,
    int row_chunks, int rc_offset, float* __restrict__ part_m, float* __restrict__ part_s,
    const float* __restrict__ lse2, int group_max, int causal, float* __restrict__ out,
    const DeferList& defer, const int bx, const int by, const int bz, const int gy, const int gz) {
  static_assert(MODE == 0 || (EMIT && TASK_MAX), "modes 1 and 2 are forms of the max-pooling emit pass");
  constexpr bool RECENTRE = MODE == 1;
  constexpr int WK = 4 / WQ;        // waves along the keys
  constexpr int NT = 4 / WK;        // 32-key tiles per wave per macro tile
  constexpr bool PIPE = NT % 2 == 0;
  __shared__ __attribute__((aligned(1024))) unsigned char kbuf[MF_NBUF][MF_KBUF];
  __shared__ float red[EMIT ? 3 : 1][8][EMIT ? MF_TILE : 1];   // EMIT: per (q block | wave, key)
  __shared__ float stat[EMIT ? 1 : 4][2][32][2];               // STATS: per wave (max, sum)
  __shared__ __attribute__((aligned(16))) float lse_s[EMIT ? MF_RCHUNK : 4];   // EMIT: -lse2 of the row chunk

  // blockIdx.z = layer: one launch covers every layer, so that workgroups of the
  // next layer start as those of this one finish and only the very first ones wait
  // for their first tile with nothing else running.
  // blockIdx.x runs over the (sequence, chunk) pairs of the batch, sequence by
  // sequence: the grid holds no empty slots, and consecutive workgroup ids, which
  // the hardware deals round-robin to the eight XCDs, carry equal work whatever the
  // mix of sequence lengths (a chunk-major grid gave XCD j the j-th chunk of every
  // sequence: twice the time on a batch of 5k..29k-token sequences).
  const int layer = bz;
  const int chunk_shift = __builtin_ctz(chunk_keys);   // chunk_keys is a power of two (host-checked)
  int b = 0, chunk = bx;
  for (; b < batch - 1; ++b) {
    const int nc = (seq.cu[b + 1] - seq.cu[b] + chunk_keys - 1) >> chunk_shift;
    if (chunk < nc) break;
    chunk -= nc;
  }
  const int zid = layer * batch + b;
  const uint16_t* __restrict__ q_layer = static_cast<const uint16_t*>(q_tab.p[layer]);
  const uint16_t* __restrict__ k_layer = static_cast<const uint16_t*>(k_tab.p[layer]);
  if (EMIT) out += (size_t)layer * out_layer_stride;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int key_begin = chunk * chunk_keys;
  if (key_begin >= n) return;
  const int key_end = min(n, key_begin + chunk_keys);
  const int hkv = gy / row_chunks;
  const int h = by / row_chunks, rc = by - h * row_chunks + rc_offset;
  const int R = group * window;
  const int row0 = rc * MF_RCHUNK;
  const int nqb = (min(R, row0 + MF_RCHUNK) - row0) / 32;   // q blocks in this row chunk
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wq = wave % WQ, wk = wave / WQ;
  const int col = lane & 31, half = lane >> 5;
  const uint16_t* k_chunk = k_layer + ((size_t)h * total + tok0 + key_begin) * MF_D;

  const int span = key_end - key_begin;
  const int nfull = span / MF_TILE;             // macro tiles with all 128 keys
  const int tail = span - nfull * MF_TILE;      // keys of the ragged last tile (0 = none)
  const int ntiles = nfull + (tail > 0);

  // ---- direct global->LDS tile loads ----
  // load j of this thread: tile row 16 j + 4 wave + lane/16, LDS slot lane%16
  const int drow = wave * 4 + (lane >> 4);
  const int dpiece = (lane & 15) ^ (drow & 15);          // piece of the row that lands in my slot
  const uint32_t kbuf_lds =
      (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)(&kbuf[0][0]);
  const uint32_t dma_lds = __builtin_amdgcn_readfirstlane(kbuf_lds + wave * 1024);
  const uint32_t dvoff = (uint32_t)(drow * MF_D + dpiece * 8) * 2u;   // byte offset of load 0
  auto issue_tile = [&](int t) {
    // scalar tile base; load j adds 16 rows (4096 bytes) to it
    const uint64_t addr = reinterpret_cast<uint64_t>(k_chunk) + (uint64_t)t * MF_KBUF;
    // readfirstlane returns a signed int: widen through uint32_t, or a low half
    // with bit 31 set would sign-extend into the high half
    const uint64_t tile =
        ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(addr >> 32)) << 32) |
        (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)addr);
    const uint32_t dst = dma_lds + (uint32_t)(t & 1) * MF_KBUF;
    if (t < nfull) {
#pragma unroll
      for (int j = 0; j < MF_DMA; ++j)
        lds_dma16_s(reinterpret_cast<const void*>(tile + j * 4096), dvoff, dst + j * 4096);
    } else {   // ragged: rows past the sequence re-read the last valid row (masked later)
#pragma unroll
      for (int j = 0; j < MF_DMA; ++j)
        lds_dma16_s(reinterpret_cast<const void*>(tile),
                    (uint32_t)(min(16 * j + drow, tail - 1) * MF_D + dpiece * 8) * 2u, dst + j * 4096);
    }
  };
  issue_tile(0);

  // ---- query fragments: registers for the whole kernel ----
  uint4 qf[2][8];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int blk = wq * 2 + qb;
    const int r = row0 + blk * 32 + col;
    const bool ok = blk < nqb;
    // the G query heads of a KV head are contiguous, so row r of the group is
    // simply row r after the group's first query row
    const size_t qrow = ((size_t)b * hq + h * group) * window + (ok ? r : 0);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ok) v = *reinterpret_cast<const uint4*>(q_layer + qrow * MF_D + ks * 16 + half * 8);
      qf[qb][ks] = v;
    }
  }

  // EMIT: minus lse2 of this row chunk goes through LDS (one coalesced load)
  float my_nl = 0.f;
  if (EMIT && (int)threadIdx.x < nqb * 32)
    my_nl = -lse2[((size_t)zid * hq + h * group) * window + row0 + threadIdx.x];
  float nl[2][16];   // EMIT: minus lse2 of the lane's accumulator rows, filled after the first barrier
  float nbase[2] = {0.f, 0.f};   // RECENTRE: minus lse2 of the first row of each q block

  float mrun[2] = {NEG_BIG, NEG_BIG}, srun[2] = {0.f, 0.f};   // STATS, in log2 units
  const int bpg = window / 32;                                 // q blocks per query head
  const int gcount = nqb / bpg;                                // query heads in this row chunk
  // EMIT, window <= 64: a wave holds whole query heads, so it finishes the task
  // aggregate itself and stores one partial group value per key (slot = wq).
  const bool wave_groups = bpg <= 2;
  const float inv_window = 1.f / float(window);

  // fragment address inside a buffer, key tile 0: k-step ks is at fbase ^ (32 ks)
  // (the slot swizzle only touches address bits 4-7, the k-step bits 5-7)
  const int fbase = col * 256 + ((half ^ (col & 15)) << 4);

  // Two accumulator sets; one tile is always "pending" (its vector work runs behind
  // the MFMAs of the next one).  STATS: a pending set full of -inf folds to exactly
  // nothing (its maximum never wins, every 2^(-inf) is 0).  EMIT: the pending set
  // of the very first phase is zeros and lands in a red[] buffer nobody reads.
  f32x16 acc[2][2];
  const float ninf = -__builtin_inff();
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc[1][0][r] = EMIT ? 0.f : ninf; acc[1][1][r] = EMIT ? 0.f : ninf; }

  auto load_frags = [&](uint4 (&kf)[8], const unsigned char* kp) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[ks] = *reinterpret_cast<const uint4*>(kp + (fbase ^ (32 * ks)));
  };
  auto mfma_tile = [&](f32x16 (&a)[2], const uint4 (&kf)[8]) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      a[0][r] = (EMIT && TASK_MAX && RECENTRE) ? nl[0][r] : 0.f;
      a[1][r] = (EMIT && TASK_MAX && RECENTRE) ? nl[1][r] : 0.f;
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 kfr = as_bf16x8(kf[ks]);
      if (EMIT) {   // rows = queries, columns = keys
        a[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qf[0][ks]), kfr, a[0], 0, 0, 0);
        a[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qf[1][ks]), kfr, a[1], 0, 0, 0);
      } else {      // rows = keys, columns = queries
        a[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, as_bf16x8(qf[0][ks]), a[0], 0, 0, 0);
        a[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, as_bf16x8(qf[1][ks]), a[1], 0, 0, 0);
      }
    }
  };
  // EMIT: per-block task aggregates (both half-waves hold them) -> red[buf]
  auto red_store = [&](const float (&v)[2], int buf, int kt) {
    const int blk0 = wq * 2;
    if (wave_groups) {
      float part;
      if (bpg == 2) {
        const float tv = TASK_MAX ? fmaxf(v[0], v[1]) : v[0] + v[1];
        part = blk0 < nqb ? (TASK_MAX ? fast_exp2(tv) : tv * inv_window) : 0.f;
      } else {
        const float s0 = blk0 < nqb ? (TASK_MAX ? fast_exp2(v[0]) : v[0] * inv_window) : 0.f;
        const float s1 = blk0 + 1 < nqb ? (TASK_MAX ? fast_exp2(v[1]) : v[1] * inv_window) : 0.f;
        part = group_max ? fmaxf(s0, s1) : s0 + s1;
      }
      if (half == 0) red[buf][wq][kt * 32 + col] = part;
    } else {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
        if (half == 0 && blk0 + qb < nqb) red[buf][blk0 + qb][kt * 32 + col] = v[qb];
    }
  };
  auto emit_store = [&](const f32x16 (&a)[2], int buf, int kt) {
    float v[2];
    v[0] = emit_fold<TASK_MAX, RECENTRE>(a[0], c2, nl[0], nbase[0]);
    v[1] = emit_fold<TASK_MAX, RECENTRE>(a[1], c2, nl[1], nbase[1]);
    red_store(v, buf, kt);
  };
  // EMIT: threads 0..127 turn red[buf] into the group value of one key each
  // (even tiles: waves 0-1, odd tiles: waves 2-3, so the extra work is shared)
  auto epilogue = [&](int t, int keys) {
    const int ekey = threadIdx.x & (MF_TILE - 1);
    if ((int)(threadIdx.x >> 7) == (t & 1) && ekey < keys) {
      const int buf = t % 3;
      // all partials are read before any is used (one LDS round trip, not eight)
      const int nslots = wave_groups ? (nqb + 1) >> 1 : nqb;
      const float neutral = (!wave_groups && TASK_MAX) ? NEG_BIG : 0.f;
      float x[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) x[i] = i < nslots ? red[buf][i][ekey] : neutral;
      float gacc;
      if (wave_groups) {
        // finished group partials of the waves, all >= 0, so 0 is neutral for max and sum
        gacc = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) gacc = group_max ? fmaxf(gacc, x[i]) : gacc + x[i];
      } else {
        // a query head spans 4 or 8 blocks: two heads of 4, or one of 8
        float t0 = x[0], t1 = x[4];
#pragma unroll
        for (int i = 1; i < 4; ++i) {
          t0 = TASK_MAX ? fmaxf(t0, x[i]) : t0 + x[i];
          t1 = TASK_MAX ? fmaxf(t1, x[4 + i]) : t1 + x[4 + i];
        }
        if (bpg > 8) {
          // the query head continues in other row chunks: hand on the raw task partial
          gacc = TASK_MAX ? fmaxf(t0, t1) : t0 + t1;
        } else if (bpg == 8) {
          const float tv = TASK_MAX ? fmaxf(t0, t1) : t0 + t1;
          gacc = TASK_MAX ? fast_exp2(tv) : tv * inv_window;
        } else {
          gacc = TASK_MAX ? fast_exp2(t0) : t0 * inv_window;
          if (gcount > 1) {
            const float s1 = TASK_MAX ? fast_exp2(t1) : t1 * inv_window;
            gacc = group_max ? fmaxf(gacc, s1) : gacc + s1;
          }
        }
      }
      out[((size_t)rc * hkv + h) * total + tok0 + key_begin + t * MF_TILE + ekey] = gacc;
    }
  };
  // One key tile at a time with masking of keys past `keys_here` (ragged tile, or
  // every tile when the wave has an odd number of key tiles).
  // causal tail: task-token index of the first row of each of the wave's q blocks
  // (blocks are 32-aligned and window % 32 == 0, so a block never wraps) and the
  // last key position every row sees
  const int mbase[2] = {(row0 + (wq * 2) * 32) % window, (row0 + (wq * 2 + 1) * 32) % window};
  const int all_see = n - window;
  auto serial_tile = [&](int t, int keys_here) {
    const unsigned char* kb = kbuf[t & 1];
    for (int j = 0; j < NT; ++j) {
      const int kt = wk + j * WK;
      if (kt * 32 >= keys_here) break;          // wave-uniform
      uint4 kf[8];
      load_frags(kf, kb + kt * 8192);
      mfma_tile(acc[0], kf);
      const int kpos0 = key_begin + t * MF_TILE + kt * 32;       // position of the tile's first key
      const bool masked = causal && kpos0 + 31 > all_see;        // wave-uniform
      if (!EMIT) {
        if (kt * 32 + 32 > keys_here) {      // keys past the sequence drop out
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (kt * 32 + acc_row(r, half) >= keys_here) { acc[0][0][r] = NEG_BIG; acc[0][1][r] = NEG_BIG; }
        }
        if (masked) {                         // rows = keys, my column = one task token
#pragma unroll
          for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (kpos0 + acc_row(r, half) > all_see + mbase[qb] + col) acc[0][qb][r] = NEG_BIG;
        }
        stats_fold(acc[0][0], c2, mrun[0], srun[0]);
        stats_fold(acc[0][1], c2, mrun[1], srun[1]);
      } else {
        if (masked) {                         // rows = task tokens, my column = one key
#pragma unroll
          for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (kpos0 + col > all_see + mbase[qb] + acc_row(r, half)) acc[0][qb][r] = NEG_BIG;
        }
        emit_store(acc[0], t % 3, kt);
      }
    }
  };

  // STATS runs the chunk with the reference frozen after 256 keys; if a sum
  // overflowed (a later logit more than 2^127 above the reference: never seen on
  // attention-like data, possible on adversarial input) the whole workgroup runs
  // the chunk once more with the maxima tracked throughout.
  bool track_all = false;
  for (;;) {
  // Tile 0 has landed (and the query fragments); tile 1 is requested only now, so
  // that at kernel start, when every workgroup asks at once, all first tiles are
  // served before any second one.
  wait_vmcnt<0>();
  if (EMIT) lse_s[threadIdx.x] = my_nl;
  if (ntiles > 1) issue_tile(1);
  int issued = ntiles > 1 ? 1 : 0;            // highest tile requested so far
  __syncthreads();

  // MODE 1: the re-centred form needs the rows of each block close to its first row;
  // a workgroup that finds them too far apart hands itself to the exact kernel
  if (MODE == 1) {
    const bool far = (int)threadIdx.x < nqb * 32 &&
                     fabsf(my_nl - lse_s[threadIdx.x & ~31]) > EMIT_SPREAD_LIMIT;
    if (__syncthreads_or(far)) {
      wait_vmcnt<0>();   // tile loads in flight must land before this workgroup's LDS is given back
      if (threadIdx.x == 0) {
        const uint32_t slot = atomicAdd(defer.count, 1u);
        if (slot < defer.capacity)
          defer.entries[slot] = (uint64_t)(uint32_t)bx | ((uint64_t)(uint32_t)by << 32) | ((uint64_t)(uint32_t)bz << 56);
      }
      return;
    }
  }
  // EMIT: minus lse2 of the 16 accumulator rows of each q block held by this lane
  // (register r is row 8 (r/4) + 4 half + r%4: four consecutive rows per 16 bytes)
  if (EMIT) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int blk = wq * 2 + qb;
      const bool ok = blk < nqb;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ok) v = *reinterpret_cast<const float4*>(&lse_s[blk * 32 + 8 * i + 4 * half]);
        nl[qb][4 * i + 0] = v.x; nl[qb][4 * i + 1] = v.y; nl[qb][4 * i + 2] = v.z; nl[qb][4 * i + 3] = v.w;
      }
    }
    if (TASK_MAX && RECENTRE) {   // accumulators start from -(lse2 - lse2[first row])/c2
      const float inv_c2 = 1.f / c2;
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const int blk = wq * 2 + qb;
        // wave-uniform (the block index depends on the wave only): a scalar register
        nbase[qb] = __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane(
            (int)__float_as_uint(blk < nqb ? lse_s[blk * 32] : 0.f)));
#pragma unroll
        for (int r = 0; r < 16; ++r) nl[qb][r] = (nl[qb][r] - nbase[qb]) * inv_c2;
      }
    }
  }

  // tiles [0, npipe) run through the software pipeline
  int npipe = PIPE ? nfull : 0;
  if (causal) npipe = max(0, min(npipe, (all_see + 1 - key_begin) / MF_TILE));
  if (PIPE) {
    uint4 kf[8];
    load_frags(kf, kbuf[0] + wk * 8192);
    // Two workgroups share a CU and the hardware favours the older one; alternating
    // the wave priority per tile keeps them advancing at the same pace.
    const int prio_phase = (by * 2 >= gy) ? 1 : 0;
    for (int it = 0; it < npipe; ++it) {
      if ((it + prio_phase) & 1) __builtin_amdgcn_s_setprio(1);
      else __builtin_amdgcn_s_setprio(0);
      // STATS: the running maxima are taken from the first two macro tiles (256 keys)
      // and then frozen as the reference of the sums (see stats_slice)
      const bool track = track_all || it < 2;
      const unsigned char* kb = kbuf[it & 1];
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int kt = wk + j * WK;
        const int p = j & 1;
        const unsigned char* nkb;       // fragments to prefetch during this phase
        if (j + 1 < NT) {
          nkb = kb + (kt + WK) * 8192;
        } else {
          // all fragments of tile `it` are in registers: hand its buffer over
          if (it + 1 < ntiles) wait_vmcnt<0>();
          __syncthreads();
          if (EMIT && it > 0) epilogue(it - 1, MF_TILE);
          if (it + 2 < ntiles) { issue_tile(it + 2); issued = it + 2; }
          // next pipelined tile's first fragments (or a harmless re-read of this tile's)
          nkb = (it + 1 < npipe ? kbuf[(it + 1) & 1] : kb) + wk * 8192;
        }
        StatsCarry carry;
        float ev[2];
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int ks = i >> 1, qb = i & 1;
          const bf16x8 kfr = as_bf16x8(kf[ks]);
          f32x16 cin = acc[p][qb];
          if (ks == 0) {
            cin = zero;
            if (EMIT && TASK_MAX && RECENTRE) {
#pragma unroll
              for (int r = 0; r < 16; ++r) cin[r] = nl[qb][r];
            }
          }
          if (EMIT)   // rows = queries, columns = keys
            acc[p][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qf[qb][ks]), kfr, cin, 0, 0, 0);
          else        // rows = keys, columns = queries
            acc[p][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, as_bf16x8(qf[qb][ks]), cin, 0, 0, 0);
          if (qb == 1) kf[ks] = *reinterpret_cast<const uint4*>(nkb + (fbase ^ (32 * ks)));
          if (!EMIT) {
            stats_slice(i, acc[p ^ 1][0], acc[p ^ 1][1], c2, mrun, srun, carry, track);
            // The slice results feed nothing until the end of the tile, so without an
            // anchor the optimiser sinks the whole slice past the tile barrier (all
            // vector work of a tile would then run after its MFMAs, not beside them).
            if (i < 2) { if (track) asm volatile("" : "+v"(carry.amax[i])); }
            else if (i == 2) asm volatile("" : "+v"(carry.s[0]), "+v"(carry.s[1]), "+v"(carry.nmn[0]), "+v"(carry.nmn[1]));
            else asm volatile("" : "+v"(carry.s[0]), "+v"(carry.s[1]), "+v"(carry.e[0]), "+v"(carry.e[1]));
          } else {
            emit_slice<TASK_MAX, RECENTRE>(i, acc[p ^ 1][0], acc[p ^ 1][1], c2, nl, nbase, ev);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if (EMIT) {
          // the pending tile: previous key tile of this macro tile, or the last
          // key tile of the previous one (tile -1 goes to a buffer nobody reads)
          const int ptile = j == 0 ? it + 2 : it;            // == it - 1 (mod 3) for j == 0
          const int pkt = j == 0 ? wk + (NT - 1) * WK : kt - WK;
          red_store(ev, ptile % 3, pkt);
        }
      }
    }
    __builtin_amdgcn_s_setprio(0);
    // the last key tile of the last pipelined macro tile is still pending
    if (!EMIT) {
      stats_fold(acc[1][0], c2, mrun[0], srun[0]);
      stats_fold(acc[1][1], c2, mrun[1], srun[1]);
    } else if (npipe > 0) {
      emit_store(acc[1], (npipe - 1) % 3, wk + (NT - 1) * WK);
    }
  }
  // The other tiles one key tile at a time: the ragged last tile, tiles under the
  // causal mask, every tile when the wave has an odd number of key tiles.  Tile t
  // is in buffer t&1; tile t+1 is requested once every wave is done with tile t-1.
  for (int t = npipe; t < ntiles; ++t) {
    wait_vmcnt<0>();
    __syncthreads();
    if (EMIT && t > 0) epilogue(t - 1, MF_TILE);
    if (issued < t + 1 && t + 1 < ntiles) { issue_tile(t + 1); issued = t + 1; }
    serial_tile(t, t < nfull ? MF_TILE : tail);
  }
  __syncthreads();
  if (EMIT && ntiles > 0) epilogue(ntiles - 1, tail > 0 ? tail : MF_TILE);
  if (EMIT || track_all) break;
  // inf or NaN, tested on the bits: the library is compiled with the assumption that
  // no NaN occurs, under which a floating-point comparison may drop the NaN case (a
  // sum that overflowed to inf turns into NaN when a later tile rescales it by 0)
  const int overflowed = (__float_as_uint(srun[0]) & 0x7f800000u) == 0x7f800000u ||
                         (__float_as_uint(srun[1]) & 0x7f800000u) == 0x7f800000u;
  if (!__syncthreads_or(overflowed)) break;
  track_all = true;
  mrun[0] = mrun[1] = NEG_BIG;
  srun[0] = srun[1] = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc[1][0][r] = ninf; acc[1][1][r] = ninf; }
  issue_tile(0);
  }

  if (!EMIT) {
    // lanes l and l+32 hold the same query over different keys
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const float m2 = __shfl_xor(mrun[qb], 32), s2 = __shfl_xor(srun[qb], 32);
      const float mn = fmaxf(mrun[qb], m2);
      srun[qb] = srun[qb] * fast_exp2(mrun[qb] - mn) + s2 * fast_exp2(m2 - mn);
      mrun[qb] = mn;
      if (half == 0) { stat[wave][qb][col][0] = mrun[qb]; stat[wave][qb][col][1] = srun[qb]; }
    }
    __syncthreads();
    // one thread per query row of the row chunk merges the WK key-split waves
    const int t = threadIdx.x;
    if (t < nqb * 32) {
      const int blk = t >> 5, j = t & 31;
      const int sq = blk >> 1, qb = blk & 1;
      float mm = NEG_BIG;
#pragma unroll
      for (int k2 = 0; k2 < WK; ++k2) mm = fmaxf(mm, stat[k2 * WQ + sq][qb][j][0]);
      float ss = 0.f;
#pragma unroll
      for (int k2 = 0; k2 < WK; ++k2)
        ss += stat[k2 * WQ + sq][qb][j][1] * fast_exp2(stat[k2 * WQ + sq][qb][j][0] - mm);
      const int r = row0 + blk * 32 + j;
      // row index over all layers and sequences of the launch
      const size_t qrow = ((size_t)zid * hq + h * group) * window + r;
      // partial statistics are stored chunk-major so the merge reads coalesced
      const size_t rows_all = (size_t)gz * batch * hq * window;
      part_m[(size_t)chunk * rows_all + qrow] = mm;
      part_s[(size_t)chunk * rows_all + qrow] = ss;
    }
  }
}

// The grid-indexed kernel: workgroup (blockIdx) = ((sequence, chunk) pair, KV head x row chunk, layer).
template <bool EMIT, bool TASK_MAX, int WQ>
__global__ __launch_bounds__(MF_THREADS, 2) void score_mfma(
    PtrTable q_tab, PtrTable k_tab, int batch, size_t out_layer_stride, SeqTable seq,
    int hq, int group, int window, int total, float c2, int chunk_keys, int row_chunks,
    int rc_offset, float* __restrict__ part_m, float* __restrict__ part_s, const float* __restrict__ lse2,
    int group_max, int causal, float* __restrict__ out, DeferList defer) {
  score_mfma_body<EMIT, TASK_MAX, WQ, (EMIT && TASK_MAX) ? 1 : 0>(
      q_tab, k_tab, batch, out_layer_stride, seq, hq, group, window, total, c2, chunk_keys,
      row_chunks, rc_offset, part_m, part_s, lse2, group_max, causal, out, defer,
      (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, (int)gridDim.y, (int)gridDim.z);
}

// The list-driven kernel: redoes, in the exact form, the workgroups of the max-pooling
// emit launch with grid (gx, gy, gz) that put themselves on the list.  Workgroup i takes
// entries i, i + gridDim.x, ...; an empty list costs one load per workgroup.
template <int WQ>
__global__ __launch_bounds__(MF_THREADS, 2) void score_mfma_listed(
    PtrTable q_tab, PtrTable k_tab, int batch, size_t out_layer_stride, SeqTable seq,
    int hq, int group, int window, int total, float c2, int chunk_keys, int row_chunks,
    int rc_offset, const float* __restrict__ lse2, int group_max, int causal,
    float* __restrict__ out, DeferList defer, int gx, int gy, int gz) {
  const uint32_t listed = min(*defer.count, defer.capacity);     // appended by the launch before this one
  for (uint32_t i = blockIdx.x; i < listed; i += gridDim.x) {
    const uint64_t e = defer.entries[i];
    const int bx = (int)(uint32_t)(e & 0xffffffffu), by = (int)((e >> 32) & 0xffffffu), bz = (int)(e >> 56);
    if (bx < gx && by < gy && bz < gz)     // entries are this library's own block indices; checked all the same
      score_mfma_body<true, true, WQ, 2>(q_tab, k_tab, batch, out_layer_stride, seq, hq, group, window,
                                         total, c2, chunk_keys, row_chunks, rc_offset, nullptr, nullptr,
                                         lse2, group_max, causal, out, defer, bx, by, bz, gy, gz);
    __syncthreads();   // the next entry reuses the LDS
  }
}

// Windows up to 256 task tokens must divide 256 (a row chunk then holds whole
// query heads); larger windows must be multiples of 256 (a query head then
// spans window/256 whole row chunks).
inline bool mfma_supported(const Problem& pb) {
  if (pb.dtype != KVC_BF16 || pb.d != MF_D || pb.window % 32 != 0) return false;
  return pb.window <= MF_RCHUNK ? MF_RCHUNK % pb.window == 0 : pb.window % MF_RCHUNK == 0;
}

}  // namespace
}  // namespace kvc
