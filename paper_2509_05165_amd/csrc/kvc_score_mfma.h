// bf16 matrix-core kernels of kvc_score (d = 128, window in {32,64,128,256}).
// Included by kvc_score.hip only.
//
// One workgroup (4 waves) handles one KV head x one chunk of keys x up to 256
// query rows (8 blocks of 32 rows).  A wave owns two query blocks whose
// fragments stay in registers; K streams through LDS in 128-key macro tiles.
// v_mfma_f32_32x32x16_bf16 fragment layout (wave64): operand lane l holds, for
// row/column (l % 32), the 8 consecutive k-values 8*(l/32) .. +7; accumulator
// register r of lane l is element (row 8*(r/4) + 4*(l/32) + r%4, column l%32).
#pragma once

namespace kvc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int MF_D = 128;
constexpr int MF_TILE = 128;                 // keys per LDS macro tile
constexpr int MF_ROWB = MF_D * 2 + 16;       // padded LDS row: 272 bytes
constexpr int MF_RCHUNK = 256;               // query rows per workgroup
constexpr int MF_KBUF = MF_TILE * MF_ROWB;   // bytes per K buffer

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// Eight 16-byte pieces per thread cover one 128-key x 256-byte macro tile:
// piece i of thread t is row 16*i + t/16, bytes 16*(t%16) .. +15.
struct KStage { uint4 a, b, c, d, e, f, g, h; };

// Full tile: every row exists.  src points at this thread's piece 0 of the tile.
__device__ __forceinline__ void stage_load_full(KStage& s, const uint16_t* src) {
  constexpr int STEP = 16 * MF_D;   // 16 rows further
  s.a = *reinterpret_cast<const uint4*>(src);
  s.b = *reinterpret_cast<const uint4*>(src + STEP);
  s.c = *reinterpret_cast<const uint4*>(src + 2 * STEP);
  s.d = *reinterpret_cast<const uint4*>(src + 3 * STEP);
  s.e = *reinterpret_cast<const uint4*>(src + 4 * STEP);
  s.f = *reinterpret_cast<const uint4*>(src + 5 * STEP);
  s.g = *reinterpret_cast<const uint4*>(src + 6 * STEP);
  s.h = *reinterpret_cast<const uint4*>(src + 7 * STEP);
}
// Ragged tile: rows at or past `rows_left` re-read the last valid row.
__device__ __forceinline__ uint4 ld_clamped(const uint16_t* tile, int rows_left, int i) {
  const int row = min(16 * i + ((int)threadIdx.x >> 4), rows_left - 1);
  return *reinterpret_cast<const uint4*>(tile + (size_t)row * MF_D + ((int)threadIdx.x & 15) * 8);
}
__device__ __forceinline__ void stage_load_ragged(KStage& s, const uint16_t* tile, int rows_left) {
  s.a = ld_clamped(tile, rows_left, 0); s.b = ld_clamped(tile, rows_left, 1);
  s.c = ld_clamped(tile, rows_left, 2); s.d = ld_clamped(tile, rows_left, 3);
  s.e = ld_clamped(tile, rows_left, 4); s.f = ld_clamped(tile, rows_left, 5);
  s.g = ld_clamped(tile, rows_left, 6); s.h = ld_clamped(tile, rows_left, 7);
}
__device__ __forceinline__ void stage_store(const KStage& s, unsigned char* dst) {
  constexpr int STEP = 16 * MF_ROWB;
  *reinterpret_cast<uint4*>(dst) = s.a;
  *reinterpret_cast<uint4*>(dst + STEP) = s.b;
  *reinterpret_cast<uint4*>(dst + 2 * STEP) = s.c;
  *reinterpret_cast<uint4*>(dst + 3 * STEP) = s.d;
  *reinterpret_cast<uint4*>(dst + 4 * STEP) = s.e;
  *reinterpret_cast<uint4*>(dst + 5 * STEP) = s.f;
  *reinterpret_cast<uint4*>(dst + 6 * STEP) = s.g;
  *reinterpret_cast<uint4*>(dst + 7 * STEP) = s.h;
}

struct KFrag { uint4 v[8]; };
__device__ __forceinline__ void frag_load(KFrag& f, const unsigned char* kp) {
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) f.v[ks] = *reinterpret_cast<const uint4*>(kp + ks * 32);
}

// grid: (chunks, Hkv * row_chunks, Bt), 256 threads.  WQ = waves along the query
// rows (each owns 2 blocks of 32 rows); the other 4/WQ waves split the key tiles.
template <bool EMIT, bool TASK_MAX, int WQ>
__global__ __launch_bounds__(256, 2) void score_mfma(
    const uint16_t* __restrict__ q_layer, const uint16_t* __restrict__ k_layer, SeqTable seq,
    int hq, int group, int window, int total, float c2, int chunk_keys, int max_chunks,
    int row_chunks, float* __restrict__ part_m, float* __restrict__ part_s,
    const float* __restrict__ lse2, int group_max, float* __restrict__ out) {
  constexpr int WK = 4 / WQ;        // waves along the keys
  constexpr int NT = 4 / WK;        // 32-key tiles per wave per macro tile
  __shared__ __attribute__((aligned(16))) unsigned char kbuf[2][MF_KBUF];
  __shared__ float red[EMIT ? 2 : 1][8][EMIT ? MF_TILE : 1];   // EMIT: (q block, key) task aggregate
  __shared__ float stat[EMIT ? 1 : 4][2][32][2];               // STATS: per wave (max, sum)

  const int b = blockIdx.z;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int key_begin = blockIdx.x * chunk_keys;
  if (key_begin >= n) return;
  const int key_end = min(n, key_begin + chunk_keys);
  const int hkv = gridDim.y / row_chunks;
  const int h = blockIdx.y / row_chunks, rc = blockIdx.y - h * row_chunks;
  const int R = group * window;
  const int row0 = rc * MF_RCHUNK;
  const int nqb = (min(R, row0 + MF_RCHUNK) - row0) / 32;   // q blocks in this row chunk
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wq = wave % WQ, wk = wave / WQ;
  const int col = lane & 31, half = lane >> 5;
  const uint16_t* k_chunk = k_layer + ((size_t)h * total + tok0 + key_begin) * MF_D;

  // ---- query fragments: registers for the whole kernel ----
  uint4 qf[2][8];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int blk = wq * 2 + qb;
    const int r = row0 + blk * 32 + col;
    const bool ok = blk < nqb;
    const int g = ok ? r / window : 0, m = ok ? r % window : 0;
    const size_t qrow = ((size_t)b * hq + h * group + g) * window + m;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ok) v = *reinterpret_cast<const uint4*>(q_layer + qrow * MF_D + ks * 16 + half * 8);
      qf[qb][ks] = v;
    }
  }

  // EMIT: minus lse2 of the 16 accumulator rows of each q block held by this lane
  float nl[2][16];
  if (EMIT) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int blk = wq * 2 + qb;
      const bool ok = blk < nqb;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = 0.f;
        if (ok) {
          const int rr = row0 + blk * 32 + acc_row(r, half);
          v = -lse2[((size_t)b * hq + h * group + rr / window) * window + rr % window];
        }
        nl[qb][r] = v;
      }
    }
  }

  float mrun[2] = {NEG_BIG, NEG_BIG}, srun[2] = {0.f, 0.f};   // STATS, in log2 units
  const int bpg = window / 32;                                 // q blocks per query head
  const int gcount = nqb / bpg;                                // query heads in this row chunk

  const int span = key_end - key_begin;
  const int nfull = span / MF_TILE;             // macro tiles with all 128 keys
  const int tail = span - nfull * MF_TILE;      // keys of the ragged last tile (0 = none)
  const int ntiles = nfull + (tail > 0);

  // this thread's piece 0 inside a macro tile, in global memory and in LDS
  const uint16_t* gsrc = k_chunk + (size_t)(threadIdx.x >> 4) * MF_D + (threadIdx.x & 15) * 8;
  const int lds_piece = (threadIdx.x >> 4) * MF_ROWB + (threadIdx.x & 15) * 16;
  // this lane's fragment base inside a macro tile (key tile 0, k-step 0)
  const int lds_frag = col * MF_ROWB + half * 16;

  KStage st;
  if (nfull > 0) stage_load_full(st, gsrc);
  else stage_load_ragged(st, k_chunk, tail);
  stage_store(st, kbuf[0] + lds_piece);
  __syncthreads();

  for (int it = 0; it < ntiles; ++it) {
    const int cur = it & 1;
    const int key0 = key_begin + it * MF_TILE;
    const bool more = it + 1 < ntiles;
    if (more) {
      const uint16_t* nxt = k_chunk + (size_t)(it + 1) * MF_TILE * MF_D;
      if (it + 1 < nfull) stage_load_full(st, gsrc + (size_t)(it + 1) * MF_TILE * MF_D);
      else stage_load_ragged(st, nxt, tail);
    }

    const int keys_here = it < nfull ? MF_TILE : tail;
    const unsigned char* kb = kbuf[cur] + lds_frag;
    KFrag kf;
    frag_load(kf, kb + (wk * 32) * MF_ROWB);
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int kt = wk + j * WK;
      if (kt * 32 >= keys_here) break;          // wave-uniform; only in the ragged tile
      f32x16 acc0, acc1;
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 kfr = as_bf16x8(kf.v[ks]);
        if (EMIT) {   // rows = queries, columns = keys
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qf[0][ks]), kfr, acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qf[1][ks]), kfr, acc1, 0, 0, 0);
        } else {      // rows = keys, columns = queries
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, as_bf16x8(qf[0][ks]), acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, as_bf16x8(qf[1][ks]), acc1, 0, 0, 0);
        }
      }
      // fragments of the wave's next key tile: issued while the MFMAs drain
      if (j + 1 < NT) frag_load(kf, kb + ((kt + WK) * 32) * MF_ROWB);

      if (!EMIT) {
        if (kt * 32 + 32 > keys_here) {      // ragged: keys past the sequence drop out
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (kt * 32 + acc_row(r, half) >= keys_here) { acc0[r] = NEG_BIG; acc1[r] = NEG_BIG; }
        }
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const f32x16& acc = qb ? acc1 : acc0;
          float amax = acc[0];
#pragma unroll
          for (int r = 1; r < 16; ++r) amax = fmaxf(amax, acc[r]);
          const float mn = fmaxf(mrun[qb], amax * c2);
          float s = srun[qb] * fast_exp2(mrun[qb] - mn);
          const float nmn = -mn;
#pragma unroll
          for (int r = 0; r < 16; ++r) s += fast_exp2(fmaf(acc[r], c2, nmn));
          srun[qb] = s;
          mrun[qb] = mn;
        }
      } else {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const f32x16& acc = qb ? acc1 : acc0;
          float v = TASK_MAX ? NEG_BIG : 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float t = fmaf(acc[r], c2, nl[qb][r]);
            v = TASK_MAX ? fmaxf(v, t) : v + fast_exp2(t);
          }
          const float o = __shfl_xor(v, 32);
          v = TASK_MAX ? fmaxf(v, o) : v + o;
          const int blk = wq * 2 + qb;
          if (half == 0 && blk < nqb) red[cur][blk][kt * 32 + col] = v;
        }
      }
    }

    if (more) stage_store(st, kbuf[cur ^ 1] + lds_piece);
    __syncthreads();

    if (EMIT) {
      // threads 0..127: one key each; combine q blocks -> task -> group
      if ((int)threadIdx.x < keys_here) {
        float gacc = 0.f;
        for (int g = 0; g < gcount; ++g) {
          float tv = TASK_MAX ? NEG_BIG : 0.f;
          for (int j = 0; j < bpg; ++j) {
            const float x = red[cur][g * bpg + j][threadIdx.x];
            tv = TASK_MAX ? fmaxf(tv, x) : tv + x;
          }
          const float sv = TASK_MAX ? fast_exp2(tv) : tv / float(window);
          gacc = group_max ? fmaxf(gacc, sv) : gacc + sv;
        }
        out[((size_t)rc * hkv + h) * total + tok0 + key0 + threadIdx.x] = gacc;
      }
    }
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
      const size_t qrow = ((size_t)b * hq + h * group + r / window) * window + r % window;
      // partial statistics are stored chunk-major so the merge reads coalesced
      const size_t rows_layer = (size_t)gridDim.z * hq * window;
      part_m[(size_t)blockIdx.x * rows_layer + qrow] = mm;
      part_s[(size_t)blockIdx.x * rows_layer + qrow] = ss;
    }
  }
}

inline bool mfma_supported(const Problem& pb) {
  return pb.dtype == KVC_BF16 && pb.d == MF_D && pb.window % 32 == 0 && pb.window <= MF_RCHUNK &&
         MF_RCHUNK % pb.window == 0;
}

}  // namespace
}  // namespace kvc
