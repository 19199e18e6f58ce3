// kvc_score: attention of the window queries over all cached keys, aggregated
// as in Section 3.2.2 of the paper (task tokens -> GQA group -> head mean).
//
// The attention tensor A[l,q,c,m] is never stored.  Per layer:
//   stats : logits t = (q.k) * scale * log2(e) for every (query row, key);
//           per key-chunk running (max, sum 2^(t-max)) for every query row
//   merge : lse2[row] = log2 sum_c 2^t over all chunks of the row's sequence
//   emit  : logits again; p = 2^(t - lse2); Agg_task over m, Agg_group over g
//   finish: combine row-chunk partials, add the mean over KV heads
// Two implementations of stats/emit: a bf16 matrix-core (MFMA) kernel for
// d = 128, and a plain fp32 kernel for everything else (f32 inputs, other
// head sizes, windows that are not a multiple of 32).
#include "kvc_internal.h"

namespace kvc {

namespace {

constexpr float NEG_BIG = -1.0e30f;
constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float load_as_float(const float* p) { return *p; }
__device__ __forceinline__ float load_as_float(const uint16_t* p) {
  return __uint_as_float(uint32_t(*p) << 16);
}

// ---------------------------------------------------------------------------
// Plain fp32 path
// ---------------------------------------------------------------------------
constexpr int GEN_TILE = 32;     // keys per LDS tile
constexpr int GEN_MGROUPS = 8;   // 256 threads = 32 key lanes x 8 row groups
constexpr int GEN_ROWS = 8;      // query rows per thread per row block
constexpr int GEN_RB = GEN_MGROUPS * GEN_ROWS;  // 64 query rows per row block

template <typename T>
__device__ __forceinline__ void gen_load_ktile(float* lds, const T* k_head, int tok0, int key0,
                                               int n, int d) {
  // lds[key][d+1]; rows beyond the sequence are clamped (masked by the caller)
  for (int e = threadIdx.x; e < GEN_TILE * d; e += blockDim.x) {
    int r = e / d, j = e - r * d;
    int key = min(key0 + r, n - 1);
    lds[r * (d + 1) + j] = load_as_float(k_head + (size_t)(tok0 + key) * d + j);
  }
}

// grid: (chunks, Hq * row_blocks, Bt); one query head's <=64 rows x one key chunk
template <typename T>
__global__ __launch_bounds__(256) void score_stats_generic(
    const T* __restrict__ q_layer, const T* __restrict__ k_layer, SeqTable seq, int hq, int group,
    int window, int d, int total, float c2, int chunk_keys, int max_chunks, float* part_m,
    float* part_s) {
  extern __shared__ float lds[];
  const int b = blockIdx.z;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int key_begin = blockIdx.x * chunk_keys;
  if (key_begin >= n) return;
  const int key_end = min(n, key_begin + chunk_keys);
  const int row_blocks = (window + GEN_RB - 1) / GEN_RB;
  const int qh = blockIdx.y / row_blocks, rb = blockIdx.y - qh * row_blocks;
  const int hkv = hq / group;
  const T* k_head = k_layer + (size_t)(qh / group) * total * d;
  const T* q_head = q_layer + ((size_t)b * hq + qh) * window * d;
  const int kc = threadIdx.x % GEN_TILE, mg = threadIdx.x / GEN_TILE;
  (void)hkv;

  float mrun[GEN_ROWS], srun[GEN_ROWS];
#pragma unroll
  for (int i = 0; i < GEN_ROWS; ++i) { mrun[i] = NEG_BIG; srun[i] = 0.f; }

  for (int key0 = key_begin; key0 < key_end; key0 += GEN_TILE) {
    __syncthreads();
    gen_load_ktile(lds, k_head, tok0, key0, n, d);
    __syncthreads();
    const bool valid = key0 + kc < key_end;
    const float* krow = lds + kc * (d + 1);
#pragma unroll
    for (int i = 0; i < GEN_ROWS; ++i) {
      const int m = rb * GEN_RB + i * GEN_MGROUPS + mg;
      if (m >= window) continue;
      const T* qrow = q_head + (size_t)m * d;
      float acc = 0.f;
      for (int j = 0; j < d; ++j) acc = fmaf(load_as_float(qrow + j), krow[j], acc);
      const float t = valid ? acc * c2 : NEG_BIG;
      const float mn = fmaxf(mrun[i], t);
      srun[i] = srun[i] * fast_exp2(mrun[i] - mn) + (valid ? fast_exp2(t - mn) : 0.f);
      mrun[i] = mn;
    }
  }
  // combine the 32 key lanes of every row (lanes of one half-wave)
#pragma unroll
  for (int i = 0; i < GEN_ROWS; ++i) {
    float mm = mrun[i], ss = srun[i];
    for (int off = 16; off >= 1; off >>= 1) {
      const float m2 = __shfl_xor(mm, off), s2 = __shfl_xor(ss, off);
      const float mn = fmaxf(mm, m2);
      ss = ss * fast_exp2(mm - mn) + s2 * fast_exp2(m2 - mn);
      mm = mn;
    }
    const int m = rb * GEN_RB + i * GEN_MGROUPS + mg;
    if (kc == 0 && m < window) {
      const size_t row = ((size_t)b * hq + qh) * window + m;
      part_m[row * max_chunks + blockIdx.x] = mm;
      part_s[row * max_chunks + blockIdx.x] = ss;
    }
  }
}

// grid: (chunks, Hkv, Bt); all G query heads of one KV head x one key chunk
template <typename T>
__global__ __launch_bounds__(256) void score_emit_generic(
    const T* __restrict__ q_layer, const T* __restrict__ k_layer, SeqTable seq, int hq, int group,
    int window, int d, int total, float c2, int chunk_keys, const float* __restrict__ lse2,
    int task_max, int group_max, float* __restrict__ out /* [Hkv][T] un-normalised */) {
  extern __shared__ float lds[];
  float* red = lds + GEN_TILE * (d + 1);  // [GEN_MGROUPS][GEN_TILE]
  const int b = blockIdx.z, h = blockIdx.y;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int key_begin = blockIdx.x * chunk_keys;
  if (key_begin >= n) return;
  const int key_end = min(n, key_begin + chunk_keys);
  const T* k_head = k_layer + (size_t)h * total * d;
  const int kc = threadIdx.x % GEN_TILE, mg = threadIdx.x / GEN_TILE;
  const int row_blocks = (window + GEN_RB - 1) / GEN_RB;

  for (int key0 = key_begin; key0 < key_end; key0 += GEN_TILE) {
    __syncthreads();
    gen_load_ktile(lds, k_head, tok0, key0, n, d);
    __syncthreads();
    const float* krow = lds + kc * (d + 1);
    float gacc = group_max ? 0.f : 0.f;  // probabilities are >= 0
    for (int g = 0; g < group; ++g) {
      const int qh = h * group + g;
      const T* q_head = q_layer + ((size_t)b * hq + qh) * window * d;
      const float* lse_head = lse2 + ((size_t)b * hq + qh) * window;
      float tacc = task_max ? NEG_BIG : 0.f;   // max of t, or sum of p
      for (int rb = 0; rb < row_blocks; ++rb) {
        float v = task_max ? NEG_BIG : 0.f;
#pragma unroll
        for (int i = 0; i < GEN_ROWS; ++i) {
          const int m = rb * GEN_RB + i * GEN_MGROUPS + mg;
          if (m >= window) continue;
          const T* qrow = q_head + (size_t)m * d;
          float acc = 0.f;
          for (int j = 0; j < d; ++j) acc = fmaf(load_as_float(qrow + j), krow[j], acc);
          const float t = acc * c2 - lse_head[m];
          v = task_max ? fmaxf(v, t) : v + fast_exp2(t);
        }
        red[mg * GEN_TILE + kc] = v;
        __syncthreads();
        if (mg == 0) {
          for (int w = 0; w < GEN_MGROUPS; ++w) {
            const float x = red[w * GEN_TILE + kc];
            tacc = task_max ? fmaxf(tacc, x) : tacc + x;
          }
        }
        __syncthreads();
      }
      const float sv = task_max ? fast_exp2(tacc) : tacc / float(window);
      gacc = group_max ? fmaxf(gacc, sv) : gacc + sv;
    }
    if (mg == 0 && key0 + kc < key_end) out[(size_t)h * total + tok0 + key0 + kc] = gacc;
  }
}

// ---------------------------------------------------------------------------
// lse merge: one thread per query row of the layer
// ---------------------------------------------------------------------------
__global__ void score_merge(SeqTable seq, int rows_per_seq, int chunk_keys, int max_chunks,
                            const float* __restrict__ part_m, const float* __restrict__ part_s,
                            float* __restrict__ lse2) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= rows_per_seq * seq.batch) return;
  const int b = row / rows_per_seq;
  const int n = seq.cu[b + 1] - seq.cu[b];
  const int chunks = (n + chunk_keys - 1) / chunk_keys;
  if (chunks == 0) return;
  const float* pm = part_m + (size_t)row * max_chunks;
  const float* ps = part_s + (size_t)row * max_chunks;
  float mm = NEG_BIG;
  for (int c = 0; c < chunks; ++c) mm = fmaxf(mm, pm[c]);
  float ss = 0.f;
  for (int c = 0; c < chunks; ++c) ss += ps[c] * fast_exp2(pm[c] - mm);
  lse2[row] = mm + __log2f(ss);
}

// ---------------------------------------------------------------------------
// finish: combine row-chunk partials, normalise the group mean, add head mean.
// One thread per token; in place when part == S and row_chunks == 1.
// ---------------------------------------------------------------------------
__global__ void score_finish(const float* part, int row_chunks, int hkv, int total,
                             float group_norm, int group_max, int add_head_mean, float* S) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= total) return;
  float sum = 0.f;
  float vals[8];
  for (int h0 = 0; h0 < hkv; h0 += 8) {
    // first sweep: values of up to 8 heads (kept so the in-place write is safe)
    for (int i = 0; i < 8 && h0 + i < hkv; ++i) {
      float v = part[((size_t)0 * hkv + h0 + i) * total + c];
      for (int rc = 1; rc < row_chunks; ++rc) {
        const float x = part[((size_t)rc * hkv + h0 + i) * total + c];
        v = group_max ? fmaxf(v, x) : v + x;
      }
      v *= group_norm;
      vals[i] = v;
      sum += v;
    }
    if (hkv <= 8) {
      const float mean = add_head_mean ? sum / float(hkv) : 0.f;
      for (int i = 0; i < hkv; ++i) S[(size_t)i * total + c] = vals[i] + mean;
      return;
    }
  }
  // more than 8 KV heads: recompute values in a second sweep (part != S is
  // guaranteed by the launcher in that case)
  const float mean = add_head_mean ? sum / float(hkv) : 0.f;
  for (int h = 0; h < hkv; ++h) {
    float v = part[((size_t)0 * hkv + h) * total + c];
    for (int rc = 1; rc < row_chunks; ++rc) {
      const float x = part[((size_t)rc * hkv + h) * total + c];
      v = group_max ? fmaxf(v, x) : v + x;
    }
    S[(size_t)h * total + c] = v * group_norm + mean;
  }
}

// ---------------------------------------------------------------------------
// bf16 matrix-core path (d = 128, window a multiple of 32 that divides 256)
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int MF_D = 128;
constexpr int MF_TILE = 128;                 // keys per LDS macro tile
constexpr int MF_ROWB = MF_D * 2 + 16;       // padded LDS row: 272 bytes
constexpr int MF_RCHUNK = 256;               // query rows per workgroup
constexpr int MF_KBUF = MF_TILE * MF_ROWB;   // bytes per K buffer

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// row i of a 32x32 accumulator held in register r of lane l: 8*(r/4) + 4*(l/32) + r%4
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// grid: (chunks, Hkv * row_chunks, Bt), 256 threads.
template <bool EMIT, bool TASK_MAX>
__global__ __launch_bounds__(256, 2) void score_mfma(
    const uint16_t* __restrict__ q_layer, const uint16_t* __restrict__ k_layer, SeqTable seq,
    int hq, int group, int window, int total, float c2, int chunk_keys, int max_chunks,
    int row_chunks, float* __restrict__ part_m, float* __restrict__ part_s,
    const float* __restrict__ lse2, int group_max, float* __restrict__ out) {
  __shared__ __attribute__((aligned(16))) unsigned char kbuf[2 * MF_KBUF];
  __shared__ float red[2][8][MF_TILE];       // EMIT: per (q block, key) task aggregate
  __shared__ float stat[4][2][32][2];        // STATS: per wave (m, s)

  const int b = blockIdx.z;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int key_begin = blockIdx.x * chunk_keys;
  if (key_begin >= n) return;
  const int key_end = min(n, key_begin + chunk_keys);
  const int h = blockIdx.y / row_chunks, rc = blockIdx.y - h * row_chunks;
  const int R = group * window;
  const int row0 = rc * MF_RCHUNK;
  const int nqb = (min(R, row0 + MF_RCHUNK) - row0) / 32;   // q blocks in this row chunk
  const int WQ = (nqb + 1) / 2;
  const int WK = 4 / WQ;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wq = wave % WQ, wk = wave / WQ;
  const bool active = wk < WK;
  const int col = lane & 31, half = lane >> 5;

  const uint16_t* k_head = k_layer + (size_t)h * total * MF_D;

  // ---- query fragments (registers, whole kernel) ----
  uint4 qf[2][8];
  int grow[2];          // global stats row of this lane's query (column role)
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int blk = wq * 2 + qb;
    const int r = row0 + blk * 32 + col;
    const bool ok = active && blk < nqb;
    const int g = ok ? r / window : 0, m = ok ? r % window : 0;
    const size_t qrow = ((size_t)b * hq + h * group + g) * window + m;
    grow[qb] = ok ? (int)qrow : -1;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ok) v = *reinterpret_cast<const uint4*>(q_layer + qrow * MF_D + ks * 16 + half * 8);
      qf[qb][ks] = v;
    }
  }

  // EMIT: lse2 of the 16 accumulator rows of each q block held by this lane
  float lrow[2][16];
  if (EMIT) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int blk = wq * 2 + qb;
      const bool ok = active && blk < nqb;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = 0.f;
        if (ok) {
          const int rr = row0 + blk * 32 + acc_row(r, half);
          v = lse2[((size_t)b * hq + h * group + rr / window) * window + rr % window];
        }
        lrow[qb][r] = v;
      }
    }
  }

  float mrun[2] = {NEG_BIG, NEG_BIG}, srun[2] = {0.f, 0.f};

  // ---- K macro tiles through LDS, register-staged double buffering ----
  uint4 stage[8];
  auto gload = [&](int key0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int id = i * 256 + threadIdx.x;
      const int r = id >> 4, c = id & 15;
      const int key = min(key0 + r, n - 1);
      stage[i] = *reinterpret_cast<const uint4*>(k_head + (size_t)(tok0 + key) * MF_D + c * 8);
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int id = i * 256 + threadIdx.x;
      const int r = id >> 4, c = id & 15;
      *reinterpret_cast<uint4*>(kbuf + buf * MF_KBUF + r * MF_ROWB + c * 16) = stage[i];
    }
  };

  gload(key_begin);
  lstore(0);
  __syncthreads();

  int it = 0;
  for (int key0 = key_begin; key0 < key_end; key0 += MF_TILE, ++it) {
    const int cur = it & 1;
    const bool more = key0 + MF_TILE < key_end;
    if (more) gload(key0 + MF_TILE);

    if (active) {
      const unsigned char* kb = kbuf + cur * MF_KBUF;
      for (int kt = wk; kt < MF_TILE / 32; kt += WK) {
        const int tkey0 = key0 + kt * 32;
        if (tkey0 >= key_end) break;
        f32x16 acc[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[qb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const uint4 kv = *reinterpret_cast<const uint4*>(kb + (kt * 32 + col) * MF_ROWB +
                                                           (2 * ks + half) * 16);
          const bf16x8 kf = as_bf16x8(kv);
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) {
            if (EMIT)   // rows = queries, columns = keys
              acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(qf[qb][ks]), kf, acc[qb], 0, 0, 0);
            else        // rows = keys, columns = queries
              acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, as_bf16x8(qf[qb][ks]), acc[qb], 0, 0, 0);
          }
        }
        if (!EMIT) {
          const bool ragged = tkey0 + 32 > key_end;
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) {
            float t[16];
            float tmax = NEG_BIG;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              t[r] = acc[qb][r] * c2;
              if (ragged && tkey0 + acc_row(r, half) >= key_end) t[r] = NEG_BIG;
              tmax = fmaxf(tmax, t[r]);
            }
            const float mn = fmaxf(mrun[qb], tmax);
            float s = srun[qb] * fast_exp2(mrun[qb] - mn);
#pragma unroll
            for (int r = 0; r < 16; ++r) s += fast_exp2(t[r] - mn);
            srun[qb] = s;
            mrun[qb] = mn;
          }
        } else {
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) {
            float v = TASK_MAX ? NEG_BIG : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const float t = acc[qb][r] * c2 - lrow[qb][r];
              v = TASK_MAX ? fmaxf(v, t) : v + fast_exp2(t);
            }
            const float o = __shfl_xor(v, 32);
            v = TASK_MAX ? fmaxf(v, o) : v + o;
            const int blk = wq * 2 + qb;
            if (half == 0 && blk < nqb) red[cur][blk][kt * 32 + col] = v;
          }
        }
      }
    }

    if (more) lstore(cur ^ 1);
    __syncthreads();

    if (EMIT) {
      // threads 0..127: one key each; combine q blocks -> task -> group
      const int key = key0 + (int)threadIdx.x;
      if (threadIdx.x < MF_TILE && key < key_end) {
        const int bpg = window / 32;            // q blocks per query head
        const int gcount = nqb / bpg;           // query heads in this row chunk
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
        out[((size_t)rc * (gridDim.y / row_chunks) + h) * total + tok0 + key] = gacc;
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
      for (int k2 = 0; k2 < WK; ++k2) mm = fmaxf(mm, stat[k2 * WQ + sq][qb][j][0]);
      float ss = 0.f;
      for (int k2 = 0; k2 < WK; ++k2)
        ss += stat[k2 * WQ + sq][qb][j][1] * fast_exp2(stat[k2 * WQ + sq][qb][j][0] - mm);
      const int r = row0 + blk * 32 + j;
      const size_t qrow = ((size_t)b * hq + h * group + r / window) * window + r % window;
      part_m[qrow * max_chunks + blockIdx.x] = mm;
      part_s[qrow * max_chunks + blockIdx.x] = ss;
    }
  }
  (void)grow;
}

inline bool mfma_supported(const Problem& pb) {
  return pb.dtype == KVC_BF16 && pb.d == MF_D && pb.window % 32 == 0 && pb.window <= MF_RCHUNK &&
         MF_RCHUNK % pb.window == 0;
}

constexpr int GEN_CHUNK = 256;
constexpr int MF_CHUNK = 1024;
constexpr int MIN_CHUNK = 256;   // workspace is sized for the smallest chunk in use

struct ScoreLayout {
  size_t off_m, off_s, off_lse, off_part, total;
  int max_chunks, rows_layer, row_chunks;
};

ScoreLayout score_layout(const Problem& pb) {
  ScoreLayout L{};
  L.rows_layer = pb.batch * pb.hq * pb.window;
  L.max_chunks = int((pb.max_seqlen + MIN_CHUNK - 1) / MIN_CHUNK);
  if (L.max_chunks < 1) L.max_chunks = 1;
  L.row_chunks = mfma_supported(pb) ? (pb.group * pb.window + MF_RCHUNK - 1) / MF_RCHUNK : 1;
  size_t cur = 0;
  L.off_m = cur;    cur += align_up(size_t(L.rows_layer) * L.max_chunks * 4);
  L.off_s = cur;    cur += align_up(size_t(L.rows_layer) * L.max_chunks * 4);
  L.off_lse = cur;  cur += align_up(size_t(L.rows_layer) * 4);
  L.off_part = cur;
  // partials are needed when row chunks must be combined, or when more than 8
  // KV heads make the in-place finish impossible
  if (L.row_chunks > 1 || pb.hkv > 8)
    cur += align_up(size_t(L.row_chunks) * pb.hkv * size_t(pb.total) * 4);
  L.total = cur;
  return L;
}

}  // namespace

size_t score_workspace_bytes(const Problem& pb) { return score_layout(pb).total; }

kvc_status launch_score(const Problem& pb, const void* const* q, const void* const* k, float* S,
                        void* ws, hipStream_t stream) {
  const ScoreLayout L = score_layout(pb);
  char* w = static_cast<char*>(ws);
  float* part_m = reinterpret_cast<float*>(w + L.off_m);
  float* part_s = reinterpret_cast<float*>(w + L.off_s);
  float* lse2 = reinterpret_cast<float*>(w + L.off_lse);
  const bool separate = L.row_chunks > 1 || pb.hkv > 8;
  const float c2 = pb.scale * LOG2E;
  const int total = int(pb.total);
  const int task_max = pb.agg_task == KVC_AGG_MAX, group_max = pb.agg_group == KVC_AGG_MAX;
  const float group_norm = group_max ? 1.f : 1.f / float(pb.group);
  const bool mfma = mfma_supported(pb);
  const int chunk = mfma ? MF_CHUNK : GEN_CHUNK;
  const int chunks = int((pb.max_seqlen + chunk - 1) / chunk);
  const int rows_per_seq = pb.hq * pb.window;

  for (int l = 0; l < pb.layers; ++l) {
    float* S_l = S + size_t(l) * pb.hkv * total;
    float* part = separate ? reinterpret_cast<float*>(w + L.off_part) : S_l;
    if (mfma) {
      const uint16_t* ql = static_cast<const uint16_t*>(q[l]);
      const uint16_t* kl = static_cast<const uint16_t*>(k[l]);
      dim3 grid(chunks, pb.hkv * L.row_chunks, pb.batch);
      KVC_LAUNCH("score_mfma<stats>", stream, score_mfma<false, true><<<grid, 256, 0, stream>>>(
          ql, kl, pb.seq, pb.hq, pb.group, pb.window, total, c2, chunk, L.max_chunks,
          L.row_chunks, part_m, part_s, nullptr, group_max, nullptr));
      KVC_LAUNCH("score_merge", stream, score_merge<<<(L.rows_layer + 255) / 256, 256, 0, stream>>>(
          pb.seq, rows_per_seq, chunk, L.max_chunks, part_m, part_s, lse2));
      if (task_max) {
        KVC_LAUNCH("score_mfma<emit>", stream, score_mfma<true, true><<<grid, 256, 0, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, total, c2, chunk, L.max_chunks,
            L.row_chunks, nullptr, nullptr, lse2, group_max, part));
      } else {
        KVC_LAUNCH("score_mfma<emit>", stream, score_mfma<true, false><<<grid, 256, 0, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, total, c2, chunk, L.max_chunks,
            L.row_chunks, nullptr, nullptr, lse2, group_max, part));
      }
    } else {
      const int row_blocks = (pb.window + GEN_RB - 1) / GEN_RB;
      dim3 gs(chunks, pb.hq * row_blocks, pb.batch), ge(chunks, pb.hkv, pb.batch);
      const size_t lds_s = size_t(GEN_TILE) * (pb.d + 1) * 4;
      const size_t lds_e = lds_s + size_t(GEN_MGROUPS) * GEN_TILE * 4;
      if (pb.dtype == KVC_BF16) {
        const uint16_t* ql = static_cast<const uint16_t*>(q[l]);
        const uint16_t* kl = static_cast<const uint16_t*>(k[l]);
        KVC_LAUNCH("score_stats_generic", stream, score_stats_generic<uint16_t><<<gs, 256, lds_s, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, pb.d, total, c2, chunk, L.max_chunks,
            part_m, part_s));
        KVC_LAUNCH("score_merge", stream, score_merge<<<(L.rows_layer + 255) / 256, 256, 0, stream>>>(
            pb.seq, rows_per_seq, chunk, L.max_chunks, part_m, part_s, lse2));
        KVC_LAUNCH("score_emit_generic", stream, score_emit_generic<uint16_t><<<ge, 256, lds_e, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, pb.d, total, c2, chunk, lse2, task_max,
            group_max, part));
      } else {
        const float* ql = static_cast<const float*>(q[l]);
        const float* kl = static_cast<const float*>(k[l]);
        KVC_LAUNCH("score_stats_generic", stream, score_stats_generic<float><<<gs, 256, lds_s, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, pb.d, total, c2, chunk, L.max_chunks,
            part_m, part_s));
        KVC_LAUNCH("score_merge", stream, score_merge<<<(L.rows_layer + 255) / 256, 256, 0, stream>>>(
            pb.seq, rows_per_seq, chunk, L.max_chunks, part_m, part_s, lse2));
        KVC_LAUNCH("score_emit_generic", stream, score_emit_generic<float><<<ge, 256, lds_e, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, pb.d, total, c2, chunk, lse2, task_max,
            group_max, part));
      }
    }
    KVC_LAUNCH("score_finish", stream, score_finish<<<(total + 255) / 256, 256, 0, stream>>>(part, L.row_chunks, pb.hkv, total,
                                                          group_norm, group_max,
                                                          pb.add_head_mean, S_l));
  }
  return KVC_OK;
}

}  // namespace kvc
