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

}  // namespace
}  // namespace kvc

#include "kvc_score_mfma.h"

namespace kvc {
namespace {

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
    int window, int d, int total, float c2, int chunk_keys, int max_chunks, int causal,
    float* part_m, float* part_s) {
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
      // causal tail: task token m sees keys at positions <= n - window + m
      const bool seen = valid && (!causal || key0 + kc <= n - window + m);
      const float t = seen ? acc * c2 : NEG_BIG;
      const float mn = fmaxf(mrun[i], t);
      srun[i] = srun[i] * fast_exp2(mrun[i] - mn) + (seen ? fast_exp2(t - mn) : 0.f);
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
      const size_t rows_layer = (size_t)gridDim.z * hq * window;
      part_m[(size_t)blockIdx.x * rows_layer + row] = mm;
      part_s[(size_t)blockIdx.x * rows_layer + row] = ss;
    }
  }
}

// grid: (chunks, Hkv, Bt); all G query heads of one KV head x one key chunk
template <typename T>
__global__ __launch_bounds__(256) void score_emit_generic(
    const T* __restrict__ q_layer, const T* __restrict__ k_layer, SeqTable seq, int hq, int group,
    int window, int d, int total, float c2, int chunk_keys, const float* __restrict__ lse2,
    int task_max, int group_max, int causal, float* __restrict__ out /* [Hkv][T] un-normalised */) {
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
          if (causal && key0 + kc > n - window + m) continue;      // hidden from task token m
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
// lse merge: 16 query rows per workgroup, 16 threads per row stride over the
// key chunks (partials are stored [chunk][row], so reads are coalesced).
// ---------------------------------------------------------------------------
constexpr int MERGE_ROWS = 16;

// (Both merge kernels also clear the two counters of the emit pass's defer lists, which
// sit DEFER_COUNTER_STRIDE words apart: the merge always runs between stats and emit.)
constexpr int DEFER_COUNTER_STRIDE = 64;
__global__ __launch_bounds__(256) void score_merge(SeqTable seq, int rows_per_seq, int layers,
                                                   int chunk_keys,
                                                   const float* __restrict__ part_m,
                                                   const float* __restrict__ part_s,
                                                   float* __restrict__ lse2,
                                                   uint32_t* __restrict__ defer_counters) {
  __shared__ float sm[16][MERGE_ROWS], ss[16][MERGE_ROWS];
  if (defer_counters && blockIdx.x == 0 && threadIdx.x < 2) defer_counters[threadIdx.x * DEFER_COUNTER_STRIDE] = 0;
  const int r = threadIdx.x & (MERGE_ROWS - 1), cg = threadIdx.x >> 4;
  // rows of every layer of the launch: row = (layer * batch + sequence) * rows_per_seq + ...
  const int rows = rows_per_seq * seq.batch * layers;
  const int row = blockIdx.x * MERGE_ROWS + r;
  float mm = NEG_BIG, acc = 0.f;
  int chunks = 0;
  if (row < rows) {
    const int b = (row / rows_per_seq) % seq.batch;
    const int n = seq.cu[b + 1] - seq.cu[b];
    chunks = (n + chunk_keys - 1) / chunk_keys;
    for (int c = cg; c < chunks; c += 16) {
      const float m2 = part_m[(size_t)c * rows + row], s2 = part_s[(size_t)c * rows + row];
      const float mn = fmaxf(mm, m2);
      acc = acc * fast_exp2(mm - mn) + s2 * fast_exp2(m2 - mn);
      mm = mn;
    }
  }
  sm[cg][r] = mm;
  ss[cg][r] = acc;
  __syncthreads();
  if (cg == 0 && row < rows && chunks > 0) {
    float top = NEG_BIG;
#pragma unroll
    for (int i = 0; i < 16; ++i) top = fmaxf(top, sm[i][r]);
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) tot += ss[i][r] * fast_exp2(sm[i][r] - top);
    lse2[row] = top + __log2f(tot);
  }
}

// Same merge, one thread per row: for sequences of a few chunks (the 4096-token
// regime has one), where sixteen lanes per row would mostly idle.
__global__ __launch_bounds__(256) void score_merge_few(SeqTable seq, int rows_per_seq, int layers,
                                                       int chunk_keys,
                                                       const float* __restrict__ part_m,
                                                       const float* __restrict__ part_s,
                                                       float* __restrict__ lse2,
                                                       uint32_t* __restrict__ defer_counters) {
  if (defer_counters && blockIdx.x == 0 && threadIdx.x < 2) defer_counters[threadIdx.x * DEFER_COUNTER_STRIDE] = 0;
  const int rows = rows_per_seq * seq.batch * layers;
  const int row = blockIdx.x * 256 + threadIdx.x;
  if (row >= rows) return;
  const int b = (row / rows_per_seq) % seq.batch;
  const int n = seq.cu[b + 1] - seq.cu[b];
  const int chunks = (n + chunk_keys - 1) / chunk_keys;
  if (chunks == 0) return;
  float mm = NEG_BIG, acc = 0.f;
  for (int c = 0; c < chunks; ++c) {
    const float m2 = part_m[(size_t)c * rows + row], s2 = part_s[(size_t)c * rows + row];
    const float mn = fmaxf(mm, m2);
    acc = acc * fast_exp2(mm - mn) + s2 * fast_exp2(m2 - mn);
    mm = mn;
  }
  lse2[row] = mm + __log2f(acc);
}

// ---------------------------------------------------------------------------
// finish: combine row-chunk partials, normalise the group mean, add head mean.
// One thread per token; in place when part == S and row_chunks == 1.  blockIdx.y
// is a layer: both pointers advance by layer_stride floats per layer (one launch
// can finish all layers when they were emitted in place).
//
// vnorm (may be null): [layers][hkv, total] weights ||V[h,c,:]||; the
// weighted attention matrix of the value-norm appendix scales every entry of
// column c of head h by the same non-negative number, which commutes with the
// max / mean over task tokens and over the group, so it is applied here.
//
// chunks_per_head = 1: every row chunk holds whole query heads and its partial is
// already a group partial.  chunks_per_head = J > 1 (window of J*256 task tokens):
// row chunk g*J + j holds rows [256 j, 256 j + 256) of query head g and its
// partial is the raw task aggregate of those rows (max of the log2-domain
// logits, or sum of probabilities); the J pieces are joined, turned into the
// task score (2^max, or sum / window) and only then aggregated over g.
// ---------------------------------------------------------------------------
struct FinishArgs {
  int row_chunks, hkv, total, group_max, add_head_mean, chunks_per_head, task_max;
  int keep_first, keep_last;   // forced retention: these tokens of every sequence score +inf
  float group_norm, inv_window;
};

__device__ __forceinline__ float finish_group_value(const float* part, const FinishArgs& a, int h,
                                                    int c, const float* vnorm) {
  float v;
  if (a.chunks_per_head <= 1) {
    v = part[((size_t)0 * a.hkv + h) * a.total + c];
    for (int rc = 1; rc < a.row_chunks; ++rc) {
      const float x = part[((size_t)rc * a.hkv + h) * a.total + c];
      v = a.group_max ? fmaxf(v, x) : v + x;
    }
  } else {
    const int heads = a.row_chunks / a.chunks_per_head;
    v = 0.f;                                           // task scores are >= 0
    for (int g = 0; g < heads; ++g) {
      float tv = part[((size_t)(g * a.chunks_per_head) * a.hkv + h) * a.total + c];
      for (int j = 1; j < a.chunks_per_head; ++j) {
        const float x = part[((size_t)(g * a.chunks_per_head + j) * a.hkv + h) * a.total + c];
        tv = a.task_max ? fmaxf(tv, x) : tv + x;
      }
      const float sv = a.task_max ? fast_exp2(tv) : tv * a.inv_window;
      v = a.group_max ? fmaxf(v, sv) : v + sv;
    }
  }
  v *= a.group_norm;
  if (vnorm) v *= vnorm[(size_t)h * a.total + c];
  return v;
}

__global__ void score_finish(const float* part, FinishArgs a, SeqTable seq, float* S,
                             size_t part_layer_stride, size_t layer_stride,
                             const float* __restrict__ vnorm) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  const int hkv = a.hkv, total = a.total, add_head_mean = a.add_head_mean;
  if (c >= total) return;
  part += blockIdx.y * part_layer_stride;
  S += blockIdx.y * layer_stride;
  if (vnorm) vnorm += blockIdx.y * ((size_t)hkv * total);   // [layer][hkv, total]
  if (a.keep_first > 0 || a.keep_last > 0) {
    int b = 0;
    while (b + 1 < seq.batch && seq.cu[b + 1] <= c) ++b;          // sequence of token c
    const int pos = c - seq.cu[b], n = seq.cu[b + 1] - seq.cu[b];
    if (pos < a.keep_first || pos >= n - a.keep_last) {
      for (int h = 0; h < hkv; ++h) S[(size_t)h * total + c] = __builtin_inff();
      return;
    }
  }
  float sum = 0.f;
  float vals[8];
  for (int h0 = 0; h0 < hkv; h0 += 8) {
    // first sweep: values of up to 8 heads (kept so the in-place write is safe)
    for (int i = 0; i < 8 && h0 + i < hkv; ++i) {
      const float v = finish_group_value(part, a, h0 + i, c, vnorm);
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
  for (int h = 0; h < hkv; ++h)
    S[(size_t)h * total + c] = finish_group_value(part, a, h, c, vnorm) + mean;
}

// The common case of the finish (one row chunk per KV head, no value norms, no
// forced retention, HKV heads known at compile time): all loads of a thread are
// independent and in flight together; VEC consecutive tokens per thread.
template <int HKV, int VEC>
__global__ __launch_bounds__(256) void score_finish_plain(const float* part, float* S, int total,
                                                          float group_norm, int add_head_mean,
                                                          size_t part_layer_stride,
                                                          size_t layer_stride) {
  typedef float vec_t __attribute__((ext_vector_type(VEC)));
  const int c = (blockIdx.x * 256 + threadIdx.x) * VEC;
  if (c >= total) return;                       // total is a multiple of VEC (host-checked)
  part += blockIdx.y * part_layer_stride;
  S += blockIdx.y * layer_stride;
  vec_t v[HKV];
#pragma unroll
  for (int h = 0; h < HKV; ++h)
    v[h] = *reinterpret_cast<const vec_t*>(part + (size_t)h * total + c) * group_norm;
  vec_t sum = v[0];
#pragma unroll
  for (int h = 1; h < HKV; ++h) sum += v[h];    // same order as the general kernel
  const vec_t mean = add_head_mean ? sum / float(HKV) : (vec_t)(0.f);
#pragma unroll
  for (int h = 0; h < HKV; ++h)
    *reinterpret_cast<vec_t*>(S + (size_t)h * total + c) = v[h] + mean;
}

// ---------------------------------------------------------------------------
// value norms: w[l][h, c] = ||V_l[h, c, :]||_2 in fp32 for every layer of the table.  A group of
// 16 lanes squares and sums one row (16 bytes per lane and step), four rows
// per wave instruction.
// ---------------------------------------------------------------------------
constexpr int VN_ROWS = 4;   // rows per 16-lane group: four independent loads in flight per lane
template <typename T>
__global__ __launch_bounds__(256) void value_norm_kernel(PtrTable v_tab, size_t rows, int d,
                                                         float* __restrict__ w) {
  constexpr int PER = 16 / sizeof(T);          // elements per 16-byte piece
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  // blockIdx.y = entry of the pointer table (a layer); its weights follow those of the one before
  const T* __restrict__ v = static_cast<const T*>(v_tab.p[blockIdx.y]);
  w += (size_t)blockIdx.y * rows;
  const int sub = threadIdx.x & 15;
  const size_t row0 = (((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 4) * VN_ROWS;
  float acc[VN_ROWS];
#pragma unroll
  for (int i = 0; i < VN_ROWS; ++i) acc[i] = 0.f;
  for (int j = sub * PER; j < d; j += 16 * PER) {
    u32x4 raw[VN_ROWS];
#pragma unroll
    for (int i = 0; i < VN_ROWS; ++i) {        // V is read once: streaming loads
      const size_t row = row0 + i < rows ? row0 + i : rows - 1;   // clamped, result dropped below
      raw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(v + row * d + j));
    }
#pragma unroll
    for (int i = 0; i < VN_ROWS; ++i) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (sizeof(T) == 2) {
          const float lo = __uint_as_float(raw[i][e] << 16), hi = __uint_as_float(raw[i][e] & 0xffff0000u);
          acc[i] = fmaf(lo, lo, acc[i]);
          acc[i] = fmaf(hi, hi, acc[i]);
        } else {
          const float f = __uint_as_float(raw[i][e]);
          acc[i] = fmaf(f, f, acc[i]);
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < VN_ROWS; ++i) {
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) acc[i] += __shfl_xor(acc[i], off);
    if (row0 + i < rows && sub == 0) w[row0 + i] = sqrtf(acc[i]);
  }
}


constexpr int GEN_CHUNK = 256;
constexpr int MF_CHUNK = 2048;        // keys per workgroup of the matrix-core path ...
constexpr int MF_CHUNK_BIG = 4096;    // ... or twice that when the launch still has plenty of workgroups

// A workgroup pays a fixed price (query fragments, first tile) per chunk, so
// longer chunks are better as long as the compute units stay oversubscribed.
inline int mfma_chunk(const Problem& pb, int row_chunks) {
  const int64_t big_chunks = (pb.max_seqlen + MF_CHUNK_BIG - 1) / MF_CHUNK_BIG;
  const int64_t wgs = big_chunks * pb.hkv * row_chunks * pb.batch * pb.layers;
  return wgs >= 2048 ? MF_CHUNK_BIG : MF_CHUNK;
}
constexpr int MIN_CHUNK = 256;   // workspace is sized for the smallest chunk in use
constexpr int MF_LISTED_BLOCKS = 512;   // workgroups of the list-driven exact emit launch (two per compute unit)

struct ScoreLayout {
  size_t off_m, off_s, off_lse, off_part, off_vnorm, off_defer, total, part_layer;
  size_t defer_capacity;   // entries per defer list: an upper bound of the workgroups of one emit launch
  int max_chunks, rows_layer, row_chunks, layers_held;
};

ScoreLayout score_layout(const Problem& pb) {
  ScoreLayout L{};
  L.rows_layer = pb.batch * pb.hq * pb.window;
  L.max_chunks = int((pb.max_seqlen + MIN_CHUNK - 1) / MIN_CHUNK);
  if (L.max_chunks < 1) L.max_chunks = 1;
  const bool mfma = mfma_supported(pb);
  L.row_chunks = mfma ? (pb.group * pb.window + MF_RCHUNK - 1) / MF_RCHUNK : 1;
  // the matrix-core path runs all layers in one launch and keeps the statistics,
  // log-sum-exps and group partials of every layer; the generic path goes layer by layer
  L.layers_held = mfma ? pb.layers : 1;
  if (mfma) L.max_chunks = int((pb.max_seqlen + MF_CHUNK - 1) / MF_CHUNK) > 0
                               ? int((pb.max_seqlen + MF_CHUNK - 1) / MF_CHUNK) : 1;
  size_t cur = 0;
  L.off_m = cur;    cur += align_up(size_t(L.rows_layer) * L.layers_held * L.max_chunks * 4);
  L.off_s = cur;    cur += align_up(size_t(L.rows_layer) * L.layers_held * L.max_chunks * 4);
  L.off_lse = cur;  cur += align_up(size_t(L.rows_layer) * L.layers_held * 4);
  L.off_part = cur;
  // partials are needed when row chunks must be combined, or when more than 8
  // KV heads make the in-place finish impossible
  L.part_layer = size_t(L.row_chunks) * pb.hkv * size_t(pb.total);
  if (L.row_chunks > 1 || pb.hkv > 8) cur += align_up(L.part_layer * L.layers_held * 4);
  L.off_vnorm = cur;
  if (pb.value_norm) cur += align_up(size_t(L.layers_held) * pb.hkv * size_t(pb.total) * 4);
  // defer lists of the emit pass (matrix-core path): two counters, then two lists of block
  // indices; a launch has at most (total/chunk + batch) x hkv x row_chunks x layers workgroups
  L.off_defer = cur;
  L.defer_capacity = 0;
  if (mfma) {
    L.defer_capacity = (size_t(pb.total) / MF_CHUNK + size_t(pb.batch)) * pb.hkv * L.row_chunks * pb.layers;
    cur += align_up(2 * DEFER_COUNTER_STRIDE * 4) + align_up(2 * L.defer_capacity * 8);
  }
  L.total = cur;
  return L;
}

}  // namespace

size_t score_workspace_bytes(const Problem& pb) { return score_layout(pb).total; }

kvc_status launch_score(const Problem& pb, const void* const* q, const void* const* k,
                        const void* const* v, float* S, void* ws, hipStream_t stream) {
  const ScoreLayout L = score_layout(pb);
  char* w = static_cast<char*>(ws);
  float* part_m = reinterpret_cast<float*>(w + L.off_m);
  float* part_s = reinterpret_cast<float*>(w + L.off_s);
  float* lse2 = reinterpret_cast<float*>(w + L.off_lse);
  const bool separate = L.row_chunks > 1 || pb.hkv > 8;
  float* vnorm = v ? reinterpret_cast<float*>(w + L.off_vnorm) : nullptr;
  const bool per_layer_finish = separate || vnorm != nullptr;
  FinishArgs fa{};
  fa.row_chunks = L.row_chunks; fa.hkv = pb.hkv; fa.total = int(pb.total);
  fa.group_max = pb.agg_group == KVC_AGG_MAX; fa.add_head_mean = pb.add_head_mean;
  fa.task_max = pb.agg_task == KVC_AGG_MAX;
  // a window above 256 task tokens spreads every query head over window/256 row chunks
  fa.chunks_per_head = (mfma_supported(pb) && pb.window > MF_RCHUNK) ? pb.window / MF_RCHUNK : 1;
  fa.group_norm = fa.group_max ? 1.f : 1.f / float(pb.group);
  fa.inv_window = 1.f / float(pb.window);
  fa.keep_first = pb.keep_first; fa.keep_last = pb.keep_last;
  const float c2 = pb.scale * LOG2E;
  const int total = int(pb.total);
  const int task_max = pb.agg_task == KVC_AGG_MAX, group_max = pb.agg_group == KVC_AGG_MAX;
  const bool mfma = mfma_supported(pb);
  const int chunk = mfma ? mfma_chunk(pb, L.row_chunks) : GEN_CHUNK;
  const int chunks = int((pb.max_seqlen + chunk - 1) / chunk);
  const int rows_per_seq = pb.hq * pb.window;

  if (mfma) {
    // One launch per pass for all layers (blockIdx.z = layer * batch + sequence).
    PtrTable qt{}, kt{};
    for (int l = 0; l < pb.layers; ++l) { qt.p[l] = q[l]; kt.p[l] = k[l]; }
    float* part_all = separate ? reinterpret_cast<float*>(w + L.off_part) : S;
    const size_t out_stride = separate ? L.part_layer : size_t(pb.hkv) * total;
    // grid.x: the (sequence, chunk) pairs of the batch, no empty slots
    int flat_chunks = 0;
    for (int b = 0; b < pb.batch; ++b)
      flat_chunks += (pb.seq.cu[b + 1] - pb.seq.cu[b] + chunk - 1) / chunk;
    if ((chunk & (chunk - 1)) != 0) { set_error("internal: chunk length %d not a power of two", chunk); return KVC_ERR_INVALID_ARG; }
    const int rows_head = pb.group * pb.window;                  // query rows per KV head
    const int nqb0 = (rows_head < MF_RCHUNK ? rows_head : MF_RCHUNK) / 32;
    const int rows_all = L.rows_layer * pb.layers;
    // The last row chunk of a head may hold few rows (G = 5 at M = 64: 256 + 64).  With
    // four waves along the rows it would cost a full 256-row pass, so when it has at most
    // four 32-row blocks it gets a launch of its own in which the waves split the keys.
    const int rem_blocks = (rows_head % MF_RCHUNK) / 32;         // 0: every chunk is full
    const bool split = L.row_chunks > 1 && rem_blocks > 0 && rem_blocks <= 4;
    const int main_chunks = split ? L.row_chunks - 1 : L.row_chunks;
    const unsigned gx = flat_chunks > 0 ? flat_chunks : 1;
    // Max-pooling emit pass: a workgroup whose log-sum-exps are too far apart for the cheap
    // form puts itself on a list (one for the main launch, one for the remainder launch)
    // and a small list-driven launch right behind redoes the listed ones in the exact form.
    uint32_t* defer_counters = reinterpret_cast<uint32_t*>(w + L.off_defer);
    uint64_t* defer_entries = reinterpret_cast<uint64_t*>(w + L.off_defer + align_up(2 * DEFER_COUNTER_STRIDE * 4));
    const uint32_t defer_cap = (uint32_t)(L.defer_capacity < 0xffffffffu ? L.defer_capacity : 0xffffffffu);
    const DeferList defer_main{defer_counters, defer_entries, defer_cap};
    const DeferList defer_rem{defer_counters + DEFER_COUNTER_STRIDE, defer_entries + L.defer_capacity, defer_cap};
    const DeferList defer_none{nullptr, nullptr, 0};
#define KVC_SCORE_MFMA(NAME, EMIT, TMAX, WQ, RCS, RC0, PM, PS, LSE, OUT)                         \
  do {                                                                                           \
    const DeferList dl_ = (EMIT && TMAX) ? ((RC0) == 0 ? defer_main : defer_rem) : defer_none;   \
    KVC_LAUNCH(NAME, stream, score_mfma<EMIT, TMAX, WQ><<<dim3(gx, pb.hkv * (RCS), pb.layers), MF_THREADS, 0, stream>>>( \
        qt, kt, pb.batch, out_stride, pb.seq, pb.hq, pb.group, pb.window, total, c2, chunk,      \
        RCS, RC0, PM, PS, LSE, group_max, pb.causal_tail, OUT, dl_));                            \
    if (EMIT && TMAX)                                                                            \
      KVC_LAUNCH(NAME ",exact", stream, score_mfma_listed<WQ><<<MF_LISTED_BLOCKS, MF_THREADS, 0, stream>>>( \
          qt, kt, pb.batch, out_stride, pb.seq, pb.hq, pb.group, pb.window, total, c2, chunk,    \
          RCS, RC0, LSE, group_max, pb.causal_tail, OUT, dl_, (int)gx, pb.hkv * (RCS), pb.layers)); \
  } while (0)
#define KVC_SCORE_MFMA_BLOCKS(NAME, EMIT, TMAX, BLOCKS, RCS, RC0, PM, PS, LSE, OUT)                  \
  do {                                                                                             \
    if ((BLOCKS) <= 2) { KVC_SCORE_MFMA(NAME, EMIT, TMAX, 1, RCS, RC0, PM, PS, LSE, OUT); }          \
    else if ((BLOCKS) <= 4) { KVC_SCORE_MFMA(NAME, EMIT, TMAX, 2, RCS, RC0, PM, PS, LSE, OUT); }     \
    else { KVC_SCORE_MFMA(NAME, EMIT, TMAX, 4, RCS, RC0, PM, PS, LSE, OUT); }                        \
  } while (0)
#define KVC_SCORE_MFMA_WQ(NAME, EMIT, TMAX, PM, PS, LSE, OUT)                                                   \
  do {                                                                                                          \
    KVC_SCORE_MFMA_BLOCKS(NAME, EMIT, TMAX, nqb0, main_chunks, 0, PM, PS, LSE, OUT);                            \
    if (split) KVC_SCORE_MFMA_BLOCKS(NAME ",rem", EMIT, TMAX, rem_blocks, 1, main_chunks, PM, PS, LSE, OUT);    \
  } while (0)
    if (chunks > 0) {
      KVC_SCORE_MFMA_WQ("score_mfma<stats>", false, true, part_m, part_s, nullptr, nullptr);
      if (chunks <= 4) {
        KVC_LAUNCH("score_merge", stream, score_merge_few<<<(rows_all + 255) / 256, 256, 0, stream>>>(
            pb.seq, rows_per_seq, pb.layers, chunk, part_m, part_s, lse2, defer_counters));
      } else {
        KVC_LAUNCH("score_merge", stream, score_merge<<<(rows_all + MERGE_ROWS - 1) / MERGE_ROWS, 256, 0, stream>>>(
            pb.seq, rows_per_seq, pb.layers, chunk, part_m, part_s, lse2, defer_counters));
      }
      if (task_max) {
        KVC_SCORE_MFMA_WQ("score_mfma<emit>", true, true, nullptr, nullptr, lse2, part_all);
      } else {
        KVC_SCORE_MFMA_WQ("score_mfma<emit>", true, false, nullptr, nullptr, lse2, part_all);
      }
    }
#undef KVC_SCORE_MFMA_WQ
#undef KVC_SCORE_MFMA_BLOCKS
#undef KVC_SCORE_MFMA
    if (vnorm && pb.layers > 0 && total > 0) {   // value norms and finish of all layers, one launch each
      PtrTable vt{};
      for (int l = 0; l < pb.layers; ++l) vt.p[l] = v[l];
      const size_t rows = size_t(pb.hkv) * total;
      const dim3 vgrid(unsigned((rows + 16 * VN_ROWS - 1) / (16 * VN_ROWS)), pb.layers);
      KVC_LAUNCH("value_norm_kernel", stream, value_norm_kernel<uint16_t><<<vgrid, 256, 0, stream>>>(
          vt, rows, pb.d, vnorm));
      KVC_LAUNCH("score_finish", stream, score_finish<<<dim3((total + 255) / 256, pb.layers), 256, 0, stream>>>(
          part_all, fa, pb.seq, S, out_stride, rows, vnorm));
    } else if (pb.layers > 0 && total > 0) {
      const bool plain = L.row_chunks == 1 && pb.keep_first == 0 && pb.keep_last == 0 &&
                         (pb.hkv == 8 || pb.hkv == 4);
      // four tokens per thread need 16-byte aligned rows in every layer
      const bool vec4 = total % 4 == 0 && out_stride % 4 == 0 &&
                        (reinterpret_cast<uintptr_t>(part_all) | reinterpret_cast<uintptr_t>(S)) % 16 == 0;
      const size_t s_stride = size_t(pb.hkv) * total;
#define KVC_FINISH_PLAIN(HKV, VEC)                                                              \
  KVC_LAUNCH("score_finish", stream,                                                            \
             score_finish_plain<HKV, VEC><<<dim3((total / VEC + 255) / 256, pb.layers), 256, 0, stream>>>( \
                 part_all, S, total, fa.group_norm, pb.add_head_mean, out_stride, s_stride))
      if (plain && pb.hkv == 8 && vec4) KVC_FINISH_PLAIN(8, 4);
      else if (plain && pb.hkv == 8) KVC_FINISH_PLAIN(8, 1);
      else if (plain && pb.hkv == 4 && vec4) KVC_FINISH_PLAIN(4, 4);
      else if (plain && pb.hkv == 4) KVC_FINISH_PLAIN(4, 1);
      else
        KVC_LAUNCH("score_finish", stream, score_finish<<<dim3((total + 255) / 256, pb.layers), 256, 0, stream>>>(
            part_all, fa, pb.seq, S, out_stride, s_stride, nullptr));
#undef KVC_FINISH_PLAIN
    }
    return KVC_OK;
  }

  // generic fp32 path: layer by layer
  for (int l = 0; l < pb.layers; ++l) {
    float* S_l = S + size_t(l) * pb.hkv * total;
    float* part = separate ? reinterpret_cast<float*>(w + L.off_part) : S_l;
    {
      const int row_blocks = (pb.window + GEN_RB - 1) / GEN_RB;
      dim3 gs(chunks, pb.hq * row_blocks, pb.batch), ge(chunks, pb.hkv, pb.batch);
      const size_t lds_s = size_t(GEN_TILE) * (pb.d + 1) * 4;
      const size_t lds_e = lds_s + size_t(GEN_MGROUPS) * GEN_TILE * 4;
      if (pb.dtype == KVC_BF16) {
        const uint16_t* ql = static_cast<const uint16_t*>(q[l]);
        const uint16_t* kl = static_cast<const uint16_t*>(k[l]);
        KVC_LAUNCH("score_stats_generic", stream, score_stats_generic<uint16_t><<<gs, 256, lds_s, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, pb.d, total, c2, chunk, L.max_chunks,
            pb.causal_tail, part_m, part_s));
        KVC_LAUNCH("score_merge", stream, score_merge<<<(L.rows_layer + MERGE_ROWS - 1) / MERGE_ROWS, 256, 0, stream>>>(
            pb.seq, rows_per_seq, 1, chunk, part_m, part_s, lse2, nullptr));
        KVC_LAUNCH("score_emit_generic", stream, score_emit_generic<uint16_t><<<ge, 256, lds_e, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, pb.d, total, c2, chunk, lse2, task_max,
            group_max, pb.causal_tail, part));
      } else {
        const float* ql = static_cast<const float*>(q[l]);
        const float* kl = static_cast<const float*>(k[l]);
        KVC_LAUNCH("score_stats_generic", stream, score_stats_generic<float><<<gs, 256, lds_s, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, pb.d, total, c2, chunk, L.max_chunks,
            pb.causal_tail, part_m, part_s));
        KVC_LAUNCH("score_merge", stream, score_merge<<<(L.rows_layer + MERGE_ROWS - 1) / MERGE_ROWS, 256, 0, stream>>>(
            pb.seq, rows_per_seq, 1, chunk, part_m, part_s, lse2, nullptr));
        KVC_LAUNCH("score_emit_generic", stream, score_emit_generic<float><<<ge, 256, lds_e, stream>>>(
            ql, kl, pb.seq, pb.hq, pb.group, pb.window, pb.d, total, c2, chunk, lse2, task_max,
            group_max, pb.causal_tail, part));
      }
    }
    // with separate partials (or one buffer of value norms) each layer is finished
    // before the next one reuses them
    if (vnorm) {
      const size_t rows = size_t(pb.hkv) * total;
      const unsigned blocks = unsigned((rows + 16 * VN_ROWS - 1) / (16 * VN_ROWS));
      PtrTable vt{};
      vt.p[0] = v[l];                       // one layer at a time on this path
      if (pb.dtype == KVC_BF16)
        KVC_LAUNCH("value_norm_kernel", stream, value_norm_kernel<uint16_t><<<blocks, 256, 0, stream>>>(
            vt, rows, pb.d, vnorm));
      else
        KVC_LAUNCH("value_norm_kernel", stream, value_norm_kernel<float><<<blocks, 256, 0, stream>>>(
            vt, rows, pb.d, vnorm));
    }
    if (per_layer_finish)
      KVC_LAUNCH("score_finish", stream, score_finish<<<(total + 255) / 256, 256, 0, stream>>>(
          part, fa, pb.seq, S_l, 0, 0, vnorm));
  }
  // emitted in place: one launch finishes every layer
  if (!per_layer_finish && pb.layers > 0 && total > 0)
    KVC_LAUNCH("score_finish", stream, score_finish<<<dim3((total + 255) / 256, pb.layers), 256, 0, stream>>>(
        S, fa, pb.seq, S, size_t(pb.hkv) * total, size_t(pb.hkv) * total, nullptr));
  return KVC_OK;
}

}  // namespace kvc
