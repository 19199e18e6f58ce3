// kvc_gather: K'[l][h,k,:] = K[l][h, idx[l,h,k], :] for k < N_l, same for V
// (Section 3.3, final selection equations), written as dense per-layer blocks
// [Hkv, N_l, d] into one pool (uniform per-layer layout, constraint C2 of the
// problem statement).
//
// The grid runs over the rows of the output pool, so it is sized by the budget
// alone; lengths and offsets are read on the device.  Each row is moved as
// 16-byte pieces by adjacent lanes: writes are fully coalesced, reads are
// whole rows at random positions.
//
// Blocks of the pool: (sequence, layer) holding [Hkv, N_l, d], or, in the
// unstructured variant, (sequence, layer, head) holding [N_{l,h}, d].
//
// Position order: the retained prefix idx[l,h,0..N) of every head is first
// turned into its ascending permutation: one bit per token marks the retained
// positions, a prefix sum over the bit counts gives every marked position its
// output slot.  The gather then reads that list instead of idx.
#include "kvc_internal.h"

namespace kvc {

namespace {

constexpr int GA_THREADS = 256;
constexpr int GA_BATCH = 2;   // row groups in flight per lane (measured: 2 beats 1, 3, 4 and 8)

// Every byte the gather moves is touched once, so loads and stores carry the
// streaming (non-temporal) hint: measured 0.70 -> 0.63 ms at the 128k shape,
// most of it from the stores.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4 load_stream(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void store_stream(u32x4* p, u32x4 v) { __builtin_nontemporal_store(v, p); }

// Each wave takes 64 consecutive rows of the output pool.  Lane i first resolves
// pool row (group*64 + i): which (sequence, layer) block it lies in (binary
// search in `offsets`), its head and rank inside the block, and from `idx` the
// address of the source row.  Then the wave copies the rows a few at a time:
// `pieces` adjacent lanes move one row as 16-byte pieces, the source address
// comes from the owning lane by a cross-lane read.
// heads_per_block = Hkv (block = layer) or 1 (block = one head of a layer)
__global__ __launch_bounds__(GA_THREADS) void gather_kernel(
    PtrTable k_tab, PtrTable v_tab, int has_v, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ lengths, const int64_t* __restrict__ offsets, SeqTable seq,
    int layers, int hkv, int heads_per_block, int total, int pieces, int64_t pool_rows,
    uint4* __restrict__ k_out, uint4* __restrict__ v_out) {
  const int lane = threadIdx.x & 63;
  const int64_t wave_id = (int64_t)blockIdx.x * (GA_THREADS / 64) + (threadIdx.x >> 6);
  const int64_t wave_count = (int64_t)gridDim.x * (GA_THREADS / 64);
  const int blocks_per_layer = hkv / heads_per_block;
  const int nblk = seq.batch * layers * blocks_per_layer;
  const int hpb = heads_per_block;
  const int rows_per_step = 64 / pieces;            // rows copied by one wave instruction
  const int sub = lane / pieces, piece = lane - sub * pieces;
  const bool mover = sub < rows_per_step;
  const int steps = (64 + rows_per_step - 1) / rows_per_step;

  for (int64_t group = wave_id; group * 64 < pool_rows; group += wave_count) {
    // ---- resolve my row ----
    const int64_t row = group * 64 + lane;
    uint64_t ksrc = 0, vsrc = 0;                    // 0 = nothing to copy
    if (row < pool_rows) {
      int lo = 0, hi = nblk;   // invariant: offsets[lo]*hpb <= row < offsets[hi]*hpb
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (offsets[mid] * hpb <= row) lo = mid; else hi = mid;
      }
      const int bl = lo / blocks_per_layer, h0 = lo - bl * blocks_per_layer;   // (b,l), first head
      const int b = bl / layers, l = bl - b * layers;
      const int len = lengths[lo];
      const int64_t local = row - offsets[lo] * hpb;
      if (len > 0 && local < (int64_t)len * hpb) {   // else: inconsistent lengths/offsets
        const int hh = (int)(local / len), kk = (int)(local - (int64_t)hh * len);
        const int h = h0 * hpb + hh;
        const int n_b = seq.cu[b + 1] - seq.cu[b];
        if (kk < n_b) {
          const int p = idx[((size_t)l * hkv + h) * total + seq.cu[b] + kk];
          if (p >= 0 && p < n_b) {                   // never read outside the cache
            const size_t src = ((size_t)h * total + seq.cu[b] + p) * pieces;
            ksrc = reinterpret_cast<uint64_t>(static_cast<const uint4*>(k_tab.p[l]) + src);
            if (has_v) vsrc = reinterpret_cast<uint64_t>(static_cast<const uint4*>(v_tab.p[l]) + src);
          }
        }
      }
    }
    // ---- copy the 64 rows, GA_BATCH wave instructions of loads in flight ----
    for (int s0 = 0; s0 < steps; s0 += GA_BATCH) {
      u32x4 kd[GA_BATCH], vd[GA_BATCH];
      uint64_t kp[GA_BATCH], vp[GA_BATCH];
#pragma unroll
      for (int j = 0; j < GA_BATCH; ++j) {
        const int r = min((s0 + j) * rows_per_step + sub, 63);   // owning lane
        const uint32_t klo = __shfl((uint32_t)ksrc, r), khi = __shfl((uint32_t)(ksrc >> 32), r);
        kp[j] = ((uint64_t)khi << 32) | klo;
        if (!mover || (s0 + j) * rows_per_step + sub > 63) kp[j] = 0;
        if (has_v) {
          const uint32_t vlo = __shfl((uint32_t)vsrc, r), vhi = __shfl((uint32_t)(vsrc >> 32), r);
          vp[j] = kp[j] ? (((uint64_t)vhi << 32) | vlo) : 0;
        } else {
          vp[j] = 0;
        }
      }
#pragma unroll
      for (int j = 0; j < GA_BATCH; ++j) {
        if (kp[j]) kd[j] = load_stream(reinterpret_cast<const u32x4*>(kp[j]) + piece);
        if (vp[j]) vd[j] = load_stream(reinterpret_cast<const u32x4*>(vp[j]) + piece);
      }
#pragma unroll
      for (int j = 0; j < GA_BATCH; ++j) {
        const int64_t orow = group * 64 + (s0 + j) * rows_per_step + sub;
        if (kp[j]) store_stream(reinterpret_cast<u32x4*>(k_out) + ((size_t)orow * pieces + piece), kd[j]);
        if (vp[j]) store_stream(reinterpret_cast<u32x4*>(v_out) + ((size_t)orow * pieces + piece), vd[j]);
      }
    }
  }
}

// ---- position order ----
// mask: one bit per (layer, head, token of the packed batch), [layers*hkv][words]
// with words = ceil(total/32); sel: int32 [layers, hkv, total] like idx.
__global__ void order_clear(uint32_t* mask, size_t words) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words;
       i += (size_t)gridDim.x * blockDim.x)
    mask[i] = 0;
}

// grid: (rank blocks, layers*hkv, batch): marks idx[l,h,k], k < N of the block
__global__ void order_mark(const int32_t* __restrict__ idx, const int32_t* __restrict__ lengths,
                           SeqTable seq, int layers, int hkv, int heads_per_block, int total,
                           int words, uint32_t* __restrict__ mask) {
  const int b = blockIdx.z, lh = blockIdx.y, l = lh / hkv, h = lh - l * hkv;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int bpl = hkv / heads_per_block;
  const int len = min(n, lengths[(b * layers + l) * bpl + h / heads_per_block]);
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= len) return;
  const int p = idx[(size_t)lh * total + tok0 + k];
  if (p < 0 || p >= n) return;                       // never mark outside the sequence
  const int bit = tok0 + p;
  atomicOr(&mask[(size_t)lh * words + (bit >> 5)], 1u << (bit & 31));
}

// grid: (layers*hkv, batch), 1024 threads: sel[l,h,tok0 + j] = position of the j-th set bit
// of the sequence's bit range, ascending.
__global__ __launch_bounds__(1024) void order_compact(const uint32_t* __restrict__ mask,
                                                      SeqTable seq, int total, int words,
                                                      int32_t* __restrict__ sel) {
  __shared__ uint32_t wave_sum[16];
  __shared__ uint32_t carry;
  const int b = blockIdx.y, lh = blockIdx.x;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  if (n == 0) return;
  const int w_first = tok0 >> 5, w_last = (tok0 + n - 1) >> 5;
  const uint32_t* row = mask + (size_t)lh * words;
  int32_t* out = sel + (size_t)lh * total + tok0;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int w0 = w_first; w0 <= w_last; w0 += 1024) {
    const int w = w0 + tid;
    uint32_t bits = 0;
    if (w <= w_last) {
      bits = row[w];
      // bits of neighbouring sequences that share the first / last word drop out
      if (w == w_first) bits &= ~0u << (tok0 & 31);
      if (w == w_last) bits &= ~0u >> (31 - ((tok0 + n - 1) & 31));
    }
    const uint32_t cnt = __popc(bits);
    uint32_t incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t o = __shfl_up(incl, off);
      if (lane >= off) incl += o;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t before = carry;
    for (int i = 0; i < wave; ++i) before += wave_sum[i];
    uint32_t slot = before + incl - cnt;
    while (bits) {
      const int bit = __ffs(bits) - 1;
      bits &= bits - 1;
      if (slot < (uint32_t)n) out[slot] = (w << 5) + bit - tok0;   // slot < retained count <= n
      ++slot;
    }
    __syncthreads();
    if (tid == 1023) carry = before + incl;
    __syncthreads();
  }
}

// Plain streaming copy (16 bytes per lane, same hints as the gather), used to
// calibrate hardware counters against a known byte count and as the copy rate
// the gather is compared with.
__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src,
                                                         uint4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
       i += (size_t)gridDim.x * blockDim.x)
    store_stream(reinterpret_cast<u32x4*>(dst) + i,
                 load_stream(reinterpret_cast<const u32x4*>(src) + i));
}

}  // namespace

kvc_status launch_copy_probe(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  KVC_LAUNCH("copy_probe_kernel", stream, copy_probe_kernel<<<8192, 256, 0, stream>>>(
      static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16));
  return KVC_OK;
}

struct GatherLayout { size_t off_sel, off_mask, total; int words; };

static GatherLayout gather_layout(const Problem& pb) {
  GatherLayout L{};
  if (pb.order != KVC_ORDER_POSITION) return L;
  const size_t lh = size_t(pb.layers) * pb.hkv;
  L.words = int((pb.total + 31) / 32);
  L.off_sel = 0;
  L.off_mask = align_up(lh * size_t(pb.total) * 4);
  L.total = L.off_mask + align_up(lh * size_t(L.words) * 4);
  return L;
}

size_t gather_workspace_bytes(const Problem& pb) { return gather_layout(pb).total; }

kvc_status launch_gather(const Problem& pb, const void* const* k, const void* const* v,
                         const int32_t* idx, const int32_t* lengths, const int64_t* offsets,
                         int64_t total_budget, void* k_out, void* v_out, void* ws,
                         hipStream_t stream) {
  PtrTable kt{}, vt{};
  for (int l = 0; l < pb.layers; ++l) { kt.p[l] = k[l]; vt.p[l] = v ? v[l] : nullptr; }
  const int pieces = pb.d * esize(pb.dtype) / 16;
  const int hpb = pb.unstructured ? 1 : pb.hkv;
  const int64_t pool_rows = total_budget * hpb;
  if (pb.order == KVC_ORDER_POSITION && pb.total > 0) {
    const GatherLayout G = gather_layout(pb);
    int32_t* sel = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + G.off_sel);
    uint32_t* mask = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + G.off_mask);
    const int lh = pb.layers * pb.hkv;
    const size_t words_all = size_t(lh) * G.words;
    KVC_LAUNCH("order_clear", stream, order_clear<<<1024, 256, 0, stream>>>(mask, words_all));
    if (pb.max_seqlen > 0) {
      dim3 gm((unsigned)((pb.max_seqlen + 255) / 256), lh, pb.batch);
      KVC_LAUNCH("order_mark", stream, order_mark<<<gm, 256, 0, stream>>>(
          idx, lengths, pb.seq, pb.layers, pb.hkv, hpb, int(pb.total), G.words, mask));
      KVC_LAUNCH("order_compact", stream, order_compact<<<dim3(lh, pb.batch), 1024, 0, stream>>>(
          mask, pb.seq, int(pb.total), G.words, sel));
    }
    idx = sel;
  }
  const int64_t groups = (pool_rows + 63) / 64;                  // one wave per 64 pool rows
  int64_t blocks = (groups + GA_THREADS / 64 - 1) / (GA_THREADS / 64);
  const int64_t cap = 256 * 32;
  if (blocks > cap) blocks = cap;
  KVC_LAUNCH("gather_kernel", stream, gather_kernel<<<(unsigned)blocks, GA_THREADS, 0, stream>>>(
      kt, vt, v != nullptr, idx, lengths, offsets, pb.seq, pb.layers, pb.hkv, hpb, int(pb.total),
      pieces, pool_rows, static_cast<uint4*>(k_out), static_cast<uint4*>(v_out)));
  return KVC_OK;
}

}  // namespace kvc
