// kvc_gather: K'[l][h,k,:] = K[l][h, idx[l,h,k], :] for k < N_l, same for V
// (Section 3.3, final selection equations), written as dense per-layer blocks
// [Hkv, N_l, d] into one pool (uniform per-layer layout, constraint C2 of the
// problem statement).
//
// The grid runs over the rows of the output pool, so it is sized by the budget
// alone; lengths and offsets are read on the device.  Each row is moved as
// 16-byte pieces by adjacent lanes: writes are fully coalesced, reads are
// whole rows at random positions.
#include "kvc_internal.h"

namespace kvc {

namespace {

constexpr int GA_THREADS = 256;
constexpr int GA_BATCH = 4;   // row groups in flight per lane

// Each wave takes 64 consecutive rows of the output pool.  Lane i first resolves
// pool row (group*64 + i): which (sequence, layer) block it lies in (binary
// search in `offsets`), its head and rank inside the block, and from `idx` the
// address of the source row.  Then the wave copies the rows a few at a time:
// `pieces` adjacent lanes move one row as 16-byte pieces, the source address
// comes from the owning lane by a cross-lane read.
__global__ __launch_bounds__(GA_THREADS) void gather_kernel(
    PtrTable k_tab, PtrTable v_tab, int has_v, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ lengths, const int64_t* __restrict__ offsets, SeqTable seq,
    int layers, int hkv, int total, int pieces, int64_t pool_rows, uint4* __restrict__ k_out,
    uint4* __restrict__ v_out) {
  const int lane = threadIdx.x & 63;
  const int64_t wave_id = (int64_t)blockIdx.x * (GA_THREADS / 64) + (threadIdx.x >> 6);
  const int64_t wave_count = (int64_t)gridDim.x * (GA_THREADS / 64);
  const int nblk = seq.batch * layers;
  const int rows_per_step = 64 / pieces;            // rows copied by one wave instruction
  const int sub = lane / pieces, piece = lane - sub * pieces;
  const bool mover = sub < rows_per_step;
  const int steps = (64 + rows_per_step - 1) / rows_per_step;

  for (int64_t group = wave_id; group * 64 < pool_rows; group += wave_count) {
    // ---- resolve my row ----
    const int64_t row = group * 64 + lane;
    uint64_t ksrc = 0, vsrc = 0;                    // 0 = nothing to copy
    if (row < pool_rows) {
      int lo = 0, hi = nblk;   // invariant: offsets[lo]*hkv <= row < offsets[hi]*hkv
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (offsets[mid] * hkv <= row) lo = mid; else hi = mid;
      }
      const int b = lo / layers, l = lo - b * layers;
      const int len = lengths[lo];
      const int64_t local = row - offsets[lo] * hkv;
      if (len > 0 && local < (int64_t)len * hkv) {   // else: inconsistent lengths/offsets
        const int h = (int)(local / len), kk = (int)(local - (int64_t)h * len);
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
      uint4 kd[GA_BATCH], vd[GA_BATCH];
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
        if (kp[j]) kd[j] = reinterpret_cast<const uint4*>(kp[j])[piece];
        if (vp[j]) vd[j] = reinterpret_cast<const uint4*>(vp[j])[piece];
      }
#pragma unroll
      for (int j = 0; j < GA_BATCH; ++j) {
        const int64_t orow = group * 64 + (s0 + j) * rows_per_step + sub;
        if (kp[j]) k_out[(size_t)orow * pieces + piece] = kd[j];
        if (vp[j]) v_out[(size_t)orow * pieces + piece] = vd[j];
      }
    }
  }
}

// Plain streaming copy (16 bytes per lane), used only to calibrate hardware
// counters against a known byte count.
__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src,
                                                         uint4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
       i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

}  // namespace

kvc_status launch_copy_probe(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  KVC_LAUNCH("copy_probe_kernel", stream, copy_probe_kernel<<<8192, 256, 0, stream>>>(
      static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16));
  return KVC_OK;
}

kvc_status launch_gather(const Problem& pb, const void* const* k, const void* const* v,
                         const int32_t* idx, const int32_t* lengths, const int64_t* offsets,
                         int64_t total_budget, void* k_out, void* v_out, hipStream_t stream) {
  PtrTable kt{}, vt{};
  for (int l = 0; l < pb.layers; ++l) { kt.p[l] = k[l]; vt.p[l] = v ? v[l] : nullptr; }
  const int pieces = pb.d * esize(pb.dtype) / 16;
  const int64_t pool_rows = total_budget * pb.hkv;
  const int64_t groups = (pool_rows + 63) / 64;                  // one wave per 64 pool rows
  int64_t blocks = (groups + GA_THREADS / 64 - 1) / (GA_THREADS / 64);
  const int64_t cap = 256 * 32;
  if (blocks > cap) blocks = cap;
  KVC_LAUNCH("gather_kernel", stream, gather_kernel<<<(unsigned)blocks, GA_THREADS, 0, stream>>>(
      kt, vt, v != nullptr, idx, lengths, offsets, pb.seq, pb.layers, pb.hkv, int(pb.total),
      pieces, pool_rows, static_cast<uint4*>(k_out), static_cast<uint4*>(v_out)));
  return KVC_OK;
}

}  // namespace kvc
