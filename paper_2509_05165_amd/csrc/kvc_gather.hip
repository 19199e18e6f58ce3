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

// grid: (row blocks); `pieces` = 16-byte pieces per row (power of two not required)
__global__ __launch_bounds__(GA_THREADS) void gather_kernel(
    PtrTable k_tab, PtrTable v_tab, int has_v, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ lengths, const int64_t* __restrict__ offsets, SeqTable seq,
    int layers, int hkv, int total, int pieces, int64_t pool_rows, uint4* __restrict__ k_out,
    uint4* __restrict__ v_out) {
  const int rows_per_block = GA_THREADS / pieces;
  const int piece = threadIdx.x % pieces;
  const int rsub = threadIdx.x / pieces;
  if (rsub >= rows_per_block) return;
  const int nblk = seq.batch * layers;
  for (int64_t row = (int64_t)blockIdx.x * rows_per_block + rsub; row < pool_rows;
       row += (int64_t)gridDim.x * rows_per_block) {
    // block (b,l) whose rows [offsets*hkv, offsets_next*hkv) contain `row`
    int lo = 0, hi = nblk;   // invariant: offsets[lo]*hkv <= row < offsets[hi]*hkv
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (offsets[mid] * hkv <= row) lo = mid; else hi = mid;
    }
    const int b = lo / layers, l = lo - b * layers;
    const int len = lengths[lo];
    const int64_t local = row - offsets[lo] * hkv;
    if (len <= 0 || local >= (int64_t)len * hkv) continue;   // inconsistent lengths/offsets
    const int h = (int)(local / len), kk = (int)(local - (int64_t)h * len);
    const int n_b = seq.cu[b + 1] - seq.cu[b];
    const int p = idx[((size_t)l * hkv + h) * total + seq.cu[b] + kk];
    if (kk >= n_b || p < 0 || p >= n_b) continue;            // never read outside the cache
    const int tok = seq.cu[b] + p;
    const size_t src = ((size_t)h * total + tok) * pieces + piece;
    const size_t dst = (size_t)row * pieces + piece;
    k_out[dst] = static_cast<const uint4*>(k_tab.p[l])[src];
    if (has_v) v_out[dst] = static_cast<const uint4*>(v_tab.p[l])[src];
  }
}

}  // namespace

kvc_status launch_gather(const Problem& pb, const void* const* k, const void* const* v,
                         const int32_t* idx, const int32_t* lengths, const int64_t* offsets,
                         int64_t total_budget, void* k_out, void* v_out, hipStream_t stream) {
  PtrTable kt{}, vt{};
  for (int l = 0; l < pb.layers; ++l) { kt.p[l] = k[l]; vt.p[l] = v ? v[l] : nullptr; }
  const int pieces = pb.d * esize(pb.dtype) / 16;
  const int64_t pool_rows = total_budget * pb.hkv;
  const int rows_per_block = GA_THREADS / pieces;
  int64_t blocks = (pool_rows + rows_per_block - 1) / rows_per_block;
  const int64_t cap = 256 * 64;
  if (blocks > cap) blocks = cap;
  KVC_LAUNCH("gather_kernel", stream, gather_kernel<<<(unsigned)blocks, GA_THREADS, 0, stream>>>(
      kt, vt, v != nullptr, idx, lengths, offsets, pb.seq, pb.layers, pb.hkv, int(pb.total),
      pieces, pool_rows, static_cast<uint4*>(k_out), static_cast<uint4*>(v_out)));
  return KVC_OK;
}

}  // namespace kvc
