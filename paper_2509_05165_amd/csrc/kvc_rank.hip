// kvc_head_rank: per (layer, KV head, sequence) stable descending argsort of
// the scores (Section 3.3, eq. 17) and the rank-aligned scores S'.
//
// One workgroup sorts one segment with a least-significant-digit radix sort,
// 8 bits per pass, on the order-preserving integer image of the fp32 scores
// (inverted, so that ascending keys are descending scores).  LSD passes are
// stable, which yields the ascending-index order of equal scores for free.
// Within a tile every wave ranks its items with ballot-based digit matching
// and lane prefix counts; per-wave digit counters live in LDS.
#include "kvc_internal.h"

namespace kvc {

namespace {

constexpr int RK_THREADS = 1024;
constexpr int RK_WAVES = RK_THREADS / 64;
constexpr int RK_ITEMS = 4;
constexpr int RK_TILE = RK_THREADS * RK_ITEMS;
constexpr int RK_BINS = 256;

__device__ __forceinline__ uint32_t desc_key(float f) { return ~float_to_ordered(f); }
__device__ __forceinline__ float desc_key_to_float(uint32_t k) { return ordered_to_float(~k); }

// lanes (among `valid`) whose 8-bit digit equals mine
__device__ __forceinline__ uint64_t match_digit(uint32_t digit, uint64_t valid) {
  uint64_t mask = valid;
#pragma unroll
  for (int bit = 0; bit < 8; ++bit) {
    const bool set = (digit >> bit) & 1u;
    const uint64_t bal = __ballot(set);
    mask &= set ? bal : ~bal;
  }
  return mask;
}

__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi(uint32_t(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(uint32_t(mask), 0));
}

// grid: (layers * hkv, batch); block: RK_THREADS
__global__ __launch_bounds__(RK_THREADS) void head_rank_kernel(
    const float* __restrict__ S, SeqTable seq, int total, int32_t* __restrict__ idx_out,
    float* __restrict__ sorted_out, uint32_t* __restrict__ tmp_keys,
    int32_t* __restrict__ tmp_idx) {
  __shared__ uint32_t hist[4][RK_BINS];
  __shared__ uint32_t bucket[RK_BINS];            // next free slot of each digit
  __shared__ uint32_t wave_cnt[RK_WAVES][RK_BINS];
  __shared__ uint32_t wave_tot[4];

  const int b = blockIdx.y;
  const int n = seq.cu[b + 1] - seq.cu[b];
  if (n == 0) return;
  const size_t seg = (size_t)blockIdx.x * total + seq.cu[b];
  const float* src_f = S + seg;
  uint32_t* a_keys = tmp_keys + seg;
  int32_t* a_idx = tmp_idx + seg;
  uint32_t* b_keys = reinterpret_cast<uint32_t*>(sorted_out) + seg;
  int32_t* b_idx = idx_out + seg;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  // ---- histograms of all four digits in one sweep ----
  for (int i = tid; i < 4 * RK_BINS; i += RK_THREADS) (&hist[0][0])[i] = 0;
  __syncthreads();
  for (int i = tid; i < n; i += RK_THREADS) {
    const uint32_t key = desc_key(src_f[i]);
    atomicAdd(&hist[0][key & 255u], 1u);
    atomicAdd(&hist[1][(key >> 8) & 255u], 1u);
    atomicAdd(&hist[2][(key >> 16) & 255u], 1u);
    atomicAdd(&hist[3][key >> 24], 1u);
  }
  __syncthreads();

  for (int pass = 0; pass < 4; ++pass) {
    const int shift = pass * 8;
    // exclusive scan of hist[pass] -> bucket (first 256 threads = 4 waves)
    if (tid < RK_BINS) {
      const uint32_t c = hist[pass][tid];
      uint32_t incl = c;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_up(incl, off);
        if (lane >= off) incl += o;
      }
      if (lane == 63) wave_tot[wave] = incl;
      bucket[tid] = incl - c;   // exclusive within the wave
    }
    __syncthreads();
    if (tid < RK_BINS) {
      uint32_t add = 0;
      for (int w = 0; w < wave; ++w) add += wave_tot[w];
      bucket[tid] += add;
    }
    __syncthreads();

    const uint32_t* src_k = (pass == 2) ? b_keys : a_keys;   // pass 0 reads S itself
    const int32_t* src_i = (pass == 2) ? b_idx : a_idx;
    uint32_t* dst_k = (pass & 1) ? b_keys : a_keys;
    int32_t* dst_i = (pass & 1) ? b_idx : a_idx;

    for (int base = 0; base < n; base += RK_TILE) {
      uint32_t key[RK_ITEMS];
      int32_t val[RK_ITEMS];
      uint32_t rank[RK_ITEMS];
      const int wbase = base + wave * 64 * RK_ITEMS;
#pragma unroll
      for (int e = 0; e < RK_ITEMS; ++e) {
        const int pos = wbase + e * 64 + lane;
        key[e] = 0xffffffffu;
        val[e] = 0;
        if (pos < n) {
          if (pass == 0) { key[e] = desc_key(src_f[pos]); val[e] = pos; }
          else { key[e] = src_k[pos]; val[e] = src_i[pos]; }
        }
      }
      // zero this wave's counters
#pragma unroll
      for (int i = 0; i < RK_BINS / 64; ++i) wave_cnt[wave][i * 64 + lane] = 0;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int e = 0; e < RK_ITEMS; ++e) {
        const int pos = wbase + e * 64 + lane;
        const bool valid = pos < n;
        const uint64_t vmask = __ballot(valid);
        const uint32_t digit = (key[e] >> shift) & 255u;
        const uint64_t mask = match_digit(digit, vmask);
        const int below = lanes_below(mask);
        uint32_t prev = 0;
        if (valid) prev = wave_cnt[wave][digit];
        rank[e] = prev + below;
        __builtin_amdgcn_wave_barrier();
        if (valid && below == 0) wave_cnt[wave][digit] = prev + (uint32_t)__popcll(mask);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
      __syncthreads();
      // per digit: turn per-wave counts into absolute start slots
      if (tid < RK_BINS) {
        uint32_t run = bucket[tid];
#pragma unroll
        for (int w = 0; w < RK_WAVES; ++w) {
          const uint32_t c = wave_cnt[w][tid];
          wave_cnt[w][tid] = run;
          run += c;
        }
        bucket[tid] = run;
      }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < RK_ITEMS; ++e) {
        const int pos = wbase + e * 64 + lane;
        if (pos < n) {
          const uint32_t digit = (key[e] >> shift) & 255u;
          const uint32_t dst = wave_cnt[wave][digit] + rank[e];
          if (pass == 3) {
            sorted_out[seg + dst] = desc_key_to_float(key[e]);
            b_idx[dst] = val[e];
          } else {
            dst_k[dst] = key[e];
            dst_i[dst] = val[e];
          }
        }
      }
      __syncthreads();
    }
    // make this pass's global writes visible to the whole workgroup
    __threadfence_block();
    __syncthreads();
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
  dim3 grid((unsigned)((pb.total + 255) / 256), pb.layers);
  KVC_LAUNCH("composite_kernel", stream, composite_kernel<<<grid, 256, 0, stream>>>(S_sorted, pb.hkv, int(pb.total),
                                             pb.agg_head == KVC_AGG_MAX, I));
  return KVC_OK;
}

}  // namespace kvc
