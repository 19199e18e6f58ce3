// Measurement aid: what the matrix cores of this GPU sustain on a loop that
// never leaves the registers, in the shape the score kernels issue their
// MFMAs (v_mfma_f32_32x32x16_bf16, two accumulator blocks per key fragment,
// eight k-steps per 32x32 tile, two waves per SIMD).  It is the measured
// ceiling the score kernels' matrix-core fraction is quoted against beside
// the nominal one.  Not part of the pass.
#include "kvc_internal.h"

namespace kvc {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PR_THREADS = 256;
constexpr int PR_BLOCKS = 512;          // two workgroups on each of the 256 compute units
constexpr int PR_FRAGS = 24;            // 16-byte operand fragments per lane: 2 x 8 "query", 8 "key"
constexpr int PR_MFMA_PER_ITER = 16;

__device__ __forceinline__ bf16x8 frag(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// MODE 0: MFMAs only.  MODE 1: behind every MFMA the vector work the
// statistics pass of kvc_score does for the 2 x 64 logits of one accumulator
// register pair: scale-and-shift FMA, exp2, add.
template <int MODE>
__global__ __launch_bounds__(PR_THREADS, 2) void mfma_probe_kernel(const uint4* __restrict__ operands,
                                                                   int iterations,
                                                                   float* __restrict__ sink,
                                                                   int64_t* __restrict__ cycles) {
  uint4 qa[8], qb[8], kf[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    qa[i] = operands[(size_t)i * PR_THREADS + threadIdx.x];
    qb[i] = operands[(size_t)(8 + i) * PR_THREADS + threadIdx.x];
    kf[i] = operands[(size_t)(16 + i) * PR_THREADS + threadIdx.x];
  }
  f32x16 acc0, acc1;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
  // vector side of MODE 1: 32 "logits" per lane, refreshed from themselves
  float x[2] = {__uint_as_float(qa[0].x & 0x3fffffffu), __uint_as_float(qb[0].x & 0x3fffffffu)};
  float sum[2] = {0.f, 0.f};
  __syncthreads();
  const int64_t c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iterations; ++it) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(kf[ks]), frag(qa[ks]), acc0, 0, 0, 0);
      if (MODE == 1) {
        sum[0] += __builtin_amdgcn_exp2f(fmaf(x[0], 0.1275f, -20.f));
        sum[1] += __builtin_amdgcn_exp2f(fmaf(x[1], 0.1275f, -20.f));
        __builtin_amdgcn_sched_barrier(0);
      }
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(kf[ks]), frag(qb[ks]), acc1, 0, 0, 0);
      if (MODE == 1) {
        sum[0] += __builtin_amdgcn_exp2f(fmaf(x[1], 0.1275f, -21.f));
        sum[1] += __builtin_amdgcn_exp2f(fmaf(x[0], 0.1275f, -21.f));
        // keep the inputs changing so that nothing is hoisted out of the loop
        asm volatile("" : "+v"(x[0]), "+v"(x[1]));
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  const int64_t c1 = clock64(), w1 = wall_clock64();
  float s = sum[0] + sum[1];
#pragma unroll
  for (int r = 0; r < 16; ++r) s += acc0[r] + acc1[r];
  sink[(size_t)blockIdx.x * PR_THREADS + threadIdx.x] = s;
  if (cycles && blockIdx.x == 0 && threadIdx.x == 0) { cycles[0] = c1 - c0; cycles[1] = w1 - w0; }
}

}  // namespace

kvc_status launch_mfma_probe(const void* operands, int iterations, int mode, float* sink,
                             int64_t* cycles, double* flops, hipStream_t stream) {
  const uint4* ops = static_cast<const uint4*>(operands);
  if (mode == 0)
    KVC_LAUNCH("mfma_probe_kernel", stream, mfma_probe_kernel<0><<<PR_BLOCKS, PR_THREADS, 0, stream>>>(ops, iterations, sink, cycles));
  else
    KVC_LAUNCH("mfma_probe_kernel", stream, mfma_probe_kernel<1><<<PR_BLOCKS, PR_THREADS, 0, stream>>>(ops, iterations, sink, cycles));
  if (flops)
    *flops = double(PR_BLOCKS) * (PR_THREADS / 64) * double(iterations) * PR_MFMA_PER_ITER *
             (2.0 * 32 * 32 * 16);
  return KVC_OK;
}

static_assert(KVC_MFMA_PROBE_OPERAND_BYTES == PR_FRAGS * PR_THREADS * 16, "operand buffer size");
static_assert(KVC_MFMA_PROBE_SINK_FLOATS == PR_BLOCKS * PR_THREADS, "sink size");

}  // namespace kvc
