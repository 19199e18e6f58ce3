// Internal declarations shared by the host API and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvc.h"

namespace kvc {

// Sequence table passed to kernels by value (no device copy of cu_seqlens).
struct SeqTable {
  int32_t batch;
  int32_t cu[KVC_MAX_BATCH + 1];
};

// Per-layer device pointers passed by value.
struct PtrTable {
  const void* p[KVC_MAX_LAYERS];
};

struct Problem {
  int32_t batch, layers, hq, hkv, group, d, window, dtype;
  int32_t agg_task, agg_group, agg_head, add_head_mean;
  int32_t value_norm, order, min_per_layer, unstructured, causal_tail, keep_first, keep_last;
  int32_t sel_rows;   // rows of the selection pool per sequence: layers, or layers*hkv
  float scale;        // softmax scale actually used
  int64_t total;      // T
  int64_t max_seqlen;
  SeqTable seq;
};

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
inline int esize(int dtype) { return dtype == KVC_BF16 ? 2 : 4; }

// Host-side error plumbing (thread local message).
void set_error(const char* fmt, ...);
kvc_status hip_fail(hipError_t e, const char* what);

// Optional event pair around a launch (see kvc_profile_enable).
void prof_begin(const char* name, hipStream_t stream);
void prof_end(hipStream_t stream);

// Launch a kernel (the variadic part is the launch expression), bracket it
// with timing events when profiling is on, and turn a launch failure into
// KVC_ERR_HIP.
#define KVC_LAUNCH(name, stream, ...)                       \
  do {                                                      \
    kvc::prof_begin(name, stream);                          \
    __VA_ARGS__;                                            \
    kvc::prof_end(stream);                                  \
    hipError_t e__ = hipGetLastError();                     \
    if (e__ != hipSuccess) return kvc::hip_fail(e__, name); \
  } while (0)

// ---------------------------------------------------------------------------
// Stage launchers (each enqueues on `stream`, validates nothing).
// ---------------------------------------------------------------------------
size_t score_workspace_bytes(const Problem& pb);
kvc_status launch_score(const Problem& pb, const void* const* q, const void* const* k,
                        const void* const* v, float* S, void* ws, hipStream_t stream);

size_t rank_workspace_bytes(const Problem& pb);
kvc_status launch_head_rank(const Problem& pb, const float* S, int32_t* idx, float* S_sorted,
                            void* ws, hipStream_t stream);

kvc_status launch_composite(const Problem& pb, const float* S_sorted, float* I,
                            hipStream_t stream);

size_t select_workspace_bytes(const Problem& pb);
kvc_status launch_global_select(const Problem& pb, const float* I, const int64_t* budget,
                                float* tau, int32_t* lengths, int64_t* offsets, void* ws,
                                hipStream_t stream);

// Device address of the current GPU's file-scope scratch array of the select
// stage (KVC_SELECT_STATIC_BYTES bytes, 256-byte aligned).
kvc_status select_static_scratch(void** ptr);

size_t gather_workspace_bytes(const Problem& pb);
kvc_status launch_gather(const Problem& pb, const void* const* k, const void* const* v,
                         const int32_t* idx, const int32_t* lengths, const int64_t* offsets,
                         int64_t total_budget, void* k_out, void* v_out, void* ws,
                         hipStream_t stream);

kvc_status launch_copy_probe(void* dst, const void* src, size_t bytes, hipStream_t stream);
kvc_status launch_mfma_probe(const void* operands, int iterations, int mode, float* sink,
                             int64_t* cycles, double* flops, hipStream_t stream);

// ---------------------------------------------------------------------------
// Device helpers
// ---------------------------------------------------------------------------
// Wait until at most N of this wave's vector-memory operations (loads, stores,
// atomics) are still outstanding.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Monotone map from float to unsigned: a < b  <=>  key(a) < key(b); -0 maps to
// the same key as +0.
__device__ __forceinline__ uint32_t float_to_ordered(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_float(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(u);
}

}  // namespace kvc
