/*
 * kvc.h - C ABI of the KVCompose prefill-time KV-cache compression pass for
 * AMD MI355X (gfx950).
 *
 * The pass (paper Sections 3.2.2 and 3.3), per sequence:
 *   1. kvc_score          S[l,h,c]  attention of the M observation-window (task)
 *                         queries over all N cached keys, aggregated over task
 *                         tokens, over the query heads of a KV group, plus the
 *                         mean over KV heads            (Section 3.2.2)
 *   2. kvc_head_rank      idx[l,h,:] stable descending argsort of S[l,h,:] and
 *                         the rank-aligned scores S'     (Section 3.3, eq. 17)
 *   3. kvc_composite      I[l,k] = Agg_h S'[l,h,k]       (Section 3.3)
 *   4. kvc_global_select  top-B_total of the pool of all I[l,k]; N_l = how many
 *                         of them lie in layer l         (Section 3.3)
 *   5. kvc_gather         K'[l][h,k,:] = K[l][h, idx[l,h,k], :], k < N_l, same
 *                         for V                          (Section 3.3, last eqs.)
 *   kvc_compress runs 1-5 back to back on one stream.
 *
 * Variants, all off by default (kvc_params): value-norm weighting of the
 * attention matrix (appendix on value norms), position-ordered output rows, a
 * per-layer floor on N_l, and the unstructured selection of the appendix on
 * unstructured eviction (no step 3; every head keeps its own prefix).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * Notation: Bt sequences, Lyr layers, Hq query heads, Hkv KV heads, G = Hq/Hkv,
 * d head dimension, M window (task) tokens, N_b tokens of sequence b,
 * T = sum_b N_b.  All indices are 0-based.
 *
 * Memory: every pointer marked "device" is memory of the current HIP device,
 * owned by the caller; pointers marked "host" are ordinary host memory read
 * before the call returns.  The library allocates no device memory, keeps no
 * pointer after return and never synchronises the stream: all work is
 * enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream).
 * Results are valid once the stream has been synchronised by the caller.
 *
 * Layouts (row-major, innermost last):
 *   q[l]   device, [Bt, Hq, M, d]       task queries of layer l (already
 *                                       position-encoded; used as given)
 *   k[l]   device, [Hkv, T, d]          keys of layer l; sequence b owns tokens
 *   v[l]   device, [Hkv, T, d]          [cu_seqlens[b], cu_seqlens[b+1])
 *   q, k, v themselves are host arrays of Lyr device pointers.
 *   cu_seqlens  host, int64 [Bt+1], cu_seqlens[0] = 0, non-decreasing.
 *   S, S_sorted device, float [Lyr, Hkv, T]
 *   idx         device, int32 [Lyr, Hkv, T]; values are token positions inside
 *               their own sequence (0 .. N_b-1)
 *   I           device, float [Lyr, T]
 *   lengths     device, int32 [Bt*Lyr], lengths[b*Lyr+l] = N_{b,l}
 *   offsets     device, int64 [Bt*Lyr+1], exclusive prefix sum of lengths in
 *               that order; offsets[Bt*Lyr] = sum_b budget[b]
 *   k_out,v_out device pools of (sum_b budget[b]) * Hkv * d elements of the
 *               input dtype.  Block (b,l) is the dense tensor [Hkv, N_{b,l}, d]
 *               (the uniform per-layer layout of the problem statement,
 *               constraint C2) starting at element offsets[b*Lyr+l]*Hkv*d.
 *               Rows are in descending-importance (rank) order, or in
 *               ascending token position with KVC_ORDER_POSITION.
 *   unstructured = 1: lengths is int32 [Bt*Lyr*Hkv] (N_{b,l,h}), offsets int64
 *               [Bt*Lyr*Hkv+1]; block (b,l,h) is the dense tensor [N_{b,l,h}, d]
 *               starting at element offsets[(b*Lyr+l)*Hkv+h]*d; the pools hold
 *               (sum_b budget[b]) * d elements and budget[b] counts
 *               (head, token) entries, 0 <= budget[b] <= Lyr*Hkv*N_b.
 *
 * Readings of the paper fixed by this library: no attention mask (each task
 * query sees all N_b cached keys of its sequence, softmax over exactly those);
 * query head q belongs to KV head q / G; equal scores rank by ascending token
 * index; ties at the global threshold are taken by ascending (layer, rank);
 * a layer may keep 0 tokens; nothing is force-kept; sequences of a batch are
 * independent, each with its own budget.  Non-finite inputs are undefined.
 *
 * Errors: every function returns a kvc_status.  All argument checks run on the
 * host before the first HIP call; on any error nothing has been enqueued,
 * except KVC_ERR_HIP which reports a failed launch (kvc_last_error() has the
 * HIP message).  No function aborts or throws.
 *
 * Limits: Bt <= KVC_MAX_BATCH, Lyr <= KVC_MAX_LAYERS, T < 2^30, every N_b < 2^29,
 * d * sizeof(element) a multiple of 16 bytes and d <= 256.  The sequence table and
 * the per-layer pointer tables travel to the kernels as by-value arguments (no device
 * copy, no allocation, nothing to keep alive), and a kernel's argument block holds
 * 4 KB: hence 256 sequences and 128 layers per call (the largest argument block is
 * 3.4 KB).  Sequences of a batch are independent (own budget, own threshold), so a
 * larger batch is compressed as several calls with identical results; at the
 * 4096-token contexts of the paper's evaluation 256 sequences are a million tokens.
 */
#ifndef KVC_H
#define KVC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVC_MAX_BATCH 256
#define KVC_MAX_LAYERS 128

typedef enum {
  KVC_OK = 0,
  KVC_ERR_INVALID_ARG = 1, /* null pointer, inconsistent sizes, out-of-range value */
  KVC_ERR_UNSUPPORTED = 2, /* well-formed but outside the supported shapes */
  KVC_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or too small */
  KVC_ERR_HIP = 4          /* a HIP runtime call failed */
} kvc_status;

typedef enum { KVC_F32 = 0, KVC_BF16 = 1 } kvc_dtype;
typedef enum { KVC_AGG_MAX = 0, KVC_AGG_MEAN = 1 } kvc_agg;
typedef enum {
  KVC_ORDER_RANK = 0,    /* rows k_out[h,k,:] = K[h, idx[h,k], :]: the paper's literal order */
  KVC_ORDER_POSITION = 1 /* the same retained rows of each head in ascending token position:
                            a full budget then reproduces K and V bit for bit */
} kvc_order;

/* Problem description.  Defaults of the paper's experiments (Section 4.2):
 * agg_task = MAX, agg_group = MEAN, agg_head = MEAN, add_head_mean = 1. */
typedef struct kvc_params {
  int32_t batch;         /* Bt  */
  int32_t layers;        /* Lyr */
  int32_t hq;            /* Hq  */
  int32_t hkv;           /* Hkv, divides Hq */
  int32_t head_dim;      /* d   */
  int32_t window;        /* M   */
  int32_t dtype;         /* kvc_dtype of q, k, v, k_out, v_out */
  int32_t agg_task;      /* kvc_agg over the M task tokens        (eq. 14) */
  int32_t agg_group;     /* kvc_agg over the G heads of a KV group (eq. 15) */
  int32_t agg_head;      /* kvc_agg over KV heads for I            (Section 3.3) */
  int32_t add_head_mean; /* 1: add the mean over KV heads to S (Section 3.2.2) */
  float softmax_scale;   /* 0 => 1/sqrt(d) (Preliminary eq. 3) */
  /* ---- variants; 0 everywhere is the pass of Sections 3.2.2-3.3 ---- */
  int32_t value_norm;    /* 1: A[q,m,c] is multiplied by ||V[l,h,c,:]||_2, h = q/G, before
                            any aggregation (appendix on value norms, v-norm) */
  int32_t order;         /* kvc_order of the output rows */
  int32_t min_per_layer; /* m >= 0: ranks 0..min(m,N_b)-1 of every layer (of every head
                            when unstructured) are kept first; only the other pool
                            entries compete for the rest of the budget.  The paper
                            defines no floor; this is the library's reading. */
  int32_t unstructured;  /* 1: no head aggregation; the pool holds all Lyr*Hkv*N_b
                            rank-aligned scores and every head keeps its own prefix
                            (appendix on unstructured eviction) */
  int32_t causal_tail;   /* 1: the M task tokens are the last M tokens of the context
                            (task-agnostic setting, Section 3.2.1): task token m sits at
                            position N_b-M+m and attends to cached keys at positions
                            <= N_b-M+m only (softmax over those; the rest of its row of
                            A is 0).  Needs N_b >= M.  0: no mask, the library's default
                            reading. */
  int32_t keep_first;    /* forced retention (not part of the paper's method; the sink /
                            recent-window conventions of its related work): the first
                            keep_first and the last keep_last tokens of every sequence
                            get S = +inf in every head of every layer, rank first
                            (ascending position) and are retained whenever
                            budget >= rows * (number of forced tokens) */
  int32_t keep_last;     /* see keep_first */
} kvc_params;

typedef struct kvc_inputs {
  const void* const* q;      /* host array [Lyr] of device pointers */
  const void* const* k;      /* host array [Lyr] of device pointers */
  const void* const* v;      /* host array [Lyr] of device pointers */
  const int64_t* cu_seqlens; /* host, [Bt+1] */
  const int64_t* budget;     /* host, [Bt]: B_total of each sequence, in
                                [R*min(min_per_layer, N_b), R*N_b] with R = Lyr
                                (Lyr*Hkv when unstructured) */
} kvc_inputs;

typedef struct kvc_outputs {
  void* k_out;      /* device pool, see layouts */
  void* v_out;      /* device pool */
  int32_t* lengths; /* device [Bt*Lyr] */
  int64_t* offsets; /* device [Bt*Lyr+1] */
  /* Optional taps on the intermediates; each may be NULL (then it lives in the
   * workspace).  Shapes as in "Layouts". */
  float* scores;   /* S */
  int32_t* idx;    /* idx */
  float* s_sorted; /* S' */
  float* composite;/* I */
  float* tau;      /* device [Bt]: smallest retained composite score
                      (+inf when budget[b] == 0) */
} kvc_outputs;

int kvc_version(void);
const char* kvc_status_string(int status);
/* Message of the last KVC_ERR_* raised on the calling thread ("" if none). */
const char* kvc_last_error(void);

/* floor(keep_percent/100 * layers * n) in integer arithmetic: the paper's
 * B_total = floor((1 - r_target) * L * N) with 1 - r_target = keep_percent/100
 * (Section 3.3).  Returns -1 on invalid arguments. */
int64_t kvc_budget(int32_t keep_percent, int32_t layers, int64_t n);

/* Bytes of device workspace that suffice for kvc_compress and for every stage
 * entry point on this problem.  max_seqlen = max_b N_b.  The workspace must be
 * 256-byte aligned; its contents on entry are irrelevant and on exit
 * unspecified. */
kvc_status kvc_workspace_size(const kvc_params* params, int64_t total_tokens,
                              int64_t max_seqlen, size_t* bytes);

/* Stage 1, Section 3.2.2.  For every sequence b, layer l, KV head h, token c:
 *   A[q,m,c]  = softmax_c( Q[l,b,q,m,:] . K[l,h,c,:] * scale )   (all N_b keys)
 *   S_task    = Agg_task over m;  S_group = Agg_group over q in [hG, hG+G);
 *   S[l,h,c]  = S_group[h,c] + (add_head_mean ? mean_i S_group[i,c] : 0).
 * bf16 inputs are multiplied on the matrix cores with fp32 accumulation; all
 * later arithmetic is fp32.  Writes S (device, float [Lyr,Hkv,T]).
 * v (host array [Lyr] of device pointers, layout of k) is read only when
 * params->value_norm is set, and must then be given; else it may be NULL.  The
 * weight ||V[l,h,c,:]|| does not depend on q or m, so it is applied to
 * S_group[h,c] (it commutes with max and mean over m and over g). */
kvc_status kvc_score(const kvc_params* params, const void* const* q,
                     const void* const* k, const void* const* v,
                     const int64_t* cu_seqlens, float* S, void* workspace,
                     size_t workspace_bytes, void* stream);

/* Stage 2, Section 3.3 eq. 17 and the rank-aligned scores after it.  For each
 * (l,h) and sequence: idx = positions sorted by S descending, equal scores in
 * ascending position; S_sorted[k] = S[idx[k]].  -0 and +0 compare equal. */
kvc_status kvc_head_rank(const kvc_params* params, const float* S,
                         const int64_t* cu_seqlens, int32_t* idx, float* S_sorted,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Stage 3, Section 3.3 composite importance: I[l,k] = Agg_head over h of
 * S_sorted[l,h,k]; the mean is summed in ascending h in fp32. */
kvc_status kvc_composite(const kvc_params* params, const float* S_sorted,
                         const int64_t* cu_seqlens, float* I, void* stream);

/* Stage 4, Section 3.3 pool / budget / N_l.  Per sequence: tau = budget-th
 * largest of the Lyr*N_b values I[l, seq tokens]; lengths = count of I > tau
 * plus, in ascending layer order, as many I == tau as still fit the budget.
 * offsets = exclusive prefix sum of lengths over (b,l).  tau may be NULL.
 * With min_per_layer = m the first min(m,N_b) ranks of each layer are counted
 * in unconditionally and tau is the threshold of the competition for the rest
 * (+inf if nothing is left to compete for).  With unstructured = 1, I is
 * S_sorted (float [Lyr*Hkv, T]) and a "layer" above reads "(layer, head)". */
kvc_status kvc_global_select(const kvc_params* params, const float* I,
                             const int64_t* cu_seqlens, const int64_t* budget,
                             float* tau, int32_t* lengths, int64_t* offsets,
                             void* workspace, size_t workspace_bytes, void* stream);

/* kvc_global_select for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and errors as kvc_global_select
 * minus the workspace: the histograms, counters and tickets live in a buffer of
 * KVC_SELECT_STATIC_BYTES bytes that is part of the library's device image (one
 * copy per GPU, held until the process ends).  The call allocates nothing and
 * clears what it needs with a kernel on `stream`.  Problems whose select
 * workspace would exceed that size (very many sequences times rows times
 * tokens) return KVC_ERR_UNSUPPORTED with nothing enqueued.  Every call on a
 * GPU shares that GPU's buffer: calls that may overlap on one GPU (different
 * streams, different threads) race and must be serialised by the caller. */
#define KVC_SELECT_STATIC_BYTES (4u << 20)
kvc_status kvc_global_select_static(const kvc_params* params, const float* I,
                                    const int64_t* cu_seqlens, const int64_t* budget,
                                    float* tau, int32_t* lengths, int64_t* offsets,
                                    void* stream);

/* Stage 5, Section 3.3 final selection.  Copies rows idx[l,h,0..N_{b,l}) of
 * K and V (bit copies) into the pools; lengths/offsets are read on the device.
 * total_budget = sum_b budget[b] (host value, sizes the launch).  v and v_out
 * may both be NULL to gather keys only.  KVC_ORDER_POSITION first turns every
 * retained prefix idx[l,h,0..N) into its ascending permutation (a bit mask per
 * head and a prefix sum over it) and needs workspace (kvc_workspace_size
 * covers it); with KVC_ORDER_RANK workspace may be NULL. */
kvc_status kvc_gather(const kvc_params* params, const void* const* k,
                      const void* const* v, const int32_t* idx,
                      const int32_t* lengths, const int64_t* offsets,
                      const int64_t* cu_seqlens, int64_t total_budget, void* k_out,
                      void* v_out, void* workspace, size_t workspace_bytes,
                      void* stream);

/* The whole pass: stages 1-5 on one stream, no host synchronisation.  With
 * unstructured = 1 stage 3 is skipped and out->composite is not written. */
kvc_status kvc_compress(const kvc_params* params, const kvc_inputs* in,
                        const kvc_outputs* out, void* workspace,
                        size_t workspace_bytes, void* stream);

/* ---- optional per-kernel timing (measurement aid, not part of the pass) ----
 * While enabled, every kernel the library launches on the calling thread is
 * bracketed by a pair of HIP events recorded on the launch stream.
 * kvc_profile_collect synchronises those events, sums the elapsed time per
 * kernel name into `out` (at most `capacity` entries, in first-launch order),
 * forgets them and returns the number of distinct names (or -1 on a HIP
 * error).  Enabling allocates host-side event objects only; it slightly
 * serialises back-to-back launches, so throughput is timed with it off. */
typedef struct kvc_profile_entry {
  char name[48];
  int32_t launches;
  float total_ms;
} kvc_profile_entry;
void kvc_profile_enable(int on);
int kvc_profile_collect(kvc_profile_entry* out, int capacity);

/* Measurement aid: one plain device-to-device streaming copy of `bytes` bytes
 * (a positive multiple of 16; dst and src are device buffers that must not
 * overlap).  Its known traffic (bytes read + bytes written) is what hardware
 * byte counters are scaled against. */
kvc_status kvc_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

/* Measurement aid: a bf16 MFMA loop that never leaves the registers, issued in
 * the shape of the score kernels (v_mfma_f32_32x32x16_bf16, 512 workgroups of
 * four waves = two waves per SIMD on 256 compute units, 16 MFMAs per wave and
 * iteration).  What it sustains is the measured matrix-core ceiling of the GPU
 * it runs on, under the clocks the power management grants such a load.
 *   operands   device, KVC_MFMA_PROBE_OPERAND_BYTES bytes of bf16 values, read
 *              once; fill them with values distributed like the workload
 *              (matrix-core power, hence clock, depends on operand bits)
 *   iterations > 0; mode 0: MFMAs only; mode 1: each MFMA is followed by the
 *              vector work the statistics pass of kvc_score does per MFMA (two
 *              scale-and-shift FMAs, two exp2, two adds)
 *   sink       device, KVC_MFMA_PROBE_SINK_FLOATS floats, overwritten
 *   cycles     device int64[2] or NULL: shader-clock cycles and ticks of the
 *              constant 100 MHz counter that elapsed over the loop of one wave
 *              (their ratio is the shader clock the loop ran at)
 *   flops      host, or NULL: floating-point operations issued by the launch
 * Asynchronous on `stream`; time it with events. */
#define KVC_MFMA_PROBE_OPERAND_BYTES (24 * 256 * 16)
#define KVC_MFMA_PROBE_SINK_FLOATS (512 * 256)
kvc_status kvc_mfma_probe(const void* operands, int32_t iterations, int32_t mode, float* sink,
                          int64_t* cycles, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVC_H */
