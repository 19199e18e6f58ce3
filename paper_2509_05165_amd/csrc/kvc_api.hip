// Host side of the C ABI: argument validation, workspace carving and the
// stream-ordered sequence of stage launches.  All checks run before the first
// HIP call so every error path can be exercised without a GPU.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "kvc_internal.h"

namespace kvc {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

kvc_status hip_fail(hipError_t e, const char* what) {
  set_error("%s: %s", what, hipGetErrorString(e));
  return KVC_ERR_HIP;
}

// ---- per-kernel timing records (thread local, host objects only) ----
struct ProfRec { const char* name; hipEvent_t start, stop; };
static thread_local bool g_prof_on = false;
static thread_local std::vector<ProfRec> g_prof;

void prof_begin(const char* name, hipStream_t stream) {
  if (!g_prof_on) return;
  ProfRec r{name, nullptr, nullptr};
  if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) return;
  (void)hipEventRecord(r.start, stream);
  g_prof.push_back(r);
}

void prof_end(hipStream_t stream) {
  if (!g_prof_on || g_prof.empty()) return;
  (void)hipEventRecord(g_prof.back().stop, stream);
}

static kvc_status check_params(const kvc_params* p) {
  if (!p) { set_error("params is NULL"); return KVC_ERR_INVALID_ARG; }
  if (p->batch < 1 || p->layers < 1 || p->hq < 1 || p->hkv < 1 || p->head_dim < 1 ||
      p->window < 1) {
    set_error("batch, layers, hq, hkv, head_dim and window must be positive");
    return KVC_ERR_INVALID_ARG;
  }
  if (p->hq % p->hkv != 0) { set_error("hkv must divide hq"); return KVC_ERR_INVALID_ARG; }
  if (p->dtype != KVC_F32 && p->dtype != KVC_BF16) {
    set_error("unknown dtype %d", p->dtype); return KVC_ERR_INVALID_ARG;
  }
  const int32_t aggs[3] = {p->agg_task, p->agg_group, p->agg_head};
  for (int32_t a : aggs)
    if (a != KVC_AGG_MAX && a != KVC_AGG_MEAN) {
      set_error("unknown aggregation operator %d", a); return KVC_ERR_INVALID_ARG;
    }
  if (p->add_head_mean != 0 && p->add_head_mean != 1) {
    set_error("add_head_mean must be 0 or 1"); return KVC_ERR_INVALID_ARG;
  }
  if (!(p->softmax_scale >= 0.0f) || !std::isfinite(p->softmax_scale)) {
    set_error("softmax_scale must be finite and >= 0"); return KVC_ERR_INVALID_ARG;
  }
  if ((p->value_norm | p->unstructured | p->causal_tail) & ~1) {
    set_error("value_norm, unstructured and causal_tail must be 0 or 1"); return KVC_ERR_INVALID_ARG;
  }
  if (p->order != KVC_ORDER_RANK && p->order != KVC_ORDER_POSITION) {
    set_error("unknown output order %d", p->order); return KVC_ERR_INVALID_ARG;
  }
  if (p->min_per_layer < 0) { set_error("min_per_layer must be >= 0"); return KVC_ERR_INVALID_ARG; }
  if (p->keep_first < 0 || p->keep_last < 0) {
    set_error("keep_first and keep_last must be >= 0"); return KVC_ERR_INVALID_ARG;
  }
  if (p->batch > KVC_MAX_BATCH) {
    set_error("batch %d exceeds KVC_MAX_BATCH", p->batch); return KVC_ERR_UNSUPPORTED;
  }
  if (p->layers > KVC_MAX_LAYERS) {
    set_error("layers %d exceeds KVC_MAX_LAYERS", p->layers); return KVC_ERR_UNSUPPORTED;
  }
  if (p->head_dim > 256 || (p->head_dim * esize(p->dtype)) % 16 != 0) {
    set_error("head_dim %d unsupported (row bytes must be a multiple of 16, d <= 256)",
              p->head_dim);
    return KVC_ERR_UNSUPPORTED;
  }
  if (p->window > 4096 || p->hq > 1024) {
    set_error("window > 4096 or hq > 1024 unsupported"); return KVC_ERR_UNSUPPORTED;
  }
  if (int64_t(p->layers) * p->hkv > 65535) {
    set_error("layers * hkv > 65535 unsupported"); return KVC_ERR_UNSUPPORTED;
  }
  return KVC_OK;
}

static kvc_status make_problem(const kvc_params* p, const int64_t* cu, Problem* pb) {
  kvc_status st = check_params(p);
  if (st != KVC_OK) return st;
  if (!cu) { set_error("cu_seqlens is NULL"); return KVC_ERR_INVALID_ARG; }
  if (cu[0] != 0) { set_error("cu_seqlens[0] must be 0"); return KVC_ERR_INVALID_ARG; }
  int64_t mx = 0;
  for (int b = 0; b < p->batch; ++b) {
    int64_t n = cu[b + 1] - cu[b];
    if (n < 0) { set_error("cu_seqlens must be non-decreasing"); return KVC_ERR_INVALID_ARG; }
    if (p->causal_tail && n > 0 && n < p->window) {
      set_error("causal_tail needs N_b >= window (sequence %d has %lld tokens)", b, (long long)n);
      return KVC_ERR_INVALID_ARG;
    }
    if (n > mx) mx = n;
  }
  if (cu[p->batch] >= (int64_t(1) << 30)) {
    set_error("total tokens must be below 2^30"); return KVC_ERR_UNSUPPORTED;
  }
  if (mx >= (int64_t(1) << 29)) {   // 8-byte items of one sequence are addressed with 32-bit byte offsets
    set_error("every sequence must be shorter than 2^29 tokens"); return KVC_ERR_UNSUPPORTED;
  }
  pb->batch = p->batch; pb->layers = p->layers; pb->hq = p->hq; pb->hkv = p->hkv;
  pb->group = p->hq / p->hkv; pb->d = p->head_dim; pb->window = p->window;
  pb->dtype = p->dtype; pb->agg_task = p->agg_task; pb->agg_group = p->agg_group;
  pb->agg_head = p->agg_head; pb->add_head_mean = p->add_head_mean;
  pb->value_norm = p->value_norm; pb->order = p->order; pb->min_per_layer = p->min_per_layer;
  pb->unstructured = p->unstructured; pb->causal_tail = p->causal_tail;
  pb->keep_first = p->keep_first; pb->keep_last = p->keep_last;
  pb->sel_rows = p->unstructured ? p->layers * p->hkv : p->layers;
  pb->scale = p->softmax_scale > 0.0f ? p->softmax_scale
                                      : 1.0f / std::sqrt(float(p->head_dim));
  pb->total = cu[p->batch];
  pb->max_seqlen = mx;
  pb->seq.batch = p->batch;
  for (int b = 0; b <= p->batch; ++b) pb->seq.cu[b] = int32_t(cu[b]);
  for (int b = p->batch + 1; b <= KVC_MAX_BATCH; ++b) pb->seq.cu[b] = int32_t(cu[p->batch]);
  return KVC_OK;
}

static kvc_status check_ptr_table(const void* const* t, int n, const char* name) {
  if (!t) { set_error("%s is NULL", name); return KVC_ERR_INVALID_ARG; }
  for (int i = 0; i < n; ++i)
    if (!t[i]) { set_error("%s[%d] is NULL", name, i); return KVC_ERR_INVALID_ARG; }
  return KVC_OK;
}

static kvc_status check_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return KVC_OK;
  if (!ws) { set_error("workspace is NULL (%zu bytes needed)", need); return KVC_ERR_WORKSPACE; }
  if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) {
    set_error("workspace must be 256-byte aligned"); return KVC_ERR_WORKSPACE;
  }
  if (have < need) {
    set_error("workspace too small: %zu < %zu bytes", have, need); return KVC_ERR_WORKSPACE;
  }
  return KVC_OK;
}

static kvc_status check_budget(const Problem& pb, const int64_t* cu, const int64_t* budget,
                               int64_t* total) {
  if (!budget) { set_error("budget is NULL"); return KVC_ERR_INVALID_ARG; }
  int64_t sum = 0;
  for (int b = 0; b < pb.batch; ++b) {
    int64_t n = cu[b + 1] - cu[b];
    const int64_t floor_b = pb.min_per_layer < n ? pb.min_per_layer : n;
    if (budget[b] < int64_t(pb.sel_rows) * floor_b || budget[b] > int64_t(pb.sel_rows) * n) {
      set_error("budget[%d]=%lld outside [rows*min(min_per_layer,N_b)=%lld, rows*N_b=%lld]", b,
                (long long)budget[b], (long long)(int64_t(pb.sel_rows) * floor_b),
                (long long)(int64_t(pb.sel_rows) * n));
      return KVC_ERR_INVALID_ARG;
    }
    sum += budget[b];
  }
  if (total) *total = sum;
  return KVC_OK;
}

// Workspace of kvc_compress: [S][idx][S_sorted][I][tau] (each only when the
// caller gave no tap for it) followed by one region shared by the stages.
struct CompressLayout {
  size_t off_S, off_idx, off_sorted, off_I, off_tau, off_stage, total;
};

static CompressLayout compress_layout(const Problem& pb) {
  CompressLayout L{};
  size_t lht = size_t(pb.layers) * pb.hkv * size_t(pb.total);
  size_t cur = 0;
  L.off_S = cur;      cur += align_up(lht * 4);
  L.off_idx = cur;    cur += align_up(lht * 4);
  L.off_sorted = cur; cur += align_up(lht * 4);
  L.off_I = cur;      cur += align_up(size_t(pb.layers) * size_t(pb.total) * 4);
  L.off_tau = cur;    cur += align_up(size_t(pb.batch) * 4);
  L.off_stage = cur;
  size_t stage = score_workspace_bytes(pb);
  size_t r = rank_workspace_bytes(pb);
  if (r > stage) stage = r;
  size_t s = select_workspace_bytes(pb);
  if (s > stage) stage = s;
  size_t g = gather_workspace_bytes(pb);
  if (g > stage) stage = g;
  cur += align_up(stage);
  L.total = cur;
  return L;
}

}  // namespace kvc

using namespace kvc;

extern "C" {

int kvc_version(void) { return 100; }

const char* kvc_status_string(int status) {
  switch (status) {
    case KVC_OK: return "KVC_OK";
    case KVC_ERR_INVALID_ARG: return "KVC_ERR_INVALID_ARG";
    case KVC_ERR_UNSUPPORTED: return "KVC_ERR_UNSUPPORTED";
    case KVC_ERR_WORKSPACE: return "KVC_ERR_WORKSPACE";
    case KVC_ERR_HIP: return "KVC_ERR_HIP";
    default: return "KVC_ERR_UNKNOWN";
  }
}

const char* kvc_last_error(void) { return g_err; }

void kvc_profile_enable(int on) { g_prof_on = on != 0; }

int kvc_profile_collect(kvc_profile_entry* out, int capacity) {
  int count = 0;
  bool failed = false;
  for (ProfRec& r : g_prof) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess ||
        hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
      failed = true;
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
    int slot = -1;
    for (int i = 0; i < count && i < capacity; ++i)
      if (std::strncmp(out[i].name, r.name, sizeof(out[i].name) - 1) == 0) { slot = i; break; }
    if (slot < 0) {
      if (count < capacity && out) {
        std::memset(&out[count], 0, sizeof(out[count]));
        std::strncpy(out[count].name, r.name, sizeof(out[count].name) - 1);
        slot = count;
      }
      ++count;
    }
    if (slot >= 0 && slot < capacity && out) { out[slot].launches += 1; out[slot].total_ms += ms; }
  }
  g_prof.clear();
  return failed ? -1 : count;
}

int64_t kvc_budget(int32_t keep_percent, int32_t layers, int64_t n) {
  if (keep_percent < 0 || keep_percent > 100 || layers < 0 || n < 0) return -1;
  return (int64_t(keep_percent) * layers * n) / 100;
}

kvc_status kvc_workspace_size(const kvc_params* params, int64_t total_tokens,
                              int64_t max_seqlen, size_t* bytes) {
  kvc_status st = check_params(params);
  if (st != KVC_OK) return st;
  if (!bytes) { set_error("bytes is NULL"); return KVC_ERR_INVALID_ARG; }
  if (total_tokens < 0 || max_seqlen < 0 || max_seqlen > total_tokens ||
      total_tokens >= (int64_t(1) << 30)) {
    set_error("need 0 <= max_seqlen <= total_tokens < 2^30"); return KVC_ERR_INVALID_ARG;
  }
  // A synthetic sequence table with the same totals is enough for sizing.
  Problem pb{};
  int64_t cu[KVC_MAX_BATCH + 1];
  cu[0] = 0;
  for (int b = 1; b <= params->batch; ++b) cu[b] = (b == params->batch) ? total_tokens : 0;
  if (params->batch > 1) cu[1] = max_seqlen < total_tokens ? max_seqlen : total_tokens;
  for (int b = 2; b < params->batch; ++b) cu[b] = cu[1];
  st = make_problem(params, cu, &pb);
  if (st != KVC_OK) return st;
  pb.max_seqlen = max_seqlen;
  *bytes = compress_layout(pb).total;
  return KVC_OK;
}

kvc_status kvc_score(const kvc_params* params, const void* const* q, const void* const* k,
                     const void* const* v, const int64_t* cu_seqlens, float* S, void* workspace,
                     size_t workspace_bytes, void* stream) {
  Problem pb{};
  kvc_status st = make_problem(params, cu_seqlens, &pb);
  if (st != KVC_OK) return st;
  if ((st = check_ptr_table(q, pb.layers, "q")) != KVC_OK) return st;
  if ((st = check_ptr_table(k, pb.layers, "k")) != KVC_OK) return st;
  if (pb.value_norm && (st = check_ptr_table(v, pb.layers, "v")) != KVC_OK) return st;
  if (!S) { set_error("S is NULL"); return KVC_ERR_INVALID_ARG; }
  if ((st = check_ws(workspace, workspace_bytes, score_workspace_bytes(pb))) != KVC_OK) return st;
  if (pb.total == 0) return KVC_OK;
  return launch_score(pb, q, k, pb.value_norm ? v : nullptr, S, workspace,
                      static_cast<hipStream_t>(stream));
}

kvc_status kvc_head_rank(const kvc_params* params, const float* S, const int64_t* cu_seqlens,
                         int32_t* idx, float* S_sorted, void* workspace,
                         size_t workspace_bytes, void* stream) {
  Problem pb{};
  kvc_status st = make_problem(params, cu_seqlens, &pb);
  if (st != KVC_OK) return st;
  if (!S || !idx || !S_sorted) { set_error("S, idx or S_sorted is NULL"); return KVC_ERR_INVALID_ARG; }
  if ((st = check_ws(workspace, workspace_bytes, rank_workspace_bytes(pb))) != KVC_OK) return st;
  if (pb.total == 0) return KVC_OK;
  return launch_head_rank(pb, S, idx, S_sorted, workspace, static_cast<hipStream_t>(stream));
}

kvc_status kvc_composite(const kvc_params* params, const float* S_sorted,
                         const int64_t* cu_seqlens, float* I, void* stream) {
  Problem pb{};
  kvc_status st = make_problem(params, cu_seqlens, &pb);
  if (st != KVC_OK) return st;
  if (!S_sorted || !I) { set_error("S_sorted or I is NULL"); return KVC_ERR_INVALID_ARG; }
  if (pb.total == 0) return KVC_OK;
  return launch_composite(pb, S_sorted, I, static_cast<hipStream_t>(stream));
}

kvc_status kvc_global_select(const kvc_params* params, const float* I,
                             const int64_t* cu_seqlens, const int64_t* budget, float* tau,
                             int32_t* lengths, int64_t* offsets, void* workspace,
                             size_t workspace_bytes, void* stream) {
  Problem pb{};
  kvc_status st = make_problem(params, cu_seqlens, &pb);
  if (st != KVC_OK) return st;
  if ((st = check_budget(pb, cu_seqlens, budget, nullptr)) != KVC_OK) return st;
  if (!lengths || !offsets) { set_error("lengths or offsets is NULL"); return KVC_ERR_INVALID_ARG; }
  if (!I && pb.total > 0) { set_error("I is NULL"); return KVC_ERR_INVALID_ARG; }
  if ((st = check_ws(workspace, workspace_bytes, select_workspace_bytes(pb))) != KVC_OK) return st;
  return launch_global_select(pb, I, budget, tau, lengths, offsets, workspace,
                              static_cast<hipStream_t>(stream));
}

kvc_status kvc_global_select_static(const kvc_params* params, const float* I,
                                    const int64_t* cu_seqlens, const int64_t* budget, float* tau,
                                    int32_t* lengths, int64_t* offsets, void* stream) {
  Problem pb{};
  kvc_status st = make_problem(params, cu_seqlens, &pb);
  if (st != KVC_OK) return st;
  if ((st = check_budget(pb, cu_seqlens, budget, nullptr)) != KVC_OK) return st;
  if (!lengths || !offsets) { set_error("lengths or offsets is NULL"); return KVC_ERR_INVALID_ARG; }
  if (!I && pb.total > 0) { set_error("I is NULL"); return KVC_ERR_INVALID_ARG; }
  const size_t need = select_workspace_bytes(pb);
  if (need > size_t(KVC_SELECT_STATIC_BYTES)) {
    set_error("problem needs %zu bytes of select scratch, the static buffer holds %zu", need,
              size_t(KVC_SELECT_STATIC_BYTES));
    return KVC_ERR_UNSUPPORTED;
  }
  void* scratch_ptr = nullptr;
  if ((st = select_static_scratch(&scratch_ptr)) != KVC_OK) return st;
  return launch_global_select(pb, I, budget, tau, lengths, offsets, scratch_ptr,
                              static_cast<hipStream_t>(stream));
}

kvc_status kvc_gather(const kvc_params* params, const void* const* k, const void* const* v,
                      const int32_t* idx, const int32_t* lengths, const int64_t* offsets,
                      const int64_t* cu_seqlens, int64_t total_budget, void* k_out, void* v_out,
                      void* workspace, size_t workspace_bytes, void* stream) {
  Problem pb{};
  kvc_status st = make_problem(params, cu_seqlens, &pb);
  if (st != KVC_OK) return st;
  if ((st = check_ptr_table(k, pb.layers, "k")) != KVC_OK) return st;
  if ((v == nullptr) != (v_out == nullptr)) {
    set_error("v and v_out must both be given or both be NULL"); return KVC_ERR_INVALID_ARG;
  }
  if (v && (st = check_ptr_table(v, pb.layers, "v")) != KVC_OK) return st;
  if (!idx || !lengths || !offsets) {
    set_error("idx, lengths or offsets is NULL"); return KVC_ERR_INVALID_ARG;
  }
  if (total_budget < 0 || total_budget > int64_t(pb.sel_rows) * pb.total) {
    set_error("total_budget outside [0, rows*T]"); return KVC_ERR_INVALID_ARG;
  }
  if ((st = check_ws(workspace, workspace_bytes, gather_workspace_bytes(pb))) != KVC_OK) return st;
  if (total_budget == 0) return KVC_OK;
  if (!k_out) { set_error("k_out is NULL"); return KVC_ERR_INVALID_ARG; }
  return launch_gather(pb, k, v, idx, lengths, offsets, total_budget, k_out, v_out, workspace,
                       static_cast<hipStream_t>(stream));
}

kvc_status kvc_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes == 0 || bytes % 16 != 0) {
    set_error("copy probe needs non-null buffers and a positive multiple of 16 bytes");
    return KVC_ERR_INVALID_ARG;
  }
  return launch_copy_probe(dst, src, bytes, static_cast<hipStream_t>(stream));
}

kvc_status kvc_mfma_probe(const void* operands, int32_t iterations, int32_t mode, float* sink,
                          int64_t* cycles, double* flops, void* stream) {
  if (!operands || !sink || iterations < 1 || (mode != 0 && mode != 1)) {
    set_error("mfma probe needs operands, a sink, iterations >= 1 and mode 0 or 1");
    return KVC_ERR_INVALID_ARG;
  }
  return launch_mfma_probe(operands, iterations, mode, sink, cycles, flops,
                           static_cast<hipStream_t>(stream));
}

kvc_status kvc_compress(const kvc_params* params, const kvc_inputs* in, const kvc_outputs* out,
                        void* workspace, size_t workspace_bytes, void* stream) {
  if (!in || !out) { set_error("inputs or outputs is NULL"); return KVC_ERR_INVALID_ARG; }
  Problem pb{};
  kvc_status st = make_problem(params, in->cu_seqlens, &pb);
  if (st != KVC_OK) return st;
  if ((st = check_ptr_table(in->q, pb.layers, "q")) != KVC_OK) return st;
  if ((st = check_ptr_table(in->k, pb.layers, "k")) != KVC_OK) return st;
  if ((in->v == nullptr) != (out->v_out == nullptr)) {
    set_error("v and v_out must both be given or both be NULL"); return KVC_ERR_INVALID_ARG;
  }
  if (in->v && (st = check_ptr_table(in->v, pb.layers, "v")) != KVC_OK) return st;
  if (pb.value_norm && !in->v) { set_error("value_norm needs v"); return KVC_ERR_INVALID_ARG; }
  int64_t total_budget = 0;
  if ((st = check_budget(pb, in->cu_seqlens, in->budget, &total_budget)) != KVC_OK) return st;
  if (!out->lengths || !out->offsets) {
    set_error("lengths or offsets is NULL"); return KVC_ERR_INVALID_ARG;
  }
  if (total_budget > 0 && !out->k_out) { set_error("k_out is NULL"); return KVC_ERR_INVALID_ARG; }
  CompressLayout L = compress_layout(pb);
  if ((st = check_ws(workspace, workspace_bytes, L.total)) != KVC_OK) return st;

  char* ws = static_cast<char*>(workspace);
  float* S = out->scores ? out->scores : reinterpret_cast<float*>(ws + L.off_S);
  int32_t* idx = out->idx ? out->idx : reinterpret_cast<int32_t*>(ws + L.off_idx);
  float* sorted = out->s_sorted ? out->s_sorted : reinterpret_cast<float*>(ws + L.off_sorted);
  float* I = out->composite ? out->composite : reinterpret_cast<float*>(ws + L.off_I);
  float* tau = out->tau ? out->tau : reinterpret_cast<float*>(ws + L.off_tau);
  void* stage = ws + L.off_stage;
  hipStream_t s = static_cast<hipStream_t>(stream);

  if (pb.total > 0) {
    if ((st = launch_score(pb, in->q, in->k, pb.value_norm ? in->v : nullptr, S, stage, s)) !=
        KVC_OK)
      return st;
    if ((st = launch_head_rank(pb, S, idx, sorted, stage, s)) != KVC_OK) return st;
    if (!pb.unstructured && (st = launch_composite(pb, sorted, I, s)) != KVC_OK) return st;
  }
  // unstructured: the pool is the rank-aligned per-head scores themselves
  if ((st = launch_global_select(pb, pb.unstructured ? sorted : I, in->budget, tau, out->lengths,
                                 out->offsets, stage, s)) != KVC_OK)
    return st;
  if (total_budget > 0) {
    st = launch_gather(pb, in->k, in->v, idx, out->lengths, out->offsets, total_budget,
                       out->k_out, out->v_out, stage, s);
  }
  return st;
}

}  // extern "C"
