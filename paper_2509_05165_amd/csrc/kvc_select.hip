// kvc_global_select: the budget-th largest composite score of each sequence's
// pool {I[l,k]} and the per-layer lengths N_l it induces (Section 3.3: global
// pool, B_total, N_l).
//
// Radix select on the order-preserving integer image of the fp32 scores, three
// digits of 11/11/10 bits from the top: each pass histograms the candidates
// that match the prefix found so far, a one-workgroup step picks the digit
// that holds the wanted rank.  A last sweep counts, per layer, the entries
// above the threshold and those equal to it; ties are granted in ascending
// layer order until the budget is met (within a layer the tied entries are the
// ranks right after the ones above the threshold, so each layer keeps a prefix).
//
// A "layer" here is a row of the pool: a layer, or a (layer, head) pair in the
// unstructured variant.  With a per-row floor f the first f ranks of every row
// are kept unconditionally and stay out of the histograms; the budget that is
// searched for is what remains after them.
#include "kvc_internal.h"

namespace kvc {

namespace {

constexpr int SEL_BINS = 2048;
constexpr int SEL_THREADS = 256;
constexpr int SEL_PER_BLOCK = SEL_THREADS * 8;

struct SelState {
  uint32_t prefix;       // bits of the threshold key fixed so far
  uint32_t pad;
  uint64_t remaining;    // rank still to descend inside the prefix bucket (1-based)
};

struct BudgetTable { int64_t b[KVC_MAX_BATCH]; };

__device__ __forceinline__ void digit_of(int pass, uint32_t key, uint32_t* digit, uint32_t* hi) {
  // pass 0: bits 31..21, pass 1: bits 20..10, pass 2: bits 9..0
  if (pass == 0) { *digit = key >> 21; *hi = 0; }
  else if (pass == 1) { *digit = (key >> 10) & 2047u; *hi = key >> 21; }
  else { *digit = key & 1023u; *hi = key >> 10; }
}

// budget.b[] already excludes the floor entries
__global__ void select_init(uint32_t* hist, int count, SelState* state, BudgetTable budget,
                            int batch) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) hist[i] = 0;
  if (i < batch) { state[i].prefix = 0; state[i].pad = 0; state[i].remaining = (uint64_t)budget.b[i]; }
}

// grid: (token blocks, layers, batch)
__global__ __launch_bounds__(SEL_THREADS) void select_hist(
    const float* __restrict__ I, SeqTable seq, int total, int pass, int floor_rank,
    const SelState* __restrict__ state, uint32_t* __restrict__ hist /* [batch][3][SEL_BINS] */) {
  __shared__ uint32_t lh[SEL_BINS];
  const int b = blockIdx.z;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int begin = max(blockIdx.x * SEL_PER_BLOCK, floor_rank);   // ranks below the floor do not compete
  if (begin >= n || begin >= (int)(blockIdx.x + 1) * SEL_PER_BLOCK) return;
  const int end = min(n, (int)(blockIdx.x + 1) * SEL_PER_BLOCK);
  for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS) lh[i] = 0;
  __syncthreads();
  const uint32_t want_hi = pass == 0 ? 0u : (pass == 1 ? state[b].prefix >> 21 : state[b].prefix >> 10);
  const float* row = I + (size_t)blockIdx.y * total + tok0;
  for (int i = begin + threadIdx.x; i < end; i += SEL_THREADS) {
    uint32_t digit, hi;
    digit_of(pass, float_to_ordered(row[i]), &digit, &hi);
    if (hi == want_hi) atomicAdd(&lh[digit], 1u);
  }
  __syncthreads();
  uint32_t* gh = hist + ((size_t)b * 3 + pass) * SEL_BINS;
  for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS)
    if (lh[i]) atomicAdd(&gh[i], lh[i]);
}

// grid: (batch); picks the digit whose bucket holds the wanted rank, walking
// from the largest digit down.
__global__ __launch_bounds__(SEL_THREADS) void select_find(int pass, const uint32_t* __restrict__ hist,
                                                           SelState* state) {
  __shared__ uint32_t sums[SEL_THREADS];
  const int b = blockIdx.x;
  const uint64_t want = state[b].remaining;
  if (want == 0) return;                       // budget 0: nothing to find
  const uint32_t* gh = hist + ((size_t)b * 3 + pass) * SEL_BINS;
  const int bins = pass == 2 ? 1024 : SEL_BINS;
  const int per = bins / SEL_THREADS;          // 8 or 4 bins per thread
  // thread t owns bins [bins - (t+1)*per, bins - t*per): descending order
  const int t = threadIdx.x;
  uint32_t mine = 0;
  for (int j = 0; j < per; ++j) mine += gh[bins - 1 - (t * per + j)];
  sums[t] = mine;
  __syncthreads();
  if (t == 0) {
    uint64_t run = 0;
    int owner = SEL_THREADS - 1;
    for (int i = 0; i < SEL_THREADS; ++i) {
      if (run + sums[i] >= want) { owner = i; break; }
      run += sums[i];
    }
    uint32_t digit = 0;
    for (int j = 0; j < per; ++j) {
      const int bin = bins - 1 - (owner * per + j);
      const uint32_t c = gh[bin];
      if (run + c >= want) { digit = (uint32_t)bin; break; }
      run += c;
      digit = (uint32_t)bin;
    }
    const uint32_t shift = pass == 0 ? 21u : (pass == 1 ? 10u : 0u);
    state[b].prefix |= digit << shift;
    state[b].remaining = want - run;           // rank inside the chosen bucket
  }
}

// grid: (token blocks, layers, batch): counts[b][l] = {#(I > tau), #(I == tau)}
__global__ __launch_bounds__(SEL_THREADS) void select_count(
    const float* __restrict__ I, SeqTable seq, int total, int layers, int floor_rank,
    const SelState* __restrict__ state, uint32_t* __restrict__ counts) {
  __shared__ uint32_t sh[2];
  const int b = blockIdx.z;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int begin = max(blockIdx.x * SEL_PER_BLOCK, floor_rank);
  if (begin >= n || begin >= (int)(blockIdx.x + 1) * SEL_PER_BLOCK) return;
  const int end = min(n, (int)(blockIdx.x + 1) * SEL_PER_BLOCK);
  if (threadIdx.x < 2) sh[threadIdx.x] = 0;
  __syncthreads();
  const uint32_t tau = state[b].prefix;
  const float* row = I + (size_t)blockIdx.y * total + tok0;
  uint32_t gt = 0, eq = 0;
  for (int i = begin + threadIdx.x; i < end; i += SEL_THREADS) {
    const uint32_t key = float_to_ordered(row[i]);
    gt += key > tau;
    eq += key == tau;
  }
  for (int off = 32; off >= 1; off >>= 1) { gt += __shfl_xor(gt, off); eq += __shfl_xor(eq, off); }
  if ((threadIdx.x & 63) == 0) { atomicAdd(&sh[0], gt); atomicAdd(&sh[1], eq); }
  __syncthreads();
  if (threadIdx.x < 2 && sh[threadIdx.x])
    atomicAdd(&counts[((size_t)b * layers + blockIdx.y) * 2 + threadIdx.x], sh[threadIdx.x]);
}

// One thread per sequence.  The retained total of a sequence is its budget (known
// on the host), so every thread derives its own first offset from the table.
__global__ void select_finalize(SeqTable seq, int layers, int floor_rank, BudgetTable budget,
                                const SelState* __restrict__ state,
                                const uint32_t* __restrict__ counts, float* tau,
                                int32_t* lengths, int64_t* offsets) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= seq.batch) return;
  int64_t off = 0;       // rows retained by the sequences before mine
  for (int p = 0; p < b; ++p) {
    const int n_p = seq.cu[p + 1] - seq.cu[p];
    off += budget.b[p] + (int64_t)layers * (floor_rank < n_p ? floor_rank : n_p);
  }
  const int64_t want = budget.b[b];
  const int n_b = seq.cu[b + 1] - seq.cu[b];
  const int64_t kept_first = floor_rank < n_b ? floor_rank : n_b;   // the floor entries
  if (tau) tau[b] = want > 0 ? ordered_to_float(state[b].prefix) : __builtin_inff();
  int64_t above = 0;
  if (want > 0)
    for (int l = 0; l < layers; ++l) above += counts[((size_t)b * layers + l) * 2];
  int64_t ties_left = want - above;
  for (int l = 0; l < layers; ++l) {
    int64_t len = kept_first;
    if (want > 0) {
      const int64_t gt = counts[((size_t)b * layers + l) * 2];
      const int64_t eq = counts[((size_t)b * layers + l) * 2 + 1];
      const int64_t take = eq < ties_left ? eq : ties_left;
      ties_left -= take;
      len += gt + take;
    }
    lengths[b * layers + l] = (int32_t)len;
    offsets[b * layers + l] = off;
    off += len;
  }
  if (b == seq.batch - 1) offsets[seq.batch * layers] = off;
}

struct SelectLayout { size_t off_hist, off_counts, off_state, total; int words; };

SelectLayout select_layout(const Problem& pb) {
  SelectLayout L{};
  size_t cur = 0;
  const size_t hist_words = size_t(pb.batch) * 3 * SEL_BINS;
  const size_t count_words = size_t(pb.batch) * pb.sel_rows * 2;
  L.off_hist = cur;   cur += hist_words * 4;
  L.off_counts = cur; cur += align_up(count_words * 4);
  L.words = int((cur) / 4);                   // hist and counts are zeroed together
  L.off_state = cur;  cur += align_up(size_t(pb.batch) * sizeof(SelState));
  L.total = cur;
  return L;
}

}  // namespace

size_t select_workspace_bytes(const Problem& pb) { return select_layout(pb).total; }

kvc_status launch_global_select(const Problem& pb, const float* I, const int64_t* budget,
                                float* tau, int32_t* lengths, int64_t* offsets, void* ws,
                                hipStream_t stream) {
  const SelectLayout L = select_layout(pb);
  char* w = static_cast<char*>(ws);
  uint32_t* hist = reinterpret_cast<uint32_t*>(w + L.off_hist);
  uint32_t* counts = reinterpret_cast<uint32_t*>(w + L.off_counts);
  SelState* state = reinterpret_cast<SelState*>(w + L.off_state);
  const int rows = pb.sel_rows, floor_rank = pb.min_per_layer;
  BudgetTable bt{};   // what is left to compete for after the floor entries
  for (int b = 0; b < pb.batch; ++b) {
    const int64_t n_b = pb.seq.cu[b + 1] - pb.seq.cu[b];
    bt.b[b] = budget[b] - int64_t(rows) * (floor_rank < n_b ? floor_rank : n_b);
  }
  const int total = int(pb.total);

  KVC_LAUNCH("select_init", stream, select_init<<<(L.words + 255) / 256, 256, 0, stream>>>(hist, L.words, state, bt, pb.batch));
  if (pb.max_seqlen > 0) {
    dim3 grid((unsigned)((pb.max_seqlen + SEL_PER_BLOCK - 1) / SEL_PER_BLOCK), rows, pb.batch);
    for (int pass = 0; pass < 3; ++pass) {
      KVC_LAUNCH("select_hist", stream, select_hist<<<grid, SEL_THREADS, 0, stream>>>(I, pb.seq, total, pass, floor_rank, state, hist));
      KVC_LAUNCH("select_find", stream, select_find<<<pb.batch, SEL_THREADS, 0, stream>>>(pass, hist, state));
    }
    KVC_LAUNCH("select_count", stream, select_count<<<grid, SEL_THREADS, 0, stream>>>(I, pb.seq, total, rows, floor_rank, state, counts));
  }
  KVC_LAUNCH("select_finalize", stream, select_finalize<<<1, 64, 0, stream>>>(pb.seq, rows, floor_rank, bt, state, counts, tau,
                                        lengths, offsets));
  return KVC_OK;
}

}  // namespace kvc
