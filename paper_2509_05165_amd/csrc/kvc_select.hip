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
// The digit search after a histogram pass and the final bookkeeping run in the
// last workgroup of the sequence to finish (each workgroup takes a ticket once its
// atomic updates are complete; the one that draws the last ticket reads the totals
// with device-scope atomic loads), so a call is five launches instead of eleven.
//
// A "layer" here is a row of the pool: a layer, or a (layer, head) pair in the
// unstructured variant.  With a per-row floor f the first f ranks of every row
// are kept unconditionally and stay out of the histograms; the budget that is
// searched for is what remains after them.
#include <mutex>

#include "kvc_internal.h"

namespace kvc {

namespace {

// Scratch of kvc_global_select_static: the histograms, counters, tickets and
// per-sequence state that kvc_global_select takes from the caller's workspace.
// One copy per GPU, held until the process ends.  In host code the array's name
// is only a stand-in for the symbol; its device address is looked up once per
// device (static_scratch) and that pointer is what kernels receive.
static __device__ __align__(256) unsigned char scratch[KVC_SELECT_STATIC_BYTES];

constexpr int SEL_BINS = 2048;
constexpr int SEL_THREADS = 256;
constexpr int SEL_PER_BLOCK = SEL_THREADS * 8;   // fewest elements of a row per workgroup

struct SelState {
  uint32_t prefix;       // bits of the threshold key fixed so far
  uint32_t bad;          // set when a histogram did not add up (see find_digit)
  uint64_t remaining;    // rank still to descend inside the prefix bucket (1-based)
  uint64_t expect;       // candidates the next histogram pass must count: the pool, then
                         // the population of the bucket chosen by the pass before
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
                            SeqTable seq, int rows, int floor_rank) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) hist[i] = 0;
  if (i < seq.batch) {
    const int n = seq.cu[i + 1] - seq.cu[i];
    state[i].prefix = 0;
    state[i].bad = 0;
    state[i].remaining = (uint64_t)budget.b[i];
    state[i].expect = (uint64_t)rows * (uint64_t)max(n - floor_rank, 0);   // entries that compete
  }
}

__device__ __forceinline__ uint32_t load_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Ticket of a workgroup that has finished its part for sequence b: true for the
// one that drew the last of `expected` tickets.
//
// INVARIANT: inside one kernel, workgroups hand data to the last one through
// device-scope atomic read-modify-writes ONLY (histogram bins, row counts).  Those
// are performed at the device's coherence point and are complete once the issuing
// wave's vector-memory counter has drained; so the release side is that wait, not a
// device-scope release fence (whose write-back of the whole L2 cost 150 us per
// launch here, 2048 workgroups each paying it).  The last workgroup reads the totals
// with device-scope atomic loads.  A plain store would NOT be visible to the last
// workgroup this way: anything else a kernel produces (state[], lengths, offsets) is
// written by the last workgroup itself and read by a later kernel.  This relies on
// returned-less atomics counting in vmcnt and being performed in L2, which holds on
// gfx950; find_digit checks that every histogram adds up to the population it must
// cover, so a violation cannot pass silently (tau becomes NaN).
// Tickets are drawn in two levels (groups of SEL_GROUP workgroups, then the groups
// of a sequence), each counter on a cache line of its own: two thousand
// workgroups drawing from one address took 30 us per launch.
constexpr int SEL_GROUP = 64;
constexpr int SEL_TICKET_WORDS = 32;   // one 128-byte line per counter

// tickets: [4 kernels][batch][groups + 1][SEL_TICKET_WORDS]; slot `groups` is the second level
__device__ __forceinline__ bool last_workgroup(uint32_t* tickets, int kernel_id, int batch, int b) {
  __shared__ uint32_t is_last;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  wait_vmcnt<0>();                             // my atomics have been performed
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t nblocks = gridDim.x * gridDim.y;
    const uint32_t groups = (nblocks + SEL_GROUP - 1) / SEL_GROUP;
    const uint32_t flat = blockIdx.y * gridDim.x + blockIdx.x, g = flat / SEL_GROUP;
    const uint32_t in_group = min((uint32_t)SEL_GROUP, nblocks - g * SEL_GROUP);
    uint32_t* base = tickets + ((size_t)(kernel_id * batch + b) * (groups + 1)) * SEL_TICKET_WORDS;
    uint32_t last = atomicAdd(base + (size_t)g * SEL_TICKET_WORDS, 1u) == in_group - 1;
    if (last) last = atomicAdd(base + (size_t)groups * SEL_TICKET_WORDS, 1u) == groups - 1;
    is_last = last;
  }
  __syncthreads();
  const bool last = is_last != 0;
  if (last) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return last;
}

// Inclusive prefix sum over the SEL_THREADS threads of a workgroup; *total = sum of all.
__device__ __forceinline__ uint64_t block_scan_incl(uint64_t v, uint64_t* total) {
  __shared__ uint64_t wave_tot[SEL_THREADS / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint64_t incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint64_t o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  __syncthreads();                              // the previous call's readers are done
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint64_t add = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < SEL_THREADS / 64; ++w) {
    const uint64_t x = wave_tot[w];
    if (w < wave) add += x;
    tot += x;
  }
  *total = tot;
  return incl + add;
}

// One workgroup: picks the digit whose bucket holds the wanted rank, walking from
// the largest digit down.  Thread t owns bins [bins - (t+1)*per, bins - t*per) in
// descending order; a prefix sum over the threads names the owner of the rank.
__device__ __forceinline__ void find_digit(int pass, int b, const uint32_t* __restrict__ hist,
                                           SelState* state) {
  const uint64_t want = state[b].remaining;    // uniform
  if (want == 0) return;                       // budget 0: nothing to find
  const uint64_t expect = state[b].expect;     // uniform; read before anyone updates it
  const uint32_t* gh = hist + ((size_t)b * 3 + pass) * SEL_BINS;
  const int bins = pass == 2 ? 1024 : SEL_BINS;
  const int per = bins / SEL_THREADS;          // 8 or 4 bins per thread
  const int t = threadIdx.x;
  uint32_t c[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) c[j] = j < per ? load_agent(&gh[bins - 1 - (t * per + j)]) : 0u;
  uint64_t mine = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) mine += c[j];
  uint64_t total;
  const uint64_t incl = block_scan_incl(mine, &total);
  uint64_t run = incl - mine;
  // every candidate of this pass must have been counted (see last_workgroup)
  if (t == 0 && total != expect) state[b].bad = 1;
  // the thread whose range holds the rank; a rank past the pool ends in the last bin
  if (run < want && (want <= incl || t == SEL_THREADS - 1)) {
    uint32_t digit = 0, population = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (j < per) {
        const int bin = bins - 1 - (t * per + j);
        digit = (uint32_t)bin;
        population = c[j];
        if (run + c[j] >= want) break;
        run += c[j];
      }
    }
    const uint32_t shift = pass == 0 ? 21u : (pass == 1 ? 10u : 0u);
    state[b].prefix |= digit << shift;
    state[b].remaining = want - run;           // rank inside the chosen bucket
    state[b].expect = population;              // what the next pass must count
  }
}

// grid: (token blocks, layers, batch)
__global__ __launch_bounds__(SEL_THREADS) void select_hist(
    const float* __restrict__ I, SeqTable seq, int total, int pass, int floor_rank, int per_block,
    SelState* state, uint32_t* __restrict__ hist /* [batch][3][SEL_BINS] */,
    uint32_t* __restrict__ tickets) {
  __shared__ uint32_t lh[SEL_BINS];
  const int b = blockIdx.z;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int begin = max((int)blockIdx.x * per_block, floor_rank);   // ranks below the floor do not compete
  const bool active = begin < n && begin < (int)(blockIdx.x + 1) * per_block;   // uniform in the workgroup
  if (active) {
    const int end = min(n, (int)(blockIdx.x + 1) * per_block);
    for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS) lh[i] = 0;
    __syncthreads();
    const uint32_t want_hi = pass == 0 ? 0u : (pass == 1 ? state[b].prefix >> 21 : state[b].prefix >> 10);
    const float* row = I + (size_t)blockIdx.y * total + tok0;
    // Four loads in flight per thread.  Rows are usually sorted, so the 64 elements of
    // a wave step mostly share one digit: then one lane adds the whole count instead
    // of 64 atomics on one address.
    const int lane = threadIdx.x & 63;
    for (int i0 = begin; i0 < end; i0 += SEL_THREADS * 4) {
      float x[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = i0 + e * SEL_THREADS + (int)threadIdx.x;
        x[e] = row[i < end ? i : end - 1];              // clamped; dropped below
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = i0 + e * SEL_THREADS + (int)threadIdx.x;
        uint32_t digit, hi;
        digit_of(pass, float_to_ordered(x[e]), &digit, &hi);
        const bool ok = i < end && hi == want_hi;
        const uint64_t all = __ballot(ok);
        if (all == 0) continue;                          // wave-uniform
        const int leader = __ffsll((unsigned long long)all) - 1;
        const uint32_t d0 = __builtin_amdgcn_readlane(digit, leader);
        const uint64_t same = __ballot(ok && digit == d0);
        if (same == all) {
          if (lane == leader) atomicAdd(&lh[d0], (uint32_t)__popcll(all));
        } else if (ok) {
          atomicAdd(&lh[digit], 1u);
        }
      }
    }
    __syncthreads();
    uint32_t* gh = hist + ((size_t)b * 3 + pass) * SEL_BINS;
    for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS)
      if (lh[i]) atomicAdd(&gh[i], lh[i]);
  }
  // every workgroup of the sequence takes a ticket, the idle ones included
  if (last_workgroup(tickets, pass, seq.batch, b))
    find_digit(pass, b, hist, state);
}

// Lengths and offsets of sequence b from its per-row counts, by one workgroup.
// The retained total of a sequence is its budget (known on the host), so the first
// offset of every sequence comes from the table.  Ties at the threshold go to the
// rows in ascending order until the budget is met: row l takes
// min(eq_l, max(0, ties - sum of eq over the rows before it)).  AGENT: counts are
// read with device-scope loads (inside the kernel that accumulated them).
template <bool AGENT>
__device__ __forceinline__ void finalize_sequence(int b, const SeqTable& seq, int layers,
                                                  int floor_rank, const BudgetTable& budget,
                                                  const SelState* state, const uint32_t* counts,
                                                  float* tau, int32_t* lengths, int64_t* offsets) {
  int64_t off = 0;       // rows retained by the sequences before mine
  for (int p = 0; p < b; ++p) {
    const int n_p = seq.cu[p + 1] - seq.cu[p];
    off += budget.b[p] + (int64_t)layers * (floor_rank < n_p ? floor_rank : n_p);
  }
  const int64_t want = budget.b[b];
  const int n_b = seq.cu[b + 1] - seq.cu[b];
  const int64_t kept_first = floor_rank < n_b ? floor_rank : n_b;   // the floor entries
  const int t = threadIdx.x;
  if (tau && t == 0) {
    // stored through the integer image: the library is compiled under the assumption
    // that no NaN occurs, which a floating-point select of a NaN need not survive
    const uint32_t bits = want > 0 ? __float_as_uint(ordered_to_float(state[b].prefix)) : 0x7f800000u;
    reinterpret_cast<uint32_t*>(tau)[b] = state[b].bad ? 0x7fc00000u : bits;
  }
  auto count_at = [&](size_t i) -> uint64_t { return AGENT ? load_agent(&counts[i]) : counts[i]; };
  uint64_t above_mine = 0;
  if (want > 0)
    for (int l = t; l < layers; l += SEL_THREADS) above_mine += count_at(((size_t)b * layers + l) * 2);
  uint64_t above;
  block_scan_incl(above_mine, &above);
  const int64_t ties = want - (int64_t)above;
  uint64_t eq_before = 0, len_before = 0;      // carried over the chunks of SEL_THREADS rows
  for (int l0 = 0; l0 < layers; l0 += SEL_THREADS) {
    const int l = l0 + t;
    const bool live = l < layers;
    uint64_t gt = 0, eq = 0;
    if (live && want > 0) {
      gt = count_at(((size_t)b * layers + l) * 2);
      eq = count_at(((size_t)b * layers + l) * 2 + 1);
    }
    uint64_t eq_chunk, len_chunk;
    const uint64_t eq_excl = eq_before + block_scan_incl(eq, &eq_chunk) - eq;
    int64_t take = ties - (int64_t)eq_excl;
    take = take < 0 ? 0 : (take > (int64_t)eq ? (int64_t)eq : take);
    const uint64_t len = live ? uint64_t(kept_first) + gt + uint64_t(take) : 0;
    const uint64_t len_excl = len_before + block_scan_incl(len, &len_chunk) - len;
    if (live) {
      lengths[b * layers + l] = (int32_t)len;
      offsets[b * layers + l] = off + (int64_t)len_excl;
    }
    eq_before += eq_chunk;
    len_before += len_chunk;
  }
  if (b == seq.batch - 1 && t == 0) offsets[seq.batch * layers] = off + (int64_t)len_before;
}

// grid: (token blocks, layers, batch): counts[b][l] = {#(I > tau), #(I == tau)}; the
// last workgroup of a sequence then writes its lengths and offsets.
__global__ __launch_bounds__(SEL_THREADS) void select_count(
    const float* __restrict__ I, SeqTable seq, int total, int layers, int floor_rank, int per_block,
    BudgetTable budget, const SelState* __restrict__ state, uint32_t* __restrict__ counts,
    uint32_t* __restrict__ tickets, float* tau, int32_t* lengths, int64_t* offsets) {
  __shared__ uint32_t sh[2];
  const int b = blockIdx.z;
  const int tok0 = seq.cu[b], n = seq.cu[b + 1] - tok0;
  const int begin = max((int)blockIdx.x * per_block, floor_rank);
  const bool active = begin < n && begin < (int)(blockIdx.x + 1) * per_block;   // uniform in the workgroup
  if (active) {
    const int end = min(n, (int)(blockIdx.x + 1) * per_block);
    if (threadIdx.x < 2) sh[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t tau_key = state[b].prefix;
    const float* row = I + (size_t)blockIdx.y * total + tok0;
    uint32_t gt = 0, eq = 0;
    for (int i = begin + threadIdx.x; i < end; i += SEL_THREADS) {
      const uint32_t key = float_to_ordered(row[i]);
      gt += key > tau_key;
      eq += key == tau_key;
    }
    for (int off = 32; off >= 1; off >>= 1) { gt += __shfl_xor(gt, off); eq += __shfl_xor(eq, off); }
    if ((threadIdx.x & 63) == 0) { atomicAdd(&sh[0], gt); atomicAdd(&sh[1], eq); }
    __syncthreads();
    if (threadIdx.x < 2 && sh[threadIdx.x])
      atomicAdd(&counts[((size_t)b * layers + blockIdx.y) * 2 + threadIdx.x], sh[threadIdx.x]);
  }
  if (last_workgroup(tickets, 3, seq.batch, b))
    finalize_sequence<true>(b, seq, layers, floor_rank, budget, state, counts, tau, lengths, offsets);
}

// Batches whose sequences are all empty launch nothing else.  grid: (batch)
__global__ __launch_bounds__(SEL_THREADS) void select_finalize(
    SeqTable seq, int layers, int floor_rank, BudgetTable budget,
    const SelState* __restrict__ state, const uint32_t* __restrict__ counts, float* tau,
    int32_t* lengths, int64_t* offsets) {
  finalize_sequence<false>(blockIdx.x, seq, layers, floor_rank, budget, state, counts, tau, lengths, offsets);
}

// Elements of a row per workgroup: every workgroup clears and flushes a 2048-bin
// histogram, so big pools (many rows) get longer stretches per workgroup, about
// 4096 workgroups per sequence at most.
inline int select_per_block(const Problem& pb) {
  int per = SEL_PER_BLOCK;
  while (per < (1 << 20) && ((pb.max_seqlen + per - 1) / per) * int64_t(pb.sel_rows) > 4096) per *= 2;
  return per;
}

struct SelectLayout { size_t off_hist, off_counts, off_tickets, off_state, total; int words; };

SelectLayout select_layout(const Problem& pb) {
  SelectLayout L{};
  size_t cur = 0;
  const size_t hist_words = size_t(pb.batch) * 3 * SEL_BINS;
  const size_t count_words = size_t(pb.batch) * pb.sel_rows * 2;
  L.off_hist = cur;   cur += hist_words * 4;
  L.off_counts = cur; cur += align_up(count_words * 4);
  // 3 passes + the count sweep, each with one counter line per group of workgroups + 1
  // (sized for the shortest stretch per workgroup, so that the size never shrinks when
  // max_seqlen grows: callers may size the workspace with an upper bound)
  const size_t sel_blocks = size_t((pb.max_seqlen + SEL_PER_BLOCK - 1) / SEL_PER_BLOCK) * pb.sel_rows;
  const size_t sel_groups = (sel_blocks + SEL_GROUP - 1) / SEL_GROUP;
  L.off_tickets = cur; cur += align_up(4 * size_t(pb.batch) * (sel_groups + 1) * SEL_TICKET_WORDS * 4);
  L.words = int((cur) / 4);                   // hist, counts and tickets are zeroed together
  L.off_state = cur;  cur += align_up(size_t(pb.batch) * sizeof(SelState));
  L.total = cur;
  return L;
}

}  // namespace

size_t select_workspace_bytes(const Problem& pb) { return select_layout(pb).total; }

// Device address of this GPU's copy of `scratch` (looked up on the first call on
// each device, with that device current).
kvc_status select_static_scratch(void** ptr) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static void* per_device[MAX_DEVICES] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= MAX_DEVICES) {
    set_error("device ordinal %d outside [0, %d)", dev, MAX_DEVICES);
    return KVC_ERR_UNSUPPORTED;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (!per_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p) { set_error("hipGetSymbolAddress(scratch) returned NULL"); return KVC_ERR_HIP; }
    per_device[dev] = p;
  }
  *ptr = per_device[dev];
  return KVC_OK;
}

kvc_status launch_global_select(const Problem& pb, const float* I, const int64_t* budget,
                                float* tau, int32_t* lengths, int64_t* offsets, void* ws,
                                hipStream_t stream) {
  const SelectLayout L = select_layout(pb);
  char* w = static_cast<char*>(ws);
  uint32_t* hist = reinterpret_cast<uint32_t*>(w + L.off_hist);
  uint32_t* counts = reinterpret_cast<uint32_t*>(w + L.off_counts);
  uint32_t* tickets = reinterpret_cast<uint32_t*>(w + L.off_tickets);
  SelState* state = reinterpret_cast<SelState*>(w + L.off_state);
  const int rows = pb.sel_rows, floor_rank = pb.min_per_layer;
  BudgetTable bt{};   // what is left to compete for after the floor entries
  for (int b = 0; b < pb.batch; ++b) {
    const int64_t n_b = pb.seq.cu[b + 1] - pb.seq.cu[b];
    bt.b[b] = budget[b] - int64_t(rows) * (floor_rank < n_b ? floor_rank : n_b);
  }
  const int total = int(pb.total);

  KVC_LAUNCH("select_init", stream, select_init<<<(L.words + 255) / 256, 256, 0, stream>>>(hist, L.words, state, bt, pb.seq, rows, floor_rank));
  if (pb.max_seqlen > 0) {
    const int per_block = select_per_block(pb);
    dim3 grid((unsigned)((pb.max_seqlen + per_block - 1) / per_block), rows, pb.batch);
    for (int pass = 0; pass < 3; ++pass)
      KVC_LAUNCH("select_hist", stream, select_hist<<<grid, SEL_THREADS, 0, stream>>>(I, pb.seq, total, pass, floor_rank, per_block, state, hist, tickets));
    KVC_LAUNCH("select_count", stream, select_count<<<grid, SEL_THREADS, 0, stream>>>(I, pb.seq, total, rows, floor_rank, per_block, bt, state, counts,
                                                                                     tickets, tau, lengths, offsets));
  } else {
    KVC_LAUNCH("select_finalize", stream, select_finalize<<<pb.batch, SEL_THREADS, 0, stream>>>(pb.seq, rows, floor_rank, bt, state, counts, tau,
                                          lengths, offsets));
  }
  return KVC_OK;
}

}  // namespace kvc
