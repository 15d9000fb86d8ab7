// Dispatching order -> per-expert index lists (the "indices" of Algorithm 1; worked example of
// Section 3.3.3: order 2,3,1,2,0,3,2,0 gives [4,7] [2] [0,3,6] [1,5]).
//
// The position of assignment a = t*k + j in its expert's queue is the number of earlier assignments
// to the same expert.  It is computed without order-dependent atomics, so the permutation is
// identical on every run and on every rank of a tensor-parallel group:
//   1. every wavefront owns a segment of seg_assign consecutive assignments (64 when this file counts
//      them; the tokens of one block when the gating kernel has already counted them on the way)
//      and counts, per local expert, how many of them it holds (ballot + popcount, counts kept in
//      registers);
//   2. one wavefront per expert turns the per-segment counts into exclusive prefix sums;
//   3. every wavefront walks its segment again, 64 assignments at a time: rank inside the step by
//      ballot/popcount, plus the running count carried in registers, plus the segment's prefix.
// counts/offsets (capacity-clamped, exclusive scan over the local experts) are rebuilt by every
// wavefront of step 3 from the expert totals, which costs a few shuffles, and written by the first.

#include <mutex>

#include "common.h"

namespace ppmoe {

// Scratch of the allocation-free dispatch call (per-segment counters of the permutation): a
// file-scope array in device memory, kStaticScratchBytes on every device the library runs on, held
// until the process ends.  In host code the name below is only a stand-in for the symbol: its device
// address is looked up once per device (static_scratch_of) and that pointer is what kernels get.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxScratchDevices = 64;
void* g_scratch_ptr[kMaxScratchDevices] = {};
std::mutex g_scratch_mutex;
}  // namespace

hipError_t static_scratch_of_current_device(void** ptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxScratchDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // (this device's copy: the device is current)
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return hipSuccess;
}

constexpr int kRegs = kMaxExperts / kWave;  // lane i holds experts i, i+64, i+128, i+192

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// For a uniform expert id e: value of run[e / 64] held by lane e % 64.
__device__ __forceinline__ int read_slot(const int (&run)[kRegs], int e) {
  int v = 0;
#pragma unroll
  for (int c = 0; c < kRegs; ++c)
    if ((e >> 6) == c) v = __builtin_amdgcn_readlane(run[c], e & 63);
  return v;
}

__device__ __forceinline__ void add_slot(int (&run)[kRegs], int e, int amount) {
#pragma unroll
  for (int c = 0; c < kRegs; ++c)
    if ((e >> 6) == c && lane_id() == (e & 63)) run[c] += amount;
}

// Step 1.  seg_count[i * n_seg + seg] = number of assignments of segment seg that picked local
// expert i.
__device__ __forceinline__ void count_segment(const int32_t* __restrict__ expert_idx,
                                              int32_t* seg_count, int seg, int64_t n_assign,
                                              int n_seg, int seg_assign, int local_begin, int n_local) {
  const int lane = lane_id();
  int run[kRegs] = {0, 0, 0, 0};
  const int64_t base = static_cast<int64_t>(seg) * seg_assign;
  const int64_t end = min(n_assign, base + seg_assign);
  for (int step = 0; step * kWave < seg_assign; ++step) {
    int64_t a = base + step * kWave + lane;
    int e = -1;
    if (a < end) {
      unsigned le = static_cast<unsigned>(expert_idx[a] - local_begin);
      if (le < static_cast<unsigned>(n_local)) e = static_cast<int>(le);
    }
    unsigned long long todo = __ballot(e >= 0);
    while (todo) {
      int leader = __ffsll(static_cast<long long>(todo)) - 1;
      int e0 = __builtin_amdgcn_readlane(e, leader);
      unsigned long long same = __ballot(e == e0);
      add_slot(run, e0, __popcll(same));
      todo &= ~same;
    }
  }
#pragma unroll
  for (int c = 0; c < kRegs; ++c) {
    int i = c * kWave + lane;
    if (i < n_local) seg_count[static_cast<int64_t>(i) * n_seg + seg] = run[c];
  }
}

__global__ __launch_bounds__(256) void segment_count_kernel(const int32_t* __restrict__ expert_idx,
                                                            int32_t* __restrict__ seg_count,
                                                            int64_t n_assign, int n_seg,
                                                            int seg_assign, int local_begin,
                                                            int n_local) {
  const int seg = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (seg < n_seg)
    count_segment(expert_idx, seg_count, seg, n_assign, n_seg, seg_assign, local_begin, n_local);
}

// Step 2.  One block per local expert: seg_base = exclusive scan of seg_count over segments (may be
// done in place), totals[i] = queue length of expert i before any capacity clamp.  A thread adds up a
// run of consecutive segments, the 256 run sums are scanned (butterfly inside a wavefront, the four
// wavefront totals in order), and every thread then writes the prefixes of its run.
constexpr int kScanThreads = 256;
__device__ __forceinline__ void scan_expert(const int32_t* seg_count, int32_t* seg_base,
                                            int32_t* totals, int i, int n_seg) {
  __shared__ int wave_total[4];
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  const int32_t* in = seg_count + static_cast<int64_t>(i) * n_seg;
  int32_t* out = seg_base + static_cast<int64_t>(i) * n_seg;
  const int run = (n_seg + kScanThreads - 1) / kScanThreads;
  const int s0 = threadIdx.x * run, s1 = min(n_seg, s0 + run);
  int sum = 0;
  for (int s = s0; s < s1; ++s) sum += in[s];
  int incl = sum;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    int up = __shfl_up(incl, off, 64);
    if (lane >= off) incl += up;
  }
  if (lane == kWave - 1) wave_total[wave] = incl;
  __syncthreads();
  int before = incl - sum;
  for (int w = 0; w < wave; ++w) before += wave_total[w];
  for (int s = s0; s < s1; ++s) {
    const int v = in[s];
    out[s] = before;
    before += v;
  }
  if (threadIdx.x == kScanThreads - 1) totals[i] = before;
}

// Blocks 0 .. n_local-1 scan one expert each.  One more block, when the gating kernel has left
// per-segment partial sums for the balance loss (Algorithm 1's l_aux; see aux.hip for the formula),
// adds them up in segment order (fixed order: bitwise reproducible) and writes the loss.
__global__ __launch_bounds__(kScanThreads) void segment_scan_kernel(const int32_t* __restrict__ seg_count,
                                                          int32_t* __restrict__ seg_base,
                                                          int32_t* __restrict__ totals, int n_seg,
                                                          int n_local, AuxOut aux) {
  if (static_cast<int>(blockIdx.x) < n_local) {
    scan_expert(seg_count, seg_base, totals, blockIdx.x, n_seg);
    return;
  }
  __shared__ float term[kMaxExperts];
  for (int e = threadIdx.x; e < aux.E; e += kScanThreads) {
    float prob = 0.f;
    int cnt = 0;
    for (int g = 0; g < aux.n_part; ++g) {
      prob += aux.part_prob[static_cast<size_t>(g) * aux.E + e];
      cnt += aux.part_cnt[static_cast<size_t>(g) * aux.E + e];
    }
    const float mp = aux.T > 0 ? prob / static_cast<float>(aux.T) : 0.f;
    if (aux.mean_prob != nullptr) aux.mean_prob[e] = mp;
    if (aux.first_counts != nullptr) aux.first_counts[e] = cnt;
    term[e] = aux.T > 0 ? mp * (static_cast<float>(cnt) / static_cast<float>(aux.T)) : 0.f;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float sum = 0.f;
    for (int e = 0; e < aux.E; ++e) sum += term[e];   // ascending expert order
    *aux.l_aux = static_cast<float>(aux.E) * sum;
  }
}

// Step 3.
__device__ __forceinline__ void rank_segment(
    const int32_t* __restrict__ expert_idx, const int32_t* seg_base, const int32_t* totals,
    int32_t* __restrict__ counts, int32_t* __restrict__ offsets, int32_t* __restrict__ perm,
    int32_t* __restrict__ inv_perm, int seg, int64_t n_assign, int n_seg, int seg_assign,
    int local_begin, int n_local, int cap /* INT_MAX when unlimited */) {
  const int lane = lane_id();

  // Kept queue lengths and their exclusive scan over the local experts (ascending expert id).
  int kept[kRegs], off[kRegs], run[kRegs];
  int carry = 0;
#pragma unroll
  for (int c = 0; c < kRegs; ++c) {
    int i = c * kWave + lane;
    kept[c] = i < n_local ? min(totals[i], cap) : 0;
    int incl = kept[c];
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      int up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    off[c] = carry + incl - kept[c];
    carry += __shfl(incl, kWave - 1, 64);
    run[c] = i < n_local ? seg_base[static_cast<int64_t>(i) * n_seg + seg] : 0;
    if (seg == 0 && i < n_local) {
      counts[i] = kept[c];
      offsets[i] = off[c];
    }
  }
  if (seg == 0 && lane == 0) offsets[n_local] = carry;

  const int64_t base = static_cast<int64_t>(seg) * seg_assign;
  const int64_t end = min(n_assign, base + seg_assign);
  for (int step = 0; step * kWave < seg_assign; ++step) {
    int64_t a = base + step * kWave + lane;
    int e = -1;
    if (a < end) {
      unsigned le = static_cast<unsigned>(expert_idx[a] - local_begin);
      if (le < static_cast<unsigned>(n_local)) e = static_cast<int>(le);
    }
    int row = -1;
    const unsigned long long below = (1ull << lane) - 1ull;
    unsigned long long todo = __ballot(e >= 0);
    while (todo) {
      int leader = __ffsll(static_cast<long long>(todo)) - 1;
      int e0 = __builtin_amdgcn_readlane(e, leader);
      unsigned long long same = __ballot(e == e0);
      int pos0 = read_slot(run, e0);   // queue position of the first of this group
      int off0 = read_slot(off, e0);
      if (e == e0) {
        int pos = pos0 + __popcll(same & below);
        if (pos < cap) row = off0 + pos;
      }
      add_slot(run, e0, __popcll(same));
      todo &= ~same;
    }
    if (a < end) {
      inv_perm[a] = row;
      if (row >= 0) perm[row] = static_cast<int32_t>(a);
    }
  }
}

__global__ __launch_bounds__(256) void rank_kernel(
    const int32_t* __restrict__ expert_idx, const int32_t* __restrict__ seg_base,
    const int32_t* __restrict__ totals, int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm, int64_t n_assign, int n_seg,
    int seg_assign, int local_begin, int n_local, int cap) {
  const int seg = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (seg < n_seg)
    rank_segment(expert_idx, seg_base, totals, counts, offsets, perm, inv_perm, seg, n_assign, n_seg,
                 seg_assign, local_begin, n_local, cap);
}

hipError_t launch_permute(const moe_config& c, int64_t cap, const int32_t* expert_idx,
                          int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                          int32_t* seg_scratch, hipStream_t s, int seg_assign, bool counted,
                          const AuxOut* aux) {
  const int64_t n_assign = static_cast<int64_t>(c.T) * c.top_k;
  const int n_seg = static_cast<int>((n_assign + seg_assign - 1) / seg_assign);
  const int N = c.local_count;
  int32_t* seg_count = seg_scratch;
  int32_t* seg_base = seg_scratch + static_cast<int64_t>(N) * n_seg;
  int32_t* totals = seg_base + static_cast<int64_t>(N) * n_seg;
  const int cap_i = (cap < 0 || cap > 0x7fffffff) ? 0x7fffffff : static_cast<int>(cap);
  const int blocks = n_seg > 0 ? (n_seg + 3) / 4 : 0;
  if (blocks > 0 && !counted)
    segment_count_kernel<<<blocks, 256, 0, s>>>(expert_idx, seg_count, n_assign, n_seg, seg_assign,
                                                c.local_begin, N);
  AuxOut no_aux = {};
  const bool with_aux = aux != nullptr && aux->l_aux != nullptr;
  segment_scan_kernel<<<N + (with_aux ? 1 : 0), kScanThreads, 0, s>>>(seg_count, seg_base, totals, n_seg, N,
                                                            with_aux ? *aux : no_aux);
  if (blocks > 0) {
    rank_kernel<<<blocks, 256, 0, s>>>(expert_idx, seg_base, totals, counts, offsets, perm,
                                       inv_perm, n_assign, n_seg, seg_assign, c.local_begin, N, cap_i);
  } else {
    // T == 0: counts and offsets are still defined (all zero); one wavefront writes them.
    rank_kernel<<<1, 64, 0, s>>>(expert_idx, seg_base, totals, counts, offsets, perm, inv_perm, 0, 1,
                                 seg_assign, c.local_begin, N, cap_i);
  }
  return hipGetLastError();
}

}  // namespace ppmoe
