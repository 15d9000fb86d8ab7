// Gating module: router GEMM + softmax + top-k in one pass over the token matrix.
// Section 3.3.3 of the paper (linear mapping, softmax score function, gating schedule);
// Algorithm 1: logits = wg(hidden_states); scores = softmax(logits); gate_function(scores).
//
// The router GEMM is skinny (N = E <= 256) and reads x exactly once, so it is HBM-bound; it runs on
// the 16x16x32 bf16 MFMA so that the arithmetic never becomes the limit at E = 64.  Softmax and the
// top-k selection are float32 (the paper keeps the gating module in float32, Section 4.1).

#include "common.h"

namespace ppmoe {


// One token: softmax over all E logits, then k picks in descending (logit, then ascending index)
// order.  Picks are found without a "taken" mask: the next pick is the largest element that comes
// strictly after the previous pick in that order.
__device__ __forceinline__ void softmax_topk_row(const float* lg, int E, int k, int renorm,
                                                 int32_t* idx_out, float* w_out,
                                                 int32_t* idx_copy = nullptr, float* max_out = nullptr,
                                                 float* sum_out = nullptr) {
  float m = lg[0];
  for (int e = 1; e < E; ++e) m = fmaxf(m, lg[e]);
  float sum = 0.f;
  for (int e = 0; e < E; ++e) sum += expf(lg[e] - m);
  float pv = __builtin_inff();
  int pe = -1;
  float wsum = 0.f;
  for (int j = 0; j < k; ++j) {
    int best = -1;
    float bv = 0.f;
    for (int e = 0; e < E; ++e) {
      float v = lg[e];
      bool after_prev = (v < pv) || (v == pv && e > pe);
      if (after_prev && (best < 0 || v > bv)) {
        best = e;
        bv = v;
      }
    }
    float w = expf(bv - m) / sum;
    idx_out[j] = best;
    if (idx_copy != nullptr) idx_copy[j] = best;
    w_out[j] = w;
    wsum += w;
    pv = bv;
    pe = best;
  }
  if (renorm) {
    for (int j = 0; j < k; ++j) w_out[j] = w_out[j] / wsum;
  }
  if (max_out != nullptr) *max_out = m;
  if (sum_out != nullptr) *sum_out = sum;
}

// The same routine for a row of at most EP logits sitting in LDS: they are read into registers in
// one go (the loops above would pay one LDS latency per element) and every loop is unrolled over EP
// with the elements past E switched off.  Same arithmetic in the same order as softmax_topk_row:
// the two give the same bits.  On return the row holds the logits still, or, if probs_out, the
// softmax probabilities.
template <int EP>
__device__ __forceinline__ void softmax_topk_row_regs(float* lg, const float* __restrict__ bias,
                                                      float* __restrict__ logits_out, int E, int k,
                                                      int renorm, int32_t* idx_out, float* w_out,
                                                      int32_t* idx_copy, bool probs_out) {
  float v[EP];
#pragma unroll
  for (int e = 0; e < EP; ++e) v[e] = lg[e];
  if (bias != nullptr) {
#pragma unroll
    for (int e = 0; e < EP; ++e)
      if (e < E) v[e] += bias[e];
  }
  if (logits_out != nullptr) {
#pragma unroll
    for (int e = 0; e < EP; ++e)
      if (e < E) logits_out[e] = v[e];
  }
  float m = v[0];
#pragma unroll
  for (int e = 1; e < EP; ++e)
    if (e < E) m = fmaxf(m, v[e]);
  float p[EP];
  float sum = 0.f;
#pragma unroll
  for (int e = 0; e < EP; ++e)
    if (e < E) {
      p[e] = expf(v[e] - m);
      sum += p[e];
    }
  float pv = __builtin_inff();
  int pe = -1;
  float wsum = 0.f;
  for (int j = 0; j < k; ++j) {
    int best = -1;
    float bv = 0.f, bp = 0.f;
#pragma unroll
    for (int e = 0; e < EP; ++e) {
      const bool after_prev = (v[e] < pv) || (v[e] == pv && e > pe);
      if (e < E && after_prev && (best < 0 || v[e] > bv)) {
        best = e;
        bv = v[e];
        bp = p[e];
      }
    }
    const float w = bp / sum;
    idx_out[j] = best;
    if (idx_copy != nullptr) idx_copy[j] = best;
    w_out[j] = w;
    wsum += w;
    pv = bv;
    pe = best;
  }
  if (renorm) {
    for (int j = 0; j < k; ++j) w_out[j] = w_out[j] / wsum;
  }
  if (probs_out) {
#pragma unroll
    for (int e = 0; e < EP; ++e)
      if (e < E) lg[e] = p[e] / sum;
  }
}

// What a block adds once it has scored its tokens (one segment of the permutation that follows):
// its picks per local expert (seg_count), and the sums of the softmax probabilities and of the first
// picks per expert (part_prob, part_cnt: partial sums of the balance loss).  One thread per expert
// walks the block's tokens in order, so everything is bitwise reproducible.
// tile[tok * ld + e]: probabilities (zeros for tokens past T); picks[tok * k + j]: picks (-1 past T).
__device__ __forceinline__ void block_segment_sums(const float* tile, int ld, const int32_t* picks,
                                                   int n_tok, int k, int E, int local_begin,
                                                   int n_local, int seg, int n_seg,
                                                   int32_t* __restrict__ seg_count,
                                                   float* __restrict__ part_prob,
                                                   int32_t* __restrict__ part_cnt) {
  for (int e = threadIdx.x; e < max(E, n_local); e += blockDim.x) {
    if (seg_count != nullptr && e < n_local) {
      int cnt = 0;
      for (int a = 0; a < n_tok * k; ++a) cnt += picks[a] == local_begin + e;
      seg_count[static_cast<size_t>(e) * n_seg + seg] = cnt;
    }
    if (part_prob != nullptr && e < E) {
      float p = 0.f;
      int first = 0;
      for (int tok = 0; tok < n_tok; ++tok) {
        p += tile[tok * ld + e];
        first += picks[tok * k] == e;
      }
      part_prob[static_cast<size_t>(seg) * E + e] = p;
      part_cnt[static_cast<size_t>(seg) * E + e] = first;
    }
  }
}

// One token's share of the tail: softmax + top-k on its row of the logits tile, outputs, and what
// block_segment_sums needs.
template <int EP>
__device__ __forceinline__ void score_token(float* lg, int t, int T, int E, int k, int renorm,
                                            const float* __restrict__ bias,
                                            float* __restrict__ logits_out,
                                            int32_t* __restrict__ expert_idx,
                                            float* __restrict__ gate_w, int32_t* pk, bool extras,
                                            bool probs) {
  if (t < T) {
    float* lo = logits_out != nullptr ? logits_out + static_cast<size_t>(t) * E : nullptr;
    if constexpr (EP > 0) {
      softmax_topk_row_regs<EP>(lg, bias, lo, E, k, renorm, expert_idx + static_cast<size_t>(t) * k,
                                gate_w + static_cast<size_t>(t) * k, extras ? pk : nullptr, probs);
    } else {
      if (bias != nullptr)
        for (int e = 0; e < E; ++e) lg[e] += bias[e];
      if (lo != nullptr)
        for (int e = 0; e < E; ++e) lo[e] = lg[e];
      float m, sum;
      softmax_topk_row(lg, E, k, renorm, expert_idx + static_cast<size_t>(t) * k,
                       gate_w + static_cast<size_t>(t) * k, extras ? pk : nullptr, &m, &sum);
      if (probs)
        for (int e = 0; e < E; ++e) lg[e] = expf(lg[e] - m) / sum;
    }
  } else if (extras) {
    for (int j = 0; j < k; ++j) pk[j] = -1;
    for (int e = 0; e < E; ++e) lg[e] = 0.f;
  }
}

// 16-bit router, direct operand loads (used for more than 64 experts): a block owns 16*MT tokens; its 4 wavefronts split d between them (span-interleaved)
// and their partial logits are added in wavefront order through LDS, so the float32 sum order is
// fixed.  MFMA operands come straight from global memory: lane (r = lane%16, g = lane/16) holds 8
// consecutive k of row r, which is exactly a 16-byte load; four such loads cover 64 contiguous
// bytes of each of the 16 rows.
template <int NT, int MT, int DT>
__global__ __launch_bounds__(256) void gate_bf16_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wg, const float* __restrict__ bias,
    float* __restrict__ logits_out, int32_t* __restrict__ expert_idx, float* __restrict__ gate_w,
    int32_t* __restrict__ seg_count, float* __restrict__ part_prob, int32_t* __restrict__ part_cnt,
    int T, int d, int E, int k, int renorm, int local_begin, int n_local) {
  constexpr int kTok = 16 * MT;
  constexpr int kLd = NT * 16 + 1;
  __shared__ float red[kTok * kLd];
  __shared__ int32_t picks[kTok * kMaxTopK];
  const bool extras = seg_count != nullptr || part_prob != nullptr;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, g = lane >> 4;
  const int t0 = blockIdx.x * kTok;
  const int nchunk = d >> 3;  // 16-byte chunks per row

  const u32x4* xrow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int t = min(t0 + mt * 16 + r, T - 1);
    xrow[mt] = reinterpret_cast<const u32x4*>(x + static_cast<size_t>(t) * d);
  }
  const u32x4* wrow[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int e = min(nt * 16 + r, E - 1);
    wrow[nt] = reinterpret_cast<const u32x4*>(Wg + static_cast<size_t>(e) * d);
  }

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // U spans of 128 k-values per iteration: all their loads are issued before the first MFMA, so a
  // wavefront keeps U * (MT + NT) * 4 16-byte loads in flight.
  constexpr int U = (NT * MT == 1) ? 4 : (NT * MT <= 4) ? 2 : 1;
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  for (int c0 = wave * 16; c0 < nchunk; c0 += 64 * U) {
    u32x4 a[U][MT][4], b[U][NT][4];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = c0 + u * 64 + i * 4 + g;
        const bool ok = c < nchunk;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[u][mt][i] = ok ? __builtin_nontemporal_load(xrow[mt] + c) : zero;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) b[u][nt][i] = ok ? wrow[nt][c] : zero;
      }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[mt][nt] = Elem16<DT>::mfma16(__builtin_bit_cast(typename Elem16<DT>::vec8, a[u][mt][i]),
                                             __builtin_bit_cast(typename Elem16<DT>::vec8, b[u][nt][i]),
                                             acc[mt][nt]);
  }

  // D layout of the 16x16 MFMA: lane holds column (lane % 16), rows (lane / 16) * 4 + i.
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float* p = &red[(mt * 16 + g * 4 + i) * kLd + nt * 16 + r];
            *p = (w == 0) ? acc[mt][nt][i] : (*p + acc[mt][nt][i]);
          }
    }
    __syncthreads();
  }

  // The tail: one thread per token (rows of up to 64 experts go through registers).
  if (threadIdx.x < kTok)
    score_token<(NT <= 4 ? NT * 16 : 0)>(&red[threadIdx.x * kLd], t0 + threadIdx.x, T, E, k, renorm, bias,
                                         logits_out, expert_idx, gate_w, picks + threadIdx.x * k, extras,
                                         part_prob != nullptr);
  if (extras) {   // the block's tokens are one segment of the permutation that follows
    __syncthreads();
    block_segment_sums(red, kLd, picks, kTok, k, E, local_begin, n_local, blockIdx.x, gridDim.x,
                       seg_count, part_prob, part_cnt);
  }
}

// The same router with the token rows read as whole rows: a block brings its 16*MT token rows in
// through LDS, 2048/MT columns at a time, every wavefront load covering one contiguous kilobyte of a
// row (the direct operand loads above fetch 64 bytes of each of 16 rows per instruction, which costs
// a fifth to a quarter of the achievable read bandwidth); the MFMA operands of the tokens then come
// from LDS (rows 16 bytes apart from a multiple of the bank width: conflict free), those of the
// router matrix straight from global memory (L2) as above.  The next chunk's rows are in flight, in
// registers, while the current one is multiplied.  Partial logits of the four wavefronts (which
// split the columns of a chunk) are added in wavefront order: fixed float32 sum order.
template <int NT, int MT, int DT>
__global__ __launch_bounds__(256) void gate_rows_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ Wg, const float* __restrict__ bias,
    float* __restrict__ logits_out, int32_t* __restrict__ expert_idx, float* __restrict__ gate_w,
    int32_t* __restrict__ seg_count, float* __restrict__ part_prob, int32_t* __restrict__ part_cnt,
    int T, int d, int E, int k, int renorm, int local_begin, int n_local) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int kTok = 16 * MT;
  constexpr int kLd = NT * 16 + 1;
  constexpr int CK = 2048 / MT;               // columns per chunk
  constexpr int kPiecesRow = CK / 8;          // 16-byte pieces of a row per chunk
  constexpr int kRowBytes = CK * 2 + 16;      // one token row of a chunk in LDS
  constexpr int kStepsWave = CK / 32 / 4;     // MFMA steps per wavefront per chunk
  unsigned char* xt = smem;                                                 // [kTok][kRowBytes]
  float* red = reinterpret_cast<float*>(smem + kTok * kRowBytes);           // [kTok][kLd]
  int32_t* picks = reinterpret_cast<int32_t*>(red + kTok * kLd);            // [kTok][k]
  const bool extras = seg_count != nullptr || part_prob != nullptr;
  typedef typename Elem16<DT>::vec8 vec8;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, g = lane >> 4;
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  const int n_groups = (T + kTok - 1) / kTok;   // a group of kTok tokens = one segment of the permutation
  const int n_chunks = (d + CK - 1) / CK;

  // staging: kTok * kPiecesRow = 4096 pieces per chunk, 16 per thread, consecutive threads on
  // consecutive pieces of a row
  u32x4 st[16];
  auto load_chunk = [&](int grp, int ck) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int p = threadIdx.x + 256 * i;
      const int row = p / kPiecesRow, col = ck * CK + (p % kPiecesRow) * 8;
      const int t = min(grp * kTok + row, T - 1);
      st[i] = col < d ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(x + static_cast<size_t>(t) * d + col)) : zero;
    }
  };
  const bf16_t* wrow[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) wrow[nt] = Wg + static_cast<size_t>(min(nt * 16 + r, E - 1)) * d;

  // The block walks over groups of tokens; the rows of the next chunk -- of this group or of the
  // block's next one -- are always in flight, also during the softmax / top-k tail.
  int grp = blockIdx.x;
  if (grp < n_groups) load_chunk(grp, 0);
  for (; grp < n_groups; grp += gridDim.x) {
    const int t0 = grp * kTok;
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int ck = 0; ck < n_chunks; ++ck) {
      // this wavefront's router operands of the chunk (steps wave, wave + 4, ...): on their way first
      u32x4 b[kStepsWave][NT];
#pragma unroll
      for (int j = 0; j < kStepsWave; ++j) {
        const int col = ck * CK + 32 * (wave + 4 * j) + 8 * g;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          b[j][nt] = col < d ? *reinterpret_cast<const u32x4*>(wrow[nt] + col) : zero;
      }
      __syncthreads();   // the previous chunk has been multiplied (and the previous group's tail is over)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int p = threadIdx.x + 256 * i;
        *reinterpret_cast<u32x4*>(xt + (p / kPiecesRow) * kRowBytes + (p % kPiecesRow) * 16) = st[i];
      }
      __syncthreads();
      if (ck + 1 < n_chunks) load_chunk(grp, ck + 1);
      else if (grp + static_cast<int>(gridDim.x) < n_groups) load_chunk(grp + gridDim.x, 0);
#pragma unroll
      for (int j = 0; j < kStepsWave; ++j) {
        const int off = (32 * (wave + 4 * j) + 8 * g) * 2;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const vec8 a = *reinterpret_cast<const vec8*>(xt + (mt * 16 + r) * kRowBytes + off);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[mt][nt] = Elem16<DT>::mfma16(a, __builtin_bit_cast(vec8, b[j][nt]), acc[mt][nt]);
        }
      }
    }

    // D layout of the 16x16 MFMA: lane holds column (lane % 16), rows (lane / 16) * 4 + i.
    for (int w = 0; w < 4; ++w) {
      if (wave == w) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              float* p = &red[(mt * 16 + g * 4 + i) * kLd + nt * 16 + r];
              *p = (w == 0) ? acc[mt][nt][i] : (*p + acc[mt][nt][i]);
            }
      }
      __syncthreads();
    }
    if (threadIdx.x < kTok)
      score_token<(NT <= 4 ? NT * 16 : 0)>(&red[threadIdx.x * kLd], t0 + threadIdx.x, T, E, k, renorm, bias,
                                           logits_out, expert_idx, gate_w, picks + threadIdx.x * k, extras,
                                           part_prob != nullptr);
    if (extras) {
      __syncthreads();
      block_segment_sums(red, kLd, picks, kTok, k, E, local_begin, n_local, grp, n_groups, seg_count,
                         part_prob, part_cnt);
    }
  }
}

// float32 router (the small parity configuration): one wavefront per token, experts four at a time,
// fixed butterfly reduction order.
__global__ __launch_bounds__(256) void gate_f32_kernel(
    const float* __restrict__ x, const float* __restrict__ Wg, const float* __restrict__ bias,
    float* __restrict__ logits_out, int32_t* __restrict__ expert_idx, float* __restrict__ gate_w,
    int T, int d, int E, int k, int renorm) {
  __shared__ float red[4][kMaxExperts];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;  // whole wavefront leaves; no block-wide barrier below
  const float4* xr = reinterpret_cast<const float4*>(x + static_cast<size_t>(t) * d);
  const int nq = d >> 2;
  for (int e0 = 0; e0 < E; e0 += 4) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int q = lane; q < nq; q += 64) {
      float4 xv = xr[q];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int e = min(e0 + j, E - 1);
        float4 wv = reinterpret_cast<const float4*>(Wg + static_cast<size_t>(e) * d)[q];
        acc[j] = fmaf(xv.x, wv.x, acc[j]);
        acc[j] = fmaf(xv.y, wv.y, acc[j]);
        acc[j] = fmaf(xv.z, wv.z, acc[j]);
        acc[j] = fmaf(xv.w, wv.w, acc[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float v = acc[j];
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
      if (lane == 0 && e0 + j < E) red[wave][e0 + j] = v + (bias ? bias[e0 + j] : 0.f);
    }
  }
  __builtin_amdgcn_wave_barrier();
  if (lane == 0) {
    float* lg = red[wave];
    if (logits_out != nullptr)
      for (int e = 0; e < E; ++e) logits_out[static_cast<size_t>(t) * E + e] = lg[e];
    softmax_topk_row(lg, E, k, renorm, expert_idx + static_cast<size_t>(t) * k,
                     gate_w + static_cast<size_t>(t) * k);
  }
}

// Logits handed in by the caller: one thread per token.
__global__ __launch_bounds__(256) void gate_from_logits_kernel(
    const float* __restrict__ logits_in, float* __restrict__ logits_out,
    int32_t* __restrict__ expert_idx, float* __restrict__ gate_w, int T, int E, int k, int renorm) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float* lg = logits_in + static_cast<size_t>(t) * E;
  if (logits_out != nullptr && logits_out != logits_in)
    for (int e = 0; e < E; ++e) logits_out[static_cast<size_t>(t) * E + e] = lg[e];
  softmax_topk_row(lg, E, k, renorm, expert_idx + static_cast<size_t>(t) * k,
                   gate_w + static_cast<size_t>(t) * k);
}

template <int NT, int MT>
static hipError_t launch_bf16(const moe_config& c, const void* x, const void* Wg, const float* bias,
                              float* logits_out, int32_t* expert_idx, float* gate_w, hipStream_t s,
                              GateFusion* fusion) {
  constexpr int kTok = 16 * MT;
  constexpr size_t lds = kTok * (2048 / MT * 2 + 16) + kTok * (NT * 16 + 1) * sizeof(float) +
                         kTok * kMaxTopK * sizeof(int32_t);
  static std::atomic<uint64_t> attr_set{0};
  const hipError_t attr = once_per_device(attr_set, [] {
    const void* kernels[] = {reinterpret_cast<const void*>(gate_rows_kernel<NT, MT, MOE_BF16>),
                             reinterpret_cast<const void*>(gate_rows_kernel<NT, MT, MOE_F16>)};
    for (const void* kern : kernels) {
      hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  });
  if (attr != hipSuccess) return attr;
  const int n_groups = (c.T + kTok - 1) / kTok;
  const int blocks = n_groups < 512 ? n_groups : 512;   // two resident blocks per compute unit walk over the groups
#define PPMOE_GATE(DT)                                                                                 \
  gate_rows_kernel<NT, MT, DT><<<blocks, 256, lds, s>>>(                                               \
      static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(Wg), bias, logits_out, expert_idx,     \
      gate_w, fusion != nullptr ? fusion->seg_count : nullptr,                                         \
      fusion != nullptr ? fusion->part_prob : nullptr, fusion != nullptr ? fusion->part_cnt : nullptr, \
      c.T, c.d, c.E, c.top_k, c.renorm_topk, c.local_begin, c.local_count)
  if (c.in_dtype == MOE_F16) PPMOE_GATE(MOE_F16);
  else PPMOE_GATE(MOE_BF16);
#undef PPMOE_GATE
  if (fusion != nullptr) {
    fusion->seg_assign = kTok * c.top_k;
    fusion->n_seg = n_groups;
  }
  return hipGetLastError();
}

// The direct-operand kernel (more than 64 experts: the whole-row kernel's register budget does not
// reach that far).
template <int NT, int MT>
static hipError_t launch_bf16_direct(const moe_config& c, const void* x, const void* Wg, const float* bias,
                                     float* logits_out, int32_t* expert_idx, float* gate_w, hipStream_t s,
                                     GateFusion* fusion) {
  int blocks = (c.T + 16 * MT - 1) / (16 * MT);
#define PPMOE_GATE(DT)                                                                                 \
  gate_bf16_kernel<NT, MT, DT><<<blocks, 256, 0, s>>>(                                                 \
      static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(Wg), bias, logits_out, expert_idx,     \
      gate_w, fusion != nullptr ? fusion->seg_count : nullptr,                                         \
      fusion != nullptr ? fusion->part_prob : nullptr, fusion != nullptr ? fusion->part_cnt : nullptr, \
      c.T, c.d, c.E, c.top_k, c.renorm_topk, c.local_begin, c.local_count)
  if (c.in_dtype == MOE_F16) PPMOE_GATE(MOE_F16);
  else PPMOE_GATE(MOE_BF16);
#undef PPMOE_GATE
  if (fusion != nullptr) {
    fusion->seg_assign = 16 * MT * c.top_k;
    fusion->n_seg = blocks;
  }
  return hipGetLastError();
}

// Can launch_gate honour a GateFusion request for this configuration?  (The 16-bit router kernel can.)
bool gate_is_fused_kernel(const moe_config& c) { return is_16bit(c.in_dtype) && c.T > 0; }

hipError_t launch_gate(const moe_config& c, const void* x, const void* Wg, const float* bias,
                       const float* logits_in, float* logits_out, int32_t* expert_idx,
                       float* gate_w, hipStream_t s, GateFusion* fusion) {
  if (fusion != nullptr) fusion->seg_assign = fusion->n_seg = 0;
  if (c.T == 0) return hipSuccess;
  if (logits_in != nullptr) {
    gate_from_logits_kernel<<<(c.T + 255) / 256, 256, 0, s>>>(logits_in, logits_out, expert_idx,
                                                              gate_w, c.T, c.E, c.top_k,
                                                              c.renorm_topk);
    return hipGetLastError();
  }
  if (c.in_dtype == MOE_F32) {
    gate_f32_kernel<<<(c.T + 3) / 4, 256, 0, s>>>(static_cast<const float*>(x),
                                                  static_cast<const float*>(Wg), bias, logits_out,
                                                  expert_idx, gate_w, c.T, c.d, c.E, c.top_k,
                                                  c.renorm_topk);
    return hipGetLastError();
  }
  // Up to 16 experts: more tokens per block where that still leaves two blocks per compute unit -- the
  // router rows, fetched once per block, then cost a half or a quarter of the L2 -> CU traffic.
  if (c.E <= 16 && c.T >= 64 * 512) return launch_bf16<1, 4>(c, x, Wg, bias, logits_out, expert_idx, gate_w, s, fusion);
  if (c.E <= 16 && c.T >= 32 * 512) return launch_bf16<1, 2>(c, x, Wg, bias, logits_out, expert_idx, gate_w, s, fusion);
  if (c.E <= 16) return launch_bf16<1, 1>(c, x, Wg, bias, logits_out, expert_idx, gate_w, s, fusion);
  if (c.E <= 32) return launch_bf16<2, 2>(c, x, Wg, bias, logits_out, expert_idx, gate_w, s, fusion);
  if (c.E <= 64) return launch_bf16<4, 4>(c, x, Wg, bias, logits_out, expert_idx, gate_w, s, fusion);
  if (c.E <= 128) return launch_bf16_direct<8, 4>(c, x, Wg, bias, logits_out, expert_idx, gate_w, s, fusion);
  return launch_bf16_direct<16, 2>(c, x, Wg, bias, logits_out, expert_idx, gate_w, s, fusion);
}

}  // namespace ppmoe
