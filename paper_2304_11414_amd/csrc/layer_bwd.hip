// Backward of the layer around the expert FFN (the paper prints no backward algorithm -- Section 3.2,
// footnote to Eq. 1, only prices it; this is the chain rule of Algorithm 1's forward, picks held
// fixed):
//   dY[r, :]       = gate_w[t, j] * d_out[t, :]          for the kept local assignment (t, j) in row r
//   d_gate_w[t, j] = <d_out[t, :], y_sliced[r, :]>        (0 for dropped / non-local picks)
//   dlogits        through the (renormalised) top-k weights and the softmax
//   dx[t, :]       = sum over kept local (t, j) of dX_sliced[r, :]  +  dlogits[t, :] Wg
//   dWg            = dlogits^T x,   dbias = column sums of dlogits
// All of it is this device's partial sum, like the forward output.  Row movement kernels are
// HBM-bound; every sum has a fixed order (bitwise reproducible).

#include "common.h"

namespace ppmoe {

namespace {

constexpr int kThreads = 256;

template <int D>
__device__ __forceinline__ void widen8(const void* p, float (&f)[8]) {
  if constexpr (D == MOE_F32) {
    const f32x4 a = reinterpret_cast<const f32x4*>(p)[0], b = reinterpret_cast<const f32x4*>(p)[1];
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
  } else {
    const u32x4 v = *reinterpret_cast<const u32x4*>(p);
    Elem16<D>::widen2(v.x, f[0], f[1]);
    Elem16<D>::widen2(v.y, f[2], f[3]);
    Elem16<D>::widen2(v.z, f[4], f[5]);
    Elem16<D>::widen2(v.w, f[6], f[7]);
  }
}

template <int D>
__device__ __forceinline__ u32x4 pack8(const float (&f)[8]) {
  return u32x4{Elem16<D>::pack2(f[0], f[1]), Elem16<D>::pack2(f[2], f[3]), Elem16<D>::pack2(f[4], f[5]),
               Elem16<D>::pack2(f[6], f[7])};
}

// dY[r, :] = gate_w[perm[r]] * d_out[perm[r] / k, :]; a thread moves 8 elements per row.
template <int DOUT, int DT>
__global__ __launch_bounds__(kThreads) void gather_scale_kernel(const void* __restrict__ d_out,
                                                                const int32_t* __restrict__ perm,
                                                                const int32_t* __restrict__ offsets,
                                                                const float* __restrict__ gate_w,
                                                                bf16_t* __restrict__ dY, int n_local, int top_k,
                                                                int d) {
  const int rows = offsets[n_local];
  constexpr int in_bytes = DOUT == MOE_F32 ? 4 : 2;
  const unsigned char* src = static_cast<const unsigned char*>(d_out);
  for (int r = blockIdx.x; r < rows; r += gridDim.x) {
    const int a = perm[r];
    const int t = top_k == 1 ? a : a / top_k;
    const float w = gate_w[a];
    for (int c = threadIdx.x * 8; c < d; c += kThreads * 8) {
      float f[8];
      widen8<DOUT>(src + (static_cast<int64_t>(t) * d + c) * in_bytes, f);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] *= w;
      *reinterpret_cast<u32x4*>(dY + static_cast<int64_t>(r) * d + c) = pack8<DT>(f);
    }
  }
}

// One thread per token.  p = softmax(logits);  w_j = p[e_j], or p[e_j] / S with S = sum_j p[e_j] when
// renormalised (gate_w holds the w_j the forward used).  d_gate_w[j] = row_dot[row] / w_j for a kept
// local pick (row_dot = <dY, y_sliced> = w_j <d_out, y_sliced>), else 0.
// Without renormalisation dp[e_j] = dw_j; with it dp[e_j] = (dw_j - sum_i dw_i w_i) / S.
// Softmax: dlogits[e] = p[e] (dp[e] - sum_e' dp[e'] p[e']).
__global__ __launch_bounds__(kThreads) void gate_backward_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ expert_idx, const float* __restrict__ gate_w,
    const int32_t* __restrict__ inv_perm, const float* __restrict__ row_dot, float* __restrict__ dlogits, int T,
    int E, int k, int renorm) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float* lg = logits + static_cast<int64_t>(t) * E;
  float m = lg[0];
  for (int e = 1; e < E; ++e) m = fmaxf(m, lg[e]);
  float sum = 0.f;
  for (int e = 0; e < E; ++e) sum += expf(lg[e] - m);
  float dw[kMaxTopK], pj[kMaxTopK];
  float S = 0.f, dww = 0.f;
  for (int j = 0; j < k; ++j) {
    const int a = t * k + j;
    const int row = inv_perm[a];
    const float w = gate_w[a];
    dw[j] = row >= 0 ? row_dot[row] / w : 0.f;
    pj[j] = expf(lg[expert_idx[a]] - m) / sum;
    S += pj[j];
    dww = fmaf(dw[j], w, dww);
  }
  float dot = 0.f;   // sum_e dp[e] p[e]
  for (int j = 0; j < k; ++j) {
    dw[j] = renorm ? (dw[j] - dww) / S : dw[j];   // now dp at the picked expert
    dot = fmaf(dw[j], pj[j], dot);
  }
  float* out = dlogits + static_cast<int64_t>(t) * E;
  for (int e = 0; e < E; ++e) out[e] = -(expf(lg[e] - m) / sum) * dot;
  for (int j = 0; j < k; ++j) out[expert_idx[t * k + j]] += pj[j] * dw[j];   // (a token picks an expert at most once)
}

// dx: kTok tokens per block iteration, a thread owns 8 columns; the router rows are read once per
// kTok tokens.
constexpr int kTok = 8;
template <int DT>
__global__ __launch_bounds__(kThreads) void dx_kernel(const bf16_t* __restrict__ dXs,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ dlogits,
                                                      const bf16_t* __restrict__ Wg, bf16_t* __restrict__ dx, int T,
                                                      int d, int E, int k) {
  __shared__ float dl[kTok][kMaxExperts];
  for (int t0 = blockIdx.x * kTok; t0 < T; t0 += gridDim.x * kTok) {
    __syncthreads();
    for (int i = threadIdx.x; i < kTok * E; i += kThreads) {
      const int tt = i / E, e = i - tt * E;
      dl[tt][e] = t0 + tt < T ? dlogits[static_cast<int64_t>(t0 + tt) * E + e] : 0.f;
    }
    __syncthreads();
    for (int c = threadIdx.x * 8; c < d; c += kThreads * 8) {
      float acc[kTok][8];
#pragma unroll
      for (int tt = 0; tt < kTok; ++tt) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[tt][e] = 0.f;
        const int t = t0 + tt;
        if (t < T) {
          for (int j = 0; j < k; ++j) {
            const int r = inv_perm[static_cast<int64_t>(t) * k + j];
            if (r >= 0) {
              float f[8];
              widen8<DT>(dXs + static_cast<int64_t>(r) * d + c, f);
#pragma unroll
              for (int e = 0; e < 8; ++e) acc[tt][e] += f[e];
            }
          }
        }
      }
      for (int e = 0; e < E; ++e) {
        float w[8];
        widen8<DT>(Wg + static_cast<int64_t>(e) * d + c, w);
#pragma unroll
        for (int tt = 0; tt < kTok; ++tt) {
          const float g = dl[tt][e];
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[tt][q] = fmaf(g, w[q], acc[tt][q]);
        }
      }
#pragma unroll
      for (int tt = 0; tt < kTok; ++tt)
        if (t0 + tt < T) *reinterpret_cast<u32x4*>(dx + static_cast<int64_t>(t0 + tt) * d + c) = pack8<DT>(acc[tt]);
    }
  }
}

// dWg: the tokens are cut into kChunks chunks; block (column block, chunk) adds up its chunk for its
// 2048 columns (8 per thread), eight experts at a time, and stores a partial sum; a second launch
// adds the chunks in order.
constexpr int kChunks = 256;
constexpr int kEG = 8;
template <int DT>
__global__ __launch_bounds__(kThreads) void dwg_partial_kernel(const bf16_t* __restrict__ x,
                                                               const float* __restrict__ dlogits,
                                                               float* __restrict__ part, float* __restrict__ part_bias,
                                                               int T, int d, int E) {
  const int chunk = blockIdx.y;
  const int per = (T + kChunks - 1) / kChunks;
  const int tb = chunk * per, te = min(T, tb + per);
  const int c = (blockIdx.x * kThreads + threadIdx.x) * 8;
  for (int e0 = 0; e0 < E; e0 += kEG) {
    float acc[kEG][8];
#pragma unroll
    for (int g = 0; g < kEG; ++g)
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[g][q] = 0.f;
    float bsum = 0.f;   // (thread g of column block 0 also adds up dlogits[:, e0 + g])
    // four tokens at a time: their loads go out together, the sums keep the token order
    for (int t0 = tb; t0 < te; t0 += 4) {
      float dl[4][kEG];
      u32x4 xr[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int t = min(t0 + j, te - 1);
        xr[j] = (c < d && t0 + j < te) ? *reinterpret_cast<const u32x4*>(x + static_cast<int64_t>(t) * d + c) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int g = 0; g < kEG; ++g)
          dl[j][g] = (t0 + j < te && e0 + g < E) ? dlogits[static_cast<int64_t>(t) * E + e0 + g] : 0.f;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (blockIdx.x == 0 && threadIdx.x < kEG) {
#pragma unroll
          for (int g = 0; g < kEG; ++g)
            if (static_cast<int>(threadIdx.x) == g) bsum += dl[j][g];
        }
        float f[8];
        const uint32_t w4[4] = {xr[j].x, xr[j].y, xr[j].z, xr[j].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) Elem16<DT>::widen2(w4[q], f[2 * q], f[2 * q + 1]);
#pragma unroll
        for (int g = 0; g < kEG; ++g)
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[g][q] = fmaf(dl[j][g], f[q], acc[g][q]);
      }
    }
    if (c < d) {
#pragma unroll
      for (int g = 0; g < kEG; ++g)
        if (e0 + g < E) {
          float* o = part + (static_cast<int64_t>(chunk) * E + e0 + g) * d + c;
          *reinterpret_cast<f32x4*>(o) = f32x4{acc[g][0], acc[g][1], acc[g][2], acc[g][3]};
          *reinterpret_cast<f32x4*>(o + 4) = f32x4{acc[g][4], acc[g][5], acc[g][6], acc[g][7]};
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < kEG && e0 + static_cast<int>(threadIdx.x) < E)
      part_bias[static_cast<int64_t>(chunk) * E + e0 + threadIdx.x] = bsum;
  }
}

__global__ __launch_bounds__(kThreads) void dwg_final_kernel(const float* __restrict__ part,
                                                             const float* __restrict__ part_bias,
                                                             float* __restrict__ dWg, float* __restrict__ dbias, int d,
                                                             int E) {
  const int64_t n = static_cast<int64_t>(E) * d;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < n; i += static_cast<int64_t>(gridDim.x) * kThreads) {
    float sum = 0.f;
    for (int ch = 0; ch < kChunks; ++ch) sum += part[ch * n + i];
    dWg[i] = sum;
  }
  if (dbias != nullptr && blockIdx.x == 0)
    for (int e = threadIdx.x; e < E; e += kThreads) {
      float sum = 0.f;
      for (int ch = 0; ch < kChunks; ++ch) sum += part_bias[ch * E + e];
      dbias[e] = sum;
    }
}

}  // namespace

hipError_t launch_gather_scale(const moe_config& c, const void* d_out, const int32_t* perm,
                               const int32_t* offsets, const float* gate_w, void* dY, int64_t max_rows,
                               hipStream_t s) {
  if (max_rows == 0 || c.T == 0) return hipSuccess;
  const int blocks = static_cast<int>(max_rows < 256 * 16 ? max_rows : 256 * 16);
  bf16_t* dy = static_cast<bf16_t*>(dY);
#define PPMOE_GS(DOUT, DT) \
  gather_scale_kernel<DOUT, DT><<<blocks, kThreads, 0, s>>>(d_out, perm, offsets, gate_w, dy, c.local_count, c.top_k, c.d)
  if (c.in_dtype == MOE_F16) {
    if (c.out_dtype == MOE_F32) PPMOE_GS(MOE_F32, MOE_F16);
    else PPMOE_GS(MOE_F16, MOE_F16);
  } else {
    if (c.out_dtype == MOE_F32) PPMOE_GS(MOE_F32, MOE_BF16);
    else PPMOE_GS(MOE_BF16, MOE_BF16);
  }
#undef PPMOE_GS
  return hipGetLastError();
}

hipError_t launch_gate_backward(const moe_config& c, const float* logits, const int32_t* expert_idx,
                                const float* gate_w, const int32_t* inv_perm, const float* row_dot,
                                float* dlogits, hipStream_t s) {
  if (c.T == 0) return hipSuccess;
  gate_backward_kernel<<<(c.T + kThreads - 1) / kThreads, kThreads, 0, s>>>(
      logits, expert_idx, gate_w, inv_perm, row_dot, dlogits, c.T, c.E, c.top_k, c.renorm_topk);
  return hipGetLastError();
}

hipError_t launch_dx(const moe_config& c, const void* dX_sliced, const int32_t* inv_perm,
                     const float* dlogits, const void* Wg, void* dx, hipStream_t s) {
  if (c.T == 0) return hipSuccess;
  const int64_t want = (static_cast<int64_t>(c.T) + kTok - 1) / kTok;
  const int blocks = static_cast<int>(want < 256 * 8 ? want : 256 * 8);
  if (c.in_dtype == MOE_F16)
    dx_kernel<MOE_F16><<<blocks, kThreads, 0, s>>>(static_cast<const bf16_t*>(dX_sliced), inv_perm, dlogits,
                                                   static_cast<const bf16_t*>(Wg), static_cast<bf16_t*>(dx), c.T, c.d,
                                                   c.E, c.top_k);
  else
    dx_kernel<MOE_BF16><<<blocks, kThreads, 0, s>>>(static_cast<const bf16_t*>(dX_sliced), inv_perm, dlogits,
                                                    static_cast<const bf16_t*>(Wg), static_cast<bf16_t*>(dx), c.T, c.d,
                                                    c.E, c.top_k);
  return hipGetLastError();
}

size_t dwg_scratch_bytes(const moe_config& c) {
  return static_cast<size_t>(kChunks) * c.E * (static_cast<size_t>(c.d) + 1) * sizeof(float) + 256;
}

hipError_t launch_dwg(const moe_config& c, const void* x, const float* dlogits, float* dWg, float* dbias,
                      void* scratch, hipStream_t s) {
  float* part = static_cast<float*>(scratch);
  float* part_bias = part + static_cast<size_t>(kChunks) * c.E * c.d;
  const dim3 grid((c.d + kThreads * 8 - 1) / (kThreads * 8), kChunks);
  if (c.in_dtype == MOE_F16)
    dwg_partial_kernel<MOE_F16><<<grid, kThreads, 0, s>>>(static_cast<const bf16_t*>(x), dlogits, part, part_bias,
                                                          c.T, c.d, c.E);
  else
    dwg_partial_kernel<MOE_BF16><<<grid, kThreads, 0, s>>>(static_cast<const bf16_t*>(x), dlogits, part, part_bias,
                                                           c.T, c.d, c.E);
  const int64_t n = static_cast<int64_t>(c.E) * c.d;
  const int blocks = static_cast<int>((n + kThreads - 1) / kThreads < 1024 ? (n + kThreads - 1) / kThreads : 1024);
  dwg_final_kernel<<<blocks, kThreads, 0, s>>>(part, part_bias, dWg, dbias, c.d, c.E);
  return hipGetLastError();
}

}  // namespace ppmoe
