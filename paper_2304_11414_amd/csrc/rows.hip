// The two row-movement kernels of the layer, both bound by HBM bandwidth:
//   slice   -- x_sliced[r, :] = x[perm[r] / k, :], the index selection that replaces the first
//              all-to-all (Sections 3.3.1, 3.3.3; Algorithm 1: hidden_states.index_select);
//   combine -- out[t, :] = sum_j gate_w[t, j] * y_sliced[inv_perm[t, j], :], the placement of the
//              expert outputs into a zero-initialised output that replaces the second all-to-all
//              (Algorithm 1: zeros_like + index assignment).  It is written as a gather per output
//              row, so each row of `out` is stored exactly once, zeros included: no atomics, no
//              separate memset, bitwise reproducible.
// Rows are moved as 16-byte pieces; a block owns kRowsPerBlock rows per iteration so that enough
// loads are in flight per CU.

#include "common.h"

namespace ppmoe {

constexpr int kCopyThreads = 256;

// ---- slice ------------------------------------------------------------------------------------

__global__ __launch_bounds__(kCopyThreads) void slice_rows_kernel(
    const u32x4* __restrict__ x, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ offsets, u32x4* __restrict__ x_sliced, int n_local, int top_k,
    int chunks_per_row /* d * sizeof(elem) / 16 */) {
  const int total_rows = offsets[n_local];
  const int64_t total_chunks = static_cast<int64_t>(total_rows) * chunks_per_row;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kCopyThreads * 4;
  for (int64_t c0 = (static_cast<int64_t>(blockIdx.x) * 4) * kCopyThreads + threadIdx.x;
       c0 < total_chunks; c0 += stride) {
    u32x4 v[4];
    int64_t c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      c[i] = c0 + static_cast<int64_t>(i) * kCopyThreads;
      if (c[i] < total_chunks) {
        int r = static_cast<int>(c[i] / chunks_per_row);
        int col = static_cast<int>(c[i] - static_cast<int64_t>(r) * chunks_per_row);
        int t = perm[r] / top_k;
        v[i] = __builtin_nontemporal_load(x + static_cast<int64_t>(t) * chunks_per_row + col);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (c[i] < total_chunks) __builtin_nontemporal_store(v[i], x_sliced + c[i]);
  }
}

hipError_t launch_slice(const moe_config& c, const void* x, const int32_t* perm,
                        const int32_t* offsets, void* x_sliced, int64_t max_rows, hipStream_t s) {
  if (max_rows == 0 || c.T == 0) return hipSuccess;
  const int elem = c.in_dtype == MOE_BF16 ? 2 : 4;
  const int chunks_per_row = c.d * elem / 16;
  int64_t max_chunks = max_rows * chunks_per_row;
  int64_t want = (max_chunks + kCopyThreads * 4 - 1) / (kCopyThreads * 4);
  int blocks = static_cast<int>(want < 256 * 16 ? want : 256 * 16);
  slice_rows_kernel<<<blocks, kCopyThreads, 0, s>>>(
      static_cast<const u32x4*>(x), perm, offsets, static_cast<u32x4*>(x_sliced), c.local_count,
      c.top_k, chunks_per_row);
  return hipGetLastError();
}

// ---- combine ----------------------------------------------------------------------------------

template <typename T>
struct Elems;  // how many elements a 16-byte piece holds and how to widen them
template <>
struct Elems<bf16_t> {
  static constexpr int n = 8;
  __device__ static void widen(const u32x4& v, float* f) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <>
struct Elems<float> {
  static constexpr int n = 4;
  __device__ static void widen(const u32x4& v, float* f) {
    f[0] = __uint_as_float(v.x);
    f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z);
    f[3] = __uint_as_float(v.w);
  }
};

// One thread produces Elems<TIn>::n consecutive output elements of one token.
template <typename TIn, typename TOut>
__global__ __launch_bounds__(kCopyThreads) void combine_kernel(
    const u32x4* __restrict__ y, const int32_t* __restrict__ inv_perm,
    const float* __restrict__ gate_w, TOut* __restrict__ out, int T, int d, int top_k) {
  constexpr int n = Elems<TIn>::n;
  const int pieces_per_row = d / n;
  const int64_t total = static_cast<int64_t>(T) * pieces_per_row;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kCopyThreads;
  for (int64_t p = static_cast<int64_t>(blockIdx.x) * kCopyThreads + threadIdx.x; p < total;
       p += stride) {
    const int t = static_cast<int>(p / pieces_per_row);
    const int col = static_cast<int>(p - static_cast<int64_t>(t) * pieces_per_row);
    float acc[n];
#pragma unroll
    for (int i = 0; i < n; ++i) acc[i] = 0.f;
    for (int j = 0; j < top_k; ++j) {
      const int r = inv_perm[static_cast<int64_t>(t) * top_k + j];
      if (r >= 0) {
        const float w = gate_w[static_cast<int64_t>(t) * top_k + j];
        float f[n];
        Elems<TIn>::widen(
            __builtin_nontemporal_load(y + static_cast<int64_t>(r) * pieces_per_row + col), f);
#pragma unroll
        for (int i = 0; i < n; ++i) acc[i] = fmaf(w, f[i], acc[i]);
      }
    }
    TOut* o = out + static_cast<int64_t>(t) * d + static_cast<int64_t>(col) * n;
    if constexpr (sizeof(TOut) == 2) {
      static_assert(n == 8, "bf16 output comes from bf16 input");
      u32x4 v;
      v.x = pack_bf16x2(acc[0], acc[1]);
      v.y = pack_bf16x2(acc[2], acc[3]);
      v.z = pack_bf16x2(acc[4], acc[5]);
      v.w = pack_bf16x2(acc[6], acc[7]);
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(o));
    } else {
#pragma unroll
      for (int i = 0; i < n; i += 4) {
        f32x4 v = {acc[i], acc[i + 1], acc[i + 2], acc[i + 3]};
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(o + i));
      }
    }
  }
}

hipError_t launch_combine(const moe_config& c, const void* y_sliced, const int32_t* inv_perm,
                          const float* gate_w, void* out, hipStream_t s) {
  if (c.T == 0) return hipSuccess;
  const int n = c.in_dtype == MOE_BF16 ? 8 : 4;
  int64_t total = static_cast<int64_t>(c.T) * (c.d / n);
  int64_t want = (total + kCopyThreads - 1) / kCopyThreads;
  int blocks = static_cast<int>(want < 256 * 32 ? want : 256 * 32);
  const u32x4* y = static_cast<const u32x4*>(y_sliced);
  if (c.in_dtype == MOE_BF16 && c.out_dtype == MOE_BF16)
    combine_kernel<bf16_t, bf16_t><<<blocks, kCopyThreads, 0, s>>>(
        y, inv_perm, gate_w, static_cast<bf16_t*>(out), c.T, c.d, c.top_k);
  else if (c.in_dtype == MOE_BF16)
    combine_kernel<bf16_t, float><<<blocks, kCopyThreads, 0, s>>>(
        y, inv_perm, gate_w, static_cast<float*>(out), c.T, c.d, c.top_k);
  else
    combine_kernel<float, float><<<blocks, kCopyThreads, 0, s>>>(
        y, inv_perm, gate_w, static_cast<float*>(out), c.T, c.d, c.top_k);
  return hipGetLastError();
}

}  // namespace ppmoe
