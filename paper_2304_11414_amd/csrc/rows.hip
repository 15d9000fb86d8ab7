// The two row-movement kernels of the layer, both bound by HBM bandwidth:
//   slice   -- x_sliced[r, :] = x[perm[r] / k, :], the index selection that replaces the first
//              all-to-all (Sections 3.3.1, 3.3.3; Algorithm 1: hidden_states.index_select);
//   combine -- out[t, :] = sum_j gate_w[t, j] * y_sliced[inv_perm[t, j], :], the placement of the
//              expert outputs into a zero-initialised output that replaces the second all-to-all
//              (Algorithm 1: zeros_like + index assignment).  It is written as a gather per output
//              row, so each row of `out` is stored exactly once, zeros included: no atomics, no
//              separate memset, bitwise reproducible.
// Rows are moved as 16-byte pieces; a block owns a few rows per iteration so that enough loads are in
// flight per CU.

#include "common.h"

namespace ppmoe {

constexpr int kCopyThreads = 256;

// ---- slice ------------------------------------------------------------------------------------

// Measured on 67 MB (T=8192, d=2048) and 1.3 GB (T=32768, d=5120, top-2) of rows, launches replayed from
// a graph: the slice is fastest with 8 rows per block iteration (8 x 16 bytes in flight per thread)
// and up to 16 blocks per CU; the combine, which has a dependent index load in front of every row
// load, with one row per block iteration and up to 32 blocks per CU (more blocks hide that chain).
constexpr int kRowsPerIter = 8;    // slice: rows a block moves per iteration
constexpr int kSliceBlocksPerCu = 16;
constexpr int kCombineRows = 1;    // combine: output rows a block produces per iteration
constexpr int kCombineBlocksPerCu = 32;

__global__ __launch_bounds__(kCopyThreads) void slice_rows_kernel(
    const u32x4* __restrict__ x, const int32_t* __restrict__ perm,
    const int32_t* __restrict__ offsets, u32x4* __restrict__ x_sliced, int n_local, int top_k,
    int chunks_per_row /* d * sizeof(elem) / 16 */, int max_rows, int T) {
  // The row count lives on the device.  It is not waited for before the first loads go out: perm is
  // read for every row below max_rows (stale entries past the real count are clamped to a valid
  // token and their copies dropped at the store), so the loads of offsets, perm and x overlap.
  const int total_rows = offsets[n_local];
  for (int r0 = blockIdx.x * kRowsPerIter; r0 < max_rows; r0 += gridDim.x * kRowsPerIter) {
    const u32x4* src[kRowsPerIter];
#pragma unroll
    for (int i = 0; i < kRowsPerIter; ++i) {
      const int r = min(r0 + i, max_rows - 1);
      const int a = perm[r];
      const int t = top_k == 1 ? a : a / top_k;
      src[i] = x + static_cast<int64_t>(min(max(t, 0), T - 1)) * chunks_per_row;
    }
    for (int col = threadIdx.x; col < chunks_per_row; col += kCopyThreads) {
      u32x4 v[kRowsPerIter];
#pragma unroll
      for (int i = 0; i < kRowsPerIter; ++i) v[i] = __builtin_nontemporal_load(src[i] + col);
#pragma unroll
      for (int i = 0; i < kRowsPerIter; ++i)
        if (r0 + i < total_rows)
          __builtin_nontemporal_store(v[i], x_sliced + static_cast<int64_t>(r0 + i) * chunks_per_row + col);
    }
    if (r0 + gridDim.x * kRowsPerIter >= total_rows) break;   // uniform: nothing left for this block
  }
}

hipError_t launch_slice(const moe_config& c, const void* x, const int32_t* perm,
                        const int32_t* offsets, void* x_sliced, int64_t max_rows, hipStream_t s) {
  if (max_rows == 0 || c.T == 0) return hipSuccess;
  const int elem = is_16bit(c.in_dtype) ? 2 : 4;
  const int chunks_per_row = c.d * elem / 16;
  int64_t want = (max_rows + kRowsPerIter - 1) / kRowsPerIter;
  int blocks = static_cast<int>(want < 256 * kSliceBlocksPerCu ? want : 256 * kSliceBlocksPerCu);
  slice_rows_kernel<<<blocks, kCopyThreads, 0, s>>>(
      static_cast<const u32x4*>(x), perm, offsets, static_cast<u32x4*>(x_sliced), c.local_count,
      c.top_k, chunks_per_row, static_cast<int>(max_rows), c.T);
  return hipGetLastError();
}

// ---- zero rows of the output (fused layer path) ---------------------------------------------
// When the second GEMM places the expert outputs itself (top-1), rows of tokens without a kept local
// pick are written by nobody: they are set to +0 here (Algorithm 1's zeros_like).
__global__ __launch_bounds__(kCopyThreads) void zero_unrouted_rows_kernel(
    const int32_t* __restrict__ inv_perm, u32x4* __restrict__ out, int T, int chunks_per_row) {
  for (int t = blockIdx.x; t < T; t += gridDim.x) {
    if (inv_perm[t] >= 0) continue;   // (uniform: one row per block iteration)
    for (int col = threadIdx.x; col < chunks_per_row; col += kCopyThreads)
      __builtin_nontemporal_store(u32x4{0u, 0u, 0u, 0u}, out + static_cast<int64_t>(t) * chunks_per_row + col);
  }
}

hipError_t launch_zero_unrouted_rows(const moe_config& c, const int32_t* inv_perm, void* out,
                                     hipStream_t s) {
  if (c.T == 0) return hipSuccess;
  const int elem = is_16bit(c.out_dtype) ? 2 : 4;
  const int blocks = c.T < 256 * 16 ? c.T : 256 * 16;
  zero_unrouted_rows_kernel<<<blocks, kCopyThreads, 0, s>>>(inv_perm, static_cast<u32x4*>(out), c.T,
                                                            c.d * elem / 16);
  return hipGetLastError();
}

// ---- plain copy (reference kernel of known traffic, for calibrating hardware byte counters) ----

__global__ __launch_bounds__(kCopyThreads) void copy_bytes_kernel(const u32x4* __restrict__ src,
                                                                  u32x4* __restrict__ dst,
                                                                  int64_t pieces) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kCopyThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kCopyThreads + threadIdx.x; i < pieces; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

hipError_t launch_copy_bytes(const void* src, void* dst, int64_t bytes, hipStream_t s) {
  const int64_t pieces = bytes / 16;
  if (pieces == 0) return hipSuccess;
  int64_t want = (pieces + kCopyThreads - 1) / kCopyThreads;
  // four blocks per CU: the fastest of the grid sizes and unroll factors tried on a 1 GiB copy
  int blocks = static_cast<int>(want < 256 * 4 ? want : 256 * 4);
  copy_bytes_kernel<<<blocks, kCopyThreads, 0, s>>>(static_cast<const u32x4*>(src),
                                                    static_cast<u32x4*>(dst), pieces);
  return hipGetLastError();
}

// ---- combine ----------------------------------------------------------------------------------

// A thread produces 16 bytes of each output row it works on (n = 8 bf16 or 4 float32 elements), so
// that the lanes of a wavefront store one contiguous kilobyte per instruction whatever the input
// type; it reads the matching n elements of y: 16 bytes, or 8 when bf16 is combined into float32.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// DIN / DOUT: moe_dtype of y_sliced and of out.
template <int DIN, int N>
struct Piece;
template <int DIN>
struct Piece<DIN, 8> {   // eight 16-bit elements
  typedef u32x4 type;
  __device__ static void widen(const u32x4& v, float* f) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) Elem16<DIN>::widen2(w[i], f[2 * i], f[2 * i + 1]);
  }
};
template <int DIN>
struct Piece<DIN, 4> {   // four 16-bit elements
  typedef u32x2 type;
  __device__ static void widen(const u32x2& v, float* f) {
    Elem16<DIN>::widen2(v.x, f[0], f[1]);
    Elem16<DIN>::widen2(v.y, f[2], f[3]);
  }
};
template <>
struct Piece<MOE_F32, 4> {
  typedef u32x4 type;
  __device__ static void widen(const u32x4& v, float* f) {
    f[0] = __uint_as_float(v.x);
    f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z);
    f[3] = __uint_as_float(v.w);
  }
};

// A block produces kCombineRows output rows per iteration.
template <int DIN, int DOUT>
__global__ __launch_bounds__(kCopyThreads) void combine_kernel(
    const void* __restrict__ y_sliced, const int32_t* __restrict__ inv_perm,
    const float* __restrict__ gate_w, void* __restrict__ out_v, int T, int d, int top_k, int skip_single) {
  constexpr int out_bytes = DOUT == MOE_F32 ? 4 : 2;
  constexpr int n = 16 / out_bytes;
  typedef Piece<DIN, n> P;
  const typename P::type* __restrict__ y = static_cast<const typename P::type*>(y_sliced);
  unsigned char* out = static_cast<unsigned char*>(out_v);
  const int pieces_per_row = d / n;
  for (int t0 = blockIdx.x * kCombineRows; t0 < T; t0 += gridDim.x * kCombineRows) {
    // Rows already in place (skip_single: tokens with exactly one kept local pick, stored by the
    // second expert GEMM) are neither read nor written.  (Uniform over the block.)
    bool skip[kCombineRows];
#pragma unroll
    for (int i = 0; i < kCombineRows; ++i) {
      skip[i] = false;
      if (skip_single && t0 + i < T) {
        int kept = 0;
        for (int j = 0; j < top_k; ++j) kept += inv_perm[static_cast<int64_t>(t0 + i) * top_k + j] >= 0;
        skip[i] = kept == 1;
      }
    }
    for (int col = threadIdx.x; col < pieces_per_row; col += kCopyThreads) {
      float acc[kCombineRows][n];
#pragma unroll
      for (int i = 0; i < kCombineRows; ++i) {
#pragma unroll
        for (int e = 0; e < n; ++e) acc[i][e] = 0.f;
        if (skip[i]) continue;
        const int t = min(t0 + i, T - 1);
        for (int j = 0; j < top_k; ++j) {
          const int r = inv_perm[static_cast<int64_t>(t) * top_k + j];
          if (r >= 0) {
            const float w = gate_w[static_cast<int64_t>(t) * top_k + j];
            float f[n];
            P::widen(__builtin_nontemporal_load(y + static_cast<int64_t>(r) * pieces_per_row + col), f);
#pragma unroll
            for (int e = 0; e < n; ++e) acc[i][e] = fmaf(w, f[e], acc[i][e]);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < kCombineRows; ++i) {
        if (t0 + i >= T) continue;
        if (skip[i]) continue;
        unsigned char* o = out + (static_cast<int64_t>(t0 + i) * pieces_per_row + col) * 16;
        if constexpr (DOUT != MOE_F32) {
          u32x4 v;
          v.x = Elem16<DOUT>::pack2(acc[i][0], acc[i][1]);
          v.y = Elem16<DOUT>::pack2(acc[i][2], acc[i][3]);
          v.z = Elem16<DOUT>::pack2(acc[i][4], acc[i][5]);
          v.w = Elem16<DOUT>::pack2(acc[i][6], acc[i][7]);
          __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(o));
        } else {
          f32x4 v = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
          __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(o));
        }
      }
    }
  }
}

hipError_t launch_combine(const moe_config& c, const void* y_sliced, const int32_t* inv_perm,
                          const float* gate_w, void* out, hipStream_t s, bool skip_single) {
  if (c.T == 0) return hipSuccess;
  int64_t want = (static_cast<int64_t>(c.T) + kCombineRows - 1) / kCombineRows;
  int blocks = static_cast<int>(want < 256 * kCombineBlocksPerCu ? want : 256 * kCombineBlocksPerCu);
#define PPMOE_COMBINE(DIN, DOUT)                                  \
  combine_kernel<DIN, DOUT><<<blocks, kCopyThreads, 0, s>>>(y_sliced, inv_perm, gate_w, out, c.T, c.d, c.top_k, \
                                                            skip_single ? 1 : 0)
  if (c.in_dtype == MOE_BF16 && c.out_dtype == MOE_BF16) PPMOE_COMBINE(MOE_BF16, MOE_BF16);
  else if (c.in_dtype == MOE_BF16) PPMOE_COMBINE(MOE_BF16, MOE_F32);
  else if (c.in_dtype == MOE_F16 && c.out_dtype == MOE_F16) PPMOE_COMBINE(MOE_F16, MOE_F16);
  else if (c.in_dtype == MOE_F16) PPMOE_COMBINE(MOE_F16, MOE_F32);
  else PPMOE_COMBINE(MOE_F32, MOE_F32);
#undef PPMOE_COMBINE
  return hipGetLastError();
}

}  // namespace ppmoe
